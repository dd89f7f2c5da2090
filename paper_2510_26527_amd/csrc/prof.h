// Kernel launch helper with optional per-launch timing (psd_profile_enable / psd_profile_collect).
// A launcher names the kind of the kernels it is about to launch with ScopedProf; launch_kernel then
// starts the kernel normally, or - when recording - with a start and a stop event attached to the
// dispatch itself, which time the kernel alone (no launch gap in the figure).
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

namespace psd {

void prof_set_kind(int kind);
bool prof_acquire(hipEvent_t *start, hipEvent_t *stop);   // true: a slot was reserved, time this launch

struct ScopedProf {
    ScopedProf(int kind, hipStream_t) { prof_set_kind(kind); }
    ~ScopedProf() { prof_set_kind(-1); }
};

template <typename... KArgs, typename... Args>
inline void launch_kernel(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t shmem, hipStream_t stream,
                          Args... args) {
    hipEvent_t e0, e1;
    if (prof_acquire(&e0, &e1))
        hipExtLaunchKernelGGL(kernel, grid, block, (unsigned)shmem, stream, e0, e1, 0, static_cast<KArgs>(args)...);
    else
        hipLaunchKernelGGL(kernel, grid, block, (unsigned)shmem, stream, static_cast<KArgs>(args)...);
}

}  // namespace psd
