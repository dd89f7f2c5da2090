// Optional per-launch timing with HIP events (psd_profile_enable / psd_profile_collect).
// When enabled every kernel launch of the library is bracketed by two events recorded on the
// launch stream; disabled (the default) it costs one branch per launch.
#pragma once
#include <hip/hip_runtime.h>

namespace psd {

void prof_begin(int kind, hipStream_t stream);
void prof_end(hipStream_t stream);

struct ScopedProf {
    hipStream_t st;
    ScopedProf(int kind, hipStream_t stream) : st(stream) { prof_begin(kind, st); }
    ~ScopedProf() { prof_end(st); }
};

}  // namespace psd
