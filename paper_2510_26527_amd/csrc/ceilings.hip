// Measured ceilings of the machine, for stating roofline fractions against what the hardware delivers as well as
// against its published peaks (measurement aid, not part of the decoding path):
//   probe_read_kernel   a plain streaming read: every block walks an equal contiguous share of a buffer with
//                       non-temporal 16-byte loads, eight in flight per lane (the access pattern of the weight
//                       streaming and acceptance kernels, without any arithmetic);
//   probe_mfma_kernel   nothing but 32x32x16 bf16 matrix-core instructions on four independent accumulators per
//                       wavefront (the instruction of the tiled GEMM), operands held in registers.
#include "common.h"
#include "kernels.h"
#include "prof.h"
#include "../../include/psd.h"

namespace psd {
namespace {

__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4 *src, size_t n16, uint32_t *sink) {
    const size_t per_block = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t b0 = (size_t)blockIdx.x * per_block, b1 = b0 + per_block < n16 ? b0 + per_block : n16;
    uint32_t acc = 0;
    for (size_t i = b0 + threadIdx.x; i < b1; i += 256 * 8) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const size_t j = i + (size_t)u * 256;
            v[u] = j < b1 ? __builtin_nontemporal_load(src + j) : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    }
    if (acc == 0x12345678u) sink[0] = acc;        // keeps the loads alive; practically never taken
}

__global__ __launch_bounds__(256) void probe_mfma_kernel(const uint16_t *seed, float *sink, int iters) {
    // operands from memory, so that they are ordinary bf16 values of mixed magnitude rather than constants
    bf16x8 a = *reinterpret_cast<const bf16x8 *>(seed + (threadIdx.x & 63) * 8);
    bf16x8 b = *reinterpret_cast<const bf16x8 *>(seed + 512 + (threadIdx.x & 63) * 8);
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) s += acc[j][0];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

void launch_probe_read(const void *src, size_t bytes, void *sink, int blocks, hipStream_t stream) {
    launch_kernel(probe_read_kernel, blocks, 256, 0, stream, (const u32x4 *)src, bytes / 16, (uint32_t *)sink);
}
void launch_probe_mfma(const void *seed, void *sink, int blocks, int iters, hipStream_t stream) {
    launch_kernel(probe_mfma_kernel, blocks, 256, 0, stream, (const uint16_t *)seed, (float *)sink, iters);
}

}  // namespace psd
