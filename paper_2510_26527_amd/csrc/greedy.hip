// Greedy verification on gfx950 (temperature 0): the verification rule the paper lists beside
// speculative sampling in Sec. 3.1 and compares against in its ablation on acceptance-length
// variance.  A draft token is kept iff it equals the verifier's argmax at its position (lowest index
// among equal maxima); the first mismatch is replaced by that argmax; a fully matching block takes
// the argmax of the bonus row when there is one.
//
// Two launches: accept_argmax_kernel is the HBM-bound pass over the verifier's logits only (the
// drafter's rows and the uniforms are not read): per (row, chunk) the maximum raw logit and the lowest
// index attaining it; accept_greedy_finish_kernel merges the chunks per position and walks the block.
// Values are compared as stored (bf16 widened exactly), so the result is bit-exact.
#include <limits.h>

#include "common.h"
#include "kernels.h"
#include "prof.h"
#include "../../include/psd.h"

namespace psd {

namespace {

constexpr int kThreads = 256;
constexpr int kLoadsPerLane = 8;

__device__ __forceinline__ void take(float v, int idx, float &best, int &best_idx) {
    if (v > best || (v == best && idx < best_idx)) {
        best = v;
        best_idx = idx;
    }
}

template <typename T, bool VEC>
__global__ __launch_bounds__(kThreads) void accept_argmax_kernel(AcceptArgs a) {
    constexpr int EPL = VEC ? (int)(16 / sizeof(T)) : 1;
    const int tid = threadIdx.x;
    const int vec = blockIdx.x / a.n_chunksA, c = blockIdx.x % a.n_chunksA;
    const int b = vec / a.n_p_rows, r = vec % a.n_p_rows;
    const T *row = (const T *)a.p + (int64_t)b * a.p_stride + (int64_t)r * a.V;
    const int e0 = c * a.chunkA;
    const int e1 = min(a.V, e0 + a.chunkA);

    u32x4 raw[kLoadsPerLane];
    float sc[kLoadsPerLane];
    bool have[kLoadsPerLane];
#pragma unroll
    for (int i = 0; i < kLoadsPerLane; ++i) {
        const int idx = e0 + (i * kThreads + tid) * EPL;
        have[i] = idx < e1;                // chunk bounds and V are multiples of EPL: a vector load is whole
        if constexpr (VEC) {
            raw[i] = have[i] ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row + idx)) : u32x4{0u, 0u, 0u, 0u};
        } else {
            sc[i] = have[i] ? load_elem(row, idx) : -INFINITY;
        }
    }
    float best = -INFINITY;
    int best_idx = INT_MAX;
#pragma unroll
    for (int i = 0; i < kLoadsPerLane; ++i)
        if (have[i]) {
            const int idx = e0 + (i * kThreads + tid) * EPL;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                float v;
                if constexpr (!VEC) v = sc[i];
                else if constexpr (sizeof(T) == 2)
                    v = (e & 1) ? __uint_as_float(raw[i][e >> 1] & 0xffff0000u) : __uint_as_float(raw[i][e >> 1] << 16);
                else v = __uint_as_float(raw[i][e]);
                take(v, idx + e, best, best_idx);
            }
        }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float ov = __shfl_xor(best, off, 64);
        const int oi = __shfl_xor(best_idx, off, 64);
        take(ov, oi, best, best_idx);
    }
    __shared__ float sv[kThreads / 64];
    __shared__ int si[kThreads / 64];
    if ((tid & 63) == 0) {
        sv[tid >> 6] = best;
        si[tid >> 6] = best_idx;
    }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < kThreads / 64; ++w) take(sv[w], si[w], best, best_idx);
        a.stats[(size_t)vec * a.n_chunksA + c] = make_float2(best, __int_as_float(best_idx));
    }
}

// one block per sequence; thread j merges the chunks of position j, thread 0 walks the block
__global__ __launch_bounds__(128) void accept_greedy_finish_kernel(AcceptArgs a) {
    __shared__ int am[128];
    const int b = blockIdx.x, j = threadIdx.x;
    if (j < a.n_p_rows) {
        const float2 *st = a.stats + ((size_t)b * a.n_p_rows + j) * a.n_chunksA;
        float best = -INFINITY;
        int best_idx = INT_MAX;
        for (int c = 0; c < a.n_chunksA; ++c) take(st[c].x, __float_as_int(st[c].y), best, best_idx);
        am[j] = best_idx == INT_MAX ? 0 : best_idx;      // a row of NaNs only: index 0
    }
    __syncthreads();
    if (j == 0) {
        int n = 0;
        while (n < a.gamma && a.x[(size_t)b * a.gamma + n] == am[n]) ++n;
        a.out_n[b] = n;
        a.out_tok[b] = n < a.n_p_rows ? am[n] : -1;
        a.flags[b] = 0;
    }
}

template <typename T>
void launch_greedy_t(const AcceptArgs &a, bool vec_ok, hipStream_t stream) {
    dim3 grid((unsigned)a.rows * a.n_p_rows * a.n_chunksA);
    {
        ScopedProf sp(PSD_KIND_ACCEPT_STATS, stream);
        if (vec_ok) launch_kernel(accept_argmax_kernel<T, true>, grid, kThreads, 0, stream, a);
        else launch_kernel(accept_argmax_kernel<T, false>, grid, kThreads, 0, stream, a);
    }
    ScopedProf sp(PSD_KIND_ACCEPT_LOCATE, stream);
    launch_kernel(accept_greedy_finish_kernel, a.rows, 128, 0, stream, a);
}

}  // namespace

void launch_accept_greedy(const AcceptArgs &a, bool vec_ok, hipStream_t stream) {
    if (a.dtype == PSD_BF16) launch_greedy_t<uint16_t>(a, vec_ok, stream);
    else launch_greedy_t<float>(a, vec_ok, stream);
}

}  // namespace psd
