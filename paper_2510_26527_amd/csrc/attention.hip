// Verify attention on gfx950: the n_new query rows of a verify step against the model's KV
// cache, causal among the new rows, grouped-query heads sharing their K/V loads.
//
//   attn_simple_kernel   any dtype, one wavefront per (sequence, row, head): scores to LDS,
//                        softmax, then P.V.  Used by fp32 models (parity, not speed).
//   attn_mfma_kernel     bf16.  Split over the KV length (grid.x) and, inside a block, over its
//                        four wavefronts; each wavefront streams 64-key tiles of K and of the
//                        transposed V straight from HBM into MFMA operand registers with
//                        16-byte loads, computes S^T = K Q^T and O^T += V^T P^T on the matrix
//                        cores for up to 32 (d_head 128) or 64 (d_head 64) query rows - all heads
//                        of the group x all new rows; queries and probabilities go in as bf16
//                        hi + lo pairs, the cache operands as stored -
//                        and keeps an online softmax per query column with two cross-lane
//                        shuffles.  Wavefronts are merged through LDS in a fixed order, splits
//                        by attn_combine_kernel.
//
// Why V is stored transposed ([d_head][max_len]): the contraction index of P.V is the key, and an
// MFMA operand wants 8 consecutive contraction values per lane; with V^T those are one 16-byte
// load, and the score accumulator of S^T = K Q^T already holds P^T in exactly the operand layout
// the second MFMA needs (keys are numbered kb + 8g + 4t + v so that the two 16-key score tiles
// of a lane are 8 consecutive keys).
#include <cstdlib>
#include "common.h"
#include "kernels.h"
#include "prof.h"
#include "../../include/psd.h"

namespace psd {
namespace {

template <typename TC>
__global__ __launch_bounds__(64) void attn_simple_kernel(AttnArgs a, float scale) {
    extern __shared__ float sc[];
    const int lane = threadIdx.x;
    const int h = blockIdx.x, m = blockIdx.y, b = m / a.R, r = m % a.R;
    const int d_h = a.d_h;
    const int n_keys = min(a.lens[b] + r + 1, a.max_len);
    const int hk = h / (a.h_q / a.h_kv);
    const float *q = a.q + ((size_t)m * a.h_q + h) * d_h;
    const TC *K = (const TC *)a.k + ((size_t)b * a.h_kv + hk) * a.max_len * d_h;
    const TC *Vt = (const TC *)a.v + ((size_t)b * a.h_kv + hk) * d_h * (size_t)a.max_len;
    float mx = -INFINITY;
    for (int k = lane; k < n_keys; k += 64) {
        float s = 0.f;
        for (int d = 0; d < d_h; ++d) s += q[d] * load_elem(K, (size_t)k * d_h + d);
        s *= scale;
        sc[k] = s;
        mx = fmaxf(mx, s);
    }
    mx = wave_max(mx);
    float sum = 0.f;
    for (int k = lane; k < n_keys; k += 64) {
        const float e = expf(sc[k] - mx);
        sc[k] = e;
        sum += e;
    }
    sum = wave_sum(sum);
    __syncthreads();
    float *out = a.out + ((size_t)m * a.h_q + h) * d_h;
    for (int d = lane; d < d_h; d += 64) {
        float acc = 0.f;
        for (int k = 0; k < n_keys; ++k) acc += sc[k] * load_elem(Vt, (size_t)d * a.max_len + k);
        out[d] = acc / sum;
    }
}

constexpr int kKeysPerWaveIter = 64;
constexpr int kKeysPerBlockIter = 256;

template <int DH, int QT>
__global__ __launch_bounds__(256) void attn_mfma_kernel(AttnArgs a, float scale_log2, int range) {
    constexpr int KS = DH / 32;      // MFMA k-steps of S^T = K Q^T
    constexpr int DT = DH / 16;      // 16-row d tiles of O^T
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int split = blockIdx.x, qchunk = blockIdx.y;
    const int b = blockIdx.z / a.h_kv, hk = blockIdx.z % a.h_kv;
    const int group = a.h_q / a.h_kv;
    const int NQ = group * a.R;
    const int S_b = a.lens[b];
    const int n_keys = min(S_b + a.R, a.max_len);
    const int kb0 = split * range, kb1 = min(n_keys, kb0 + range);
    const size_t max_len = a.max_len;
    const uint16_t *Kc = (const uint16_t *)a.k + ((size_t)b * a.h_kv + hk) * max_len * DH;
    const uint16_t *Vt = (const uint16_t *)a.v + ((size_t)b * a.h_kv + hk) * DH * max_len;

    // Q operand (B of S^T = K Q^T): column i of tile qt is query q0 + qt*16 + i; lane group g
    // holds d_head elements [g*DH/4, (g+1)*DH/4), k-step s the 8 starting at 8*s inside them.
    bf16x8 qh[QT][KS], ql[QT][KS];
    int limit[QT];                   // last key this lane's query may see, -1 for a padding column
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int qi = (qchunk * QT + qt) * 16 + i;
        const bool valid = qi < NQ;
        const int hl = valid ? qi / a.R : 0, r = valid ? qi % a.R : 0;
        limit[qt] = valid ? S_b + r : -1;
        const float *qp = a.q + (((size_t)(b * a.R + r)) * a.h_q + hk * group + hl) * DH + g * (DH / 4);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            f32x8 v = load_f32x8(qp + 8 * s);
            if (!valid) v = f32x8{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            split_bf16(v, &qh[qt][s], &ql[qt][s]);
        }
    }

    f32x4 o[QT][DT];
    float mrun[QT], lrun[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        mrun[qt] = -INFINITY;
        lrun[qt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[qt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    for (int kt = kb0 + wave * kKeysPerWaveIter; kt < kb1; kt += kKeysPerBlockIter) {
        // issue every K and V^T load of this 64-key tile before the first MFMA (two 32-key halves)
        bf16x8 ka[2][2][KS];
        bf16x8 va[2][DT];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            // a half that starts at or beyond kb1 is fully masked; clamp its address into the tile's first half
            const int kb = (kt + sub * 32 < kb1) ? kt + sub * 32 : kt;
            // K rows of the two 16-key score tiles: row i of tile t is key kb + 8*(i/4) + 4*t + i%4
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int key = kb + 8 * (i >> 2) + 4 * t + (i & 3);     // < max_len: kb + 32 <= max_len
                const uint16_t *kp = Kc + (size_t)key * DH + g * (DH / 4);
#pragma unroll
                for (int s = 0; s < KS; ++s) ka[sub][t][s] = *reinterpret_cast<const bf16x8 *>(kp + 8 * s);
            }
            // V^T rows d = dt*16 + i, keys kb + 8g .. kb + 8g + 7
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
                va[sub][dt] = *reinterpret_cast<const bf16x8 *>(Vt + (size_t)(dt * 16 + i) * max_len + kb + 8 * g);
        }
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const int kb = kt + sub * 32;
            if (kb >= kb1) break;
            if (kb + 32 > n_keys) {          // stale cache rows may hold anything, even NaN: zero them
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    u32x4 raw = __builtin_bit_cast(u32x4, va[sub][dt]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int key = kb + 8 * g + 2 * e;
                        if (key >= n_keys) raw[e] = 0u;
                        else if (key + 1 >= n_keys) raw[e] &= 0xffffu;
                    }
                    va[sub][dt] = __builtin_bit_cast(bf16x8, raw);
                }
            }
            // scores of every query tile first, MFMAs interleaved over independent accumulators
            f32x4 c[QT][2];
#pragma unroll
            for (int qt = 0; qt < QT; ++qt)
#pragma unroll
                for (int t = 0; t < 2; ++t) c[qt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < KS; ++s) {
#pragma unroll
                for (int qt = 0; qt < QT; ++qt)
#pragma unroll
                    for (int t = 0; t < 2; ++t)
                        c[qt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[sub][t][s], qh[qt][s], c[qt][t], 0, 0, 0);
#pragma unroll
                for (int qt = 0; qt < QT; ++qt)
#pragma unroll
                    for (int t = 0; t < 2; ++t)
                        c[qt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[sub][t][s], ql[qt][s], c[qt][t], 0, 0, 0);
            }
            bf16x8 ph[QT], pl[QT];
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) {
                // lane (query column i, group g): c[qt][t][v] is key kb + 8g + 4t + v
                float tmax = -INFINITY;
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int key = kb + 8 * g + 4 * t + v;
                        const float sc = key <= limit[qt] ? c[qt][t][v] * scale_log2 : -INFINITY;
                        c[qt][t][v] = sc;
                        tmax = fmaxf(tmax, sc);
                    }
                tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
                tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
                const float mnew = fmaxf(mrun[qt], tmax);
                float p[8];
                if (mnew > -INFINITY) {
                    const float alpha = __builtin_amdgcn_exp2f(mrun[qt] - mnew);
                    float ps = 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        p[e] = __builtin_amdgcn_exp2f(c[qt][e >> 2][e & 3] - mnew);
                        ps += p[e];
                    }
                    lrun[qt] = lrun[qt] * alpha + ps;
                    if (mnew != mrun[qt]) {             // the running max moved: rescale the accumulators
#pragma unroll
                        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                            for (int v = 0; v < 4; ++v) o[qt][dt][v] *= alpha;
                    }
                    mrun[qt] = mnew;
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) p[e] = 0.f;
                }
                split_bf16(f32x8{p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7]}, &ph[qt], &pl[qt]);
            }
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int qt = 0; qt < QT; ++qt)
                    o[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[sub][dt], ph[qt], o[qt][dt], 0, 0, 0);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int qt = 0; qt < QT; ++qt)
                    o[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[sub][dt], pl[qt], o[qt][dt], 0, 0, 0);
        }
    }

    // ---- merge the four wavefronts in wavefront order through LDS
    __shared__ float sm_o[QT * 16][DH + 1];
    __shared__ float sm_m[QT * 16], sm_l[QT * 16];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        lrun[qt] += __shfl_xor(lrun[qt], 16, 64);
        lrun[qt] += __shfl_xor(lrun[qt], 32, 64);
    }
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) {
                const int qc = qt * 16 + i;
                float fo = 0.f, fn = 1.f, M = mrun[qt], L = lrun[qt];
                if (w > 0) {
                    const float mo = sm_m[qc], lo = sm_l[qc];
                    M = fmaxf(mo, mrun[qt]);
                    fo = mo > -INFINITY ? __builtin_amdgcn_exp2f(mo - M) : 0.f;
                    fn = mrun[qt] > -INFINITY ? __builtin_amdgcn_exp2f(mrun[qt] - M) : 0.f;
                    L = lo * fo + lrun[qt] * fn;
                }
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int d = dt * 16 + 4 * g + v;
                        const float mine = o[qt][dt][v] * fn;
                        sm_o[qc][d] = w > 0 ? sm_o[qc][d] * fo + mine : mine;
                    }
                __builtin_amdgcn_wave_barrier();
                if (g == 0) { sm_m[qc] = M; sm_l[qc] = L; }
            }
        }
        __syncthreads();
    }

    // ---- write: directly when there is one split, else the unnormalised partial
    for (int e = threadIdx.x; e < QT * 16 * DH; e += 256) {
        const int qc = e / DH, d = e % DH;
        const int qi = qchunk * QT * 16 + qc;
        if (qi >= NQ) continue;
        const int hl = qi / a.R, r = qi % a.R;
        const size_t row = ((size_t)(b * a.R + r)) * a.h_q + hk * group + hl;       // [B][R][h_q]
        if (a.splits == 1) {
            a.out[row * DH + d] = sm_o[qc][d] / sm_l[qc];
        } else {
            a.part_o[(row * a.splits + split) * DH + d] = sm_o[qc][d];
            if (d == 0) {
                a.part_ml[(row * a.splits + split) * 2] = sm_m[qc];
                a.part_ml[(row * a.splits + split) * 2 + 1] = sm_l[qc];
            }
        }
    }
}

// Many query rows per KV head (grouped-query verify at batch, prefill): the four wavefronts of a
// block own different 16-row query tiles and all walk the same keys, so K and V^T tiles are staged in
// LDS once per block (16-byte global loads, next tile prefetched into registers during the MFMAs) and
// read from there as MFMA operands; K/V leave HBM once for up to 128 query rows.  No cross-wavefront
// merge is needed: each wavefront finishes its own query rows.
template <int DH, int QW>
__global__ __launch_bounds__(256) void attn_mfma_wide_kernel(AttnArgs a, float scale_log2, int range) {
    constexpr int KS = DH / 32, DT = DH / 16;
    constexpr int KSTRIDE = DH + 8;            // bf16 elements per staged K row (+16 B: conflict-free reads)
    constexpr int VSTRIDE = 64 + 8;            // bf16 elements per staged V^T row
    __shared__ __attribute__((aligned(16))) uint16_t Ks[64 * KSTRIDE];
    __shared__ __attribute__((aligned(16))) uint16_t Vs[DH * VSTRIDE];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int split = blockIdx.x, qchunk = blockIdx.y;
    const int b = blockIdx.z / a.h_kv, hk = blockIdx.z % a.h_kv;
    const int group = a.h_q / a.h_kv;
    const int NQ = group * a.R;
    const int S_b = a.lens[b];
    const int n_keys = min(S_b + a.R, a.max_len);
    const int kb0 = split * range, kb1 = min(n_keys, kb0 + range);
    const size_t max_len = a.max_len;
    const uint16_t *Kc = (const uint16_t *)a.k + ((size_t)b * a.h_kv + hk) * max_len * DH;
    const uint16_t *Vt = (const uint16_t *)a.v + ((size_t)b * a.h_kv + hk) * DH * max_len;

    bf16x8 qh[QW][KS], ql[QW][KS];
    int limit[QW];
    size_t out_row[QW];
#pragma unroll
    for (int qt = 0; qt < QW; ++qt) {
        const int qi = ((qchunk * 4 + wave) * QW + qt) * 16 + i;
        const bool valid = qi < NQ;
        const int hl = valid ? qi / a.R : 0, r = valid ? qi % a.R : 0;
        limit[qt] = valid ? S_b + r : -1;
        out_row[qt] = ((size_t)(b * a.R + r)) * a.h_q + hk * group + hl;
        const float *qp = a.q + out_row[qt] * DH + g * (DH / 4);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            f32x8 v = load_f32x8(qp + 8 * s);
            if (!valid) v = f32x8{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            split_bf16(v, &qh[qt][s], &ql[qt][s]);
        }
    }
    f32x4 o[QW][DT];
    float mrun[QW], lrun[QW];
#pragma unroll
    for (int qt = 0; qt < QW; ++qt) {
        mrun[qt] = -INFINITY;
        lrun[qt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[qt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // staging: K tile 64 keys x DH (DH/8 chunks of 16 B per key), V^T tile DH rows x 64 keys (8 chunks per row)
    constexpr int KCH = 64 * DH / 8 / 256, VCH = DH * 8 / 256;
    u32x4 kreg[KCH], vreg[VCH];
    auto load_tile = [&](int kt) {
#pragma unroll
        for (int c = 0; c < KCH; ++c) {
            const int chunk = tid + c * 256, key = chunk / (DH / 8), col = (chunk % (DH / 8)) * 8;
            kreg[c] = *reinterpret_cast<const u32x4 *>(Kc + (size_t)(kt + key) * DH + col);     // kt + 64 <= max_len
        }
#pragma unroll
        for (int c = 0; c < VCH; ++c) {
            const int chunk = tid + c * 256, d = chunk >> 3, col = (chunk & 7) * 8;
            u32x4 raw = *reinterpret_cast<const u32x4 *>(Vt + (size_t)d * max_len + kt + col);
            if (kt + 64 > n_keys) {          // stale cache columns may hold anything, even NaN: zero them
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int key = kt + col + 2 * e;
                    if (key >= n_keys) raw[e] = 0u;
                    else if (key + 1 >= n_keys) raw[e] &= 0xffffu;
                }
            }
            vreg[c] = raw;
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int c = 0; c < KCH; ++c) {
            const int chunk = tid + c * 256, key = chunk / (DH / 8), col = (chunk % (DH / 8)) * 8;
            *reinterpret_cast<u32x4 *>(&Ks[key * KSTRIDE + col]) = kreg[c];
        }
#pragma unroll
        for (int c = 0; c < VCH; ++c) {
            const int chunk = tid + c * 256, d = chunk >> 3, col = (chunk & 7) * 8;
            *reinterpret_cast<u32x4 *>(&Vs[d * VSTRIDE + col]) = vreg[c];
        }
    };

    if (kb0 < kb1) {
        load_tile(kb0);
        store_tile();
    }
    __syncthreads();
    for (int kt = kb0; kt < kb1; kt += 64) {
        if (kt + 64 < kb1) load_tile(kt + 64);
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const int kb = kt + sub * 32;
            if (kb >= kb1) break;
            bf16x8 ka[2][KS], va[DT];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int key = sub * 32 + 8 * (i >> 2) + 4 * t + (i & 3);
#pragma unroll
                for (int s = 0; s < KS; ++s)
                    ka[t][s] = *reinterpret_cast<const bf16x8 *>(&Ks[key * KSTRIDE + g * (DH / 4) + 8 * s]);
            }
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
                va[dt] = *reinterpret_cast<const bf16x8 *>(&Vs[(dt * 16 + i) * VSTRIDE + sub * 32 + 8 * g]);
            // scores of every query tile first, MFMAs interleaved over independent accumulators
            f32x4 c[QW][2];
#pragma unroll
            for (int qt = 0; qt < QW; ++qt)
#pragma unroll
                for (int t = 0; t < 2; ++t) c[qt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < KS; ++s) {
#pragma unroll
                for (int qt = 0; qt < QW; ++qt)
#pragma unroll
                    for (int t = 0; t < 2; ++t)
                        c[qt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[t][s], qh[qt][s], c[qt][t], 0, 0, 0);
#pragma unroll
                for (int qt = 0; qt < QW; ++qt)
#pragma unroll
                    for (int t = 0; t < 2; ++t)
                        c[qt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[t][s], ql[qt][s], c[qt][t], 0, 0, 0);
            }
            bf16x8 ph[QW], pl[QW];
#pragma unroll
            for (int qt = 0; qt < QW; ++qt) {
                // lane (query column i, group g): c[qt][t][v] is key kb + 8g + 4t + v
                float tmax = -INFINITY;
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int key = kb + 8 * g + 4 * t + v;
                        const float sc = key <= limit[qt] ? c[qt][t][v] * scale_log2 : -INFINITY;
                        c[qt][t][v] = sc;
                        tmax = fmaxf(tmax, sc);
                    }
                tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
                tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
                const float mnew = fmaxf(mrun[qt], tmax);
                float p[8];
                if (mnew > -INFINITY) {
                    const float alpha = __builtin_amdgcn_exp2f(mrun[qt] - mnew);
                    float ps = 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        p[e] = __builtin_amdgcn_exp2f(c[qt][e >> 2][e & 3] - mnew);
                        ps += p[e];
                    }
                    lrun[qt] = lrun[qt] * alpha + ps;
                    if (mnew != mrun[qt]) {             // the running max moved: rescale the accumulators
#pragma unroll
                        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                            for (int v = 0; v < 4; ++v) o[qt][dt][v] *= alpha;
                    }
                    mrun[qt] = mnew;
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) p[e] = 0.f;
                }
                split_bf16(f32x8{p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7]}, &ph[qt], &pl[qt]);
            }
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int qt = 0; qt < QW; ++qt)
                    o[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[dt], ph[qt], o[qt][dt], 0, 0, 0);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int qt = 0; qt < QW; ++qt)
                    o[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[dt], pl[qt], o[qt][dt], 0, 0, 0);
        }
        __syncthreads();
        if (kt + 64 < kb1) store_tile();
        __syncthreads();
    }

    // each wavefront writes its own query rows: lane (query i, group g) holds d = dt*16 + 4g + v
#pragma unroll
    for (int qt = 0; qt < QW; ++qt) {
        float L = lrun[qt];
        L += __shfl_xor(L, 16, 64);
        L += __shfl_xor(L, 32, 64);
        if (limit[qt] < 0) continue;
        if (a.splits == 1) {
            const float inv = 1.0f / L;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
                *reinterpret_cast<f32x4 *>(a.out + out_row[qt] * DH + dt * 16 + 4 * g) = o[qt][dt] * inv;
        } else {
            float *po = a.part_o + (out_row[qt] * a.splits + split) * DH;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) *reinterpret_cast<f32x4 *>(po + dt * 16 + 4 * g) = o[qt][dt];
            if (g == 0) {
                a.part_ml[(out_row[qt] * a.splits + split) * 2] = mrun[qt];
                a.part_ml[(out_row[qt] * a.splits + split) * 2 + 1] = L;
            }
        }
    }
}

// one block per (sequence, row, head); thread d merges the splits in split order
__global__ void attn_combine_kernel(AttnArgs a) {
    const size_t row = blockIdx.x;
    const int d = threadIdx.x, DH = a.d_h;
    const float *ml = a.part_ml + row * a.splits * 2;
    float M = -INFINITY;
    for (int s = 0; s < a.splits; ++s) M = fmaxf(M, ml[2 * s]);
    float L = 0.f, acc = 0.f;
    for (int s = 0; s < a.splits; ++s) {
        const float ms = ml[2 * s];
        if (!(ms > -INFINITY)) continue;
        const float f = __builtin_amdgcn_exp2f(ms - M);
        L += ml[2 * s + 1] * f;
        acc += a.part_o[(row * a.splits + s) * DH + d] * f;
    }
    a.out[row * DH + d] = acc / L;
}

// query tiles of 16 per block: bounded by registers (hi+lo query operands and fp32 outputs)
inline int q_tiles(int NQ, int d_h) { return NQ <= 16 ? 1 : ((NQ <= 32 || d_h > 64) ? 2 : 4); }

}  // namespace

// more than 32 query rows per KV head: the LDS-staged kernel, 64 or 128 rows per block
inline bool use_wide(int NQ) { return NQ > 32; }
inline int wide_rows(int NQ) { return NQ <= 64 ? 64 : 128; }

int attn_pick_splits(int dtype, int B, int R, int h_q, int h_kv, int d_h, int len_bound) {
    if (dtype != PSD_BF16) return 1;
    const int NQ = (h_q / h_kv) * R;
    const int QT = q_tiles(NQ, d_h);
    const int chunks = use_wide(NQ) ? (NQ + wide_rows(NQ) - 1) / wide_rows(NQ) : (NQ + QT * 16 - 1) / (QT * 16);
    const int by_len = (len_bound + kKeysPerBlockIter - 1) / kKeysPerBlockIter;
    // the LDS-staged kernel loads its 64-128 query rows and writes as many partial rows per block: about one
    // block per CU keeps that overhead below the K/V bytes (measured at 16 x 4 KV heads x 4096 keys: 4 splits
    // 78 us, 8 splits 91 us, 16 splits 113 us per layer); the direct kernel has light blocks and wants many
    int by_grid = (use_wide(NQ) ? 256 : 1024) / (B * h_kv * chunks);
    if (by_grid < 1) by_grid = 1;
    int s = by_len < by_grid ? by_len : by_grid;
    return s < 1 ? 1 : s;
}

template <int DH>
static void launch_mfma(const AttnArgs &a, hipStream_t stream) {
    const int NQ = (a.h_q / a.h_kv) * a.R;
    const int QT = q_tiles(NQ, DH);
    const int chunks = (NQ + QT * 16 - 1) / (QT * 16);
    int range = (a.len_bound + a.splits - 1) / a.splits;
    range = (range + kKeysPerWaveIter - 1) / kKeysPerWaveIter * kKeysPerWaveIter;
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)DH);
    if (use_wide(NQ)) {
        const int rows = wide_rows(NQ);
        dim3 wgrid(a.splits, (NQ + rows - 1) / rows, a.B * a.h_kv);
        {
            ScopedProf sp(PSD_KIND_ATTN, stream);
            if (rows == 64) launch_kernel(attn_mfma_wide_kernel<DH, 1>, wgrid, 256, 0, stream, a, scale_log2, range);
            else launch_kernel(attn_mfma_wide_kernel<DH, 2>, wgrid, 256, 0, stream, a, scale_log2, range);
        }
        if (a.splits > 1) {
            ScopedProf sp(PSD_KIND_ATTN_COMBINE, stream);
            launch_kernel(attn_combine_kernel, a.B * a.R * a.h_q, DH, 0, stream, a);
        }
        return;
    }
    dim3 grid(a.splits, chunks, a.B * a.h_kv);
    {
    ScopedProf sp(PSD_KIND_ATTN, stream);
    if (QT == 1) launch_kernel(attn_mfma_kernel<DH, 1>, grid, 256, 0, stream, a, scale_log2, range);
    else if (QT == 2) launch_kernel(attn_mfma_kernel<DH, 2>, grid, 256, 0, stream, a, scale_log2, range);
    else if constexpr (DH <= 64) launch_kernel(attn_mfma_kernel<DH, 4>, grid, 256, 0, stream, a, scale_log2, range);
    }
    if (a.splits > 1) {
        ScopedProf sp(PSD_KIND_ATTN_COMBINE, stream);
        launch_kernel(attn_combine_kernel, a.B * a.R * a.h_q, DH, 0, stream, a);
    }
}

void launch_attention(int dtype, const AttnArgs &a, hipStream_t stream) {
    if (dtype == PSD_BF16 && (a.d_h == 128 || a.d_h == 64)) {
        if (a.d_h == 128) launch_mfma<128>(a, stream);
        else launch_mfma<64>(a, stream);
        return;
    }
    const float scale = 1.0f / sqrtf((float)a.d_h);
    dim3 grid(a.h_q, a.B * a.R);
    const size_t smem = (size_t)a.len_bound * sizeof(float);
    ScopedProf sp(PSD_KIND_ATTN, stream);
    if (dtype == PSD_BF16) launch_kernel(attn_simple_kernel<uint16_t>, grid, 64, smem, stream, a, scale);
    else launch_kernel(attn_simple_kernel<float>, grid, 64, smem, stream, a, scale);
}

}  // namespace psd
