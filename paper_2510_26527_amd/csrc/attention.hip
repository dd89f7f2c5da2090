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
//                        by attn_combine_kernel.  FUSED (at most 32 query rows per KV head): the kernel
//                        builds its own operands - it adds the QKV projection's partial sums, applies the
//                        RMSNorm row scale, rotates q and k by a (cos, sin) table, appends k and v to the
//                        cache and keeps the step's own rows in LDS as one more key tile - so no rotation /
//                        append kernel runs before it; a token tree's ancestor mask applies to that tile.
//   attn_mfma_wide_kernel  bf16, more query rows per KV head than that (grouped-query verify at batch,
//                        prefill): K / V^T tiles staged in LDS as fp16, one MFMA pass, each wavefront its
//                        own 16-row query tiles.
//
// Why V is stored transposed ([d_head][max_len]): the contraction index of P.V is the key, and an
// MFMA operand wants 8 consecutive contraction values per lane; with V^T those are one 16-byte
// load, and the score accumulator of S^T = K Q^T already holds P^T in exactly the operand layout
// the second MFMA needs (keys are numbered kb + 8g + 4t + v so that the two 16-key score tiles
// of a lane are 8 consecutive keys).
#include <cstdlib>
#include <type_traits>
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

// Sum over the S split-K slots (sstride floats apart) of NI pairs (src[it][0], src[it][second]) per thread.  The
// loads of SPC slots of all pairs are issued together; the additions run in slot order, the order in which the
// stand-alone rotation kernel adds them.  after_issue() runs once, between the first batch's loads and their use:
// loads the caller issues there queue up behind these and do not hold their return up.
template <int NI, typename F>
__device__ __forceinline__ void sum_pairs(const float *const *src, size_t sstride, int S, int second, float *x1, float *x2,
                                          F after_issue) {
    constexpr int SPC = 32 / NI;
#pragma unroll
    for (int it = 0; it < NI; ++it) x1[it] = x2[it] = 0.f;
    for (int sp0 = 0; sp0 < S; sp0 += SPC) {
        float t1[NI][SPC], t2[NI][SPC];
#pragma unroll
        for (int it = 0; it < NI; ++it)
#pragma unroll
            for (int u = 0; u < SPC; ++u) {
                const size_t off = (size_t)min(sp0 + u, S - 1) * sstride;
                t1[it][u] = src[it][off];
                t2[it][u] = src[it][off + second];
            }
        if (sp0 == 0) after_issue();
#pragma unroll
        for (int it = 0; it < NI; ++it)
#pragma unroll
            for (int u = 0; u < SPC; ++u)
                if (sp0 + u < S) { x1[it] += t1[it][u]; x2[it] += t2[it][u]; }
    }
}
// the same for a number of pairs known at run time (the first ni of up to 8)
template <typename F>
__device__ __forceinline__ void sum_pairs_n(int ni, const float *const *src, size_t sstride, int S, int second, float *x1, float *x2,
                                            F after_issue) {
    if (ni <= 1) sum_pairs<1>(src, sstride, S, second, x1, x2, after_issue);
    else if (ni <= 2) sum_pairs<2>(src, sstride, S, second, x1, x2, after_issue);
    else if (ni <= 4) sum_pairs<4>(src, sstride, S, second, x1, x2, after_issue);
    else sum_pairs<8>(src, sstride, S, second, x1, x2, after_issue);
}

// FUSED: the block builds its operands itself from the QKV projection's split-K partial sums: row scale of the
// folded RMSNorm, sum over the splits in split order, rotation with the (cos, sin) table of the step's positions.
// Every block does that for its own query rows; the blocks of the last split also build the step's new keys and
// values (<= 32 rows), keep them in LDS as one more 32-key tile, and the one with query chunk 0 appends them to
// the cache.  Cache reads then stop at the old length, so no block reads what another one is writing.
template <int DH, int QT, bool FUSED>
__global__ __launch_bounds__(256) void attn_mfma_kernel(AttnArgs a, float scale_log2, int range) {
    constexpr int KS = DH / 32;      // MFMA k-steps of S^T = K Q^T
    constexpr int DT = DH / 16;      // 16-row d tiles of O^T
    constexpr int HALF = DH / 2;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int split = blockIdx.x, qchunk = blockIdx.y;
    const int b = blockIdx.z / a.h_kv, hk = blockIdx.z % a.h_kv;
    const int group = a.h_q / a.h_kv;
    const int NQ = group * a.R;
    const int S_b = a.lens[b];
    const int n_keys = FUSED ? min(S_b, a.max_len) : min(S_b + a.R, a.max_len);      // keys read from the cache
    const int kb0 = split * range, kb1 = min(n_keys, kb0 + range);
    const size_t max_len = a.max_len;
    const uint16_t *Kc = (const uint16_t *)a.k + ((size_t)b * a.h_kv + hk) * max_len * DH;
    const uint16_t *Vt = (const uint16_t *)a.v + ((size_t)b * a.h_kv + hk) * DH * max_len;
    const bool new_tile = FUSED && split == (int)gridDim.x - 1;       // this block also attends to the new rows

    // LDS: the operand build (rotated queries, the new keys, the new values transposed) and, after the last tile,
    // the merge of the four wavefronts use the same bytes
    constexpr int NSLAB = QT == 1 ? 4 : 2;          // merge slabs: a wavefront each, or two wavefronts sharing one
    constexpr size_t kBuildBytes = FUSED ? (size_t)QT * 16 * (DH + 4) * 4 + 32 * (DH + 8) * 2 + (size_t)DH * 40 * 2 : 0;
    constexpr size_t kMergeBytes = (size_t)NSLAB * QT * 16 * (DH + 1) * 4 + 2 * NSLAB * QT * 16 * 4;
    __shared__ __attribute__((aligned(16))) unsigned char lds_raw[kBuildBytes > kMergeBytes ? kBuildBytes : kMergeBytes];
    float (*s_q)[DH + 4] = reinterpret_cast<float (*)[DH + 4]>(lds_raw);
    uint16_t (*s_k)[DH + 8] = reinterpret_cast<uint16_t (*)[DH + 8]>(lds_raw + (size_t)QT * 16 * (DH + 4) * 4);
    uint16_t (*s_vt)[40] = reinterpret_cast<uint16_t (*)[40]>(lds_raw + (size_t)QT * 16 * (DH + 4) * 4 + 32 * (DH + 8) * 2);
    __shared__ float s_scale[32];
    // the first 64-key tile of this wavefront is requested before anything else: its trip to HBM overlaps the
    // operand build below
    bf16x8 ka[2][2][KS];
    bf16x8 va[2][DT];
    auto load_tile = [&](int kt) {
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            // a half that starts at or beyond kb1 is fully masked; clamp its address into the tile's first half
            const int kb = (kt + sub * 32 < kb1) ? kt + sub * 32 : kt;
            // K rows of the two 16-key score tiles: row i of tile t is key kb + 8*(i/4) + 4*t + i%4
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int key = kb + 8 * (i >> 2) + 4 * t + (i & 3);     // < max_len: kb + 32 <= max_len
                // k-step s of the contraction takes d = 32 s + 8 g .. + 7: the four lane groups of a key read 64
                // contiguous bytes per load (fewer cache lines per instruction than a lane-group-major split of d)
                const uint16_t *kp = Kc + (size_t)key * DH + 8 * g;
#pragma unroll
                for (int s = 0; s < KS; ++s) ka[sub][t][s] = *reinterpret_cast<const bf16x8 *>(kp + 32 * s);
            }
            // V^T rows d = dt*16 + i, keys kb + 8g .. kb + 8g + 7
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
                va[sub][dt] = *reinterpret_cast<const bf16x8 *>(Vt + (size_t)(dt * 16 + i) * max_len + kb + 8 * g);
        }
    };
    // The wavefront's first K / V^T tile is requested ahead of the loop, so that it streams in while the operands are
    // built; but behind the loads the build waits for (returns are in order, and all blocks' tiles together are the
    // kernel's whole traffic: requested first, they would hold the build up for the time the cache takes to arrive).
    constexpr bool HOIST = QT == 1;            // two query tiles leave no registers to hold a tile across the build
    const int kt_first = kb0 + wave * kKeysPerWaveIter;
    auto hoisted_tile = [&]() {
        if (HOIST && kt_first < kb1) load_tile(kt_first);
    };
    if constexpr (!FUSED) hoisted_tile();

    if constexpr (FUSED) {
        const int tid = threadIdx.x;
        const int W = (a.h_q + 2 * a.h_kv) * DH;
        const size_t sstride = (size_t)a.B * a.R * W;
        const int S = a.qkv_splits;
        // Everything the build needs is requested before the first value is used: the sums of squares behind the
        // row scales, the (cos, sin) pairs, then the partial sums themselves.
        // RMSNorm scale of the step's rows of this sequence: one wavefront per row, the reduction order of the
        // stand-alone rotation kernel (lane-strided sum, then the butterfly)
        const bool few = a.R <= 8 && a.rs.tiles <= 256;            // then a lane holds all its terms at once
        float raw[2][4];
        if (a.rs.sumsq && few) {
#pragma unroll
            for (int rr = 0; rr < 2; ++rr)
#pragma unroll
                for (int tt = 0; tt < 4; ++tt) {
                    const int r = wave + 4 * rr, t = lane + 64 * tt;
                    raw[rr][tt] = r < a.R && t < a.rs.tiles ? a.rs.sumsq[(size_t)t * (a.B * a.R) + b * a.R + r] : 0.f;
                }
        }
        auto row_scales = [&]() {
            for (int r = wave; r < a.R; r += 4) {
                float sc = 1.0f;
                if (a.rs.sumsq) {
                    float ssq = 0.f;
                    if (few) {
#pragma unroll
                        for (int tt = 0; tt < 4; ++tt) ssq += r < 4 ? raw[0][tt] : raw[1][tt];
                    } else {
                        for (int t = lane; t < a.rs.tiles; t += 64) ssq += a.rs.sumsq[(size_t)t * (a.B * a.R) + b * a.R + r];
                    }
                    sc = 1.0f / sqrtf(wave_sum(ssq) * a.rs.inv_d + a.rs.eps);
                }
                if (lane == 0) s_scale[r] = sc;
            }
        };
        if (new_tile)                               // rows / columns past R of the new tile must read as zeros
            for (int e = tid; e < DH * 40; e += 256) {
                if (e < 32 * (DH + 8)) (&s_k[0][0])[e] = 0;
                (&s_vt[0][0])[e] = 0;
            }
        // queries of this block: (query, rotation pair) items, consecutive threads on consecutive pairs
        constexpr int NIQ = QT * 16 * HALF / 256;
        {
            const int nq = min(QT * 16, NQ - qchunk * QT * 16);       // queries of this block that exist
            const int ni = (nq * HALF + 255) / 256;
            const float *src[8];
            float x1[8], x2[8];
            float2 cs[NIQ];
            int rloc[NIQ];
#pragma unroll
            for (int it = 0; it < NIQ; ++it) {
                const int item = tid + it * 256, ql_ = item / HALF, pi = item % HALF;
                const int qi = qchunk * QT * 16 + ql_;
                const bool valid = qi < NQ;
                const int hl = valid ? qi / a.R : 0, r = valid ? qi % a.R : 0;
                rloc[it] = valid ? r : -1;
                src[it] = a.qkv_partial + (size_t)(b * a.R + r) * W + (size_t)(hk * group + hl) * DH + pi;
                cs[it] = a.rope_cs[(size_t)(b * a.R + r) * HALF + pi];
            }
            sum_pairs_n(ni, src, sstride, S, HALF, x1, x2, hoisted_tile);
            row_scales();
            __syncthreads();                        // s_scale
#pragma unroll
            for (int it = 0; it < NIQ; ++it) {
                const int item = tid + it * 256, ql_ = item / HALF, pi = item % HALF;
                float y1 = 0.f, y2 = 0.f;
                if (rloc[it] >= 0) {
                    const float sc = s_scale[rloc[it]];
                    const float v1 = x1[it] * sc, v2 = x2[it] * sc;
                    y1 = v1 * cs[it].x - v2 * cs[it].y;
                    y2 = v2 * cs[it].x + v1 * cs[it].y;
                }
                s_q[ql_][pi] = y1;
                s_q[ql_][pi + HALF] = y2;
            }
        }
        if (new_tile) {
            uint16_t *Kw = (uint16_t *)a.k + ((size_t)b * a.h_kv + hk) * max_len * DH;
            uint16_t *Vw = (uint16_t *)a.v + ((size_t)b * a.h_kv + hk) * DH * max_len;
            const bool writer = qchunk == 0;
            // keys: (row, rotation pair) items; values: (row, element pair) items; up to 32 rows x HALF of each.
            // With at most four items of each kind per thread both kinds are summed in one go.
            const int nik = (a.R * HALF + 255) / 256;               // 1 .. 8
            const bool both = nik <= 4;
            for (int pass = 0; pass < (both ? 1 : 2); ++pass) {
                const float *src[8];
                float x1[8], x2[8];
                float2 cs[8];
                // slot `it` of this pass: key items first, then (in a combined pass) the value items
                auto slot = [&](int it, bool *is_v, int *item) {
                    *is_v = both ? it >= nik : pass == 1;
                    *item = tid + (both && it >= nik ? it - nik : it) * 256;
                };
#pragma unroll
                for (int it = 0; it < 8; ++it) {
                    bool is_v;
                    int item;
                    slot(it, &is_v, &item);
                    const int r = min(item / HALF, a.R - 1), pi = item % HALF;
                    const int col0 = (is_v ? a.h_q + a.h_kv + hk : a.h_q + hk) * DH;
                    src[it] = a.qkv_partial + (size_t)(b * a.R + r) * W + col0 + pi;
                    cs[it] = a.rope_cs[(size_t)(b * a.R + r) * HALF + pi];
                }
                sum_pairs_n(both ? 2 * nik : nik, src, sstride, S, HALF, x1, x2, [] {});
#pragma unroll
                for (int it = 0; it < 8; ++it) {
                    bool is_v;
                    int item;
                    slot(it, &is_v, &item);
                    if (it >= (both ? 2 * nik : nik)) continue;
                    const int r = item / HALF, pi = item % HALF;
                    if (r >= a.R) continue;
                    const int pos = S_b + r;
                    const float sc = s_scale[r];
                    const float v1 = x1[it] * sc, v2 = x2[it] * sc;
                    if (!is_v) {
                        const uint16_t k1 = (uint16_t)f32_to_bf16_bits(v1 * cs[it].x - v2 * cs[it].y);
                        const uint16_t k2 = (uint16_t)f32_to_bf16_bits(v2 * cs[it].x + v1 * cs[it].y);
                        s_k[r][pi] = k1;
                        s_k[r][pi + HALF] = k2;
                        if (writer && pos < a.max_len) {
                            Kw[(size_t)pos * DH + pi] = k1;
                            Kw[(size_t)pos * DH + pi + HALF] = k2;
                        }
                    } else {
                        const uint16_t w1 = (uint16_t)f32_to_bf16_bits(v1), w2 = (uint16_t)f32_to_bf16_bits(v2);
                        s_vt[pi][r] = w1;
                        s_vt[pi + HALF][r] = w2;
                        if (writer && pos < a.max_len) {
                            Vw[(size_t)pi * max_len + pos] = w1;
                            Vw[(size_t)(pi + HALF) * max_len + pos] = w2;
                        }
                    }
                }
            }
        }
        __syncthreads();
    }

    // Q operand (B of S^T = K Q^T): column i of tile qt is query q0 + qt*16 + i; k-step s of lane group g
    // holds d_head elements 32 s + 8 g .. + 7, as the K operand does.
    bf16x8 qh[QT][KS], ql[QT][KS];
    int limit[QT];                   // last key this lane's query may see, -1 for a padding column
    uint32_t own_rows[QT];           // token tree: which rows of this step the query sees (bit j = row j); else unused
    uint32_t new_mask[QT];           // the mask in force for the tile being consumed: zero for cache tiles
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int qi = (qchunk * QT + qt) * 16 + i;
        const bool valid = qi < NQ;
        const int hl = valid ? qi / a.R : 0, r = valid ? qi % a.R : 0;
        limit[qt] = valid ? S_b + r : -1;
        own_rows[qt] = 0u;
        new_mask[qt] = 0u;
        if constexpr (FUSED) {
            if (a.tree_anc) {        // a node sees the cache and its ancestors among the step's rows
                limit[qt] = valid ? S_b - 1 : -1;
                own_rows[qt] = valid ? a.tree_anc[r] : 0u;
            }
        }
        const float *qp = FUSED ? &s_q[qt * 16 + i][8 * g]
                                : a.q + (((size_t)(b * a.R + r)) * a.h_q + hk * group + hl) * DH + 8 * g;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            f32x8 v = load_f32x8(qp + 32 * s);
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

    // one 32-key sub-tile: keys kb .. kb + 31, of which those below n_end exist; ka / va are its operands
    // (own_tile: the step's own rows, where a token tree's ancestor mask applies; a compile-time flag so that the
    // loop over the cache keeps the plain causal test)
    auto consume = [&](auto own_tile, int kb, int n_end, bf16x8 (&ka)[2][KS], bf16x8 (&va)[DT]) {
        if (kb + 32 > n_end) {          // stale cache rows may hold anything, even NaN: zero them
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                u32x4 raw = __builtin_bit_cast(u32x4, va[dt]);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int key = kb + 8 * g + 2 * e;
                    if (key >= n_end) raw[e] = 0u;
                    else if (key + 1 >= n_end) raw[e] &= 0xffffu;
                }
                va[dt] = __builtin_bit_cast(bf16x8, raw);
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
                    c[qt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[t][s], qh[qt][s], c[qt][t], 0, 0, 0);
#pragma unroll
            for (int qt = 0; qt < QT; ++qt)
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    c[qt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[t][s], ql[qt][s], c[qt][t], 0, 0, 0);
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
                    bool seen = key <= limit[qt];
                    if constexpr (decltype(own_tile)::value) seen = seen || ((new_mask[qt] >> ((key - kb) & 31)) & 1u);
                    const float sc = seen && key < n_end ? c[qt][t][v] * scale_log2 : -INFINITY;
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
                o[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[dt], ph[qt], o[qt][dt], 0, 0, 0);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int qt = 0; qt < QT; ++qt)
                o[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[dt], pl[qt], o[qt][dt], 0, 0, 0);
    };

    for (int kt = kt_first; kt < kb1; kt += kKeysPerBlockIter) {
        if (!HOIST || kt != kt_first) load_tile(kt); // every K and V^T load of the tile before its first MFMA
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const int kb = kt + sub * 32;
            if (kb >= kb1) break;
            consume(std::false_type{}, kb, n_keys, ka[sub], va[sub]);
        }
    }
    if constexpr (FUSED) {
        if (new_tile && wave == 3) {
            // the step's own rows as one more 32-key tile at positions S_b .. S_b + R - 1, operands from LDS
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int key = 8 * (i >> 2) + 4 * t + (i & 3);
#pragma unroll
                for (int s = 0; s < KS; ++s) ka[0][t][s] = *reinterpret_cast<const bf16x8 *>(&s_k[key][32 * s + 8 * g]);
            }
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) va[0][dt] = *reinterpret_cast<const bf16x8 *>(&s_vt[dt * 16 + i][8 * g]);
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) new_mask[qt] = own_rows[qt];
            consume(std::true_type{}, S_b, S_b + a.R, ka[0], va[0]);
        }
    }

    // ---- merge the four wavefronts through LDS: wavefront w goes to slab w % NSLAB, in round w / NSLAB (a later
    // round folds into what the slab holds); the slabs are combined in slab order when the result is written
    float (*sm_o)[QT * 16][DH + 1] = reinterpret_cast<float (*)[QT * 16][DH + 1]>(lds_raw);
    float (*sm_m)[QT * 16] = reinterpret_cast<float (*)[QT * 16]>(lds_raw + (size_t)NSLAB * QT * 16 * (DH + 1) * 4);
    float (*sm_l)[QT * 16] = sm_m + NSLAB;
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        lrun[qt] += __shfl_xor(lrun[qt], 16, 64);
        lrun[qt] += __shfl_xor(lrun[qt], 32, 64);
    }
    __syncthreads();                                // every wavefront is done with the build's LDS
    const int slab = wave % NSLAB;
    for (int round = 0; round < 4 / NSLAB; ++round) {
        if (wave / NSLAB == round) {
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) {
                const int qc = qt * 16 + i;
                float fo = 0.f, fn = 1.f, M = mrun[qt], L = lrun[qt];
                if (round > 0) {
                    const float mo = sm_m[slab][qc], lo = sm_l[slab][qc];
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
                        sm_o[slab][qc][d] = round > 0 ? sm_o[slab][qc][d] * fo + mine : mine;
                    }
                __builtin_amdgcn_wave_barrier();
                if (g == 0) { sm_m[slab][qc] = M; sm_l[slab][qc] = L; }
            }
        }
        __syncthreads();
    }

    // ---- write: directly when there is one split, else the unnormalised partial.  One thread per query row works
    // out where the row goes and how its slabs combine; the element loop then only multiplies and adds.
    __shared__ float s_f[NSLAB][QT * 16], s_M[QT * 16], s_L[QT * 16];
    __shared__ int s_row[QT * 16];
    if (threadIdx.x < QT * 16) {
        const int qc = threadIdx.x;
        const int qi = qchunk * QT * 16 + qc;
        int row = -1;
        if (qi < NQ) {
            const int hl = qi / a.R, r = qi % a.R;
            row = (b * a.R + r) * a.h_q + hk * group + hl;                           // [B][R][h_q]
        }
        float M = sm_m[0][qc];
#pragma unroll
        for (int sl = 1; sl < NSLAB; ++sl) M = fmaxf(M, sm_m[sl][qc]);
        float L = 0.f;
#pragma unroll
        for (int sl = 0; sl < NSLAB; ++sl) {
            const float ms = sm_m[sl][qc];
            const float f = ms > -INFINITY ? __builtin_amdgcn_exp2f(ms - M) : 0.f;
            s_f[sl][qc] = f;
            L += sm_l[sl][qc] * f;
        }
        s_row[qc] = row; s_M[qc] = M; s_L[qc] = L;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < QT * 16 * DH; e += 256) {
        const int qc = e / DH, d = e % DH;
        if (s_row[qc] < 0) continue;
        const size_t row = (size_t)s_row[qc];
        float acc = 0.f;
#pragma unroll
        for (int sl = 0; sl < NSLAB; ++sl) acc += sm_o[sl][qc][d] * s_f[sl][qc];
        if (a.splits == 1) {
            const float L = s_L[qc];
            a.out[row * DH + d] = acc / L;
            if (a.out16) a.out16[row * DH + d] = f32_to_f16_bits(acc / L);
        } else {
            a.part_o[(row * a.splits + split) * DH + d] = acc;
            if (d == 0) {
                a.part_ml[(row * a.splits + split) * 2] = s_M[qc];
                a.part_ml[(row * a.splits + split) * 2 + 1] = s_L[qc];
            }
        }
    }
}

// Many query rows per KV head (grouped-query verify at batch, prefill): the NW wavefronts of a
// block own different 16-row query tiles (QW each) and all walk the same keys, so K and V^T tiles are staged in
// LDS once per block and read from there as MFMA operands; K/V leave HBM once for up to 128 query rows.  No
// cross-wavefront merge is needed: each wavefront finishes its own query rows.
// Everything enters the matrix cores as fp16, one product each: cache entries are bf16, which converts to fp16
// exactly (on the way into LDS; magnitudes outside fp16's range would not, none occur in a decoder's K / V), and
// the queries and the softmax weights are rounded to fp16 (11 significant bits).  That halves the MFMAs of a
// bf16 high + low pair and frees the registers for what bounds this kernel, the bytes a CU keeps in flight: two
// 64-key tiles travel in registers (stage = tile parity) while a third is multiplied, and the next tile is stored
// into the second set of LDS tiles in the middle of the current one's MFMAs (one barrier per tile).
template <int DH, int QW, int NW>
__global__ __launch_bounds__(NW * 64) void attn_mfma_wide_kernel(AttnArgs a, float scale_log2, int range) {
    constexpr int KS = DH / 32, DT = DH / 16;
    constexpr int KSTRIDE = DH + 8;            // fp16 elements per staged K row (+16 B: conflict-free reads)
    constexpr int VSTRIDE = 64 + 8;            // fp16 elements per staged V^T row
    constexpr int kSetElems = 64 * KSTRIDE + DH * VSTRIDE;
    extern __shared__ __attribute__((aligned(16))) uint16_t lds_wide[];      // two sets of (K tile, V^T tile)
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

    f16x8 qf[QW][KS];
    int limit[QW];
    size_t out_row[QW];
#pragma unroll
    for (int qt = 0; qt < QW; ++qt) {
        const int qi = ((qchunk * NW + wave) * QW + qt) * 16 + i;
        const bool valid = qi < NQ;
        const int hl = valid ? qi / a.R : 0, r = valid ? qi % a.R : 0;
        limit[qt] = valid ? S_b + r : -1;
        out_row[qt] = ((size_t)(b * a.R + r)) * a.h_q + hk * group + hl;
        const float *qp = a.q + out_row[qt] * DH + g * (DH / 4);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            f32x8 v = load_f32x8(qp + 8 * s);
            if (!valid) v = f32x8{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            qf[qt][s] = __builtin_bit_cast(f16x8, f32x8_to_f16x8(v * scale_log2));   // scores come out in log2 units
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
    constexpr int NT = NW * 64;
    constexpr int KCH = 64 * DH / 8 / NT, VCH = DH * 8 / NT;
    u32x4 kreg[2][KCH], vreg[2][VCH];
    auto load_tile = [&](auto stage, int kt) {
        constexpr int st = decltype(stage)::value;
#pragma unroll
        for (int c = 0; c < KCH; ++c) {
            const int chunk = tid + c * NT, key = chunk / (DH / 8), col = (chunk % (DH / 8)) * 8;
            kreg[st][c] = *reinterpret_cast<const u32x4 *>(Kc + (size_t)(kt + key) * DH + col);     // kt + 64 <= max_len
        }
#pragma unroll
        for (int c = 0; c < VCH; ++c) {
            const int chunk = tid + c * NT, d = chunk >> 3, col = (chunk & 7) * 8;
            u32x4 raw = *reinterpret_cast<const u32x4 *>(Vt + (size_t)d * max_len + kt + col);
            if (kt + 64 > n_keys) {          // stale cache columns may hold anything, even NaN: zero them
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int key = kt + col + 2 * e;
                    if (key >= n_keys) raw[e] = 0u;
                    else if (key + 1 >= n_keys) raw[e] &= 0xffffu;
                }
            }
            vreg[st][c] = raw;
        }
    };
    auto store_tile = [&](auto stage, int set) {
        constexpr int st = decltype(stage)::value;
        uint16_t *Ks = lds_wide + set * kSetElems, *Vs = Ks + 64 * KSTRIDE;
#pragma unroll
        for (int c = 0; c < KCH; ++c) {
            const int chunk = tid + c * NT, key = chunk / (DH / 8), col = (chunk % (DH / 8)) * 8;
            *reinterpret_cast<u32x4 *>(&Ks[key * KSTRIDE + col]) = bf16x8_to_f16x8(kreg[st][c]);
        }
#pragma unroll
        for (int c = 0; c < VCH; ++c) {
            const int chunk = tid + c * NT, d = chunk >> 3, col = (chunk & 7) * 8;
            *reinterpret_cast<u32x4 *>(&Vs[d * VSTRIDE + col]) = bf16x8_to_f16x8(vreg[st][c]);
        }
    };
    // 32 keys of the tile in LDS set `set` (sub = which half of the tile), in two steps so that the scores of the second
    // half can be on the matrix cores while the first half's softmax runs on the vector ALU: the scores
    auto scores = [&](int set, int sub, f32x4 (&c)[QW][2]) {
        const uint16_t *Ks = lds_wide + set * kSetElems;
        f16x8 ka[2][KS];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int key = sub * 32 + 8 * (i >> 2) + 4 * t + (i & 3);
#pragma unroll
            for (int s = 0; s < KS; ++s)
                ka[t][s] = *reinterpret_cast<const f16x8 *>(&Ks[key * KSTRIDE + g * (DH / 4) + 8 * s]);
        }
        // every query tile, MFMAs interleaved over independent accumulators
#pragma unroll
        for (int qt = 0; qt < QW; ++qt)
#pragma unroll
            for (int t = 0; t < 2; ++t) c[qt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int qt = 0; qt < QW; ++qt)
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    c[qt][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka[t][s], qf[qt][s], c[qt][t], 0, 0, 0);
    };
    // ... and the softmax update and P V of keys kb .. kb + 31
    auto finish = [&](int set, int sub, int kb, f32x4 (&c)[QW][2]) {
        const uint16_t *Vs = lds_wide + set * kSetElems + 64 * KSTRIDE;
        f16x8 va[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
            va[dt] = *reinterpret_cast<const f16x8 *>(&Vs[(dt * 16 + i) * VSTRIDE + sub * 32 + 8 * g]);
        f16x8 pf[QW];
        const bool all_visible = kb + 31 <= S_b;       // every valid row sees all 32 keys: no mask (rows past NQ are never written)
#pragma unroll
        for (int qt = 0; qt < QW; ++qt) {
            // lane (query column i, group g): c[qt][t][v] is key kb + 8g + 4t + v
            float tmax = -INFINITY;
            if (!all_visible) {
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (kb + 8 * g + 4 * t + v > limit[qt]) c[qt][t][v] = -INFINITY;
            }
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) tmax = fmaxf(tmax, c[qt][t][v]);
            tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
            // The reference maximum of a row only moves when the scores outgrow it by more than 2^8: until then the
            // weights are taken against the old one (at most 256, well inside fp16 and fp32), and the accumulators
            // are rescaled a few times per row instead of at nearly every tile.  (m, l, O) stay consistent.
            if (tmax > mrun[qt] + 8.0f) {
                const float alpha = __builtin_amdgcn_exp2f(mrun[qt] - tmax);
                lrun[qt] *= alpha;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) o[qt][dt][v] *= alpha;
                mrun[qt] = tmax;
            }
            float p[8];
            if (mrun[qt] > -INFINITY) {
                float ps = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    p[e] = __builtin_amdgcn_exp2f(c[qt][e >> 2][e & 3] - mrun[qt]);
                    ps += p[e];
                }
                lrun[qt] += ps;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) p[e] = 0.f;
            }
            pf[qt] = __builtin_bit_cast(f16x8, f32x8_to_f16x8(f32x8{p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7]}));
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int qt = 0; qt < QW; ++qt)
                o[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va[dt], pf[qt], o[qt][dt], 0, 0, 0);
    };

    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;
    if (kb0 < kb1) {                             // tile t (t-th of this block) travels in stage t & 1
        load_tile(S0{}, kb0);
        store_tile(S0{}, 0);
        if (kb0 + 64 < kb1) load_tile(S1{}, kb0 + 64);
        if (kb0 + 128 < kb1) load_tile(S0{}, kb0 + 128);
    }
    __syncthreads();
    // one tile: the scores of both halves, the first half's softmax and P V, the next tile from its registers into the
    // other LDS set, those registers refilled with the tile three ahead, the second half's softmax and P V, one barrier
    // (next tile visible; this set free for the one after)
    auto k_tile = [&](auto next_stage, int kt) {
        const int set = ((kt - kb0) >> 6) & 1;
        const bool second = kt + 32 < kb1;
        f32x4 c0[QW][2], c1[QW][2];
        scores(set, 0, c0);
        if (second) scores(set, 1, c1);
        finish(set, 0, kt, c0);
        if (kt + 64 < kb1) store_tile(next_stage, set ^ 1);
        if (kt + 192 < kb1) load_tile(next_stage, kt + 192);
        if (second) finish(set, 1, kt + 32, c1);
        __syncthreads();
    };
    int kt = kb0;
    for (; kt + 64 < kb1; kt += 128) {
        k_tile(S1{}, kt);
        k_tile(S0{}, kt + 64);
    }
    if (kt < kb1) k_tile(S1{}, kt);

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
            {
                const f32x4 r = o[qt][dt] * inv;
                *reinterpret_cast<f32x4 *>(a.out + out_row[qt] * DH + dt * 16 + 4 * g) = r;
                if (a.out16)
                    *reinterpret_cast<uint2 *>(a.out16 + out_row[qt] * DH + dt * 16 + 4 * g) =
                        make_uint2(f32_to_f16_bits(r[0]) | ((uint32_t)f32_to_f16_bits(r[1]) << 16),
                                   f32_to_f16_bits(r[2]) | ((uint32_t)f32_to_f16_bits(r[3]) << 16));
            }
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
    if (a.out16) a.out16[row * DH + d] = f32_to_f16_bits(acc / L);
}

// query tiles of 16 per block: bounded by registers (hi+lo query operands and fp32 outputs)
inline int q_tiles(int NQ) { return NQ <= 16 ? 1 : 2; }

}  // namespace

// Which kernel: the LDS-staged one (64 or 128 query rows per block) from 11 query rows per KV head on, the direct one
// below that and for token trees of up to 32 rows (only it knows the ancestor mask).  The direct kernel builds its
// operands itself (no rotation kernel in front), which pays while a block's build stays small; measured per layer,
// direct kernel + combine against rotation kernel + LDS-staged kernel + combine (us): LLaMA2-7B shape, 1024 keys,
// 8 rows 18.9 / 19.9, 10 rows 19.7 / 19.9, 12 rows 20.4 / 19.9, 16 rows 22.1 / 20.1, 24 rows 31.1 / 22.8;
// LLaMA3-8B shape (4 query heads per KV head), 300 keys, 2 rows 17.1 / 17.1, 4 rows 18.1 / 17.6, 7 rows 24.6 / 17.7.
inline bool use_wide(int NQ, bool tree) { return NQ > 32 || (!tree && NQ > 10); }
inline int wide_rows(int NQ) { return NQ <= 64 ? 64 : 128; }

bool attn_fuses_rope(int dtype, int R, int h_q, int h_kv, int d_h, bool tree) {
    return dtype == PSD_BF16 && (d_h == 64 || d_h == 128) && R <= 32 && !use_wide((h_q / h_kv) * R, tree);
}

int attn_pick_splits(int dtype, int B, int R, int h_q, int h_kv, int d_h, int len_bound, bool tree) {
    if (dtype != PSD_BF16) return 1;
    const int NQ = (h_q / h_kv) * R;
    const int QT = q_tiles(NQ);
    const bool wide = use_wide(NQ, tree);
    const int chunks = wide ? (NQ + wide_rows(NQ) - 1) / wide_rows(NQ) : (NQ + QT * 16 - 1) / (QT * 16);
    // Both kernels: about one block per CU.  The LDS-staged kernel loads its 64-128 query rows and writes as many
    // partial rows per block, which that keeps below the K/V bytes (measured at 16 x 4 KV heads x 4096 keys: 4 splits
    // 78 us, 8 splits 91 us, 16 splits 113 us per layer).
    int by_grid = 256 / (B * h_kv * chunks);
    if (by_grid < 1) by_grid = 1;
    if (!wide) {
        // The direct kernel builds its own operands: the keys already in the cache are split into blocks of 256 (one
        // 64-key tile per wavefront), and one more split takes the step's own rows alone, so that building and
        // appending their K / V is nobody's prelude to a tile of cache keys.  Measured at the 7B shape, 1024 keys in
        // the cache (us per layer): 4 + 1 splits 14.7; 4 splits with the new rows riding on the last 21.4; 8 splits
        // of 128 keys 17.9; 9 splits 24.5 (every block repeats the operand build, and only one block is resident
        // per CU, so a 257th block waits for a whole block's lifetime).
        const int cached = len_bound - R > 1 ? len_bound - R : 1;
        int old_splits = (cached + kKeysPerBlockIter - 1) / kKeysPerBlockIter;
        if (old_splits > by_grid - 1) old_splits = by_grid - 1;
        return old_splits < 1 ? 1 : old_splits + 1;
    }
    const int by_len = (len_bound + kKeysPerBlockIter - 1) / kKeysPerBlockIter;
    int s = by_len < by_grid ? by_len : by_grid;
    return s < 1 ? 1 : s;
}

template <int DH>
static void launch_mfma(const AttnArgs &a, hipStream_t stream) {
    const int NQ = (a.h_q / a.h_kv) * a.R;
    const int QT = q_tiles(NQ);
    const int chunks = (NQ + QT * 16 - 1) / (QT * 16);
    const bool wide = use_wide(NQ, a.tree_anc != nullptr);
    // keys per split; the kernel that builds its own operands reads only the keys already in the cache and leaves its
    // last split (if it has several) to the step's own rows
    int range = (a.len_bound + a.splits - 1) / a.splits;
    if (!wide && a.qkv_partial && a.splits > 1) {
        const int cached = a.len_bound - a.R > 1 ? a.len_bound - a.R : 1;
        range = (cached + a.splits - 2) / (a.splits - 1);
    }
    range = (range + kKeysPerWaveIter - 1) / kKeysPerWaveIter * kKeysPerWaveIter;
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)DH);
    if (wide) {
        const int rows = wide_rows(NQ);
        dim3 wgrid(a.splits, (NQ + rows - 1) / rows, a.B * a.h_kv);
        {
            ScopedProf sp(PSD_KIND_ATTN, stream);
            // two sets of (64 keys x (DH + 8), DH x (64 + 8)) fp16 tiles: more than the 64 KB a kernel gets unasked at d_head 128
            const size_t lds = 2 * (size_t)(64 * (DH + 8) + DH * 72) * sizeof(uint16_t);
            auto go = [&](auto kernel, int threads) {
                (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
                launch_kernel(kernel, wgrid, threads, lds, stream, a, scale_log2, range);
            };
            // 128 rows: eight wavefronts with one query tile each rather than four with two.  Two wavefronts per SIMD
            // overlap each other's LDS reads, exponentials and MFMAs (measured at 16 sequences x 4 KV heads x 112 query
            // rows x 4096 keys: 43.6 us per layer against 61.1 us), although every K / V^T tile is then read from LDS
            // by eight wavefronts instead of four.
            if (rows == 64) go(attn_mfma_wide_kernel<DH, 1, 4>, 256);
            else go(attn_mfma_wide_kernel<DH, 1, 8>, 512);
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
    if (a.qkv_partial) {
        if (QT == 1) launch_kernel(attn_mfma_kernel<DH, 1, true>, grid, 256, 0, stream, a, scale_log2, range);
        else launch_kernel(attn_mfma_kernel<DH, 2, true>, grid, 256, 0, stream, a, scale_log2, range);
    } else {
        if (QT == 1) launch_kernel(attn_mfma_kernel<DH, 1, false>, grid, 256, 0, stream, a, scale_log2, range);
        else launch_kernel(attn_mfma_kernel<DH, 2, false>, grid, 256, 0, stream, a, scale_log2, range);
    }
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
