// Speculative-sampling acceptance on gfx950 (the VERIFY loop of Algorithm 1 and the residual
// draw that keeps the verifier's distribution, Sec. 3.1).
//
// Two launches per call, no host round trip:
//   1. accept_stats_kernel  one pass over every logits row of p and q (the HBM-bound part):
//      per (row, chunk) the max raw logit and sum exp((l - max)/T), fp32, wavefront
//      reductions, 8 x 16-byte loads in flight per lane.  The block whose chunk holds the
//      draft token of its position also hands on that one logit, so the ratio test later
//      needs no dependent load.
//   2. accept_draw_kernel   several blocks per sequence.  Each re-derives the first rejection
//      n of its sequence from the statistics (ratio test against the supplied uniforms, scan
//      over <= 64 flags) and accumulates, in fp64 and for the ONE position the draw needs, the
//      softmax denominators and the residual mass of its chunk.  The block of a sequence that
//      finishes last (one counter per sequence; partial sums travel as agent-scope atomic
//      stores / loads, so no cache write-back fence is needed and nothing ever waits) sums the
//      chunks in index order and locates the inverse-CDF crossing, first among the chunks,
//      then among the entries of that chunk.
// All sums are taken in a fixed order, so results do not depend on block scheduling.
#include "common.h"
#include "kernels.h"
#include "exp64.h"
#include "prof.h"
#include "../../include/psd.h"

namespace psd {

namespace {

constexpr int kThreads = 256;
constexpr int kLoadsPerLane = 8;
constexpr double kTieEps = 1e-5;
constexpr int kMaxChunksE = 256;      // draw-pass chunks per logits row: one per thread of the block that finishes a sequence
constexpr int kGroup = 8;             // consecutive entries a thread of the draw kernel takes at a time

template <typename T>
__device__ __forceinline__ const T *logits_row(const AcceptArgs &a, int b, bool is_q, int j) {
    const T *base = is_q ? (const T *)a.q + (int64_t)b * a.q_stride : (const T *)a.p + (int64_t)b * a.p_stride;
    return base + (int64_t)j * a.V;
}

template <typename T, bool VEC>
__global__ __launch_bounds__(kThreads) void accept_stats_kernel(AcceptArgs a) {
    constexpr int EPL = VEC ? (int)(16 / sizeof(T)) : 1;
    const int tid = threadIdx.x;
    const int per_seq = a.n_p_rows + a.gamma;
    const int vec = blockIdx.x / a.n_chunksA, c = blockIdx.x % a.n_chunksA;
    const int b = vec / per_seq, r = vec % per_seq;
    const bool is_q = r >= a.n_p_rows;
    const int j = is_q ? r - a.n_p_rows : r;           // position of this row inside the block of draft tokens
    const T *row = logits_row<T>(a, b, is_q, j);
    const int e0 = c * a.chunkA;
    const int e1 = min(a.V, e0 + a.chunkA);
    // the draft token of this position (none for the bonus row): its logit passes through this block's
    // registers if it lies in [e0, e1)
    int xj = -1;
    if (j < a.gamma) xj = min(max(a.x[(size_t)b * a.gamma + j], 0), a.V - 1);
    // the per-sequence arrival counters of the draw kernel start every call at zero
    if (blockIdx.x == 0)
        for (int i = tid; i < a.rows; i += kThreads) a.counter[i] = 0u;

    // keep the loaded 16-byte vectors as they are (32 registers) and unpack them twice, once for
    // the max and once for the exponentials: the small footprint keeps 8 blocks resident per CU
    u32x4 raw[kLoadsPerLane];
    float sc[kLoadsPerLane];               // scalar path
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
    auto elem = [&](int i, int e) -> float {
        if constexpr (!VEC) return sc[i];
        else if constexpr (sizeof(T) == 2)
            return (e & 1) ? __uint_as_float(raw[i][e >> 1] & 0xffff0000u) : __uint_as_float(raw[i][e >> 1] << 16);
        else return __uint_as_float(raw[i][e]);
    };
    if (xj >= e0 && xj < e1) {
        // vector v = i * kThreads + tid of the chunk holds the token's logit as its element e
        const int rel = xj - e0, v = rel / EPL, e = rel % EPL;
        if (tid == v % kThreads) {
            const int iv = v / kThreads;
            float val = 0.f;
#pragma unroll
            for (int i = 0; i < kLoadsPerLane; ++i)
#pragma unroll
                for (int ee = 0; ee < EPL; ++ee)
                    if (i == iv && ee == e) val = elem(i, ee);
            a.xlogit[((size_t)b * a.gamma + j) * 2 + (is_q ? 1 : 0)] = val;
        }
    }
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < kLoadsPerLane; ++i)
        if (have[i]) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) m = fmaxf(m, elem(i, e));
        }
    __shared__ float sm[kThreads / 64];
    __shared__ float ss[kThreads / 64];
    m = wave_max(m);
    if ((tid & 63) == 0) sm[tid >> 6] = m;
    __syncthreads();
    m = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
    float s = 0.f;
    if (m > -INFINITY) {
        const float k2 = 1.4426950408889634f / a.temperature;
#pragma unroll
        for (int i = 0; i < kLoadsPerLane; ++i)
            if (have[i]) {
#pragma unroll
                for (int e = 0; e < EPL; ++e) s += __builtin_amdgcn_exp2f((elem(i, e) - m) * k2);
            }
    }
    s = wave_sum(s);
    if ((tid & 63) == 0) ss[tid >> 6] = s;
    __syncthreads();
    if (tid == 0) a.stats[(size_t)vec * a.n_chunksA + c] = make_float2(m, ((ss[0] + ss[1]) + ss[2]) + ss[3]);
}

// (max raw logit, sum exp((l - max)/T)) of one logits row from its per-chunk statistics.  The chunk
// sums are fp32 quantities; rescaling them with the fp32 exponential loses nothing.
__device__ __forceinline__ void combine_stats(const AcceptArgs &a, int b, int r, float *M, double *Z) {
    const float2 *st = a.stats + ((size_t)b * (a.n_p_rows + a.gamma) + r) * a.n_chunksA;
    float m = -INFINITY;
    for (int c = 0; c < a.n_chunksA; ++c) m = fmaxf(m, st[c].x);
    double z = 0.0;
    const float k2 = 1.4426950408889634f / a.temperature;
    for (int c = 0; c < a.n_chunksA; ++c)
        if (st[c].x > -INFINITY) z += (double)(st[c].y * __builtin_amdgcn_exp2f((st[c].x - m) * k2));
    *M = m;
    *Z = z;
}

// fp32 statistics of every position of one sequence, kept in LDS by the block that decides it
struct SeqStats {
    float mp[65], mq[64];
    double zp[65], zq[64];
    int bits[64];
    double exp2tab[64];           // kExp2Table, for exp_core
};

// Ratio tests of sequence b and the scan to the first rejection.  Called by a whole block;
// every thread returns the same n and flags.
__device__ __forceinline__ void decide(const AcceptArgs &a, int b, SeqStats *ss, int *n_out, int *flags_out) {
    const int j = threadIdx.x;
    const double tabv = j < 64 ? kExp2Table[j] : 0.0;      // requested first, stored once the other loads are out
    double u = 0.0;
    float lpx = 0.f, lqx = 0.f;
    float Mp = 0.f, Mq = 0.f;
    double Zp = 1.0, Zq = 1.0;
    if (j < a.n_p_rows) {
        if (j < a.gamma) {                      // independent loads first
            u = (double)a.u[(size_t)b * (a.gamma + 1) + j];
            lpx = a.xlogit[((size_t)b * a.gamma + j) * 2];
            lqx = a.xlogit[((size_t)b * a.gamma + j) * 2 + 1];
        }
        combine_stats(a, b, j, &Mp, &Zp);
        ss->mp[j] = Mp;
        ss->zp[j] = Zp;
        if (j < a.gamma) {
            combine_stats(a, b, a.n_p_rows + j, &Mq, &Zq);
            ss->mq[j] = Mq;
            ss->zq[j] = Zq;
        }
    }
    if (j < 64) ss->exp2tab[j] = tabv;
    __syncthreads();
    if (j < a.gamma && j < a.n_p_rows) {
        double rho;
        if (lqx == -INFINITY) {
            rho = INFINITY;             // q[x] = 0: the token could not have been drafted; accept
        } else {
            rho = exp_any((((double)lpx - (double)Mp) - ((double)lqx - (double)Mq)) / (double)a.temperature, ss->exp2tab) * (Zq / Zp);
        }
        const int acc = u < fmin(1.0, rho) ? 1 : 0;
        const int tie = fabs(u - rho) < kTieEps ? 2 : 0;
        ss->bits[j] = acc | tie;
    }
    __syncthreads();
    int n = 0, flags = 0;
    for (int k = 0; k < a.gamma; ++k) {
        const int f = ss->bits[k];
        if (f & 2) flags |= PSD_FLAG_NEAR_TIE;
        if (!(f & 1)) break;
        ++n;
    }
    *n_out = n;
    *flags_out = flags;
}

// which position the draw reads: the rejected one (p and q) or the bonus row (p only)
struct DrawRows {
    int p_row;      // row index within p, -1: nothing to draw
    bool have_q;
};
__device__ __forceinline__ DrawRows draw_rows(const AcceptArgs &a, int n) {
    DrawRows d;
    if (n < a.gamma) { d.p_row = n; d.have_q = true; }
    else if (a.n_p_rows > a.gamma) { d.p_row = a.gamma; d.have_q = false; }
    else { d.p_row = -1; d.have_q = false; }
    return d;
}

// The draw position of one sequence.  With a_i = exp(lp_i/T - mp), b_i = exp(lq_i/T - mq) (fp64) and
// Zp = sum a, Zq = sum b, the residual weight of entry i is a_i/Zp - b_i/Zq where that is positive, i.e.
// where d_i = (lp_i/T - mp) - (lq_i/T - mq) exceeds log(Zp/Zq).  The chunk pass runs before the fp64
// Zp, Zq exist; it decides the sign against the fp32 estimate `delta` of log(Zp/Zq) from the statistics
// pass (t_i = d_i - delta > 0) and records, per chunk, the smallest positive and the largest non-positive
// t_i.  The block that finishes the sequence knows eps = log(Zp/Zq) - delta; a chunk with no t_i between
// 0 and eps was classified exactly as the fp64 residual would have been, any other chunk is summed again
// with the sign taken from a_i/Zp - b_i/Zq itself.  Nothing rests on how good the estimate is.
constexpr double kSignTol = 1e-11;      // rounding of t_i and of eps (|d_i| stays below ~1e3)

template <typename T>
struct DrawPos {
    const T *prow, *qrow;
    const double *tab;             // the block's copy of kExp2Table
    double inv_t, mp, mq, delta;
    bool have_q;
    __device__ __forceinline__ void init(const AcceptArgs &a, int b, int n, const DrawRows &d, const SeqStats &ss) {
        const float Mp = ss.mp[d.p_row], Mq = d.have_q ? ss.mq[n] : 0.f;
        const double Zp32 = ss.zp[d.p_row], Zq32 = d.have_q ? ss.zq[n] : 1.0;
        tab = ss.exp2tab;
        prow = logits_row<T>(a, b, false, d.p_row);
        qrow = logits_row<T>(a, b, true, d.have_q ? n : 0);
        inv_t = 1.0 / (double)a.temperature;
        mp = (double)Mp * inv_t;
        mq = (double)Mq * inv_t;
        const float est = logf((float)(Zp32 / Zq32));
        delta = d.have_q && est == est ? (double)est : 0.0;       // any finite value will do
        have_q = d.have_q;
    }
    // raw logits of the kGroup consecutive entries i0 .. i0 + kGroup - 1 (those at or past i_end: entry i0 again,
    // q's are 0 when there is no q row).  VEC: rows are 16-byte aligned, i0 and V are multiples of the elements
    // per 16-byte load, so whole vectors are inside the row
    template <bool VEC>
    __device__ __forceinline__ void load_group(int i0, int i_end, float (&lp)[kGroup], float (&lq)[kGroup]) const {
        if constexpr (VEC) {
            constexpr int EPL = (int)(16 / sizeof(T)), NV = kGroup / EPL;
            u32x4 rp[NV], rq[NV];
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const int i = i0 + v * EPL < i_end ? i0 + v * EPL : i0;
                rp[v] = *reinterpret_cast<const u32x4 *>(prow + i);
                rq[v] = have_q ? *reinterpret_cast<const u32x4 *>(qrow + i) : u32x4{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int j = 0; j < kGroup; ++j) {
                if constexpr (sizeof(T) == 2) {
                    const uint32_t wp = rp[j / EPL][(j % EPL) >> 1], wq = rq[j / EPL][(j % EPL) >> 1];
                    lp[j] = (j & 1) ? __uint_as_float(wp & 0xffff0000u) : __uint_as_float(wp << 16);
                    lq[j] = (j & 1) ? __uint_as_float(wq & 0xffff0000u) : __uint_as_float(wq << 16);
                } else {
                    lp[j] = __uint_as_float(rp[j / EPL][j % EPL]);
                    lq[j] = __uint_as_float(rq[j / EPL][j % EPL]);
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < kGroup; ++j) {
                const int i = i0 + j < i_end ? i0 + j : i0;
                lp[j] = load_elem(prow, i);
                lq[j] = have_q ? load_elem(qrow, i) : 0.f;
            }
        }
    }
    // (a_i, b_i, t_i) from the raw logits; without a q row b_i = 0 and t_i = +inf (every entry counts)
    __device__ __forceinline__ void eval(float lp, float lq, double *ea, double *eb, double *t) const {
        const double xa = fma((double)lp, inv_t, -mp);
        const double xb = fma((double)lq, inv_t, -mq);
        *ea = exp_nonpos(xa, tab);
        const double e = exp_nonpos(xb, tab);
        *eb = have_q ? e : 0.0;
        *t = have_q ? (xa - xb) - delta : INFINITY;
    }
};

// fixed-order block reductions of NV doubles per thread: butterfly inside each wavefront, then the four
// wavefront results left to right
template <int NV>
__device__ __forceinline__ void block_sum(double (&v)[NV], double (*red)[kThreads / 64]) {
    const int tid = threadIdx.x;
    __syncthreads();                              // red may still be read from an earlier use
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        v[k] = wave_sum(v[k]);
        if ((tid & 63) == 0) red[k][tid >> 6] = v[k];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < NV; ++k) v[k] = ((red[k][0] + red[k][1]) + red[k][2]) + red[k][3];
}
__device__ __forceinline__ double wave_min_d(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmin(v, __shfl_xor(v, o, kWave));
    return v;
}
__device__ __forceinline__ double wave_max_d(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, kWave));
    return v;
}

// per (sequence, chunk): sum a, sum b, both over the entries with t_i > 0, the smallest positive t_i and the
// largest non-positive t_i
constexpr int kPartStride = 6;

// Grid: rows x n_chunksE blocks.  Every block: first rejection of its sequence, fp64 sums of its chunk of
// the draw position; the block that arrives last at the sequence's counter finishes the draw (thread k of
// it owns chunk k: n_chunksE <= kThreads).
template <typename T, bool VEC>
__global__ __launch_bounds__(kThreads) void accept_draw_kernel(AcceptArgs a) {
    __shared__ SeqStats s_seq;
    __shared__ double s_red[6][kThreads / 64];
    __shared__ double s_scan[kThreads / 64];

    __shared__ int s_redo[kMaxChunksE];           // chunks whose sign classification has to be redone
    __shared__ int s_last, s_cstar, s_best, s_lastpos;
    __shared__ double s_base;
    const int nE = a.n_chunksE;
    const int b = blockIdx.x / nE, c = blockIdx.x % nE, tid = threadIdx.x;
    int n, flags;
    decide(a, b, &s_seq, &n, &flags);
    const DrawRows d = draw_rows(a, n);
    if (d.p_row < 0) {                            // every token accepted and no bonus row
        if (c == 0 && tid == 0) { a.out_n[b] = n; a.flags[b] = flags; a.out_tok[b] = -1; }
        return;
    }
    DrawPos<T> w;
    w.init(a, b, n, d, s_seq);

    // ---- this block's chunk
    {
        const int e0 = c * a.chunkE, e1 = min(a.V, e0 + a.chunkE);
        double acc[4] = {0.0, 0.0, 0.0, 0.0};               // sum a, sum b, positive a, positive b
        double tpos = INFINITY, tneg = -INFINITY;
        for (int i0 = e0 + tid * kGroup; i0 < e1; i0 += kGroup * kThreads) {
            float lp[kGroup], lq[kGroup];
            w.template load_group<VEC>(i0, e1, lp, lq);
            double ea[kGroup], eb[kGroup], t[kGroup];
#pragma unroll
            for (int j = 0; j < kGroup; ++j) w.eval(lp[j], lq[j], &ea[j], &eb[j], &t[j]);
#pragma unroll
            for (int j = 0; j < kGroup; ++j) {
                if (i0 + j < e1) {
                    acc[0] += ea[j];
                    acc[1] += eb[j];
                    if (t[j] > 0.0) { acc[2] += ea[j]; acc[3] += eb[j]; tpos = fmin(tpos, t[j]); }
                    if (t[j] <= 0.0) tneg = fmax(tneg, t[j]);
                }
            }
        }
        // one value per wavefront into LDS, thread 0 folds the four in wavefront order
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[k] = wave_sum(acc[k]);
        tpos = wave_min_d(tpos);
        tneg = wave_max_d(tneg);
        if ((tid & 63) == 0) {
#pragma unroll
            for (int k = 0; k < 4; ++k) s_red[k][tid >> 6] = acc[k];
            s_red[4][tid >> 6] = tpos;
            s_red[5][tid >> 6] = tneg;
        }
        __syncthreads();
        if (tid == 0) {
#pragma unroll
            for (int k = 0; k < 4; ++k) acc[k] = ((s_red[k][0] + s_red[k][1]) + s_red[k][2]) + s_red[k][3];
            tpos = fmin(fmin(s_red[4][0], s_red[4][1]), fmin(s_red[4][2], s_red[4][3]));
            tneg = fmax(fmax(s_red[5][0], s_red[5][1]), fmax(s_red[5][2], s_red[5][3]));
            // hand the results on as write-through stores, wait for them to be performed, then count this
            // block in; whoever counts last reads all of them back with loads of the same scope
            double *dst = a.part + ((size_t)b * nE + c) * kPartStride;
#pragma unroll
            for (int k = 0; k < 4; ++k) __hip_atomic_store(dst + k, acc[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(dst + 4, tpos, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(dst + 5, tneg, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            const unsigned old = __hip_atomic_fetch_add(a.counter + b, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = old == (unsigned)nE - 1u;
        }
        __syncthreads();
        if (!s_last) return;
    }

    // ---- the last block of the sequence: thread k takes chunk k's results (one round of loads)
    double pk[kPartStride] = {0.0, 0.0, 0.0, 0.0, INFINITY, -INFINITY};
    if (tid < nE) {
        const double *src = a.part + ((size_t)b * nE + tid) * kPartStride;
#pragma unroll
        for (int k = 0; k < kPartStride; ++k) pk[k] = __hip_atomic_load(src + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    const double u = (double)a.u[(size_t)b * (a.gamma + 1) + a.gamma];
    double zz[2] = {pk[0], pk[1]};
    block_sum<2>(zz, s_red);
    const double inv_zp = 1.0 / zz[0], inv_zq = d.have_q ? 1.0 / zz[1] : 0.0;
    double wk = pk[2] * inv_zp - pk[3] * inv_zq;                 // weight of chunk tid
    if (d.have_q) {
        // chunks with a t_i between 0 and eps (or too close to tell): every entry's sign again, from the fp64 weights
        const double eps = log(zz[0] / zz[1]) - w.delta;
        const double lo = fmin(0.0, eps) - kSignTol, hi = fmax(0.0, eps) + kSignTol;
        const bool redo = tid < nE && (!(eps == eps) || pk[5] >= lo || pk[4] <= hi);
        if (tid < nE) s_redo[tid] = redo ? 1 : 0;
        __syncthreads();
        for (int k = 0; k < nE; ++k) {
            if (!s_redo[k]) continue;                            // the same for the whole block
            const int f0 = k * a.chunkE, f1 = min(a.V, f0 + a.chunkE);
            double pw[2] = {0.0, 0.0};
            for (int i0 = f0 + tid * kGroup; i0 < f1; i0 += kGroup * kThreads) {
                float lp[kGroup], lq[kGroup];
                w.template load_group<VEC>(i0, f1, lp, lq);
#pragma unroll
                for (int j = 0; j < kGroup; ++j) {
                    double ea, eb, t;
                    w.eval(lp[j], lq[j], &ea, &eb, &t);
                    if (i0 + j < f1 && ea * inv_zp - eb * inv_zq > 0.0) { pw[0] += ea; pw[1] += eb; }
                }
            }
            block_sum<2>(pw, s_red);
            if (tid == k) wk = pw[0] * inv_zp - pw[1] * inv_zq;
        }
    }
    double ms[1] = {wk};
    block_sum<1>(ms, s_red);
    double mass = ms[0];
    const bool fall_back_to_p = d.have_q && !(mass > 0.0);
    if (fall_back_to_p) {                         // residual mass 0: draw from p itself
        mass = 1.0;                               // sum of a_i / Zp
        wk = pk[0] * inv_zp;
    }
    // first chunk whose inclusive prefix exceeds t
    const double t = u * mass;
    {
        double incl = wk;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const double up = __shfl_up(incl, o, 64);
            if ((tid & 63) >= o) incl += up;
        }
        if (tid == 0) { s_best = 0x7fffffff; s_lastpos = -1; s_cstar = 0x7fffffff; }
        __syncthreads();                          // s_scan: earlier readers are done
        if ((tid & 63) == 63) s_scan[tid >> 6] = incl;
        __syncthreads();
        double base = 0.0;
        for (int wvi = 0; wvi < (tid >> 6); ++wvi) base += s_scan[wvi];
        base += incl - wk;                        // weight in front of chunk tid
        const bool mine = tid < nE && base + wk > t;
        if (mine) atomicMin(&s_cstar, tid);
        if (tid < nE && wk > 0.0) atomicMax(&s_lastpos, tid);
        __syncthreads();
        const int cstar = s_cstar;
        if (cstar == 0x7fffffff) {                // rounding left no crossing: last chunk with weight
            if (tid == 0) { s_cstar = max(s_lastpos, 0); s_base = -INFINITY; }
        } else if (tid == cstar) {
            s_base = base;
        }
        __syncthreads();
        if (tid == 0) s_lastpos = -1;
    }
    __syncthreads();
    const int cs = s_cstar;
    const bool no_crossing = s_base == -INFINITY;  // then the walk only looks for the last entry with weight
    const int f0 = cs * a.chunkE, f1 = min(a.V, f0 + a.chunkE);
    // walk the chunk in tiles of 256 x kGroup entries, kGroup consecutive entries per thread, carrying the prefix
    double before = no_crossing ? 0.0 : s_base;    // weight in front of the current tile
    int found = 0x7fffffff, lastpos = -1;
    for (int t0 = f0; t0 < f1; t0 += kThreads * kGroup) {
        const int g0 = t0 + tid * kGroup;
        const bool active = g0 < f1;              // idle threads re-read the chunk's first group and count nothing
        const int i0 = active ? g0 : f0, i1 = active ? min(f1, g0 + kGroup) : f0;
        double wv[kGroup];
        double local = 0.0;
        float lp[kGroup], lq[kGroup];
        w.template load_group<VEC>(i0, active ? i1 : f1, lp, lq);
#pragma unroll
        for (int j = 0; j < kGroup; ++j) {
            double ea, eb, tt;
            w.eval(lp[j], lq[j], &ea, &eb, &tt);
            const double r = ea * inv_zp - eb * inv_zq;
            const double wj = fall_back_to_p ? ea * inv_zp : (r > 0.0 ? r : 0.0);
            wv[j] = i0 + j < i1 ? wj : 0.0;
            local += wv[j];
        }
        // exclusive prefix of `local` over threads, in thread order
        double incl = local;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const double up = __shfl_up(incl, o, 64);
            if ((tid & 63) >= o) incl += up;
        }
        __syncthreads();                          // s_scan: the previous tile's readers are done
        if ((tid & 63) == 63) s_scan[tid >> 6] = incl;
        __syncthreads();
        double run = before;
        for (int wvi = 0; wvi < (tid >> 6); ++wvi) run += s_scan[wvi];
        run += incl - local;
#pragma unroll
        for (int j = 0; j < kGroup; ++j) {
            if (i0 + j < i1) {
                if (wv[j] > 0.0) lastpos = i0 + j;
                run += wv[j];
                if (!no_crossing && run > t && found == 0x7fffffff) found = i0 + j;
            }
        }
        before += ((s_scan[0] + s_scan[1]) + s_scan[2]) + s_scan[3];
    }
    if (found != 0x7fffffff) atomicMin(&s_best, found);
    if (lastpos >= 0) atomicMax(&s_lastpos, lastpos);
    __syncthreads();
    if (tid == 0) {
        int tok = s_best;
        if (tok == 0x7fffffff) tok = s_lastpos >= 0 ? s_lastpos : f1 - 1;
        a.out_tok[b] = tok;
        a.out_n[b] = n;
        a.flags[b] = flags | (fall_back_to_p ? PSD_FLAG_ZERO_RESIDUAL : 0);
    }
}

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

}  // namespace

void accept_plan(int rows, int gamma, int n_p_rows, int V, int dtype, bool vec, AcceptArgs *a) {
    a->rows = rows; a->gamma = gamma; a->n_p_rows = n_p_rows; a->V = V; a->dtype = dtype;
    const int epl = !vec ? 1 : (dtype == PSD_BF16 ? 8 : 4);
    const int cap = kThreads * kLoadsPerLane * epl;            // elements one block can hold
    const int nA = (V + cap - 1) / cap;
    a->chunkA = round_up((V + nA - 1) / nA, epl);
    a->n_chunksA = (V + a->chunkA - 1) / a->chunkA;
    // draw pass: about 512 blocks in all.  Every block repeats the decision of its sequence, so more and smaller
    // chunks cost more than they spread (64 sequences x 32 000 entries: 4 chunks per sequence 30.7 us, 8 28.0, 16 29.9,
    // 32 41.7, 63 64.0)
    long want = ((long)V * (rows > 0 ? rows : 1) + 511) / 512;
    int ce = round_up((int)(want < 512 ? 512 : (want > 8192 ? 8192 : want)), 256);
    if ((V + ce - 1) / ce > kMaxChunksE) ce = round_up((V + kMaxChunksE - 1) / kMaxChunksE, 256);
    a->chunkE = ce;
    a->n_chunksE = (V + ce - 1) / ce;
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// workspace layout: statistics | the draft tokens' logits | chunk sums of the draw | arrival counters | flags
struct WsLayout { size_t stats, xlogit, part, counter, flags, total; };
static WsLayout ws_layout(const AcceptArgs &a) {
    const size_t rows = a.rows > 0 ? a.rows : 1;
    WsLayout l;
    size_t at = 0;
    l.stats = at;   at += align256(rows * (a.n_p_rows + a.gamma) * a.n_chunksA * sizeof(float2));
    l.xlogit = at;  at += align256(rows * (a.gamma > 0 ? a.gamma : 1) * 2 * sizeof(float));
    l.part = at;    at += align256(rows * a.n_chunksE * kPartStride * sizeof(double));
    l.counter = at; at += align256(rows * sizeof(uint32_t));
    l.flags = at;   at += align256(rows * sizeof(int32_t));
    l.total = at;
    return l;
}

size_t accept_workspace_bytes(const AcceptArgs &a) { return ws_layout(a).total; }

void accept_bind_workspace(AcceptArgs *a, void *ws, int32_t *out_flags) {
    const WsLayout l = ws_layout(*a);
    char *p = (char *)ws;
    a->stats = (float2 *)(p + l.stats);
    a->xlogit = (float *)(p + l.xlogit);
    a->part = (double *)(p + l.part);
    a->counter = (uint32_t *)(p + l.counter);
    a->flags = out_flags ? out_flags : (int32_t *)(p + l.flags);
}

template <typename T>
static void launch_accept_t(const AcceptArgs &a, bool vec_ok, hipStream_t stream) {
    const int vecs = a.rows * (a.n_p_rows + a.gamma);
    if (vecs > 0) {
        dim3 grid((unsigned)vecs * a.n_chunksA);
        ScopedProf sp(PSD_KIND_ACCEPT_STATS, stream);
        if (vec_ok) launch_kernel(accept_stats_kernel<T, true>, grid, kThreads, 0, stream, a);
        else launch_kernel(accept_stats_kernel<T, false>, grid, kThreads, 0, stream, a);
    }
    dim3 gridE((unsigned)a.rows * a.n_chunksE);
    ScopedProf sp(PSD_KIND_ACCEPT_DRAW, stream);
    if (vec_ok) launch_kernel(accept_draw_kernel<T, true>, gridE, kThreads, 0, stream, a);
    else launch_kernel(accept_draw_kernel<T, false>, gridE, kThreads, 0, stream, a);
}

void launch_accept(const AcceptArgs &a, bool vec_ok, hipStream_t stream) {
    if (a.dtype == PSD_BF16) launch_accept_t<uint16_t>(a, vec_ok, stream);
    else launch_accept_t<float>(a, vec_ok, stream);
}

}  // namespace psd
