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
#include "prof.h"
#include "../../include/psd.h"

namespace psd {

namespace {

constexpr int kThreads = 256;
constexpr int kLoadsPerLane = 8;
constexpr double kTieEps = 1e-5;
constexpr int kMaxChunksE = 1024;     // draw-pass chunks per logits row (LDS table of the locating block)
constexpr int kMaxChunkE = 8192;      // elements per draw-pass chunk
constexpr int kWalk = 8;              // consecutive entries per thread and tile when a chunk is walked

template <typename T>
__device__ __forceinline__ const T *logits_row(const AcceptArgs &a, int b, bool is_q, int j) {
    const T *base = is_q ? (const T *)a.q + (int64_t)b * a.q_stride : (const T *)a.p + (int64_t)b * a.p_stride;
    return base + (int64_t)j * a.V;
}

// exp(x) for x <= 0 in fp64, a few ulp: x = k ln2 + r with |r| <= ln2/2, degree-13 Taylor polynomial
// of exp(r) evaluated pairwise (short dependency chains), scaled by 2^k.  The draw only needs both
// sides to agree to ~1e-15 relative, which leaves the flip probability at V * 1e-15.
__device__ __forceinline__ double exp_nonpos(double x) {
    if (!(x > -745.0)) return 0.0;
    if (x > 709.0) return INFINITY;          // callers with x > 0 (the acceptance ratio) saturate
    const double kf = rint(x * 1.4426950408889634074);
    double r = fma(-kf, 6.93147180369123816490e-01, x);
    r = fma(-kf, 1.90821492927058770002e-10, r);
    const double r2 = r * r, r4 = r2 * r2, r8 = r4 * r4;
    const double p01 = 1.0 + r;
    const double p23 = fma(r, 1.0 / 6.0, 0.5);
    const double p45 = fma(r, 1.0 / 120.0, 1.0 / 24.0);
    const double p67 = fma(r, 1.0 / 5040.0, 1.0 / 720.0);
    const double p89 = fma(r, 1.0 / 362880.0, 1.0 / 40320.0);
    const double pab = fma(r, 1.0 / 39916800.0, 1.0 / 3628800.0);
    const double pcd = fma(r, 1.0 / 6227020800.0, 1.0 / 479001600.0);
    const double q0 = fma(r2, p23, p01);          // degree 0..3
    const double q1 = fma(r2, p67, p45);          // degree 4..7 (times r^4)
    const double q2 = fma(r2, pab, p89);          // degree 8..11 (times r^8)
    const double lo = fma(r4, q1, q0);
    const double hi = fma(r4, pcd, q2);           // degree 8..13 (times r^8)
    return ldexp(fma(r8, hi, lo), (int)kf);
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
};

// Ratio tests of sequence b and the scan to the first rejection.  Called by a whole block;
// every thread returns the same n and flags.
__device__ __forceinline__ void decide(const AcceptArgs &a, int b, SeqStats *ss, int *n_out, int *flags_out) {
    const int j = threadIdx.x;
    if (j < a.n_p_rows) {
        double u = 0.0;
        float lpx = 0.f, lqx = 0.f;
        if (j < a.gamma) {                      // independent loads first
            u = (double)a.u[(size_t)b * (a.gamma + 1) + j];
            lpx = a.xlogit[((size_t)b * a.gamma + j) * 2];
            lqx = a.xlogit[((size_t)b * a.gamma + j) * 2 + 1];
        }
        float Mp, Mq = 0.f;
        double Zp, Zq = 1.0;
        combine_stats(a, b, j, &Mp, &Zp);
        ss->mp[j] = Mp;
        ss->zp[j] = Zp;
        if (j < a.gamma) {
            combine_stats(a, b, a.n_p_rows + j, &Mq, &Zq);
            ss->mq[j] = Mq;
            ss->zq[j] = Zq;
            double rho;
            if (lqx == -INFINITY) {
                rho = INFINITY;             // q[x] = 0: the token could not have been drafted; accept
            } else {
                rho = exp_nonpos((((double)lpx - (double)Mp) - ((double)lqx - (double)Mq)) / (double)a.temperature) * (Zq / Zp);
            }
            const int acc = u < fmin(1.0, rho) ? 1 : 0;
            const int tie = fabs(u - rho) < kTieEps ? 2 : 0;
            ss->bits[j] = acc | tie;
        }
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
// Zp, Zq exist; it has the fp32 estimate of log(Zp/Zq) from the statistics pass (good to ~1e-6), so it
// sums the entries with d_i above the estimate by more than kSignBand as surely positive, skips those
// below it by more than that, and only counts the ones inside the band: their sign is settled with the
// fp64 denominators by the block that finishes the sequence (a_i/Zp - b_i/Zq > 0, the definition).
constexpr double kSignBand = 1e-5;

template <typename T>
struct DrawPos {
    const T *prow, *qrow;
    double inv_t, mp, mq, delta;
    bool have_q;
    __device__ __forceinline__ void init(const AcceptArgs &a, int b, int n, const DrawRows &d, const SeqStats &ss) {
        const float Mp = ss.mp[d.p_row], Mq = d.have_q ? ss.mq[n] : 0.f;
        const double Zp32 = ss.zp[d.p_row], Zq32 = d.have_q ? ss.zq[n] : 1.0;
        prow = logits_row<T>(a, b, false, d.p_row);
        qrow = logits_row<T>(a, b, true, d.have_q ? n : 0);
        inv_t = 1.0 / (double)a.temperature;
        mp = (double)Mp * inv_t;
        mq = (double)Mq * inv_t;
        delta = (double)logf((float)(Zp32 / Zq32));
        have_q = d.have_q;
    }
    // raw logits of entry i (q's is 0 when there is no q row): plain loads, so callers can issue many
    __device__ __forceinline__ void load(int i, float *lp, float *lq) const {
        *lp = load_elem(prow, i);
        *lq = have_q ? load_elem(qrow, i) : 0.f;
    }
    // (a_i, b_i, class) from the raw logits; class 1: surely positive, 2: inside the band, 0: surely not
    __device__ __forceinline__ void eval(float lp, float lq, double *ea, double *eb, int *cls) const {
        const double xa = fma((double)lp, inv_t, -mp);
        *ea = exp_nonpos(xa);
        if (have_q) {
            const double xb = fma((double)lq, inv_t, -mq);
            *eb = exp_nonpos(xb);
            const double t = (xa - xb) - delta;
            *cls = t > kSignBand ? 1 : (t >= -kSignBand ? 2 : 0);
        } else {
            *eb = 0.0;
            *cls = 1;
        }
    }
};

// fixed-order block sum of NV doubles per thread: butterfly inside each wavefront, the four totals left to right
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

constexpr int kPartStride = 6;      // doubles per (sequence, chunk): sum a, sum b, both over the surely positive
                                    // entries, number of entries inside the sign band, unused

// Grid: rows x n_chunksE blocks.  Every block: first rejection of its sequence, fp64 sums of its chunk of
// the draw position; the block that arrives last at the sequence's counter finishes the draw.
template <typename T>
__global__ __launch_bounds__(kThreads) void accept_draw_kernel(AcceptArgs a) {
    __shared__ SeqStats s_seq;
    __shared__ double s_red[5][kThreads / 64];
    __shared__ double s_scan[kThreads / 64];
    __shared__ double s_w[kMaxChunksE];           // per-chunk weights of this sequence
    __shared__ int s_und[kMaxChunksE];            // entries inside the sign band, per chunk
    __shared__ int s_last, s_cstar, s_best, s_lastpos;
    __shared__ double s_base, s_t;
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
        double acc[5] = {0.0, 0.0, 0.0, 0.0, 0.0};          // sum a, sum b, positive a, positive b, band count
        for (int i0 = e0 + tid; i0 < e1; i0 += 4 * kThreads) {
            float lp[4], lq[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)            // all loads first (out-of-range lanes re-read entry e0)
                w.load(i0 + u * kThreads < e1 ? i0 + u * kThreads : e0, &lp[u], &lq[u]);
            double ea[4], eb[4];
            int cls[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) w.eval(lp[u], lq[u], &ea[u], &eb[u], &cls[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (i0 + u * kThreads < e1) {
                    acc[0] += ea[u];
                    acc[1] += eb[u];
                    if (cls[u] == 1) { acc[2] += ea[u]; acc[3] += eb[u]; }
                    if (cls[u] == 2) acc[4] += 1.0;
                }
            }
        }
        block_sum<5>(acc, s_red);
        if (tid == 0) {
            // hand the sums on as write-through stores, wait for them to be performed, then count this
            // block in; whoever counts last reads all of them back with loads of the same scope
            double *dst = a.part + ((size_t)b * nE + c) * kPartStride;
#pragma unroll
            for (int k = 0; k < 5; ++k) __hip_atomic_store(dst + k, acc[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            const unsigned old = __hip_atomic_fetch_add(a.counter + b, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = old == (unsigned)nE - 1u;
        }
        __syncthreads();
        if (!s_last) return;
    }

    // ---- the last block of the sequence: fp64 denominators, chunk weights, the crossing
    const double *part = a.part + (size_t)b * nE * kPartStride;
    auto part_at = [&](int k, int f) -> double {
        return __hip_atomic_load(part + (size_t)k * kPartStride + f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    const double u = (double)a.u[(size_t)b * (a.gamma + 1) + a.gamma];
    double zz[2] = {0.0, 0.0};
    for (int k = tid; k < nE; k += kThreads) { zz[0] += part_at(k, 0); zz[1] += part_at(k, 1); }
    block_sum<2>(zz, s_red);
    const double inv_zp = 1.0 / zz[0], inv_zq = d.have_q ? 1.0 / zz[1] : 0.0;
    for (int k = tid; k < nE; k += kThreads) {
        s_w[k] = part_at(k, 2) * inv_zp - part_at(k, 3) * inv_zq;
        s_und[k] = (int)part_at(k, 4);
    }
    __syncthreads();
    // chunks with entries inside the sign band: their weight again, every entry's sign from the fp64 weights
    if (d.have_q) {
        for (int k = 0; k < nE; ++k) {
            if (s_und[k] == 0) continue;
            const int f0 = k * a.chunkE, f1 = min(a.V, f0 + a.chunkE);
            double pw[2] = {0.0, 0.0};
            for (int i0 = f0 + tid; i0 < f1; i0 += kThreads) {
                float lp, lq;
                w.load(i0, &lp, &lq);
                double ea, eb;
                int cls;
                w.eval(lp, lq, &ea, &eb, &cls);
                if (ea * inv_zp - eb * inv_zq > 0.0) { pw[0] += ea; pw[1] += eb; }
            }
            block_sum<2>(pw, s_red);
            if (tid == 0) s_w[k] = pw[0] * inv_zp - pw[1] * inv_zq;
        }
        __syncthreads();
    }
    double ms[1] = {0.0};
    for (int k = tid; k < nE; k += kThreads) ms[0] += s_w[k];
    block_sum<1>(ms, s_red);
    double mass = ms[0];
    const bool fall_back_to_p = d.have_q && !(mass > 0.0);
    if (fall_back_to_p) {                         // residual mass 0: draw from p itself
        mass = 1.0;                               // sum of a_i / Zp
        __syncthreads();
        for (int k = tid; k < nE; k += kThreads) s_w[k] = part_at(k, 0) * inv_zp;
        __syncthreads();
    }
    // first chunk whose inclusive prefix exceeds t: each thread owns kMaxChunksE/256 consecutive chunks
    {
        constexpr int CPT = kMaxChunksE / kThreads;
        const double t = u * mass;
        double cw[CPT], lsum = 0.0;
#pragma unroll
        for (int j = 0; j < CPT; ++j) {
            const int k = tid * CPT + j;
            cw[j] = k < nE ? s_w[k] : 0.0;
            lsum += cw[j];
        }
        double incl = lsum;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const double up = __shfl_up(incl, o, 64);
            if ((tid & 63) >= o) incl += up;
        }
        if (tid == 0) { s_best = 0x7fffffff; s_lastpos = -1; s_cstar = 0x7fffffff; }
        if ((tid & 63) == 63) s_scan[tid >> 6] = incl;
        __syncthreads();
        double base = 0.0;
        for (int wvi = 0; wvi < (tid >> 6); ++wvi) base += s_scan[wvi];
        base += incl - lsum;
        int mine = 0x7fffffff, last_nonzero = -1;
        double mybase = 0.0;
#pragma unroll
        for (int j = 0; j < CPT; ++j) {
            const int k = tid * CPT + j;
            if (k < nE) {
                if (cw[j] > 0.0) last_nonzero = k;
                if (mine == 0x7fffffff && base + cw[j] > t) { mine = k; mybase = base; }
                base += cw[j];
            }
        }
        if (mine != 0x7fffffff) atomicMin(&s_cstar, mine);
        if (last_nonzero >= 0) atomicMax(&s_lastpos, last_nonzero);
        __syncthreads();
        const int cstar = s_cstar;
        if (cstar == 0x7fffffff) {                    // rounding left no crossing: last entry with weight
            if (tid == 0) { s_cstar = max(s_lastpos, 0); s_t = INFINITY; s_base = 0.0; }
        } else if (mine == cstar) {                   // exactly one thread owns the crossing chunk
            s_t = t;
            s_base = mybase;
        }
        __syncthreads();
        if (tid == 0) s_lastpos = -1;
    }
    __syncthreads();
    const int cs = s_cstar;
    const double t = s_t;
    const int f0 = cs * a.chunkE, f1 = min(a.V, f0 + a.chunkE);
    // walk the chunk in tiles of 256 x kWalk entries, kWalk consecutive entries per thread, carrying the prefix
    double before = s_base;                       // weight in front of the current tile
    int found = 0x7fffffff, lastpos = -1;
    for (int t0 = f0; t0 < f1; t0 += kThreads * kWalk) {
        const int i0 = min(f1, t0 + tid * kWalk), i1 = min(f1, i0 + kWalk);
        double wv[kWalk];
        double local = 0.0;
        float lp[kWalk], lq[kWalk];
#pragma unroll
        for (int j = 0; j < kWalk; ++j)          // all loads first (idle slots re-read entry f0)
            w.load(i0 + j < i1 ? i0 + j : f0, &lp[j], &lq[j]);
#pragma unroll
        for (int j = 0; j < kWalk; ++j) {
            double ea, eb;
            int cls;
            w.eval(lp[j], lq[j], &ea, &eb, &cls);
            wv[j] = 0.0;
            if (i0 + j < i1) {
                const double r = ea * inv_zp - eb * inv_zq;
                if (fall_back_to_p) wv[j] = ea * inv_zp;
                else if (r > 0.0) wv[j] = r;
            }
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
        for (int j = 0; j < kWalk; ++j) {
            if (i0 + j < i1) {
                if (wv[j] > 0.0) lastpos = i0 + j;
                run += wv[j];
                if (run > t && found == 0x7fffffff) found = i0 + j;
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
    long want = ((long)V * (rows > 0 ? rows : 1) + 1023) / 1024;
    int ce = round_up((int)(want < 512 ? 512 : (want > 8192 ? 8192 : want)), 256);
    if ((V + ce - 1) / ce > kMaxChunksE) ce = kMaxChunkE;
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
    launch_kernel(accept_draw_kernel<T>, gridE, kThreads, 0, stream, a);
}

void launch_accept(const AcceptArgs &a, bool vec_ok, hipStream_t stream) {
    if (a.dtype == PSD_BF16) launch_accept_t<uint16_t>(a, vec_ok, stream);
    else launch_accept_t<float>(a, vec_ok, stream);
}

}  // namespace psd
