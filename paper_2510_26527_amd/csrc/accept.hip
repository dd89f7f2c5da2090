// Speculative-sampling acceptance on gfx950 (the VERIFY loop of Algorithm 1 and the residual
// draw that keeps the verifier's distribution, Sec. 3.1).
//
// Three launches per call, no host round trip (kernel boundaries are the cross-block
// synchronisation: device-scope fences plus a last-block counter measured several times slower):
//   1. accept_stats_kernel  one pass over every logits row of p and q (the HBM-bound part):
//      per (row, chunk) the max raw logit and sum exp((l - max)/T), fp32, wavefront
//      reductions, 8 x 16-byte loads in flight per lane.
//   2. accept_emit_kernel   each block re-derives the first rejection n of its sequence from
//      the statistics (ratio test against the supplied uniforms, prefix scan over <= 64
//      flags) and accumulates, in fp64 and for the ONE position the draw needs, the softmax
//      denominators and the residual mass of its chunk.
//   3. accept_locate_kernel one block per sequence locates the inverse-CDF crossing (chunk, then
//      entry) in index order.
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
constexpr int kMaxPer = kMaxChunkE / 256;   // elements per thread of the locating block

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
    const T *row = logits_row<T>(a, b, is_q, is_q ? r - a.n_p_rows : r);
    const int e0 = c * a.chunkA;
    const int e1 = min(a.V, e0 + a.chunkA);

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

// Ratio tests of sequence b and the scan to the first rejection.  Called by a whole block;
// every thread returns the same n and flags.
template <typename T>
__device__ __forceinline__ void decide(const AcceptArgs &a, int b, int *s_bits, int *n_out, int *flags_out) {
    const int j = threadIdx.x;
    if (j < a.gamma) {
        // the token load heads the only dependent chain (token -> its two logits): start it first
        int x = a.x[(size_t)b * a.gamma + j];
        const double u = (double)a.u[(size_t)b * (a.gamma + 1) + j];
        x = min(max(x, 0), a.V - 1);
        const double lpx = load_elem(logits_row<T>(a, b, false, j), x);
        const double lqx = load_elem(logits_row<T>(a, b, true, j), x);
        float Mp, Mq;
        double Zp, Zq;
        combine_stats(a, b, j, &Mp, &Zp);
        combine_stats(a, b, a.n_p_rows + j, &Mq, &Zq);
        double rho;
        if (lqx == -INFINITY) {
            rho = INFINITY;             // q[x] = 0: the token could not have been drafted; accept
        } else {
            rho = exp_nonpos(((lpx - (double)Mp) - (lqx - (double)Mq)) / (double)a.temperature) * (Zq / Zp);
        }
        const int acc = u < fmin(1.0, rho) ? 1 : 0;
        const int tie = fabs(u - rho) < kTieEps ? 2 : 0;
        s_bits[j] = acc | tie;
    }
    __syncthreads();
    int n = 0, flags = 0;
    for (int k = 0; k < a.gamma; ++k) {
        const int f = s_bits[k];
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

// The draw position of one sequence, as both draw kernels see it.  With a = exp(lp/T - mp),
// b = exp(lq/T - mq) (fp64), the residual weight of entry i is a_i/Zp - b_i/Zq where that is positive.
// Whether it is positive is decided in the log domain against the fp32 statistics of the first pass,
// xa - xb > log(Zp32/Zq32): a fixed rule both kernels share, which lets ONE pass accumulate sum(a),
// sum(b) and the sums over the positive set without knowing the fp64 Zp, Zq yet.  It differs from the
// sign of the fp64 residual only for entries with |p_i - q_i| < ~1e-6 q_i, whose weight is that small.
template <typename T>
struct DrawPos {
    const T *prow, *qrow;
    double inv_t, mp, mq, delta;
    bool have_q;
    __device__ __forceinline__ void init(const AcceptArgs &a, int b, int n, const DrawRows &d) {
        float Mp, Mq = 0.f;
        double Zp32, Zq32 = 1.0;
        combine_stats(a, b, d.p_row, &Mp, &Zp32);
        if (d.have_q) combine_stats(a, b, a.n_p_rows + n, &Mq, &Zq32);
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
    // (a_i, b_i, positive?) from the raw logits
    __device__ __forceinline__ void eval(float lp, float lq, double *ea, double *eb, bool *pos) const {
        const double xa = fma((double)lp, inv_t, -mp);
        *ea = exp_nonpos(xa);
        if (have_q) {
            const double xb = fma((double)lq, inv_t, -mq);
            *eb = exp_nonpos(xb);
            *pos = xa - xb > delta;
        } else {
            *eb = 0.0;
            *pos = true;
        }
    }
};

// Per chunk of the draw position: sum a, sum b, and both sums over the positive set (fp64).
template <typename T>
__global__ __launch_bounds__(kThreads) void accept_emit_kernel(AcceptArgs a) {
    __shared__ int s_bits[64];
    __shared__ double s_red[4][kThreads / 64];
    const int b = blockIdx.x / a.n_chunksE, c = blockIdx.x % a.n_chunksE, tid = threadIdx.x;
    int n, flags;
    decide<T>(a, b, s_bits, &n, &flags);
    const DrawRows d = draw_rows(a, n);
    if (c == 0 && tid == 0) {
        a.out_n[b] = n;
        a.flags[b] = flags;
        if (d.p_row < 0) a.out_tok[b] = -1;
    }
    if (d.p_row < 0) return;
    DrawPos<T> w;
    w.init(a, b, n, d);
    const int e0 = c * a.chunkE, e1 = min(a.V, e0 + a.chunkE);
    double sa = 0.0, sb = 0.0, pa = 0.0, pb = 0.0;
    for (int i0 = e0 + tid; i0 < e1; i0 += 4 * kThreads) {
        float lp[4], lq[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)            // all loads first (out-of-range lanes re-read entry e0)
            w.load(i0 + u * kThreads < e1 ? i0 + u * kThreads : e0, &lp[u], &lq[u]);
        double ea[4], eb[4];
        bool pos[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) w.eval(lp[u], lq[u], &ea[u], &eb[u], &pos[u]);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (i0 + u * kThreads < e1) {
                sa += ea[u];
                sb += eb[u];
                if (pos[u]) { pa += ea[u]; pb += eb[u]; }
            }
        }
    }
    sa = wave_sum(sa); sb = wave_sum(sb); pa = wave_sum(pa); pb = wave_sum(pb);
    if ((tid & 63) == 0) {
        const int wv = tid >> 6;
        s_red[0][wv] = sa; s_red[1][wv] = sb; s_red[2][wv] = pa; s_red[3][wv] = pb;
    }
    __syncthreads();
    if (tid == 0) {
        double t[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) t[k] = ((s_red[k][0] + s_red[k][1]) + s_red[k][2]) + s_red[k][3];
        a.zpart[(size_t)b * a.n_chunksE + c] = make_double2(t[0], t[1]);
        a.ppart[(size_t)b * a.n_chunksE + c] = make_double2(t[2], t[3]);
    }
}

// One block per sequence: fp64 Zp, Zq from the chunk sums, chunk weights, then the inverse-CDF
// crossing of u * mass, first among the chunks (index order), then among the entries of that chunk.
template <typename T>
__global__ __launch_bounds__(kThreads) void accept_locate_kernel(AcceptArgs a) {
    __shared__ double s_red[2][kThreads / 64];
    __shared__ double s_scan[kThreads / 64];
    __shared__ double s_w[kMaxChunksE];          // per-chunk weights of this sequence
    __shared__ int s_cstar, s_best, s_lastpos;
    __shared__ double s_base, s_t;
    const int b = blockIdx.x, tid = threadIdx.x;
    const int n = a.out_n[b];
    const DrawRows d = draw_rows(a, n);
    if (d.p_row < 0) return;
    const int nE = a.n_chunksE;
    const double2 *zp = a.zpart + (size_t)b * nE;
    const double2 *pp = a.ppart + (size_t)b * nE;
    const double u = (double)a.u[(size_t)b * (a.gamma + 1) + a.gamma];
    DrawPos<T> w;
    w.init(a, b, n, d);
    double za = 0.0, zb = 0.0;
    for (int k = tid; k < nE; k += kThreads) { za += zp[k].x; zb += zp[k].y; }
    za = wave_sum(za); zb = wave_sum(zb);
    if ((tid & 63) == 0) { s_red[0][tid >> 6] = za; s_red[1][tid >> 6] = zb; }
    __syncthreads();
    za = ((s_red[0][0] + s_red[0][1]) + s_red[0][2]) + s_red[0][3];
    zb = ((s_red[1][0] + s_red[1][1]) + s_red[1][2]) + s_red[1][3];
    const double inv_zp = 1.0 / za, inv_zq = d.have_q ? 1.0 / zb : 0.0;
    double mass = 0.0;
    for (int k = tid; k < nE; k += kThreads) {
        const double wk = pp[k].x * inv_zp - pp[k].y * inv_zq;
        s_w[k] = wk;
        mass += wk;
    }
    __syncthreads();                              // s_red reuse, s_w complete
    mass = wave_sum(mass);
    if ((tid & 63) == 0) s_red[0][tid >> 6] = mass;
    __syncthreads();
    mass = ((s_red[0][0] + s_red[0][1]) + s_red[0][2]) + s_red[0][3];
    const bool fall_back_to_p = d.have_q && !(mass > 0.0);
    if (fall_back_to_p) {                         // residual mass 0: draw from p itself
        mass = 1.0;                               // sum of a_i / Zp
        for (int k = tid; k < nE; k += kThreads) s_w[k] = zp[k].x * inv_zp;
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
        if (tid == 0) {
            s_lastpos = -1;
            if (fall_back_to_p) a.flags[b] |= PSD_FLAG_ZERO_RESIDUAL;
        }
    }
    __syncthreads();
    const int cs = s_cstar;
    const double t = s_t;
    const int f0 = cs * a.chunkE, f1 = min(a.V, f0 + a.chunkE);
    const int per = (f1 - f0 + kThreads - 1) / kThreads;       // consecutive entries per thread (<= kMaxPer)
    const int i0 = min(f1, f0 + tid * per), i1 = min(f1, i0 + per);
    double wv[kMaxPer];
    double local = 0.0;
    float lp[kMaxPer], lq[kMaxPer];
#pragma unroll
    for (int j = 0; j < kMaxPer; ++j)            // all loads first (idle slots re-read entry f0)
        if (j < per) w.load(i0 + j < i1 ? i0 + j : f0, &lp[j], &lq[j]);
#pragma unroll
    for (int j = 0; j < kMaxPer; ++j) {
        wv[j] = 0.0;
        if (j < per) {
            double ea, eb;
            bool pos;
            w.eval(lp[j], lq[j], &ea, &eb, &pos);
            if (i0 + j < i1) {
                if (fall_back_to_p) wv[j] = ea * inv_zp;
                else if (pos) wv[j] = ea * inv_zp - eb * inv_zq;
            }
        }
    }
#pragma unroll
    for (int j = 0; j < kMaxPer; ++j) local += wv[j];
    // exclusive prefix of `local` over threads, in thread order
    double incl = local;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const double up = __shfl_up(incl, o, 64);
        if ((tid & 63) >= o) incl += up;
    }
    if ((tid & 63) == 63) s_scan[tid >> 6] = incl;
    __syncthreads();
    double run = s_base;
    for (int wvi = 0; wvi < (tid >> 6); ++wvi) run += s_scan[wvi];
    run += incl - local;
    int found = 0x7fffffff, lastpos = -1;
#pragma unroll
    for (int j = 0; j < kMaxPer; ++j) {
        if (i0 + j < i1) {
            if (wv[j] > 0.0) lastpos = i0 + j;
            run += wv[j];
            if (run > t && found == 0x7fffffff) found = i0 + j;
        }
    }
    if (found != 0x7fffffff) atomicMin(&s_best, found);
    if (lastpos >= 0) atomicMax(&s_lastpos, lastpos);
    __syncthreads();
    if (tid == 0) {
        int tok = s_best;
        if (tok == 0x7fffffff) tok = s_lastpos >= 0 ? s_lastpos : f1 - 1;
        a.out_tok[b] = tok;
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

size_t accept_workspace_bytes(const AcceptArgs &a) {
    const size_t rows = a.rows > 0 ? a.rows : 1;
    size_t b = 0;
    b += align256(rows * (a.n_p_rows + a.gamma) * a.n_chunksA * sizeof(float2));
    b += align256(rows * a.n_chunksE * sizeof(double2));
    b += align256(rows * a.n_chunksE * sizeof(double2));
    b += align256(rows * sizeof(int32_t));
    return b;
}

void accept_bind_workspace(AcceptArgs *a, void *ws, int32_t *out_flags) {
    const size_t rows = a->rows > 0 ? a->rows : 1;
    char *p = (char *)ws;
    a->stats = (float2 *)p;   p += align256(rows * (a->n_p_rows + a->gamma) * a->n_chunksA * sizeof(float2));
    a->zpart = (double2 *)p;  p += align256(rows * a->n_chunksE * sizeof(double2));
    a->ppart = (double2 *)p;  p += align256(rows * a->n_chunksE * sizeof(double2));
    a->flags = out_flags ? out_flags : (int32_t *)p;
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
    {
        ScopedProf sp(PSD_KIND_ACCEPT_EMIT, stream);
        launch_kernel(accept_emit_kernel<T>, gridE, kThreads, 0, stream, a);
    }
    {
        ScopedProf sp(PSD_KIND_ACCEPT_LOCATE, stream);
        launch_kernel(accept_locate_kernel<T>, a.rows, kThreads, 0, stream, a);
    }
}

void launch_accept(const AcceptArgs &a, bool vec_ok, hipStream_t stream) {
    if (a.dtype == PSD_BF16) launch_accept_t<uint16_t>(a, vec_ok, stream);
    else launch_accept_t<float>(a, vec_ok, stream);
}

}  // namespace psd
