// Speculative-sampling acceptance on gfx950 (the VERIFY loop of Algorithm 1 and the residual
// draw that keeps the verifier's distribution, Sec. 3.1).
//
// Four launches per call, no host round trip (kernel boundaries are the cross-block
// synchronisation: device-scope fences plus a last-block counter measured several times slower):
//   1. accept_stats_kernel  one pass over every logits row of p and q (the HBM-bound part):
//      per (row, chunk) the max raw logit and sum exp((l - max)/T), fp32, wavefront
//      reductions, 8 x 16-byte loads in flight per lane.
//   2. accept_emit_z_kernel each block re-derives the first rejection n of its sequence from
//      the statistics (ratio test against the supplied uniforms, prefix scan over <= 64
//      flags) and accumulates, in fp64, the softmax denominators of the ONE position the
//      draw needs.
//   3. accept_emit_r_kernel fp64 residual mass per chunk.
//   4. accept_locate_kernel one block per sequence locates the inverse-CDF crossing (chunk, then
//      element) in index order.
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

// block-wide fixed-order sum of one double per thread; result valid in every thread
__device__ __forceinline__ double block_sum(double v, double *smem) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = 0.0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) t += smem[w];
    return t;
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

// (max raw logit, sum exp((l - max)/T)) of one logits row from its per-chunk statistics
__device__ __forceinline__ void combine_stats(const AcceptArgs &a, int b, int r, float *M, double *Z) {
    const float2 *st = a.stats + ((size_t)b * (a.n_p_rows + a.gamma) + r) * a.n_chunksA;
    float m = -INFINITY;
    for (int c = 0; c < a.n_chunksA; ++c) m = fmaxf(m, st[c].x);
    double z = 0.0;
    const double invT = 1.0 / (double)a.temperature;
    for (int c = 0; c < a.n_chunksA; ++c)
        if (st[c].x > -INFINITY) z += (double)st[c].y * exp(((double)st[c].x - (double)m) * invT);
    *M = m;
    *Z = z;
}

// Ratio tests of sequence b and the scan to the first rejection.  Called by a whole block;
// every thread returns the same n and flags.
template <typename T>
__device__ __forceinline__ void decide(const AcceptArgs &a, int b, int *s_bits, int *n_out, int *flags_out) {
    const int j = threadIdx.x;
    if (j < a.gamma) {
        float Mp, Mq;
        double Zp, Zq;
        combine_stats(a, b, j, &Mp, &Zp);
        combine_stats(a, b, a.n_p_rows + j, &Mq, &Zq);
        int x = a.x[(size_t)b * a.gamma + j];
        x = min(max(x, 0), a.V - 1);
        const double lpx = load_elem(logits_row<T>(a, b, false, j), x);
        const double lqx = load_elem(logits_row<T>(a, b, true, j), x);
        double rho;
        if (lqx == -INFINITY) {
            rho = INFINITY;             // q[x] = 0: the token could not have been drafted; accept
        } else {
            rho = exp(((lpx - (double)Mp) - (lqx - (double)Mq)) / (double)a.temperature) * (Zq / Zp);
        }
        const double u = (double)a.u[(size_t)b * (a.gamma + 1) + j];
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

template <typename T>
__global__ __launch_bounds__(kThreads) void accept_emit_z_kernel(AcceptArgs a) {
    __shared__ int s_bits[64];
    __shared__ double s_red[kThreads / 64];
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
    float Mp, Mq = 0.f;
    double Z_unused;
    combine_stats(a, b, d.p_row, &Mp, &Z_unused);
    if (d.have_q) combine_stats(a, b, a.n_p_rows + n, &Mq, &Z_unused);
    const double temp = (double)a.temperature;
    const double mp = (double)Mp * (1.0 / temp), mq = (double)Mq * (1.0 / temp);
    const T *prow = logits_row<T>(a, b, false, d.p_row);
    const T *qrow = logits_row<T>(a, b, true, d.have_q ? n : 0);
    const int e0 = c * a.chunkE, e1 = min(a.V, e0 + a.chunkE);
    const double inv_t = 1.0 / temp;
    double sa = 0.0, sb = 0.0;
    for (int i0 = e0 + tid; i0 < e1; i0 += 4 * kThreads) {
        double ea[4], eb[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {          // four independent elements in flight per thread
            const int i = i0 + u * kThreads;
            const bool in = i < e1;
            ea[u] = in ? exp_nonpos(fma((double)load_elem(prow, in ? i : e0), inv_t, -mp)) : 0.0;
            eb[u] = (in && d.have_q) ? exp_nonpos(fma((double)load_elem(qrow, in ? i : e0), inv_t, -mq)) : 0.0;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) { sa += ea[u]; sb += eb[u]; }
    }
    sa = block_sum(sa, s_red);
    sb = block_sum(sb, s_red);
    if (tid == 0) a.zpart[(size_t)b * a.n_chunksE + c] = make_double2(sa, sb);
}

// residual weight of element i of the draw position (unnormalised by the residual mass)
template <typename T>
struct DrawWeights {
    const T *prow, *qrow;
    double inv_t, mp, mq, inv_zp, inv_zq;
    bool have_q;
    __device__ __forceinline__ double operator()(int i) const {
        const double pi = exp_nonpos(fma((double)load_elem(prow, i), inv_t, -mp)) * inv_zp;
        if (!have_q) return pi;
        const double qi = exp_nonpos(fma((double)load_elem(qrow, i), inv_t, -mq)) * inv_zq;
        const double r = pi - qi;
        return r > 0.0 ? r : 0.0;
    }
};

template <typename T>
__global__ __launch_bounds__(kThreads) void accept_emit_r_kernel(AcceptArgs a) {
    __shared__ double s_red[kThreads / 64];
    const int b = blockIdx.x / a.n_chunksE, c = blockIdx.x % a.n_chunksE, tid = threadIdx.x;
    const int n = a.out_n[b];
    const DrawRows d = draw_rows(a, n);
    if (d.p_row < 0) return;
    const int nE = a.n_chunksE;
    const double2 *zp = a.zpart + (size_t)b * nE;
    double za = 0.0, zb = 0.0;
    for (int k = tid; k < nE; k += kThreads) { za += zp[k].x; zb += zp[k].y; }
    za = block_sum(za, s_red);
    zb = block_sum(zb, s_red);
    float Mp, Mq = 0.f;
    double Z_unused;
    combine_stats(a, b, d.p_row, &Mp, &Z_unused);
    if (d.have_q) combine_stats(a, b, a.n_p_rows + n, &Mq, &Z_unused);
    DrawWeights<T> w;
    w.prow = logits_row<T>(a, b, false, d.p_row);
    w.qrow = logits_row<T>(a, b, true, d.have_q ? n : 0);
    w.inv_t = 1.0 / (double)a.temperature;
    w.mp = (double)Mp * w.inv_t;
    w.mq = (double)Mq * w.inv_t;
    w.inv_zp = 1.0 / za;
    w.inv_zq = d.have_q ? 1.0 / zb : 0.0;
    w.have_q = d.have_q;

    const int e0 = c * a.chunkE, e1 = min(a.V, e0 + a.chunkE);
    double rs = 0.0;
    for (int i0 = e0 + tid; i0 < e1; i0 += 4 * kThreads) {
        double t[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + u * kThreads;
            t[u] = i < e1 ? w(i) : 0.0;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) rs += t[u];
    }
    rs = block_sum(rs, s_red);
    if (tid == 0) a.rpart[(size_t)b * nE + c] = rs;
}

// One block per sequence: locate the inverse-CDF crossing of u * mass, first among the chunk sums
// (index order), then among the elements of that chunk.
template <typename T>
__global__ __launch_bounds__(kThreads) void accept_locate_kernel(AcceptArgs a) {
    __shared__ double s_red[kThreads / 64];
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
    double za = 0.0, zb = 0.0;
    for (int k = tid; k < nE; k += kThreads) { za += zp[k].x; zb += zp[k].y; }
    za = block_sum(za, s_red);
    zb = block_sum(zb, s_red);
    float Mp, Mq = 0.f;
    double Z_unused;
    combine_stats(a, b, d.p_row, &Mp, &Z_unused);
    if (d.have_q) combine_stats(a, b, a.n_p_rows + n, &Mq, &Z_unused);
    DrawWeights<T> w;
    w.prow = logits_row<T>(a, b, false, d.p_row);
    w.qrow = logits_row<T>(a, b, true, d.have_q ? n : 0);
    w.inv_t = 1.0 / (double)a.temperature;
    w.mp = (double)Mp * w.inv_t;
    w.mq = (double)Mq * w.inv_t;
    w.inv_zp = 1.0 / za;
    w.inv_zq = d.have_q ? 1.0 / zb : 0.0;
    w.have_q = d.have_q;

    // ---- last block of this sequence: locate the crossing of u * mass in index order
    const double *rp = a.rpart + (size_t)b * nE;
    double mass = 0.0;
    for (int k = tid; k < nE; k += kThreads) {
        const double wk = rp[k];
        s_w[k] = wk;
        mass += wk;
    }
    mass = block_sum(mass, s_red);
    const bool fall_back_to_p = d.have_q && !(mass > 0.0);
    if (fall_back_to_p) {                  // residual mass 0: draw from p itself
        w.have_q = false;
        mass = 1.0;                        // sum of a_i / Z_p
        for (int k = tid; k < nE; k += kThreads) s_w[k] = zp[k].x * w.inv_zp;
        __syncthreads();
    }
    if (tid == 0) {
        const double u = (double)a.u[(size_t)b * (a.gamma + 1) + a.gamma];
        const double t = u * mass;
        double base = 0.0;
        int cstar = -1, last_nonzero = -1;
        for (int k = 0; k < nE; ++k) {
            const double wk = s_w[k];
            if (wk > 0.0) last_nonzero = k;
            if (base + wk > t) { cstar = k; break; }
            base += wk;
        }
        if (cstar < 0) {                   // rounding left no crossing: last element with weight
            cstar = max(last_nonzero, 0);
            s_t = INFINITY;
        } else {
            s_t = t;
        }
        s_cstar = cstar;
        s_base = base;
        s_best = 0x7fffffff;
        s_lastpos = -1;
        if (fall_back_to_p) a.flags[b] |= PSD_FLAG_ZERO_RESIDUAL;
    }
    __syncthreads();
    const int cs = s_cstar;
    const double t = s_t;
    const int f0 = cs * a.chunkE, f1 = min(a.V, f0 + a.chunkE);
    const int per = (f1 - f0 + kThreads - 1) / kThreads;       // consecutive elements per thread (<= kMaxPer)
    const int i0 = min(f1, f0 + tid * per), i1 = min(f1, i0 + per);
    double wv[kMaxPer];
    double local = 0.0;
#pragma unroll
    for (int j = 0; j < kMaxPer; ++j) {
        wv[j] = (j < per && i0 + j < i1) ? w(i0 + j) : 0.0;
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
    b += align256(rows * a.n_chunksE * sizeof(double));
    b += align256(rows * sizeof(uint32_t));
    b += align256(rows * sizeof(int32_t));
    return b;
}

void accept_bind_workspace(AcceptArgs *a, void *ws, int32_t *out_flags) {
    const size_t rows = a->rows > 0 ? a->rows : 1;
    char *p = (char *)ws;
    a->stats = (float2 *)p;   p += align256(rows * (a->n_p_rows + a->gamma) * a->n_chunksA * sizeof(float2));
    a->zpart = (double2 *)p;  p += align256(rows * a->n_chunksE * sizeof(double2));
    a->rpart = (double *)p;   p += align256(rows * a->n_chunksE * sizeof(double));
    a->counters = (uint32_t *)p; p += align256(rows * sizeof(uint32_t));
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
        ScopedProf sp(PSD_KIND_ACCEPT_EMIT_Z, stream);
        launch_kernel(accept_emit_z_kernel<T>, gridE, kThreads, 0, stream, a);
    }
    {
        ScopedProf sp(PSD_KIND_ACCEPT_EMIT_R, stream);
        launch_kernel(accept_emit_r_kernel<T>, gridE, kThreads, 0, stream, a);
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
