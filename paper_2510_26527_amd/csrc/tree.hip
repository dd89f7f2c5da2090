// Token-tree verification (Related Work, "Verification Mechanisms": token-tree-based verification; Sec. 4.6 names
// deeper and wider drafting as the next step).  The paper prints no rule; the one used is multi-round speculative
// sampling for sibling tokens drawn independently from the drafter's distribution at their parent, which leaves the
// verifier's distribution unchanged (Abstract; Sec. 3.1).
//
//   tree_setup_kernel        the tree's shape (ancestor bit masks, depths) from kernel arguments into device memory,
//                            where the embedding and attention kernels of a tree forward pass read it;
//   tree_accept_kernel       one block per sequence walks the tree from the root: at a node the children are tried in
//                            index order against the running residual of the verifier's distribution, the first
//                            accepted child is descended into, and where none is accepted one token is drawn from
//                            what is left;
//   kv_compact_tree_kernel   after acceptance: the accepted nodes' K/V rows move to consecutive cache positions.
//
// The residual after j refusals at one node needs no vector: with p, q the two distributions at the node,
//   r_0 = p,  r_{j+1} = norm(max(0, r_j - q))   =>   r_j is proportional to R_j = max(0, p - c_j q),
//   c_0 = 0,  c_{j+1} = c_j + M_j,  M_j = sum_i R_j[i]  (M_0 = 1),
// (induction: max(0, R_j / M_j - q) = max(0, p - (c_j + M_j) q) / M_j), so a refusal costs one pass over the
// vocabulary for M_{j+1}, and child j + 1 with token x is accepted with probability min(1, R_j[x] / (M_j q[x])).
// Everything that decides a token runs in fp64 with a fixed summation order.
#include "common.h"
#include "kernels.h"
#include "exp64.h"
#include "prof.h"
#include "../../include/psd.h"

namespace psd {
namespace {

constexpr int kTreeThreads = 1024;
constexpr int kTreeWaves = kTreeThreads / 64;

__global__ void tree_setup_kernel(TreeShape ts, uint32_t *anc, int32_t *depth) {
    const int t = threadIdx.x;
    // static indices into the kernel arguments, selected per lane
#pragma unroll
    for (int j = 0; j < kTreeMaxNodes; ++j)
        if (t == j && j < ts.n) {
            anc[j] = ts.anc[j];
            depth[j] = ts.depth[j];
        }
}

// block-wide sum in a fixed order: butterfly inside each wavefront, wavefronts added in order; every thread gets it
__device__ __forceinline__ double block_sum_d(double v, double *s_w) {
    v = wave_sum(v);
    __syncthreads();                                       // s_w may still be read from the previous call
    if ((threadIdx.x & 63) == 0) s_w[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = 0.0;
#pragma unroll
    for (int w = 0; w < kTreeWaves; ++w) t += s_w[w];
    return t;
}
__device__ __forceinline__ float block_max_f(float v, float *s_w) {
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_w[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = s_w[0];
#pragma unroll
    for (int w = 1; w < kTreeWaves; ++w) t = fmaxf(t, s_w[w]);
    return t;
}

template <typename T>
__global__ __launch_bounds__(kTreeThreads) void tree_accept_kernel(TreeAcceptArgs a) {
    __shared__ double s_wd[kTreeWaves];
    __shared__ float s_wf[kTreeWaves];
    __shared__ int s_par[kTreeMaxAcceptNodes];
    __shared__ int s_pick, s_lastpos;
    __shared__ unsigned long long s_best;
    __shared__ double s_exp2[64];                           // kExp2Table, for exp_nonpos
    const int row = blockIdx.x, tid = threadIdx.x, n = a.n_nodes, V = a.vocab;
    for (int j = tid; j < n; j += kTreeThreads) s_par[j] = a.parents[j];
    if (tid < 64) s_exp2[tid] = kExp2Table[tid];
    __syncthreads();
    const T *P = (const T *)a.p + (size_t)row * a.p_stride;
    const T *Q = (const T *)a.q + (size_t)row * a.q_stride;
    const int32_t *tok = a.tokens + (size_t)row * n;
    const float *u = a.uniforms ? a.uniforms + (size_t)row * (n + 1) : nullptr;
    const bool greedy = a.temperature == 0.f;
    const double Tm = (double)a.temperature, inv_t = 1.0 / Tm;
    // exp(logit / T - max / T): the scaled logit minus the row's scaled maximum is never positive
    auto ex = [&](float logit, double m) { return exp_nonpos(fma((double)logit, inv_t, -m), s_exp2); };
    int32_t *path = a.out_path + (size_t)row * n;
    int node = 0, plen = 0, flags = 0;

    while (true) {                                          // every descent moves to a larger node index: at most n rounds
        const T *lp = P + (size_t)node * V;
        const T *lq = Q + (size_t)node * V;
        if (greedy) {
            // the verifier's most likely token, lowest index among equals
            unsigned long long best = 0ull;                 // (order-preserving bits of the logit) << 32 | ~index
            for (int i = tid; i < V; i += kTreeThreads) {
                const float x = load_elem(lp, (size_t)i);
                uint32_t b = __float_as_uint(x);
                b = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
                const unsigned long long key = ((unsigned long long)b << 32) | (uint32_t)(~(uint32_t)i);
                best = key > best ? key : best;
            }
            best = wave_max(best);
            if (tid == 0) s_best = 0ull;
            __syncthreads();
            if ((tid & 63) == 0) atomicMax(&s_best, best);
            __syncthreads();
            const int top = (int)(~(uint32_t)(s_best & 0xffffffffull));
            int next = -1;
            for (int c = node + 1; c < n && next < 0; ++c)
                if (s_par[c] == node && tok[c] == top) next = c;
            __syncthreads();                                // s_best is reset by the next round
            if (next < 0) {
                if (tid == 0) { a.out_path_len[row] = plen; a.out_token[row] = top; if (a.out_flags) a.out_flags[row] = 0; }
                return;
            }
            if (tid == 0) path[plen] = next;
            ++plen;
            node = next;
            continue;
        }

        // ---- softmax statistics of the two rows at this node: s_i = logit_i / T, max, sum of exp(s_i - max)
        float mpf = -INFINITY, mqf = -INFINITY;
        for (int i = tid; i < V; i += kTreeThreads) {
            mpf = fmaxf(mpf, load_elem(lp, (size_t)i));
            mqf = fmaxf(mqf, load_elem(lq, (size_t)i));
        }
        const double mp = (double)block_max_f(mpf, s_wf) * inv_t, mq = (double)block_max_f(mqf, s_wf) * inv_t;
        double zp = 0.0, zq = 0.0;
        for (int i = tid; i < V; i += kTreeThreads) {
            zp += ex(load_elem(lp, (size_t)i), mp);
            zq += ex(load_elem(lq, (size_t)i), mq);
        }
        const double Zp = block_sum_d(zp, s_wd), Zq = block_sum_d(zq, s_wd);
        const double inv_zp = 1.0 / Zp, inv_zq = 1.0 / Zq;       // one division per row, not one per entry
        double c = 0.0, mass = 1.0;                         // the residual here is max(0, p - c q) / mass

        int next = -1;
        for (int ch = node + 1; ch < n; ++ch) {
            if (s_par[ch] != node) continue;
            int x = tok[ch];
            x = min(max(x, 0), V - 1);
            const double px = ex(load_elem(lp, (size_t)x), mp) * inv_zp;
            const double qx = ex(load_elem(lq, (size_t)x), mq) * inv_zq;
            const double rx = fmax(px - c * qx, 0.0);
            const double ratio = qx == 0.0 ? INFINITY : rx / (mass * qx);
            const double thr = fmin(1.0, ratio), uu = (double)u[ch];
            if (fabs(uu - thr) < 1e-5) flags |= PSD_FLAG_NEAR_TIE;
            if (uu < thr) { next = ch; break; }
            // refused: take the drafter's share out of what is left
            const double c2 = c + mass;
            double m2 = 0.0;
            for (int i = tid; i < V; i += kTreeThreads) {
                const double pi = ex(load_elem(lp, (size_t)i), mp) * inv_zp;
                const double qi = ex(load_elem(lq, (size_t)i), mq) * inv_zq;
                m2 += fmax(pi - c2 * qi, 0.0);
            }
            m2 = block_sum_d(m2, s_wd);
            if (m2 > 0.0) { c = c2; mass = m2; }            // mass 0: the residual equalled q, where no refusal can happen
        }
        if (next >= 0) {
            if (tid == 0) path[plen] = next;
            ++plen;
            node = next;
            continue;
        }

        // ---- no child accepted: one draw from max(0, p - c q) by inverse CDF in index order.  Thread t owns the
        // contiguous entries [t * per, (t + 1) * per); prefix sums over threads in a fixed order.
        const int per = (V + kTreeThreads - 1) / kTreeThreads;
        const int i0 = min(tid * per, V), i1 = min(i0 + per, V);
        double w = 0.0;
        int lastpos = -1;
        for (int i = i0; i < i1; ++i) {
            const double pi = ex(load_elem(lp, (size_t)i), mp) * inv_zp;
            const double qi = ex(load_elem(lq, (size_t)i), mq) * inv_zq;
            const double r = fmax(pi - c * qi, 0.0);
            if (r > 0.0) lastpos = i;
            w += r;
        }
        // inclusive prefix inside the wavefront, then the wavefronts before it
        double incl = w;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const double up = __shfl_up(incl, o, 64);
            if ((tid & 63) >= o) incl += up;
        }
        __syncthreads();
        if ((tid & 63) == 63) s_wd[tid >> 6] = incl;
        if (tid == 0) { s_pick = kTreeThreads; s_lastpos = -1; }
        __syncthreads();
        double before = 0.0, total = 0.0;
#pragma unroll
        for (int wv = 0; wv < kTreeWaves; ++wv) {
            if (wv < (tid >> 6)) before += s_wd[wv];
            total += s_wd[wv];
        }
        const double target = (double)u[n] * total;
        if (w > 0.0 && before + incl > target) atomicMin(&s_pick, tid);
        if (lastpos >= 0) atomicMax(&s_lastpos, lastpos);
        __syncthreads();
        if (tid == s_pick) {
            double cum = before + incl - w;
            int token = lastpos;                            // rounding left no crossing inside: the last positive entry
            for (int i = i0; i < i1; ++i) {
                const double pi = ex(load_elem(lp, (size_t)i), mp) * inv_zp;
                const double qi = ex(load_elem(lq, (size_t)i), mq) * inv_zq;
                cum += fmax(pi - c * qi, 0.0);
                if (cum > target) { token = i; break; }
            }
            a.out_token[row] = token;
        }
        if (tid == 0) {
            if (s_pick == kTreeThreads) a.out_token[row] = s_lastpos;      // no crossing at all: last positive entry
            a.out_path_len[row] = plen;
            if (a.out_flags) a.out_flags[row] = flags;
        }
        return;
    }
}

// One block per (layer, sequence, KV head).  Thread t moves element t of the d_h-long K row and of the V^T column of
// every accepted node, in path order: destination j is never a later source (sources grow along a path and a
// source is never below its destination), and each element has one thread, so no synchronisation is needed.
template <typename T>
__global__ __launch_bounds__(128) void kv_compact_tree_kernel(T *k, T *v, int32_t *lens, const int32_t *base,
                                                              const int32_t *path, const int32_t *path_len, int path_stride,
                                                              int n_nodes, int B, int h_kv, int d_h, int max_len, int cap) {
    const int hk = blockIdx.x % h_kv, b = (blockIdx.x / h_kv) % B;
    const size_t head = (size_t)blockIdx.x * max_len * d_h;           // blockIdx.x = (l * B + b) * h_kv + hk
    T *kh = k + head, *vh = v + head;
    const int s0 = base[b];
    int plen = path_len[b];
    plen = min(max(plen, 0), n_nodes - 1);
    for (int j = 0; j < plen; ++j) {
        const int node = path[(size_t)b * path_stride + j];
        const int src = s0 + node, dst = s0 + 1 + j;
        if (node < 1 || node >= n_nodes || src >= max_len || src == dst) continue;
        for (int t = threadIdx.x; t < d_h; t += blockDim.x) {
            kh[(size_t)dst * d_h + t] = kh[(size_t)src * d_h + t];
            vh[(size_t)t * max_len + dst] = vh[(size_t)t * max_len + src];
        }
    }
    if (blockIdx.x / (h_kv * B) == 0 && hk == 0 && threadIdx.x == 0) lens[b] = max(0, min(min(lens[b], cap), s0 + 1 + plen));
}

}  // namespace

void launch_tree_setup(const TreeShape &ts, uint32_t *anc, int32_t *depth, hipStream_t stream) {
    ScopedProf sp(PSD_KIND_LENS, stream);
    launch_kernel(tree_setup_kernel, 1, 64, 0, stream, ts, anc, depth);
}

void launch_tree_accept(int dtype, const TreeAcceptArgs &a, hipStream_t stream) {
    ScopedProf sp(PSD_KIND_ACCEPT_DRAW, stream);
    if (dtype == PSD_BF16) launch_kernel(tree_accept_kernel<uint16_t>, a.rows, kTreeThreads, 0, stream, a);
    else launch_kernel(tree_accept_kernel<float>, a.rows, kTreeThreads, 0, stream, a);
}

void launch_kv_compact_tree(int dtype, void *k, void *v, int32_t *lens, const int32_t *base, const int32_t *path,
                            const int32_t *path_len, int path_stride, int n_nodes, int L, int B, int h_kv, int d_h,
                            int max_len, int cap, hipStream_t stream) {
    ScopedProf sp(PSD_KIND_LENS, stream);
    const unsigned grid = (unsigned)((size_t)L * B * h_kv);
    if (dtype == PSD_BF16)
        launch_kernel(kv_compact_tree_kernel<uint16_t>, grid, 128, 0, stream, (uint16_t *)k, (uint16_t *)v, lens, base, path,
                      path_len, path_stride, n_nodes, B, h_kv, d_h, max_len, cap);
    else
        launch_kernel(kv_compact_tree_kernel<float>, grid, 128, 0, stream, (float *)k, (float *)v, lens, base, path,
                      path_len, path_stride, n_nodes, B, h_kv, d_h, max_len, cap);
}

}  // namespace psd
