// Internal launch interface between the C-ABI layer (api.hip) and the kernel files.
// Every launcher only enqueues work on `stream`; shapes were validated by the caller.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace psd {

// ---------------------------------------------------------------- acceptance (accept.hip)
struct AcceptArgs {
    const void *p, *q;            // logits, [rows][n_p_rows][V] / [rows][gamma][V]
    const int32_t *x;             // draft tokens [rows][gamma]
    const float *u;               // uniforms [rows][gamma+1]
    int rows, gamma, n_p_rows, V;
    int64_t p_stride, q_stride;   // elements between consecutive sequences
    int dtype;                    // PSD_F32 / PSD_BF16
    float temperature;
    int chunkA, n_chunksA;        // statistics pass: elements per block, blocks per logits row
    int chunkE, n_chunksE;        // draw pass chunking
    float2 *stats;                // [rows][n_p_rows+gamma][n_chunksA] (max raw logit, sum exp)
    double2 *zpart;               // [rows][n_chunksE] fp64 partial softmax denominators (p, q)
    double *rpart;                // [rows][n_chunksE] fp64 partial residual mass
    uint32_t *counters;           // [rows] arrival counters of the draw pass
    int32_t *out_n, *out_tok, *flags;
};
// vec: rows are 16-byte aligned and V is a multiple of the elements per 16-byte load
void accept_plan(int rows, int gamma, int n_p_rows, int V, int dtype, bool vec, AcceptArgs *a);
size_t accept_workspace_bytes(const AcceptArgs &a);
void accept_bind_workspace(AcceptArgs *a, void *ws, int32_t *out_flags);
void launch_accept(const AcceptArgs &a, bool vec_ok, hipStream_t stream);

// ---------------------------------------------------------------- GEMMs (gemm.hip)
// y[m][n] = sum_k x[m][k] * W[n][k]; W is up to three row-major [n_i][K] matrices whose
// outputs are concatenated along n (QKV, gate|up).
struct GemmArgs {
    const float *x;               // [M][K] fp32 activations
    const void *w[3];
    int n[3];
    int nseg;
    int M, K, N;                  // N = sum n[i]
    float *out;                   // [M][ldo] fp32
    int ldo;
    int accumulate;               // 0: out = y, 1: out += y (residual stream)
    float *partial;               // split-K scratch [splitk][M][N] fp32 (bf16 kernels)
    int splitk;
};
int gemm_pick_splitk(int dtype, int M, int K, int N, const int *n, int nseg);
void launch_gemm(int dtype, const GemmArgs &g, hipStream_t stream);

// ---------------------------------------------------------------- attention (attention.hip)
struct AttnArgs {
    const float *q;               // [B][R][h_q][d_h] rotated queries, fp32
    const void *k;                // this layer's K cache [B][h_kv][max_len][d_h]
    const void *v;                // this layer's V cache [B][h_kv][d_h][max_len]
    const int32_t *lens;          // [B] valid positions BEFORE this forward
    float *out;                   // [B][R][h_q*d_h] fp32
    int B, R, h_q, h_kv, d_h, max_len;
    int len_bound;                // host upper bound of lens[b] + R
    float *part_o;                // split scratch [B][h_q][R][splits][d_h]
    float *part_ml;               // [B][h_q][R][splits][2]
    int splits;
};
int attn_pick_splits(int dtype, int B, int R, int h_q, int h_kv, int d_h, int len_bound);
void launch_attention(int dtype, const AttnArgs &a, hipStream_t stream);

// ---------------------------------------------------------------- row-wise kernels (rowwise.hip)
void launch_embed(int dtype, const void *embed, const int32_t *tokens, float *x, int M, int d,
                  int vocab, hipStream_t stream);
// out = x * rsqrt(mean(x^2) + eps) * gain (fp32); gain has the model's dtype
void launch_rmsnorm(int dtype, const float *x, const void *gain, void *out, int M, int d, float eps,
                    int row_stride_x, hipStream_t stream);
// qkv fp32 [M][(h_q+2h_kv) d_h] -> rotated q (fp32), rotated k and v appended to the cache (model dtype)
void launch_rope_append(int dtype, const float *qkv, void *q_out, void *k_cache, void *v_cache,
                        const int32_t *lens, int B, int R, int h_q, int h_kv, int d_h, int max_len,
                        float theta, hipStream_t stream);
// h = silu(gu[:, :f]) * gu[:, f:] (fp32)
void launch_swiglu(int dtype, const float *gu, void *h, int M, int f, hipStream_t stream);
void launch_advance_lens(int32_t *lens, int B, int delta, int max_len, hipStream_t stream);
void launch_truncate(int32_t *lens, const int32_t *base, const int32_t *keep, int offset, int B,
                     hipStream_t stream);
void launch_truncate_to(int32_t *lens, int new_len, int B, hipStream_t stream);

}  // namespace psd
