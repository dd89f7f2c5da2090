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
    float *xlogit;                // [rows][gamma][2] the draft token's logit under p and under q
    double *part;                 // [rows][n_chunksE][6] fp64 chunk sums of the draw position (accept.hip)
    uint32_t *counter;            // [rows] chunks of the draw position done so far
    int32_t *out_n, *out_tok, *flags;
};
// vec: rows are 16-byte aligned and V is a multiple of the elements per 16-byte load
void accept_plan(int rows, int gamma, int n_p_rows, int V, int dtype, bool vec, AcceptArgs *a);
size_t accept_workspace_bytes(const AcceptArgs &a);
void accept_bind_workspace(AcceptArgs *a, void *ws, int32_t *out_flags);
void launch_accept(const AcceptArgs &a, bool vec_ok, hipStream_t stream);
// temperature 0: greedy verification (greedy.hip); reads p and x only, same workspace
void launch_accept_greedy(const AcceptArgs &a, bool vec_ok, hipStream_t stream);

// ---------------------------------------------------------------- GEMMs (gemm.hip)
// Up to this many rows (one 16-row MFMA tile) the bf16 projections stream the weights straight into MFMA
// operands (HBM-bound); above it the activation operand traffic of that scheme outgrows the weights and the
// LDS-tiled kernel wins (measured on two LLaMA2-7B-shaped layers: 0.28 ms at 16 rows; at 32 rows 0.43 ms
// streaming against 0.38 ms tiled, at 64 rows 0.66 against 0.38).
constexpr int kStreamMaxRows = 16;
// y[m][n] = sum_k x[m][k] * W[n][k]; W is up to three row-major [n_i][K] matrices whose
// outputs are concatenated along n (QKV, gate|up).
// r_m from per-tile sums of squares: rsqrt(sum_t sumsq[t * M + m] * inv_d + eps); sumsq NULL: 1
struct RowScale {
    const float *sumsq;
    int tiles;
    float inv_d, eps;
};
struct GemmArgs {
    const float *x;               // fp32 activations, K contiguous; row m is read from source row
                                  //   (m / x_rows_per_group) * x_group_stride + x_group_offset + m % x_rows_per_group
    const uint16_t *x16;          // optional: the same matrix already rounded to fp16 (what the tiled kernel multiplies)
    int x_rows_per_group, x_group_stride, x_group_offset;
    const void *w[3];
    int n[3];
    int nseg;
    int M, K, N;                  // N = sum n[i]
    const void *wpack;            // optional repacked copy of all segments (bf16, M <= kStreamMaxRows): see gemm.hip
    int pack_tiles;               //   its number of 64-row tiles
    float *partial;               // [splitk][M][N] fp32: split s holds its share of the K sum
    int splitk;
    float *reduced;               // if non-NULL: [M][N] <- sum over splits (logits), times the row scale if given
    // -- bf16, M <= kStreamMaxRows, packed weights only: RMSNorm folded into the projections around it -----------
    // rmsnorm(x) W^T = r_m * ((x * gain) W^T) with r_m = rsqrt(mean_k x[m][k]^2 + eps).  A projection with x_resid
    // set adds its output into the residual stream x_resid [M][N], writes
    // xg_out[m][n] = x_resid[m][n] * gain[n] (the operand of the next projection; gain = the next norm's)
    // and sumsq_out[strip or tile][m] = sum of x_resid[m][n]^2 over the 16 (column kernel) or 64 (unit kernel)
    // columns one block finishes; the consumer of the next projection's output multiplies by r_m (RowScale).
    float *x_resid;
    float *xg_out;
    uint16_t *xg16_out;           // optional: xg_out rounded to fp16 (the operand of the 4-bit projections)
    const void *gain;             // [N] bf16
    float *sumsq_out;             // [N/16][M] (column kernel) or [N/64][M] (unit kernel with the residual epilogue)
    unsigned *tile_counter;       // non-NULL selects the unit kernel for this projection: [N/64] arrival counters, zero
                                  //   before the launch and left at zero by it; `partial` then holds gemm_resid_slots() slots
    // -- 4-bit weights (W4A16, groups of 128 along K): wpack holds the 4-bit quad layout of
    // launch_gemm_pack_w4; the projection writes `splitk` partial slots (gemm_w4_slots)
    bool w4;
    const void *w4_scale[3], *w4_zero[3];   // M > kStreamMaxRows: w[] are the codes [n][K/2], these the bf16 scales and uint8 zero points [n][K/128]
    RowScale scale;               // applied when writing `reduced` (row = the source row of m)
    int scale_rows;               //   rows per tile slab of scale.sumsq
};
int gemm_pick_splitk(int dtype, int M, int K, int N, const int *n, int nseg);
// repacked weights for the M <= kStreamMaxRows path
int gemm_pack_tiles(const int *n, int nseg);
size_t gemm_pack_bytes(const int *n, int nseg, int K);
int gemm_w4_slots(int K, const int *n, int nseg, bool resid);  // partial slots of a 4-bit projection (resid: the arrival epilogue's grid)
int gemm_packed_splits(int M, int K, const int *n, int nseg);   // partial slots (the splitk to use) with packed weights
int gemm_stream_grid(int tiles, int K);
int gemm_stream_slots(int tiles, int K);
int gemm_resid_grid(int tiles, int K);
int gemm_resid_slots(int tiles, int K);                          // partial slots of a projection run with tile_counter
// strip_major: the layout of the column kernel (the O projection)
void launch_gemm_pack(const void *const *w, const int *n, int nseg, int K, void *dst, bool strip_major, hipStream_t stream);
// 4-bit weight-only quantised projections: q [n][K/2] bytes (low nibble = even k), scale bf16 [n][K/128],
// zero u8 [n][K/128]; w = scale * (q - zero).  Each n[s] a multiple of 64.
size_t gemm_pack_w4_bytes(const int *n, int nseg, int K);
void launch_gemm_pack_w4(const void *const *q, const void *const *scale, const void *const *zero, const int *n,
                         int nseg, int K, void *dst, hipStream_t stream);
void launch_gemm(int dtype, const GemmArgs &g, hipStream_t stream);

// ---------------------------------------------------------------- attention (attention.hip)
struct AttnArgs {
    const float *q;               // [B][R][h_q][d_h] rotated queries, fp32
    const void *k;                // this layer's K cache [B][h_kv][max_len][d_h]
    const void *v;                // this layer's V cache [B][h_kv][d_h][max_len]
    const int32_t *lens;          // [B] valid positions BEFORE this forward
    float *out;                   // [B][R][h_q*d_h] fp32
    uint16_t *out16;              // optional copy of `out` rounded to fp16 (the operand of the tiled O projection)
    int B, R, h_q, h_kv, d_h, max_len;
    int len_bound;                // host upper bound of lens[b] + R
    float *part_o;                // split scratch [B][h_q][R][splits][d_h]
    float *part_ml;               // [B][h_q][R][splits][2]
    int splits;
    // Fused operand build (bf16, at most 32 query rows per KV head and at most 32 new rows): q is not read;
    // the kernel takes q, k, v of the new rows from the QKV projection's split-K partial sums
    // qkv_partial [qkv_splits][B*R][(h_q + 2 h_kv) d_h], applies the row scale rs and the rotation by
    // rope_cs [B*R][d_h/2] = (cos, sin) of position lens[b] + r at frequency i, and appends k, v to the cache.
    const float *qkv_partial;     // NULL: q holds the rotated queries and the cache already holds the new rows
    int qkv_splits;
    RowScale rs;
    const float2 *rope_cs;
    // Token tree (fused build only): tree_anc[r] has bit j set when row j of the step is row r itself or one of its
    // ancestors; row r then sees the cache and exactly those rows.  NULL: rows see the rows before them.
    const uint32_t *tree_anc;
};
// whether launch_attention builds its operands itself for this shape (then no rotation / append kernel runs before it)
bool attn_fuses_rope(int dtype, int R, int h_q, int h_kv, int d_h, bool tree);
int attn_pick_splits(int dtype, int B, int R, int h_q, int h_kv, int d_h, int len_bound, bool tree);
void launch_attention(int dtype, const AttnArgs &a, hipStream_t stream);

// ---------------------------------------------------------------- token trees (tree.hip)
constexpr int kTreeMaxNodes = 32;          // nodes of a tree forward pass (root included): one 32-key tile of new rows
constexpr int kTreeMaxAcceptNodes = 64;    // nodes of a tree acceptance call
struct TreeShape {
    uint32_t anc[kTreeMaxNodes];  // bit j of anc[r]: node j is node r or one of its ancestors
    int32_t depth[kTreeMaxNodes];
    int n;
};
void launch_tree_setup(const TreeShape &ts, uint32_t *anc, int32_t *depth, hipStream_t stream);
struct TreeAcceptArgs {
    const void *p, *q;            // [rows][n_nodes][vocab] logits (strides in elements per sequence), q unused when greedy
    int64_t p_stride, q_stride;
    const int32_t *tokens;        // [rows][n_nodes], tokens[.][0] unused
    const float *uniforms;        // [rows][n_nodes + 1]
    float temperature;            // 0: greedy matching
    int32_t *out_path_len, *out_path, *out_token, *out_flags;   // [rows], [rows][n_nodes], [rows], [rows] or NULL
    int rows, n_nodes, vocab;
    int32_t parents[kTreeMaxAcceptNodes];
};
void launch_tree_accept(int dtype, const TreeAcceptArgs &a, hipStream_t stream);
void launch_kv_compact_tree(int dtype, void *k, void *v, int32_t *lens, const int32_t *base, const int32_t *path,
                            const int32_t *path_len, int path_stride, int n_nodes, int L, int B, int h_kv, int d_h,
                            int max_len, int cap, hipStream_t stream);

// ---------------------------------------------------------------- measured ceilings (ceilings.hip)
void launch_probe_read(const void *src, size_t bytes, void *sink, int blocks, hipStream_t stream);
void launch_probe_mfma(const void *seed, void *sink, int blocks, int iters, hipStream_t stream);

// ---------------------------------------------------------------- row-wise kernels (rowwise.hip)
// optional by-product of the embedding kernel: cs[m][i] = (cos, sin) of (the position of row m) * theta^(-2i/d_h)
struct RopeTable {
    float2 *cs;                   // [M][d_h/2], NULL: not wanted
    const int32_t *lens;
    int R, d_h;
    float theta;
    const int32_t *depth;         // token tree: row r sits at position lens[b] + depth[r]; NULL: lens[b] + r
};
struct ZeroFill {
    unsigned *words;              // n 32-bit words set to zero by the first kernel of a forward pass (NULL / 0: none)
    int n;
};
// x = embed[token]; then xn = rmsnorm(x) * gain, or (sumsq_out non-NULL) xn = x * gain and sumsq_out[m] = sum_k x[m][k]^2
void launch_embed_norm(int dtype, const void *embed, const int32_t *tokens, float *x, const void *gain, float *xn,
                       float *sumsq_out, int M, int d, int vocab, float eps, RopeTable rt, uint16_t *xn16, ZeroFill zf,
                       hipStream_t stream);
// qkv = sum over splits of partial [S][M][(h_q+2h_kv) d_h] -> rotated q (fp32), rotated k and v appended
// to the cache (model dtype)
void launch_reduce_rope_append(int dtype, const float *partial, int S, RowScale rs, float *q_out, void *k_cache,
                               void *v_cache, const int32_t *lens, int B, int R, int h_q, int h_kv, int d_h,
                               int max_len, float theta, hipStream_t stream);
// x += sum over splits of partial [S][M][d]; xn = rmsnorm(x) * gain (xn16, if given: the same rounded to fp16)
void launch_reduce_residual_norm(int dtype, const float *partial, int S, float *x, const void *gain, float *xn,
                                 int M, int d, float eps, uint16_t *xn16, hipStream_t stream);
// h = silu(g) * u with [g | u] = sum over splits of partial [S][M][2f]
void launch_reduce_swiglu(const float *partial, int S, RowScale rs, float *h, int M, int f, uint16_t *h16, hipStream_t stream);
void launch_advance_lens(int32_t *lens, int B, int delta, int max_len, hipStream_t stream);
void launch_truncate(int32_t *lens, const int32_t *base, const int32_t *keep, int offset, int cap, int B,
                     hipStream_t stream);
void launch_truncate_to(int32_t *lens, int new_len, int B, hipStream_t stream);

}  // namespace psd
