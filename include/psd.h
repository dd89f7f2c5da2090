/*
 * psd - the verify path of polybasic speculative decoding on one MI355X (gfx950).
 *
 * A chain of models M_1 (target) ... M_n (draft) shares a vocabulary; each
 * level i verifies, with ONE forward pass, the block of tokens proposed by the
 * level below it and applies the speculative-sampling acceptance test
 * (Sec. 3.1 "Problem Formulation"; Sec. 3.3 "Staged Verification";
 * Algorithm 1).  This library is that hot path:
 *
 *   psd_model_forward   p_i(. | x_<=t) = M_i(x_<=t) for the new rows of a block
 *                       (Sec. 3.1; the cost T_i of Eq. 2)
 *   psd_spec_accept     VERIFY of Algorithm 1: accept with prob. min(1, p/q),
 *                       first rejection -> one draw from norm(max(0, p - q))
 *   psd_kv_truncate     the "partial rollback" of Sec. 3.3: KV length <- accepted length
 *
 * Conventions
 *   - Every array argument marked "device" is a pointer to GPU memory owned by
 *     the caller, who keeps it alive while a handle or an enqueued call uses it.
 *     Handles (psd_model, psd_kv) are small host objects; they own no device
 *     memory.  The library allocates no device memory at all: scratch space is
 *     the caller's `workspace`, sized by the *_workspace_bytes calls.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work on that stream and never synchronise.
 *   - Arguments are checked on the host before anything is launched: a negative
 *     status means nothing was enqueued and no output was touched.
 *   - A handle may be used from one host thread at a time.
 */
#ifndef PSD_H
#define PSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t psd_status;
#define PSD_OK 0
#define PSD_ERR_NULL (-1)          /* a required pointer is NULL                         */
#define PSD_ERR_SHAPE (-2)         /* a size is out of the supported range               */
#define PSD_ERR_DTYPE (-3)         /* dtype is neither PSD_F32 nor PSD_BF16              */
#define PSD_ERR_CAPACITY (-4)      /* the KV cache cannot take n_new more positions      */
#define PSD_ERR_TEMPERATURE (-5)   /* temperature is not a finite number >= 0            */
#define PSD_ERR_WORKSPACE (-6)     /* workspace is NULL, misaligned or too small         */
#define PSD_ERR_HIP (-7)           /* a HIP launch failed (see psd_last_hip_error)       */
#define PSD_ERR_UNIMPLEMENTED (-8)

#define PSD_F32 0
#define PSD_BF16 1

/* bits of psd_spec_accept's out_flags */
#define PSD_FLAG_NEAR_TIE 1       /* some tested position had |u - p/q| < 1e-5           */
#define PSD_FLAG_ZERO_RESIDUAL 2  /* residual mass was 0: the draw used p instead        */

typedef struct psd_model psd_model;
typedef struct psd_kv psd_kv;

/* Decoder-only transformer: pre-norm, RMSNorm, rotary embedding with rotate-half pairing
 * (element i pairs with i + d_head/2, angle = position * rope_theta^(-2i/d_head)),
 * grouped-query causal attention, SwiGLU MLP, no biases, untied lm_head.
 * dtype is the storage type of every weight and of the KV cache; PSD_BF16 models
 * multiply on the bf16 matrix cores with fp32 accumulation; every activation stays
 * fp32 and enters the matrix cores as a bf16 high part plus a bf16 remainder (two
 * products per weight operand), PSD_F32 models compute in fp32 throughout.
 * Limits: d_head in {32, 64, 128} (PSD_BF16: 64 or 128); n_q_heads a multiple of
 * n_kv_heads; d_model <= 8192; d_model, d_ffn and n_q_heads*d_head multiples of 32
 * (PSD_BF16: of 128).  Anything else: PSD_ERR_SHAPE from psd_model_create. */
typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, d_head, d_ffn, vocab;
    float rope_theta, rms_eps;
    int32_t dtype;
} psd_model_desc;

const char *psd_status_string(psd_status s);
/* hipError_t of the most recent failed launch on this host thread, as an int (0 = none). */
int32_t psd_last_hip_error(void);

/* weight_ptrs: n_ptrs = 3 + 9 * n_layers device pointers in this order:
 *   embed [vocab, d_model];
 *   per layer: attn_norm [d_model], wq [n_q_heads*d_head, d_model], wk [n_kv_heads*d_head, d_model],
 *              wv [n_kv_heads*d_head, d_model], wo [d_model, n_q_heads*d_head], ffn_norm [d_model],
 *              w_gate [d_ffn, d_model], w_up [d_ffn, d_model], w_down [d_model, d_ffn];
 *   final_norm [d_model]; lm_head [vocab, d_model].
 * Every matrix is row-major [out_features, in_features] (in_features contiguous), 16-byte
 * aligned, of the model's dtype.  Pointers may alias another model's (a draft that shares
 * the target's embed / lm_head).  On success *out is a new handle. */
psd_status psd_model_create(const psd_model_desc *desc, const void *const *weight_ptrs,
                            int32_t n_ptrs, psd_model **out);
psd_status psd_model_destroy(psd_model *m);

/* A model whose seven projection matrices per layer are 4-bit weight-only quantised with groups of 128
 * input channels, the format of the paper's intermediate model M_2 ("a quantized 4-bit version of M_1",
 * group size 128: Sec. 3.3 system design and Sec. 4.1 setup): W[n][k] = scale[n][k/128] * (q[n][k] - zero[n][k/128]).
 * desc and weight_ptrs are as for psd_model_create with dtype PSD_BF16, except that the pointers of
 * wq, wk, wv, wo, w_gate, w_up, w_down address the 4-bit codes: device uint8 [n][K/2], byte b of a row holds
 * k = 2b in its low nibble and k = 2b + 1 in its high nibble.  scale_ptrs / zero_ptrs: 7 * n_layers device
 * pointers in the order (wq, wk, wv, wo, w_gate, w_up, w_down) per layer, to bf16 [n][K/128] and to uint8
 * [n][K/128] with values 0..15.  Embedding, norm gains, lm_head and the KV cache stay bf16; activations are
 * rounded to fp16 (11 significant bits) on their way into these projections; in steps of at most 16 rows no weight
 * is rounded: the codes enter the matrix cores as exact integers and scale and zero point are applied per group
 * in fp32.
 * Such a model must be packed (psd_model_pack) before its first forward (PSD_ERR_UNIMPLEMENTED otherwise).  Steps
 * of at most 16 rows (batch * n_new <= 16) stream the packed 4-bit copy and multiply the codes exactly; longer steps
 * read the caller's codes, scales and zero points and round each weight scale * (q - zero) to fp16 once.  Further limit: n_kv_heads * d_head a multiple of 64. */
psd_status psd_model_create_w4(const psd_model_desc *desc, const void *const *weight_ptrs, int32_t n_ptrs,
                               const void *const *scale_ptrs, const void *const *zero_ptrs,
                               int32_t n_quant_ptrs, psd_model **out);

/* Optional streaming copy of the projection weights for verify steps of up to 16 rows
 * (batch * n_new <= 16), where the forward pass is bound by reading the weights once from HBM.
 * psd_model_pack rewrites every projection matrix into caller memory in the order the
 * wavefronts of the streaming GEMM load it (64-row x 128-column units of 16 KB, each stored
 * as the 64 lanes' 16-byte operands, units of one projection contiguous), so that each
 * wavefront reads one contiguous byte range.  packed_mem: device, 256-byte aligned, at least
 * psd_model_packed_bytes() bytes (about the size of the weights), kept alive with the model;
 * the row-major weights stay in use for larger steps and must stay alive too.  After a
 * successful call, forwards with batch * n_new <= 16 read the packed copy; results are the same
 * up to fp32 summation order.  Call it before sizing workspaces: the workspace need changes.
 * PSD_BF16 models only (PSD_ERR_DTYPE otherwise); psd_model_packed_bytes returns 0 for others. */
size_t psd_model_packed_bytes(const psd_model *m);
psd_status psd_model_pack(psd_model *m, void *packed_mem, size_t packed_bytes, void *hip_stream);

/* Bytes of workspace psd_model_forward needs for this batch / n_new / cache length
 * (0 on a bad argument).  The workspace must be 256-byte aligned. */
size_t psd_model_workspace_bytes(const psd_model *m, int32_t batch, int32_t n_new, int32_t max_len);

/* KV cache descriptor over caller memory.  Layout (elements of the model's dtype):
 *   k_mem [n_layers][batch][n_kv_heads][max_len][d_head]
 *   v_mem [n_layers][batch][n_kv_heads][d_head][max_len]     (V is stored transposed)
 * each of psd_kv_bytes() bytes, 256-byte aligned; max_len a multiple of 64.
 * lens_dev: device int32[batch], the number of valid positions per sequence; the caller
 * initialises it and states an upper bound of its entries in len_upper_bound (the host
 * never reads lens_dev; it tracks only this bound for capacity checks).  Positions at or
 * beyond lens[b] may hold anything. */
size_t psd_kv_bytes(const psd_model *m, int32_t batch, int32_t max_len);
psd_status psd_kv_create(const psd_model *m, int32_t batch, int32_t max_len, void *k_mem,
                         void *v_mem, int32_t *lens_dev, int32_t len_upper_bound, psd_kv **out);
psd_status psd_kv_destroy(psd_kv *kv);
/* The host-side upper bound of lens (for tests and capacity planning). */
int32_t psd_kv_len_upper_bound(const psd_kv *kv);

/* One forward pass of M_i over n_new tokens per sequence (Sec. 3.1; Algorithm 1's
 * "M_2(x_<=t, x~_1:K)" / "M_1(x_<=t, accepted)").
 *   tokens_dev     device int32[batch][n_new]; sequence b's tokens go to positions
 *                  lens[b] .. lens[b]+n_new-1.  Ids outside [0, vocab) are clamped.
 *   n_logit_rows   0..n_new: the lm_head is applied to the LAST n_logit_rows rows only
 *                  (0 for a prefill that needs no logits).
 *   logits_out_dev device fp32[batch][n_logit_rows][vocab]; row r is the distribution of
 *                  the token that follows input token n_new - n_logit_rows + r.
 *                  May be NULL iff n_logit_rows == 0.
 * Appends the new rows' K/V to the cache and advances lens[b] by n_new (on the stream).
 * PSD_ERR_CAPACITY if len_upper_bound + n_new > max_len. */
psd_status psd_model_forward(psd_model *m, const int32_t *tokens_dev, int32_t n_new, psd_kv *kv,
                             float *logits_out_dev, int32_t n_logit_rows, void *workspace,
                             size_t ws_bytes, void *hip_stream);

/* Speculative-sampling acceptance for `rows` independent sequences (VERIFY loop of
 * Algorithm 1 with its break; the rule keeps the verifier's distribution, Sec. 3.1).
 *   p_logits   device [rows][n_p_rows][vocab] verifier logits, n_p_rows = gamma or gamma+1;
 *              consecutive sequences are p_seq_stride elements apart, rows are dense
 *   q_logits   device [rows][gamma][vocab] drafter logits, q_seq_stride likewise
 *   dtype      PSD_F32 or PSD_BF16, the same for both
 *   draft_tokens device int32[rows][gamma], each in [0, vocab)
 *   uniforms   device fp32[rows][gamma+1] in [0,1): u[j] decides position j, u[gamma]
 *              drives the single inverse-CDF draw
 *   temperature both distributions are softmax(logits / temperature), temperature > 0
 * For each sequence, with p_j, q_j the softmaxes of position j: accept x_j iff
 * u_j < min(1, p_j[x_j]/q_j[x_j]), stop at the first failure; n = number accepted.
 *   out_accept_len device int32[rows] <- n in [0, gamma]
 *   out_token  device int32[rows] <- if n < gamma: smallest k with
 *              sum_{i<=k} r_i > u_gamma * sum_i r_i, r = max(0, p_n - q_n) (r = p_n if that
 *              sum is 0); if n == gamma and n_p_rows == gamma+1: the same draw with
 *              r = p_gamma; else -1
 *   out_flags  device int32[rows] or NULL <- PSD_FLAG_* bits
 * The ratio test runs in fp32 (softmax statistics by wavefront reductions); the draw runs
 * in fp64 in a fixed summation order, so it is reproducible bit for bit.
 * gamma = 0 with n_p_rows = 1 is plain sampling from softmax(p_0 / temperature).
 * temperature = 0 selects greedy verification (the other rule Sec. 3.1 names, compared with
 * sampling in the paper's ablation on acceptance-length variance): x_j is kept iff it equals
 * argmax_v p_logits[j][v] (lowest index among equal maxima, values compared as stored), the
 * first mismatch is replaced by that argmax, a fully matching block emits the argmax of the
 * bonus row or -1; q_logits and uniforms are not read and may be NULL, flags are 0, the
 * result is exact.  gamma = 0 with n_p_rows = 1 is then the argmax of p_0.
 * Limits: 0 <= gamma <= 64, vocab >= 1, rows >= 0 (rows = 0 is a no-op). */
size_t psd_spec_accept_workspace_bytes(int32_t rows, int32_t gamma, int32_t n_p_rows, int32_t vocab);
psd_status psd_spec_accept(const void *p_logits, const void *q_logits, const int32_t *draft_tokens,
                           int32_t gamma, const float *uniforms, float temperature,
                           int32_t *out_accept_len, int32_t *out_token,
                           int32_t rows, int32_t n_p_rows, int32_t vocab, int32_t dtype,
                           int64_t p_seq_stride, int64_t q_seq_stride, int32_t *out_flags,
                           void *workspace, size_t ws_bytes, void *hip_stream);

/* For callers that cannot allocate device memory or size a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): psd_spec_accept on a scratch buffer that is part of the
 * library, a fixed PSD_STATIC_SCRATCH_BYTES array in device memory of every GPU the library runs on (held until
 * the process ends).  Arguments, results and error behaviour are those of psd_spec_accept without workspace /
 * ws_bytes; sizes whose psd_spec_accept_workspace_bytes() exceeds PSD_STATIC_SCRATCH_BYTES are refused with
 * PSD_ERR_WORKSPACE before anything is launched (64 x 8 x 32000 needs 0.07 MB, 16 x 16 x 152064 0.13 MB).
 * The call allocates and frees nothing and enqueues only kernels (no memset nodes); the buffer's address on the
 * current GPU is looked up on the first call there (PSD_ERR_HIP if that fails).  All calls on one GPU share
 * the buffer, which keeps the previous call's contents; whatever must start at zero is cleared by the call's
 * first kernel.  Calls that overlap in time on one GPU (different streams or threads) race on it: give
 * concurrent callers psd_spec_accept with workspaces of their own. */
#define PSD_STATIC_SCRATCH_BYTES (1u << 20)
psd_status psd_spec_accept_static(const void *p_logits, const void *q_logits, const int32_t *draft_tokens,
                                  int32_t gamma, const float *uniforms, float temperature,
                                  int32_t *out_accept_len, int32_t *out_token,
                                  int32_t rows, int32_t n_p_rows, int32_t vocab, int32_t dtype,
                                  int64_t p_seq_stride, int64_t q_seq_stride, int32_t *out_flags,
                                  void *hip_stream);

/* Rollback after verification (Sec. 3.3): on the stream, for every sequence b,
 *   lens[b] <- min(lens[b], base_lens_dev[b] + keep_dev[b] + keep_offset, new_len_upper_bound)   (never below 0).
 * base_lens_dev / keep_dev are device int32[batch] (e.g. the lengths before the verify
 * forward and psd_spec_accept's out_accept_len; keep_offset = 1 keeps the x* row too).
 * new_len_upper_bound: an upper bound, known to the host, of the lengths after the rollback: a
 * decoding loop reads the accepted lengths back to steer itself and passes the largest
 * base + keep + keep_offset.  The host-side bound behind psd_model_forward's capacity check (which
 * otherwise only grows, by n_new per forward) is lowered to it, and the device enforces it too, so
 * a loop of forward / accept / truncate needs no other call to keep that bound tight.  A negative
 * value leaves the host bound as it is.
 * No data moves; stale rows are overwritten by the next append. */
psd_status psd_kv_truncate(psd_kv *kv, const int32_t *base_lens_dev, const int32_t *keep_dev,
                           int32_t keep_offset, int32_t new_len_upper_bound, void *hip_stream);
/* Host-scalar variant: lens[b] <- min(lens[b], new_len) for all b; also lowers the host
 * upper bound to new_len. */
psd_status psd_kv_truncate_to(psd_kv *kv, int32_t new_len, void *hip_stream);

/* ---- Token-tree verification (Related Work, "Verification Mechanisms": token-tree-based verification; Sec. 4.6:
 * deeper / wider drafting).  A tree has n_nodes nodes numbered so that every parent precedes its children; node 0 is
 * the root = the last committed token, not yet in the cache (the x* row of a linear step); parents_host is a HOST
 * int32[n_nodes] with parents_host[0] = -1 and 0 <= parents_host[i] < i.  Every sequence of a call has the same shape.
 *
 * psd_model_forward_tree: psd_model_forward over the tree's nodes in one pass: node r reads the cache and its own
 *   ancestors (itself included) among the new rows and sits at position lens[b] + depth(r), so its logits row is what
 *   an ordinary pass over its root-to-node path would give.  tokens_dev: device int32[batch][n_nodes];
 *   logits_out_dev: device fp32[batch][n_nodes][vocab] (every node gets a row).  Node r's K/V go to cache slot
 *   lens[b] + r and the lengths advance by n_nodes: follow with psd_kv_compact_tree.  Workspace as for
 *   psd_model_forward(batch, n_nodes).  Limits: n_nodes <= 32, a bf16 model with d_head 64 or 128 and
 *   (n_q_heads / n_kv_heads) * n_nodes <= 32 (the attention kernel that builds its own operands); anything else
 *   PSD_ERR_UNIMPLEMENTED; a malformed parents array PSD_ERR_SHAPE.
 *
 * psd_tree_accept: one verification of the tree per sequence.  The tokens of a node's children are taken to be
 *   independent draws from softmax(q_logits[node] / T); at a node the children are tried in index order, child c with
 *   token x accepted iff uniforms[c] < min(1, r[x] / q[x]) where r starts as softmax(p_logits[node] / T) and becomes
 *   norm(max(0, r - q)) after every refusal; the first accepted child is descended into; where none is accepted (or
 *   at a leaf) one token is drawn from r by inverse CDF in index order with uniforms[n_nodes].  With one child per
 *   node this is psd_spec_accept.  temperature = 0: greedy matching (the first child that carries the verifier's most
 *   likely token, lowest index among equals; q_logits and uniforms are not read).
 *   p_logits / q_logits: device [rows][n_nodes][vocab] of `dtype` (strides in elements per sequence);
 *   tokens_dev device int32[rows][n_nodes] (entry 0 unused); uniforms device fp32[rows][n_nodes + 1] (entry 0 unused).
 *   Outputs (device): out_path_len[rows]; out_path[rows][n_nodes]: the accepted nodes root first, root excluded
 *   (entries past the length are not written); out_token[rows]; out_flags[rows] or NULL (PSD_FLAG_NEAR_TIE as in
 *   psd_spec_accept).  Everything that decides a token runs in fp64.  One block per sequence: a correctness-first
 *   kernel, several passes over two logits rows per visited node.  Limits: n_nodes <= 64.  Needs no workspace.
 *
 * psd_kv_compact_tree: after the acceptance, for every sequence b with base = base_lens_dev[b] (the length before the
 *   tree pass): the K/V rows of the accepted nodes move to slots base + 1 .. base + path_len[b] (the root stays at
 *   base), and lens[b] <- min(lens[b], base + 1 + path_len[b], new_len_upper_bound).  path_dev: device
 *   int32[batch][path_stride] as written by psd_tree_accept (path_stride >= n_nodes - 1); base_lens_dev must not be
 *   the cache's own length array.  new_len_upper_bound as in psd_kv_truncate. */
psd_status psd_model_forward_tree(psd_model *m, const int32_t *tokens_dev, int32_t n_nodes, const int32_t *parents_host,
                                  psd_kv *kv, float *logits_out_dev, void *workspace, size_t ws_bytes, void *hip_stream);
psd_status psd_tree_accept(const void *p_logits, const void *q_logits, const int32_t *tokens_dev,
                           const int32_t *parents_host, int32_t n_nodes, const float *uniforms, float temperature,
                           int32_t *out_path_len, int32_t *out_path, int32_t *out_token,
                           int32_t rows, int32_t vocab, int32_t dtype, int64_t p_seq_stride, int64_t q_seq_stride,
                           int32_t *out_flags, void *hip_stream);
psd_status psd_kv_compact_tree(psd_kv *kv, const int32_t *base_lens_dev, const int32_t *path_dev,
                               const int32_t *path_len_dev, int32_t path_stride, int32_t n_nodes,
                               int32_t new_len_upper_bound, void *hip_stream);

/* ---- measurement aid (not part of the decoding path) -------------------------------------
 * Per-kernel timing with a start and a stop HIP event attached to each kernel dispatch (they
 * time the kernel itself, on the stream it is launched on), so that a bench can state each
 * kernel's average duration against its roofline.  psd_profile_enable(n > 0) creates
 * event pairs for up to n launches and starts recording; psd_profile_enable(0) stops and
 * frees them.  psd_profile_collect waits for the recorded work, adds each launch's elapsed
 * milliseconds into ms_by_kind[kind] and counts it in launches_by_kind[kind] (host arrays of
 * PSD_KIND_COUNT entries, zeroed by the call), then rewinds.  Launches beyond n are not
 * recorded.  Not thread-safe; one process-wide recorder. */
#define PSD_KIND_EMBED 0
#define PSD_KIND_RMSNORM 1
#define PSD_KIND_GEMM_F32 2
#define PSD_KIND_GEMM_SKINNY 3       /* bf16 weight-streaming GEMM over packed 16 KB units, M <= 16 */
#define PSD_KIND_GEMM_TILED 4        /* LDS-tiled GEMM of bf16 models (fp16 MFMA), M > 16 */
#define PSD_KIND_GEMM_REDUCE 5       /* split-K reduction */
#define PSD_KIND_ROPE_APPEND 6
#define PSD_KIND_ATTN 7
#define PSD_KIND_ATTN_COMBINE 8
#define PSD_KIND_SWIGLU 9
#define PSD_KIND_LENS 10             /* length advance / truncate */
#define PSD_KIND_ACCEPT_STATS 11
#define PSD_KIND_ACCEPT_DRAW 12      /* first rejection + fp64 pass over the one position the draw reads */
#define PSD_KIND_ACCEPT_LOCATE 13    /* greedy verification: the walk over the per-position argmax */
#define PSD_KIND_GEMM_COLUMN 14      /* bf16 GEMM with the residual epilogue (O, down), M <= 16 */
#define PSD_KIND_GEMM_W4 15          /* 4-bit weight-only GEMM, M <= 16 */
#define PSD_KIND_GEMM_SLOT 16        /* bf16 GEMM on 16-column tiles x K splits, M <= 16 (one partial slot, or unpacked weights) */
#define PSD_KIND_COUNT 17
psd_status psd_profile_enable(int32_t max_launches);
psd_status psd_profile_collect(double *ms_by_kind, int64_t *launches_by_kind);

/* Two microkernels that measure what the machine delivers, so that a bench can state roofline fractions against
 * measured ceilings beside the published peaks.  Each call enqueues ONE launch on the stream; the caller times it.
 *   psd_probe_stream_read  reads `bytes` (a multiple of 16) of device memory at src_dev once, `blocks` blocks of
 *                          256 threads each on an equal contiguous share, eight non-temporal 16-byte loads in
 *                          flight per lane; sink_dev: device, >= 4 bytes (practically never written).
 *   psd_probe_mfma         `blocks` blocks of four wavefronts, each wavefront issuing 4 * iters 32x32x16 bf16
 *                          matrix-core instructions (2 * 32 * 32 * 16 flop each) on operands read from seed_dev
 *                          (device, 1024 bf16 values); sink_dev: device fp32[blocks * 256].
 * PSD_ERR_NULL / PSD_ERR_SHAPE on bad arguments, PSD_ERR_HIP if the launch fails. */
psd_status psd_probe_stream_read(const void *src_dev, size_t bytes, void *sink_dev, int32_t blocks, void *hip_stream);
psd_status psd_probe_mfma(const void *seed_dev, float *sink_dev, int32_t blocks, int32_t iters, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PSD_H */
