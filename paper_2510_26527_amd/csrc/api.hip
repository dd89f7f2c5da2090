// C ABI of the library (include/psd.h): argument validation on the host, workspace carving,
// and the launch sequence of one forward pass.  No kernel lives here.
#include <cmath>
#include <cstdlib>
#include <new>
#include <vector>

#include "../../include/psd.h"
#include "kernels.h"
#include "prof.h"

using namespace psd;

// ------------------------------------------------------------------ launch recorder
namespace {
struct Recorder {
    bool on = false;
    std::vector<hipEvent_t> ev;      // 2 per launch
    std::vector<int> kind;
    size_t used = 0, cap = 0;
} g_rec;
}  // namespace

namespace psd {
static thread_local int g_kind = -1;
void prof_set_kind(int kind) { g_kind = kind; }
bool prof_acquire(hipEvent_t *start, hipEvent_t *stop) {
    if (!g_rec.on || g_rec.used >= g_rec.cap || g_kind < 0) return false;
    g_rec.kind[g_rec.used] = g_kind;
    *start = g_rec.ev[2 * g_rec.used];
    *stop = g_rec.ev[2 * g_rec.used + 1];
    ++g_rec.used;
    return true;
}
}  // namespace psd

struct psd_model {
    psd_model_desc d;
    std::vector<const void *> w;     // the caller's weight pointers, in header order
    const void *embed() const { return w[0]; }
    const void *layer(int l, int which) const { return w[1 + 9 * l + which]; }
    const void *final_norm() const { return w[1 + 9 * d.n_layers]; }
    const void *lm_head() const { return w[2 + 9 * d.n_layers]; }
    // repacked copies for the weight-streaming path (psd_model_pack): per layer qkv, o, gate|up, down; then lm_head
    const char *packed = nullptr;
    std::vector<size_t> pack_off;    // 4 * n_layers + 1 offsets into `packed`
    const void *pack(int l, int which) const { return packed ? packed + pack_off[4 * l + which] : nullptr; }
    const void *pack_head() const { return packed ? packed + pack_off[4 * d.n_layers] : nullptr; }
    // 4-bit projections (psd_model_create_w4): per layer and projection (q, k, v, o, gate, up, down) the group
    // scales and zero points; w[] then points at the nibbles
    bool w4 = false;
    std::vector<const void *> w4_scale, w4_zero;
    const void *qscale(int l, int j) const { return w4_scale[7 * l + j]; }
    const void *qzero(int l, int j) const { return w4_zero[7 * l + j]; }
};
enum { P_QKV = 0, P_O, P_GU, P_DOWN };
enum { W_ATTN_NORM = 0, W_Q, W_K, W_V, W_O, W_FFN_NORM, W_GATE, W_UP, W_DOWN };

struct psd_kv {
    const psd_model *m;
    int batch, max_len;
    void *k, *v;
    int32_t *lens;
    int len_ub;                      // host upper bound of every lens[b]
};

static thread_local int32_t g_last_hip_error = 0;

static psd_status check_launch() {
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        g_last_hip_error = (int32_t)e;
        return PSD_ERR_HIP;
    }
    return PSD_OK;
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
static size_t elem_size(int dtype) { return dtype == PSD_BF16 ? 2 : 4; }

extern "C" {

const char *psd_status_string(psd_status s) {
    switch (s) {
        case PSD_OK: return "ok";
        case PSD_ERR_NULL: return "null pointer";
        case PSD_ERR_SHAPE: return "unsupported shape";
        case PSD_ERR_DTYPE: return "unsupported dtype";
        case PSD_ERR_CAPACITY: return "KV cache capacity exceeded";
        case PSD_ERR_TEMPERATURE: return "temperature must be finite and >= 0 (0 selects greedy verification)";
        case PSD_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case PSD_ERR_HIP: return "HIP launch failed";
        case PSD_ERR_UNIMPLEMENTED: return "not implemented";
        default: return "unknown status";
    }
}

int32_t psd_last_hip_error(void) { return g_last_hip_error; }

psd_status psd_model_create(const psd_model_desc *desc, const void *const *weight_ptrs, int32_t n_ptrs,
                            psd_model **out) {
    if (!desc || !weight_ptrs || !out) return PSD_ERR_NULL;
    const psd_model_desc &d = *desc;
    if (d.dtype != PSD_F32 && d.dtype != PSD_BF16) return PSD_ERR_DTYPE;
    if (d.n_layers < 0 || d.d_model <= 0 || d.n_q_heads <= 0 || d.n_kv_heads <= 0 || d.d_ffn <= 0 || d.vocab <= 0)
        return PSD_ERR_SHAPE;
    if (d.d_head != 32 && d.d_head != 64 && d.d_head != 128) return PSD_ERR_SHAPE;
    if (d.n_q_heads % d.n_kv_heads) return PSD_ERR_SHAPE;
    const int align = d.dtype == PSD_BF16 ? 128 : 32;      // the bf16 GEMMs step K by 128
    if (d.d_model % align || d.d_ffn % align || (d.n_q_heads * d.d_head) % align) return PSD_ERR_SHAPE;
    if (d.d_model > 8192) return PSD_ERR_SHAPE;              // the row-wise kernels keep a row in registers
    if (d.dtype == PSD_BF16 && d.d_head == 32) return PSD_ERR_SHAPE;
    if (!(d.rope_theta > 0.f) || !(d.rms_eps >= 0.f)) return PSD_ERR_SHAPE;
    if (n_ptrs != 3 + 9 * d.n_layers) return PSD_ERR_SHAPE;
    for (int i = 0; i < n_ptrs; ++i) {
        if (!weight_ptrs[i]) return PSD_ERR_NULL;
        if ((uintptr_t)weight_ptrs[i] % 16) return PSD_ERR_SHAPE;
    }
    psd_model *m = new (std::nothrow) psd_model;
    if (!m) return PSD_ERR_NULL;
    m->d = d;
    m->w.assign(weight_ptrs, weight_ptrs + n_ptrs);
    *out = m;
    return PSD_OK;
}

psd_status psd_model_destroy(psd_model *m) {
    if (!m) return PSD_ERR_NULL;
    delete m;
    return PSD_OK;
}

psd_status psd_model_create_w4(const psd_model_desc *desc, const void *const *weight_ptrs, int32_t n_ptrs,
                               const void *const *scale_ptrs, const void *const *zero_ptrs, int32_t n_quant_ptrs,
                               psd_model **out) {
    if (!desc || !scale_ptrs || !zero_ptrs) return PSD_ERR_NULL;
    if (desc->dtype != PSD_BF16) return PSD_ERR_DTYPE;
    if (n_quant_ptrs != 7 * desc->n_layers) return PSD_ERR_SHAPE;
    if ((desc->n_kv_heads * desc->d_head) % 64) return PSD_ERR_SHAPE;      // every projection a multiple of 64 wide
    for (int i = 0; i < n_quant_ptrs; ++i) {
        if (!scale_ptrs[i] || !zero_ptrs[i]) return PSD_ERR_NULL;
        if ((uintptr_t)scale_ptrs[i] % 2) return PSD_ERR_SHAPE;
    }
    psd_model *m = nullptr;
    const psd_status s = psd_model_create(desc, weight_ptrs, n_ptrs, &m);
    if (s != PSD_OK) return s;
    m->w4 = true;
    m->w4_scale.assign(scale_ptrs, scale_ptrs + n_quant_ptrs);
    m->w4_zero.assign(zero_ptrs, zero_ptrs + n_quant_ptrs);
    *out = m;
    return PSD_OK;
}

static void pack_layout(const psd_model *m, std::vector<size_t> *off, size_t *total) {
    const psd_model_desc &d = m->d;
    const int hd = d.n_q_heads * d.d_head, kvd = d.n_kv_heads * d.d_head;
    const int n_qkv[3] = {hd, kvd, kvd}, n_o[1] = {d.d_model}, n_gu[2] = {d.d_ffn, d.d_ffn}, n_v[1] = {d.vocab};
    size_t at = 0;
    off->clear();
    auto bytes = [&](const int *n, int nseg, int K) {
        return align256(m->w4 ? gemm_pack_w4_bytes(n, nseg, K) : gemm_pack_bytes(n, nseg, K));
    };
    for (int l = 0; l < d.n_layers; ++l) {
        off->push_back(at); at += bytes(n_qkv, 3, d.d_model);
        off->push_back(at); at += bytes(n_o, 1, hd);
        off->push_back(at); at += bytes(n_gu, 2, d.d_model);
        off->push_back(at); at += bytes(n_o, 1, d.d_ffn);
    }
    off->push_back(at); at += gemm_pack_bytes(n_v, 1, d.d_model);
    *total = at;
}

size_t psd_model_packed_bytes(const psd_model *m) {
    if (!m || m->d.dtype != PSD_BF16) return 0;
    std::vector<size_t> off;
    size_t total = 0;
    pack_layout(m, &off, &total);
    return total;
}

psd_status psd_model_pack(psd_model *m, void *packed_mem, size_t packed_bytes, void *hip_stream) {
    if (!m || !packed_mem) return PSD_ERR_NULL;
    if (m->d.dtype != PSD_BF16) return PSD_ERR_DTYPE;
    std::vector<size_t> off;
    size_t total = 0;
    pack_layout(m, &off, &total);
    if ((uintptr_t)packed_mem % 256 || packed_bytes < total) return PSD_ERR_WORKSPACE;
    const psd_model_desc &d = m->d;
    const int hd = d.n_q_heads * d.d_head, kvd = d.n_kv_heads * d.d_head;
    hipStream_t st = (hipStream_t)hip_stream;
    char *base = (char *)packed_mem;
    (void)hipGetLastError();
    for (int l = 0; l < d.n_layers && m->w4; ++l) {
        const int n_qkv[3] = {hd, kvd, kvd}, n_o[1] = {d.d_model}, n_gu[2] = {d.d_ffn, d.d_ffn};
        const void *qkv[3] = {m->layer(l, W_Q), m->layer(l, W_K), m->layer(l, W_V)};
        const void *qkv_s[3] = {m->qscale(l, 0), m->qscale(l, 1), m->qscale(l, 2)};
        const void *qkv_z[3] = {m->qzero(l, 0), m->qzero(l, 1), m->qzero(l, 2)};
        launch_gemm_pack_w4(qkv, qkv_s, qkv_z, n_qkv, 3, d.d_model, base + off[4 * l + P_QKV], st);
        const void *o[1] = {m->layer(l, W_O)}, *o_s[1] = {m->qscale(l, 3)}, *o_z[1] = {m->qzero(l, 3)};
        launch_gemm_pack_w4(o, o_s, o_z, n_o, 1, hd, base + off[4 * l + P_O], st);
        const void *gu[2] = {m->layer(l, W_GATE), m->layer(l, W_UP)};
        const void *gu_s[2] = {m->qscale(l, 4), m->qscale(l, 5)}, *gu_z[2] = {m->qzero(l, 4), m->qzero(l, 5)};
        launch_gemm_pack_w4(gu, gu_s, gu_z, n_gu, 2, d.d_model, base + off[4 * l + P_GU], st);
        const void *dn[1] = {m->layer(l, W_DOWN)}, *dn_s[1] = {m->qscale(l, 6)}, *dn_z[1] = {m->qzero(l, 6)};
        launch_gemm_pack_w4(dn, dn_s, dn_z, n_o, 1, d.d_ffn, base + off[4 * l + P_DOWN], st);
    }
    for (int l = 0; l < d.n_layers && !m->w4; ++l) {
        const void *qkv[3] = {m->layer(l, W_Q), m->layer(l, W_K), m->layer(l, W_V)};
        const int n_qkv[3] = {hd, kvd, kvd};
        launch_gemm_pack(qkv, n_qkv, 3, d.d_model, base + off[4 * l + P_QKV], false, st);
        const void *o[1] = {m->layer(l, W_O)};
        const int n_o[1] = {d.d_model};
        launch_gemm_pack(o, n_o, 1, hd, base + off[4 * l + P_O], true, st);
        const void *gu[2] = {m->layer(l, W_GATE), m->layer(l, W_UP)};
        const int n_gu[2] = {d.d_ffn, d.d_ffn};
        launch_gemm_pack(gu, n_gu, 2, d.d_model, base + off[4 * l + P_GU], false, st);
        const void *dn[1] = {m->layer(l, W_DOWN)};
        launch_gemm_pack(dn, n_o, 1, d.d_ffn, base + off[4 * l + P_DOWN], false, st);
    }
    const void *hw[1] = {m->lm_head()};
    const int n_v[1] = {d.vocab};
    launch_gemm_pack(hw, n_v, 1, d.d_model, base + off[4 * d.n_layers], false, st);
    const psd_status s = check_launch();
    if (s == PSD_OK) {
        m->packed = base;
        m->pack_off = off;
    }
    return s;
}

size_t psd_kv_bytes(const psd_model *m, int32_t batch, int32_t max_len) {
    if (!m || batch <= 0 || max_len <= 0 || max_len % 64) return 0;
    return (size_t)m->d.n_layers * batch * m->d.n_kv_heads * max_len * m->d.d_head * elem_size(m->d.dtype);
}

psd_status psd_kv_create(const psd_model *m, int32_t batch, int32_t max_len, void *k_mem, void *v_mem,
                         int32_t *lens_dev, int32_t len_upper_bound, psd_kv **out) {
    if (!m || !k_mem || !v_mem || !lens_dev || !out) return PSD_ERR_NULL;
    if (batch <= 0 || batch > 65535 || max_len <= 0 || max_len % 64) return PSD_ERR_SHAPE;
    if (m->d.dtype == PSD_F32 && max_len > 12288) return PSD_ERR_SHAPE;   // fp32 attention keeps a row of scores in LDS
    if (len_upper_bound < 0 || len_upper_bound > max_len) return PSD_ERR_CAPACITY;
    if ((uintptr_t)k_mem % 256 || (uintptr_t)v_mem % 256) return PSD_ERR_SHAPE;
    psd_kv *kv = new (std::nothrow) psd_kv;
    if (!kv) return PSD_ERR_NULL;
    kv->m = m; kv->batch = batch; kv->max_len = max_len; kv->k = k_mem; kv->v = v_mem;
    kv->lens = lens_dev; kv->len_ub = len_upper_bound;
    *out = kv;
    return PSD_OK;
}

psd_status psd_kv_destroy(psd_kv *kv) {
    if (!kv) return PSD_ERR_NULL;
    delete kv;
    return PSD_OK;
}

int32_t psd_kv_len_upper_bound(const psd_kv *kv) { return kv ? kv->len_ub : -1; }

}  // extern "C"

// ------------------------------------------------------------------ forward-pass workspace
namespace {

struct ForwardPlan {
    int M, width_qkv;
    int sk_qkv, sk_o, sk_gu, sk_down, sk_head, attn_splits;
    size_t off_x, off_xn, off_q, off_attn, off_h, off_partial, off_po, off_pml, off_sumsq, off_rope, off_tilectr, off_tree, total;
    size_t off_xn16, off_attn16, off_h16;
    bool half_copies;             // bf16, M > kStreamMaxRows or 4-bit projections: the producers also leave fp16 copies of the activations
    bool folded;                  // RMSNorm folded into the projections (bf16, packed weights, M <= kStreamMaxRows)
    bool fused_rope;              // the attention kernel reduces, rotates and appends q / k / v itself
};

ForwardPlan plan_forward(const psd_model *mdl, int batch, int n_new, int n_logit_rows, int len_bound, bool tree) {
    const psd_model_desc &d = mdl->d;
    ForwardPlan p{};
    const int M = batch * n_new;
    p.M = M;
    const int hd = d.n_q_heads * d.d_head, kvd = d.n_kv_heads * d.d_head;
    p.width_qkv = hd + 2 * kvd;
    const int n_qkv[3] = {hd, kvd, kvd}, n_o[1] = {d.d_model}, n_gu[2] = {d.d_ffn, d.d_ffn}, n_v[1] = {d.vocab};
    const int Ml = batch * n_logit_rows;
    p.folded = mdl->packed && d.dtype == PSD_BF16 && M <= kStreamMaxRows;
    auto splits = [&](int rows, int K, int N, const int *n, int nseg) {
        if (mdl->w4 && n != n_v && rows <= kStreamMaxRows) return gemm_w4_slots(K, n, nseg, false);
        if (mdl->packed && rows <= kStreamMaxRows) return gemm_packed_splits(rows, K, n, nseg);
        return gemm_pick_splitk(d.dtype, rows, K, N, n, nseg);
    };
    p.fused_rope = attn_fuses_rope(d.dtype, n_new, d.n_q_heads, d.n_kv_heads, d.d_head, tree);
    p.sk_qkv = splits(M, d.d_model, p.width_qkv, n_qkv, 3);
    // folded: O runs on the column kernel (one owner per output), or, 4-bit, on partial slots with the arrival epilogue
    p.sk_o = p.folded ? (mdl->w4 ? gemm_w4_slots(hd, n_o, 1, true) : 1) : splits(M, hd, d.d_model, n_o, 1);
    p.sk_gu = splits(M, d.d_model, 2 * d.d_ffn, n_gu, 2);
    // folded: the down projection runs on the unit kernel with the residual epilogue, its partials in slots
    p.sk_down = p.folded ? (mdl->w4 ? gemm_w4_slots(d.d_ffn, n_o, 1, true) : gemm_resid_slots(gemm_pack_tiles(n_o, 1), d.d_ffn))
                         : splits(M, d.d_ffn, d.d_model, n_o, 1);
    p.sk_head = Ml > 0 ? splits(Ml, d.d_model, d.vocab, n_v, 1) : 1;
    p.attn_splits = attn_pick_splits(d.dtype, batch, n_new, d.n_q_heads, d.n_kv_heads, d.d_head, len_bound, tree);
    const size_t act = 4;                                    // activations are fp32 for both dtypes
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += align256(bytes); return o; };
    p.off_x = take((size_t)M * d.d_model * 4);
    p.off_xn = take((size_t)M * d.d_model * act);
    p.off_q = take((size_t)M * hd * act);
    p.off_attn = take((size_t)M * hd * act);
    p.off_h = take((size_t)M * d.d_ffn * act);
    p.half_copies = d.dtype == PSD_BF16 && (M > kStreamMaxRows || (mdl->w4 && p.folded));
    p.off_xn16 = take(p.half_copies ? (size_t)M * d.d_model * 2 : 0);
    p.off_attn16 = take(p.half_copies ? (size_t)M * hd * 2 : 0);
    p.off_h16 = take(p.half_copies ? (size_t)M * d.d_ffn * 2 : 0);
    size_t part = 0;
    auto need = [&](int sk, int rows, int N) { const size_t b = (size_t)sk * rows * N * 4; if (b > part) part = b; };
    need(p.sk_qkv, M, p.width_qkv); need(p.sk_o, M, d.d_model); need(p.sk_gu, M, 2 * d.d_ffn);
    need(p.sk_down, M, d.d_model);
    if (p.sk_head > 1 || p.folded) need(p.sk_head, Ml, d.vocab);  // else a single split writes the logits in place
    p.off_partial = take(part);
    p.off_po = take(p.attn_splits > 1 ? (size_t)M * d.n_q_heads * p.attn_splits * d.d_head * 4 : 0);
    p.off_pml = take(p.attn_splits > 1 ? (size_t)M * d.n_q_heads * p.attn_splits * 2 * 4 : 0);
    p.off_sumsq = take(p.folded ? (size_t)(d.d_model / 16) * M * 4 : 0);
    p.off_rope = take(p.fused_rope ? (size_t)M * (d.d_head / 2) * sizeof(float2) : 0);
    p.off_tilectr = take(p.folded ? (size_t)gemm_pack_tiles(n_o, 1) * 4 : 0);
    p.off_tree = take(p.fused_rope ? (size_t)kTreeMaxNodes * 8 : 0);      // ancestor masks and depths of a tree pass
    p.total = off;
    return p;
}

bool forward_shape_ok(const psd_model *m, int batch, int n_new) {
    if (batch <= 0 || batch > 65535 || n_new <= 0) return false;
    if ((long)batch * n_new > 65535) return false;
    if ((long)batch * m->d.n_kv_heads > 65535) return false;      // grid z of the attention launch
    if ((long)(m->d.n_q_heads / m->d.n_kv_heads) * n_new > 4096) return false;
    return true;
}

}  // namespace

extern "C" {

size_t psd_model_workspace_bytes(const psd_model *m, int32_t batch, int32_t n_new, int32_t max_len) {
    if (!m || max_len <= 0 || !forward_shape_ok(m, batch, n_new)) return 0;
    // split choices depend on the cache length bound, on how many rows get logits and on whether the rows are a
    // token tree: take the largest need over all of them
    size_t worst = 0;
    for (int rows = 0; rows <= n_new; ++rows)
        for (int tree = 0; tree < 2; ++tree) {
            const size_t a = plan_forward(m, batch, n_new, rows, max_len, tree != 0).total;
            const size_t b = plan_forward(m, batch, n_new, rows, n_new, tree != 0).total;
            worst = a > worst ? a : worst;
            worst = b > worst ? b : worst;
        }
    return worst;
}

static psd_status forward_once(psd_model *m, const int32_t *tokens_dev, int32_t n_new, psd_kv *kv,
                               float *logits_out_dev, int32_t n_logit_rows, void *workspace, size_t ws_bytes,
                               void *hip_stream, const TreeShape *tree = nullptr);

psd_status psd_model_forward(psd_model *m, const int32_t *tokens_dev, int32_t n_new, psd_kv *kv,
                             float *logits_out_dev, int32_t n_logit_rows, void *workspace, size_t ws_bytes,
                             void *hip_stream) {
    if (!m || !tokens_dev || !kv) return PSD_ERR_NULL;
    if (kv->m != m) return PSD_ERR_SHAPE;
    const int B = kv->batch;
    if (!forward_shape_ok(m, B, n_new)) return PSD_ERR_SHAPE;
    if (n_logit_rows < 0 || n_logit_rows > n_new) return PSD_ERR_SHAPE;
    if (n_logit_rows > 0 && !logits_out_dev) return PSD_ERR_NULL;
    if (kv->len_ub + n_new > kv->max_len) return PSD_ERR_CAPACITY;
    if (m->w4 && !m->packed) return PSD_ERR_UNIMPLEMENTED;
    return forward_once(m, tokens_dev, n_new, kv, logits_out_dev, n_logit_rows, workspace, ws_bytes, hip_stream);
}

static psd_status forward_once(psd_model *m, const int32_t *tokens_dev, int32_t n_new, psd_kv *kv,
                               float *logits_out_dev, int32_t n_logit_rows, void *workspace, size_t ws_bytes,
                               void *hip_stream, const TreeShape *tree) {
    const psd_model_desc &d = m->d;
    const int B = kv->batch;
    const int len_bound = kv->len_ub + n_new;
    const ForwardPlan p = plan_forward(m, B, n_new, n_logit_rows, len_bound, tree != nullptr);
    if (!workspace || (uintptr_t)workspace % 256 || ws_bytes < p.total) return PSD_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;
    float *x = (float *)(ws + p.off_x);
    float *xn = (float *)(ws + p.off_xn);
    float *q = (float *)(ws + p.off_q);
    float *attn = (float *)(ws + p.off_attn);
    float *h = (float *)(ws + p.off_h);
    uint16_t *xn16 = p.half_copies ? (uint16_t *)(ws + p.off_xn16) : nullptr;
    uint16_t *attn16 = p.half_copies ? (uint16_t *)(ws + p.off_attn16) : nullptr;
    uint16_t *h16 = p.half_copies ? (uint16_t *)(ws + p.off_h16) : nullptr;
    float *partial = (float *)(ws + p.off_partial);
    const int M = p.M, hd = d.n_q_heads * d.d_head, kvd = d.n_kv_heads * d.d_head;
    const size_t kv_layer = (size_t)B * d.n_kv_heads * kv->max_len * d.d_head * elem_size(d.dtype);

    (void)hipGetLastError();
    auto norm_gain = [&](int l) { return l < d.n_layers ? m->layer(l, W_ATTN_NORM) : m->final_norm(); };
    // ql, qj: layer and index of the first segment among the layer's 4-bit projections (q k v o gate up down), if any
    auto gemm = [&](const float *xin, int rows, int K, const void *w0, int n0, const void *w1, int n1,
                    const void *w2, int n2, int sk, float *dst, const void *wpack, int ql = -1, int qj = -1) {
        GemmArgs g{};
        g.wpack = rows <= kStreamMaxRows ? wpack : nullptr;
        g.x = xin; g.x_rows_per_group = rows > 0 ? rows : 1; g.x_group_stride = 0; g.x_group_offset = 0;
        g.x16 = xin == xn ? xn16 : (xin == attn ? attn16 : (xin == h ? h16 : nullptr));
        g.w[0] = w0; g.w[1] = w1; g.w[2] = w2; g.n[0] = n0; g.n[1] = n1; g.n[2] = n2;
        g.nseg = w2 ? 3 : (w1 ? 2 : 1);
        g.M = rows; g.K = K; g.N = n0 + n1 + n2; g.partial = dst; g.splitk = sk; g.reduced = nullptr;
        g.pack_tiles = gemm_pack_tiles(g.n, g.nseg);
        g.w4 = m->w4 && qj >= 0;
        for (int sgm = 0; sgm < g.nseg && g.w4; ++sgm) { g.w4_scale[sgm] = m->qscale(ql, qj + sgm); g.w4_zero[sgm] = m->qzero(ql, qj + sgm); }
        launch_gemm(d.dtype, g, st);
    };
    // Folded mode: no RMSNorm kernel runs.  The projections that write the residual stream add into it and
    // leave behind x * gain of the next norm (in xn) and per-16-column sums of squares (one slab of M floats
    // per strip); the projections that read the residual stream take xn as it is, and the kernels that consume
    // their output multiply by the row scale rsqrt(mean x^2 + eps).
    float *sumsq = (float *)(ws + p.off_sumsq);
    const int col_tiles = d.d_model / 16;
    const int n_o_fw[1] = {d.d_model};
    RowScale rs{nullptr, 0, 1.0f / (float)d.d_model, d.rms_eps};
    if (p.folded) rs.sumsq = sumsq;
    const float *act = xn;     // what QKV / gate|up / lm_head read: rmsnorm(x) * gain, or x * gain when folded
    unsigned *tile_ctr = p.folded ? (unsigned *)(ws + p.off_tilectr) : nullptr;
    auto resid_gemm = [&](const float *xin, int K, const void *w, int sk, const void *wpack, const void *next_gain,
                          bool by_units, int ql, int qj) {
        if (p.folded) {
            GemmArgs g{};
            g.wpack = wpack; g.x = xin; g.x_rows_per_group = M; g.w[0] = w; g.n[0] = d.d_model; g.nseg = 1;
            const bool slots = by_units || m->w4;         // partial slots + arrival epilogue, else one block per 16 columns
            g.M = M; g.K = K; g.N = d.d_model; g.splitk = slots ? sk : 1; g.pack_tiles = gemm_pack_tiles(g.n, 1);
            g.x_resid = x; g.xg_out = xn; g.xg16_out = xn16; g.gain = next_gain; g.sumsq_out = sumsq; g.w4 = m->w4;
            g.x16 = xin == attn ? attn16 : (xin == h ? h16 : nullptr);
            if (slots) { g.tile_counter = tile_ctr; g.partial = partial; }
            launch_gemm(d.dtype, g, st);
            rs.tiles = slots ? g.pack_tiles : col_tiles;
        } else {
            gemm(xin, M, K, w, d.d_model, nullptr, 0, nullptr, 0, sk, partial, wpack, ql, qj);
            launch_reduce_residual_norm(d.dtype, partial, sk, x, next_gain, xn, M, d.d_model, d.rms_eps, xn16, st);
        }
    };
    RopeTable rt{};
    if (p.fused_rope) rt = RopeTable{(float2 *)(ws + p.off_rope), kv->lens, n_new, d.d_head, d.rope_theta, nullptr};
    const uint32_t *tree_anc = nullptr;
    if (tree) {
        // a token tree: positions by depth, visibility by ancestry (both only exist in the fused attention build)
        if (!p.fused_rope) return PSD_ERR_UNIMPLEMENTED;
        uint32_t *anc = (uint32_t *)(ws + p.off_tree);
        int32_t *depth = (int32_t *)(anc + kTreeMaxNodes);
        launch_tree_setup(*tree, anc, depth, st);
        rt.depth = depth;
        tree_anc = anc;
    }
    launch_embed_norm(d.dtype, m->embed(), tokens_dev, x, norm_gain(0), xn, p.folded ? sumsq : nullptr, M, d.d_model,
                      d.vocab, d.rms_eps, rt, xn16, ZeroFill{tile_ctr, p.folded ? gemm_pack_tiles(n_o_fw, 1) : 0}, st);
    rs.tiles = 1;
    for (int l = 0; l < d.n_layers; ++l) {
        gemm(act, M, d.d_model, m->layer(l, W_Q), hd, m->layer(l, W_K), kvd, m->layer(l, W_V), kvd, p.sk_qkv, partial,
             m->pack(l, P_QKV), l, 0);
        char *kl = (char *)kv->k + (size_t)l * kv_layer, *vl = (char *)kv->v + (size_t)l * kv_layer;
        if (!p.fused_rope)
            launch_reduce_rope_append(d.dtype, partial, p.sk_qkv, rs, q, kl, vl, kv->lens, B, n_new, d.n_q_heads,
                                      d.n_kv_heads, d.d_head, kv->max_len, d.rope_theta, st);
        AttnArgs a{};
        if (p.fused_rope) { a.qkv_partial = partial; a.qkv_splits = p.sk_qkv; a.rs = rs; a.rope_cs = rt.cs; a.tree_anc = tree_anc; }
        a.q = q; a.k = kl; a.v = vl; a.lens = kv->lens; a.out = attn; a.out16 = attn16;
        a.B = B; a.R = n_new; a.h_q = d.n_q_heads; a.h_kv = d.n_kv_heads; a.d_h = d.d_head; a.max_len = kv->max_len;
        a.len_bound = len_bound; a.part_o = (float *)(ws + p.off_po); a.part_ml = (float *)(ws + p.off_pml);
        a.splits = p.attn_splits;
        launch_attention(d.dtype, a, st);

        resid_gemm(attn, hd, m->layer(l, W_O), p.sk_o, m->pack(l, P_O), m->layer(l, W_FFN_NORM), false, l, 3);
        gemm(act, M, d.d_model, m->layer(l, W_GATE), d.d_ffn, m->layer(l, W_UP), d.d_ffn, nullptr, 0, p.sk_gu, partial,
             m->pack(l, P_GU), l, 4);
        launch_reduce_swiglu(partial, p.sk_gu, rs, h, M, d.d_ffn, h16, st);
        resid_gemm(h, d.d_ffn, m->layer(l, W_DOWN), p.sk_down, m->pack(l, P_DOWN), norm_gain(l + 1), true, l, 6);
    }
    if (n_logit_rows > 0) {
        // lm_head on the last n_logit_rows rows of every sequence (unfolded: xn already holds the final norm)
        GemmArgs hg{};
        hg.x = act; hg.x16 = xn16; hg.x_rows_per_group = n_logit_rows; hg.x_group_stride = n_new; hg.x_group_offset = n_new - n_logit_rows;
        hg.w[0] = m->lm_head(); hg.n[0] = d.vocab; hg.nseg = 1;
        hg.M = B * n_logit_rows; hg.K = d.d_model; hg.N = d.vocab;
        hg.wpack = hg.M <= kStreamMaxRows ? m->pack_head() : nullptr;
        hg.pack_tiles = gemm_pack_tiles(hg.n, 1);
        hg.splitk = p.sk_head;
        const bool two_step = p.sk_head > 1 || p.folded;
        hg.partial = two_step ? partial : logits_out_dev;
        hg.reduced = two_step ? logits_out_dev : nullptr;
        if (p.folded) { hg.scale = rs; hg.scale_rows = M; }
        launch_gemm(d.dtype, hg, st);
    }
    launch_advance_lens(kv->lens, B, n_new, kv->max_len, st);
    const psd_status s = check_launch();
    if (s == PSD_OK) kv->len_ub += n_new;
    return s;
}

size_t psd_spec_accept_workspace_bytes(int32_t rows, int32_t gamma, int32_t n_p_rows, int32_t vocab) {
    if (rows < 0 || gamma < 0 || gamma > 64 || vocab <= 0) return 0;
    if (n_p_rows != gamma && n_p_rows != gamma + 1) return 0;
    AcceptArgs a{};
    accept_plan(rows, gamma, n_p_rows, vocab, PSD_F32, false, &a);   // the unaligned plan needs the most
    return accept_workspace_bytes(a);
}

static psd_status spec_accept_impl(const void *p_logits, const void *q_logits, const int32_t *draft_tokens, int32_t gamma,
                                   const float *uniforms, float temperature, int32_t *out_accept_len, int32_t *out_token,
                                   int32_t rows, int32_t n_p_rows, int32_t vocab, int32_t dtype, int64_t p_seq_stride,
                                   int64_t q_seq_stride, int32_t *out_flags, void *workspace, size_t ws_bytes,
                                   void *(*late_workspace)(), void *hip_stream) {
    if (dtype != PSD_F32 && dtype != PSD_BF16) return PSD_ERR_DTYPE;
    if (rows < 0 || gamma < 0 || gamma > 64 || vocab <= 0 || vocab > (1 << 23)) return PSD_ERR_SHAPE;
    if (n_p_rows != gamma && n_p_rows != gamma + 1) return PSD_ERR_SHAPE;
    if (gamma == 0 && n_p_rows == 0) return PSD_ERR_SHAPE;
    if ((long)rows * (n_p_rows + gamma) > (1L << 24)) return PSD_ERR_SHAPE;
    if (!(temperature >= 0.f) || !std::isfinite(temperature)) return PSD_ERR_TEMPERATURE;
    const bool greedy = temperature == 0.f;              // reads neither q nor the uniforms
    if (rows == 0) return PSD_OK;
    if (!p_logits || !out_accept_len || !out_token) return PSD_ERR_NULL;
    if (!greedy && !uniforms) return PSD_ERR_NULL;
    if (gamma > 0 && (!draft_tokens || (!greedy && !q_logits))) return PSD_ERR_NULL;
    if (greedy) { q_logits = nullptr; q_seq_stride = 0; }
    if (p_seq_stride < (int64_t)n_p_rows * vocab || (gamma > 0 && !greedy && q_seq_stride < (int64_t)gamma * vocab))
        return PSD_ERR_SHAPE;
    const size_t es = elem_size(dtype);
    if ((uintptr_t)p_logits % es || (uintptr_t)q_logits % es) return PSD_ERR_SHAPE;
    const int epl = (int)(16 / es);
    const bool vec = vocab % epl == 0 && p_seq_stride % epl == 0 && q_seq_stride % epl == 0 &&
                     (uintptr_t)p_logits % 16 == 0 && (uintptr_t)q_logits % 16 == 0;
    AcceptArgs a{};
    accept_plan(rows, gamma, n_p_rows, vocab, dtype, vec, &a);
    if (ws_bytes < accept_workspace_bytes(a)) return PSD_ERR_WORKSPACE;
    if (late_workspace) workspace = late_workspace();    // the built-in buffer: looked up once the sizes are known to fit
    if (!workspace || (uintptr_t)workspace % 256) return late_workspace ? PSD_ERR_HIP : PSD_ERR_WORKSPACE;
    accept_bind_workspace(&a, workspace, out_flags);
    a.p = p_logits; a.q = q_logits; a.x = draft_tokens; a.u = uniforms;
    a.p_stride = p_seq_stride; a.q_stride = q_seq_stride; a.temperature = temperature;
    a.out_n = out_accept_len; a.out_tok = out_token;
    (void)hipGetLastError();
    if (greedy) launch_accept_greedy(a, vec, (hipStream_t)hip_stream);
    else launch_accept(a, vec, (hipStream_t)hip_stream);
    return check_launch();
}

psd_status psd_spec_accept(const void *p_logits, const void *q_logits, const int32_t *draft_tokens, int32_t gamma,
                           const float *uniforms, float temperature, int32_t *out_accept_len, int32_t *out_token,
                           int32_t rows, int32_t n_p_rows, int32_t vocab, int32_t dtype, int64_t p_seq_stride,
                           int64_t q_seq_stride, int32_t *out_flags, void *workspace, size_t ws_bytes,
                           void *hip_stream) {
    return spec_accept_impl(p_logits, q_logits, draft_tokens, gamma, uniforms, temperature, out_accept_len, out_token,
                            rows, n_p_rows, vocab, dtype, p_seq_stride, q_seq_stride, out_flags, workspace, ws_bytes,
                            nullptr, hip_stream);
}

// ---- the entry point that allocates nothing: acceptance on a scratch buffer built into the library
// One copy of the array per GPU; host code never uses its name as an address, only the device address that
// hipGetSymbolAddress returns for the current device (looked up on the first call per device and kept).
static __device__ __align__(256) unsigned char scratch[PSD_STATIC_SCRATCH_BYTES];
namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_dev[kMaxDevices] = {};
void *static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        g_last_hip_error = (int32_t)hipGetLastError();
        return nullptr;
    }
    if (!g_scratch_dev[dev]) {
        void *ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            g_last_hip_error = (int32_t)e;
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_dev[dev] = ptr;
    }
    return g_scratch_dev[dev];
}
}  // namespace

psd_status psd_spec_accept_static(const void *p_logits, const void *q_logits, const int32_t *draft_tokens, int32_t gamma,
                                  const float *uniforms, float temperature, int32_t *out_accept_len,
                                  int32_t *out_token, int32_t rows, int32_t n_p_rows, int32_t vocab, int32_t dtype,
                                  int64_t p_seq_stride, int64_t q_seq_stride, int32_t *out_flags, void *hip_stream) {
    return spec_accept_impl(p_logits, q_logits, draft_tokens, gamma, uniforms, temperature, out_accept_len, out_token,
                            rows, n_p_rows, vocab, dtype, p_seq_stride, q_seq_stride, out_flags, nullptr,
                            PSD_STATIC_SCRATCH_BYTES, static_scratch, hip_stream);
}

psd_status psd_kv_truncate(psd_kv *kv, const int32_t *base_lens_dev, const int32_t *keep_dev, int32_t keep_offset,
                           int32_t new_len_upper_bound, void *hip_stream) {
    if (!kv || !base_lens_dev || !keep_dev) return PSD_ERR_NULL;
    const int cap = new_len_upper_bound < 0 || new_len_upper_bound > kv->len_ub ? kv->len_ub : new_len_upper_bound;
    (void)hipGetLastError();
    launch_truncate(kv->lens, base_lens_dev, keep_dev, keep_offset, cap, kv->batch, (hipStream_t)hip_stream);
    const psd_status s = check_launch();
    if (s == PSD_OK) kv->len_ub = cap;
    return s;
}

// host-side check of a tree's parent array and its ancestor masks / depths
static bool tree_shape_from_parents(const int32_t *parents, int n, int max_nodes, TreeShape *ts) {
    if (!parents || n < 1 || n > max_nodes || parents[0] != -1) return false;
    for (int i = 1; i < n; ++i)
        if (parents[i] < 0 || parents[i] >= i) return false;
    if (ts) {
        ts->n = n;
        for (int i = 0; i < n; ++i) {
            ts->anc[i] = (i ? ts->anc[parents[i]] : 0u) | (1u << i);
            ts->depth[i] = i ? ts->depth[parents[i]] + 1 : 0;
        }
    }
    return true;
}

psd_status psd_model_forward_tree(psd_model *m, const int32_t *tokens_dev, int32_t n_nodes, const int32_t *parents_host,
                                  psd_kv *kv, float *logits_out_dev, void *workspace, size_t ws_bytes, void *hip_stream) {
    if (!m || !tokens_dev || !kv || !logits_out_dev || !parents_host) return PSD_ERR_NULL;
    if (kv->m != m) return PSD_ERR_SHAPE;
    const int B = kv->batch;
    TreeShape ts{};
    if (!forward_shape_ok(m, B, n_nodes) || !tree_shape_from_parents(parents_host, n_nodes, kTreeMaxNodes, &ts)) return PSD_ERR_SHAPE;
    if (kv->len_ub + n_nodes > kv->max_len) return PSD_ERR_CAPACITY;
    if (m->w4 && !m->packed) return PSD_ERR_UNIMPLEMENTED;
    return forward_once(m, tokens_dev, n_nodes, kv, logits_out_dev, n_nodes, workspace, ws_bytes, hip_stream, &ts);
}

psd_status psd_tree_accept(const void *p_logits, const void *q_logits, const int32_t *tokens_dev, const int32_t *parents_host,
                           int32_t n_nodes, const float *uniforms, float temperature, int32_t *out_path_len,
                           int32_t *out_path, int32_t *out_token, int32_t rows, int32_t vocab, int32_t dtype,
                           int64_t p_seq_stride, int64_t q_seq_stride, int32_t *out_flags, void *hip_stream) {
    if (dtype != PSD_F32 && dtype != PSD_BF16) return PSD_ERR_DTYPE;
    if (rows < 0 || vocab <= 0 || vocab > (1 << 23)) return PSD_ERR_SHAPE;
    if (!tree_shape_from_parents(parents_host, n_nodes, kTreeMaxAcceptNodes, nullptr)) return PSD_ERR_SHAPE;
    if (!(temperature >= 0.f) || !std::isfinite(temperature)) return PSD_ERR_TEMPERATURE;
    const bool greedy = temperature == 0.f;
    if (rows == 0) return PSD_OK;
    if (!p_logits || !tokens_dev || !out_path_len || !out_path || !out_token) return PSD_ERR_NULL;
    if (!greedy && (!q_logits || !uniforms)) return PSD_ERR_NULL;
    if (greedy) { q_logits = p_logits; q_seq_stride = p_seq_stride; }        // never read
    if (p_seq_stride < (int64_t)n_nodes * vocab || q_seq_stride < (int64_t)n_nodes * vocab) return PSD_ERR_SHAPE;
    const size_t es = elem_size(dtype);
    if ((uintptr_t)p_logits % es || (uintptr_t)q_logits % es) return PSD_ERR_SHAPE;
    TreeAcceptArgs a{};
    a.p = p_logits; a.q = q_logits; a.p_stride = p_seq_stride; a.q_stride = q_seq_stride;
    a.tokens = tokens_dev; a.uniforms = uniforms; a.temperature = temperature;
    a.out_path_len = out_path_len; a.out_path = out_path; a.out_token = out_token; a.out_flags = out_flags;
    a.rows = rows; a.n_nodes = n_nodes; a.vocab = vocab;
    for (int i = 0; i < n_nodes; ++i) a.parents[i] = parents_host[i];
    (void)hipGetLastError();
    launch_tree_accept(dtype, a, (hipStream_t)hip_stream);
    return check_launch();
}

psd_status psd_kv_compact_tree(psd_kv *kv, const int32_t *base_lens_dev, const int32_t *path_dev, const int32_t *path_len_dev,
                               int32_t path_stride, int32_t n_nodes, int32_t new_len_upper_bound, void *hip_stream) {
    if (!kv || !base_lens_dev || !path_dev || !path_len_dev) return PSD_ERR_NULL;
    if (n_nodes < 1 || n_nodes > kTreeMaxNodes || path_stride < n_nodes - 1) return PSD_ERR_SHAPE;
    if (base_lens_dev == kv->lens) return PSD_ERR_SHAPE;                       // the lengths are rewritten while blocks read the base
    const psd_model_desc &d = kv->m->d;
    const int cap = new_len_upper_bound < 0 || new_len_upper_bound > kv->len_ub ? kv->len_ub : new_len_upper_bound;
    (void)hipGetLastError();
    launch_kv_compact_tree(d.dtype, kv->k, kv->v, kv->lens, base_lens_dev, path_dev, path_len_dev, path_stride, n_nodes,
                           d.n_layers, kv->batch, d.n_kv_heads, d.d_head, kv->max_len, cap, (hipStream_t)hip_stream);
    const psd_status s = check_launch();
    if (s == PSD_OK) kv->len_ub = cap;
    return s;
}

psd_status psd_profile_enable(int32_t max_launches) {
    for (hipEvent_t e : g_rec.ev) (void)hipEventDestroy(e);
    g_rec.ev.clear(); g_rec.kind.clear();
    g_rec.used = g_rec.cap = 0; g_rec.on = false;
    if (max_launches < 0) return PSD_ERR_SHAPE;
    if (max_launches == 0) return PSD_OK;
    g_rec.ev.resize(2 * (size_t)max_launches);
    g_rec.kind.resize(max_launches);
    for (size_t i = 0; i < g_rec.ev.size(); ++i) {
        if (hipEventCreate(&g_rec.ev[i]) != hipSuccess) {
            for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(g_rec.ev[j]);
            g_rec.ev.clear(); g_rec.kind.clear();
            g_last_hip_error = (int32_t)hipGetLastError();
            return PSD_ERR_HIP;
        }
    }
    g_rec.cap = max_launches;
    g_rec.on = true;
    return PSD_OK;
}

psd_status psd_profile_collect(double *ms_by_kind, int64_t *launches_by_kind) {
    if (!ms_by_kind || !launches_by_kind) return PSD_ERR_NULL;
    for (int k = 0; k < PSD_KIND_COUNT; ++k) { ms_by_kind[k] = 0.0; launches_by_kind[k] = 0; }
    if (g_rec.used == 0) return PSD_OK;
    if (hipEventSynchronize(g_rec.ev[2 * g_rec.used - 1]) != hipSuccess) {
        g_last_hip_error = (int32_t)hipGetLastError();
        return PSD_ERR_HIP;
    }
    for (size_t i = 0; i < g_rec.used; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g_rec.ev[2 * i], g_rec.ev[2 * i + 1]) != hipSuccess) continue;
        const int k = g_rec.kind[i];
        if (k >= 0 && k < PSD_KIND_COUNT) { ms_by_kind[k] += ms; ++launches_by_kind[k]; }
    }
    g_rec.used = 0;
    return PSD_OK;
}

psd_status psd_probe_stream_read(const void *src_dev, size_t bytes, void *sink_dev, int32_t blocks, void *hip_stream) {
    if (!src_dev || !sink_dev) return PSD_ERR_NULL;
    if (bytes == 0 || bytes % 16 || (uintptr_t)src_dev % 16 || blocks <= 0 || blocks > (1 << 20)) return PSD_ERR_SHAPE;
    (void)hipGetLastError();
    launch_probe_read(src_dev, bytes, sink_dev, blocks, (hipStream_t)hip_stream);
    return check_launch();
}

psd_status psd_probe_mfma(const void *seed_dev, float *sink_dev, int32_t blocks, int32_t iters, void *hip_stream) {
    if (!seed_dev || !sink_dev) return PSD_ERR_NULL;
    if ((uintptr_t)seed_dev % 16 || blocks <= 0 || blocks > (1 << 20) || iters <= 0) return PSD_ERR_SHAPE;
    (void)hipGetLastError();
    launch_probe_mfma(seed_dev, sink_dev, blocks, iters, (hipStream_t)hip_stream);
    return check_launch();
}

psd_status psd_kv_truncate_to(psd_kv *kv, int32_t new_len, void *hip_stream) {
    if (!kv) return PSD_ERR_NULL;
    if (new_len < 0) return PSD_ERR_SHAPE;
    (void)hipGetLastError();
    launch_truncate_to(kv->lens, new_len, kv->batch, (hipStream_t)hip_stream);
    const psd_status s = check_launch();
    if (s == PSD_OK && new_len < kv->len_ub) kv->len_ub = new_len;
    return s;
}

}  // extern "C"
