"""Device-memory plumbing around the C boundary: owns the torch tensors a handle points at.

Nothing here computes; each method allocates or copies tensors and forwards to the binding
function of the same name in the package root.
"""
import torch

import paper_2510_26527_amd as psd

_LAYER_WEIGHTS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")
_QUANT_WEIGHTS = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def weight_order(n_layers):
    names = ["embed"]
    for l in range(n_layers):
        names += [f"l{l}.{n}" for n in _LAYER_WEIGHTS]
    return names + ["final_norm", "lm_head"]


class Model:
    """A psd_model handle plus the weight tensors it points at (kept alive here)."""

    def __init__(self, shape, weights, device="cuda", quant=None):
        # shape: any object with the psd_model_desc field names; weights: name -> tensor
        # quant: for a 4-bit model, name -> (scale bf16 [n, K/128], zero uint8 [n, K/128]) for every projection;
        #        weights[name] then holds the codes, uint8 [n, K/2]
        dt = weights["embed"].dtype
        self.dtype = dt
        self.code = psd.dtype_code(dt)
        self.device = torch.device(device)
        self.weights = {k: v.to(self.device).contiguous() for k, v in weights.items()}
        self.desc = psd.psd_model_desc(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads,
                                       shape.d_head, shape.d_ffn, shape.vocab, shape.rope_theta, shape.rms_eps,
                                       self.code)
        self.shape = shape
        ptrs = [self.weights[n].data_ptr() for n in weight_order(shape.n_layers)]
        self.quant = None
        if quant is None:
            self.handle = psd.psd_model_create(self.desc, ptrs)
        else:
            self.quant = {k: (s.to(self.device).contiguous(), z.to(self.device).contiguous()) for k, (s, z) in quant.items()}
            names = [f"l{l}.{n}" for l in range(shape.n_layers) for n in _QUANT_WEIGHTS]
            self.handle = psd.psd_model_create_w4(self.desc, ptrs, [self.quant[n][0].data_ptr() for n in names],
                                                  [self.quant[n][1].data_ptr() for n in names])
        self._ws = None
        self.packed = None

    def pack(self):
        """Build the streaming copy of the projection weights (bf16 models) for steps of <= 16 rows."""
        need = psd.psd_model_packed_bytes(self.handle)
        if need == 0:
            return self
        self.packed = torch.empty(need, dtype=torch.uint8, device=self.device)
        psd.psd_model_pack(self.handle, self.packed)
        self._ws = None
        return self

    def workspace(self, batch, n_new, max_len):
        need = psd.psd_model_workspace_bytes(self.handle, batch, n_new, max_len)
        if need == 0:
            raise ValueError("unsupported batch / n_new / max_len")
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._ws

    def workspace_upto(self, batch, max_new, max_len):
        """A workspace large enough for every n_new in 1..max_new."""
        need = max(psd.psd_model_workspace_bytes(self.handle, batch, r, max_len) for r in range(1, max_new + 1))
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._ws

    def close(self):
        if self.handle is not None:
            psd.psd_model_destroy(self.handle)
            self.handle = None


class KVCache:
    """K [L,B,h_kv,max_len,d_h] and transposed V [L,B,h_kv,d_h,max_len] tensors, the device
    length vector, and the psd_kv handle over them."""

    def __init__(self, model: Model, batch, max_len, fill_garbage=False):
        s = model.shape
        self.model, self.batch, self.max_len = model, batch, max_len
        alloc = torch.empty if not fill_garbage else (lambda *a, **k: torch.full(*a, float("nan"), **k))
        self.k = alloc((s.n_layers, batch, s.n_kv_heads, max_len, s.d_head), dtype=model.dtype, device=model.device)
        self.v = alloc((s.n_layers, batch, s.n_kv_heads, s.d_head, max_len), dtype=model.dtype, device=model.device)
        self.lens = torch.zeros(batch, dtype=torch.int32, device=model.device)
        self.handle = psd.psd_kv_create(model.handle, batch, max_len, self.k, self.v, self.lens, 0)

    def load(self, k_layers, v_layers, lens):
        """Copy given contents in: k_layers / v_layers are per-layer [B, h_kv, n_ctx, d_h] tensors
        (logical layout), lens the valid length per sequence (int or list)."""
        n_ctx = k_layers[0].shape[2]
        for l, (k, v) in enumerate(zip(k_layers, v_layers)):
            self.k[l, :, :, :n_ctx].copy_(k)
            self.v[l, :, :, :, :n_ctx].copy_(v.transpose(-1, -2))
        lens_t = torch.as_tensor(lens, dtype=torch.int32).expand(self.batch).contiguous()
        self.lens.copy_(lens_t)
        psd.psd_kv_destroy(self.handle)
        self.handle = psd.psd_kv_create(self.model.handle, self.batch, self.max_len, self.k, self.v, self.lens,
                                        int(lens_t.max()))

    def close(self):
        if self.handle is not None:
            psd.psd_kv_destroy(self.handle)
            self.handle = None


def forward(model: Model, kv: KVCache, tokens, n_logit_rows=None, logits_out=None, stream=None):
    """tokens int32 [B, n_new] on the device -> fp32 logits [B, n_logit_rows, V] (a new tensor
    unless logits_out is given)."""
    B, n_new = tokens.shape
    rows = n_new if n_logit_rows is None else n_logit_rows
    if logits_out is None and rows > 0:
        logits_out = torch.empty((B, rows, model.shape.vocab), dtype=torch.float32, device=model.device)
    ws = model.workspace(B, n_new, kv.max_len)
    psd.psd_model_forward(model.handle, tokens, n_new, kv.handle, logits_out, rows, ws, stream)
    return logits_out


def forward_tree(model: Model, kv: KVCache, tokens, parents, logits_out=None, stream=None):
    """tokens int32 [B, n_nodes] on the device, parents a host sequence (parents[0] = -1, parents[i] < i) ->
    fp32 logits [B, n_nodes, V]."""
    B, n = tokens.shape
    if logits_out is None:
        logits_out = torch.empty((B, n, model.shape.vocab), dtype=torch.float32, device=model.device)
    ws = model.workspace(B, n, kv.max_len)
    psd.psd_model_forward_tree(model.handle, tokens, n, parents, kv.handle, logits_out, ws, stream)
    return logits_out


def tree_accept(p_logits, q_logits, tokens, parents, uniforms, temperature=1.0, stream=None):
    """p, q [rows, n_nodes, V] (same dtype; q may be None when temperature is 0), tokens int32 [rows, n_nodes],
    uniforms fp32 [rows, n_nodes + 1] -> (path_len [rows], path [rows, n_nodes], token [rows], flags [rows]) int32."""
    rows, n, V = p_logits.shape
    dev = p_logits.device
    out_len = torch.empty(rows, dtype=torch.int32, device=dev)
    out_path = torch.full((rows, n), -1, dtype=torch.int32, device=dev)
    out_tok = torch.empty(rows, dtype=torch.int32, device=dev)
    out_flags = torch.empty(rows, dtype=torch.int32, device=dev)
    psd.psd_tree_accept(p_logits, q_logits, tokens, parents, n, uniforms, temperature, out_len, out_path, out_tok, rows, V,
                        psd.dtype_code(p_logits.dtype), p_logits.stride(0), q_logits.stride(0) if q_logits is not None else 0,
                        out_flags, stream)
    return out_len, out_path, out_tok, out_flags


class Acceptor:
    """Output tensors and workspace of psd_spec_accept, reused across calls."""

    def __init__(self, device="cuda"):
        self.device = torch.device(device)
        self._ws = None
        self._out = None

    def __call__(self, p_logits, q_logits, draft_tokens, uniforms, temperature=1.0, stream=None):
        """p [rows, n_p_rows, V], q [rows, gamma, V] (same dtype), tokens int32 [rows, gamma],
        uniforms fp32 [rows, gamma+1] -> (accept_len, token, flags) int32 [rows] tensors."""
        rows, n_p_rows, V = p_logits.shape
        gamma = uniforms.shape[1] - 1
        need = psd.psd_spec_accept_workspace_bytes(rows, gamma, n_p_rows, V)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(max(need, 256), dtype=torch.uint8, device=self.device)
        if self._out is None or self._out.shape[1] < rows:
            self._out = torch.empty((3, max(rows, 1)), dtype=torch.int32, device=self.device)
        n, tok, fl = self._out[0, :rows], self._out[1, :rows], self._out[2, :rows]
        q_stride = q_logits.stride(0) if gamma > 0 and q_logits is not None else 0
        psd.psd_spec_accept(p_logits, q_logits if gamma > 0 else None, draft_tokens if gamma > 0 else None, gamma,
                            uniforms, temperature, n, tok, rows, n_p_rows, V, psd.dtype_code(p_logits.dtype),
                            p_logits.stride(0), q_stride, fl, self._ws, stream)
        return n, tok, fl
