"""Seeded synthetic inputs shared by the tests, the bench and the smoke check.

This module holds none of the method's arithmetic and imports neither the
HIP binding nor the CPU oracle: it only names the model shapes of the five
workloads and draws random weights, KV contents, logits, tokens and uniform
tapes.  Both sides receive the very same arrays (the oracle as numpy views of
the torch tensors).

The paper's measurements use trained LLaMA-2 / LLaMA-3 / Qwen2 / Vicuna
checkpoints and SpecBench prompts (Sec. 4.1); none of those are available, so
the inputs below stand in for them by shape and value distribution only.
"""
from dataclasses import dataclass, asdict

import numpy as np
import torch


@dataclass(frozen=True)
class Shape:
    """Decoder-only transformer shape (RMSNorm, RoPE, GQA, SwiGLU, untied lm_head)."""
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    d_head: int
    d_ffn: int
    vocab: int
    rope_theta: float = 10000.0
    rms_eps: float = 1e-5

    def asdict(self):
        return asdict(self)


# workload 1: tiny three-level chain, fp32, shared vocabulary 512, d_head 32 everywhere
TINY_TARGET = Shape(4, 256, 8, 8, 32, 1024, 512)
TINY_INTERMEDIATE = Shape(2, 128, 4, 4, 32, 512, 512)
TINY_DRAFT = Shape(1, 64, 2, 2, 32, 256, 512)
# workload 3: LLaMA2-7B shape
LLAMA2_7B = Shape(32, 4096, 32, 32, 128, 11008, 32000, 1.0e4)
# workload 4: LLaMA3-8B-shaped target, a half-width 16-layer intermediate, a one-layer draft
LLAMA3_8B = Shape(32, 4096, 32, 8, 128, 14336, 128256, 5.0e5)
CHAIN_INTERMEDIATE = Shape(16, 2048, 32, 8, 64, 8192, 128256, 5.0e5)
CHAIN_DRAFT = Shape(1, 4096, 32, 8, 128, 14336, 128256, 5.0e5)
# workload 5: Qwen2-7B shape (its QKV biases are omitted: no biases anywhere)
QWEN2_7B = Shape(28, 3584, 28, 4, 128, 18944, 152064, 1.0e6)


def weight_names(shape: Shape):
    """Names in the order the C boundary expects its weight pointers."""
    names = ["embed"]
    for l in range(shape.n_layers):
        names += [f"l{l}.{n}" for n in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm",
                                         "w_gate", "w_up", "w_down")]
    names += ["final_norm", "lm_head"]
    return names


def weight_shape(shape: Shape, name: str):
    s = shape
    base = name.split(".")[-1]
    return {
        "embed": (s.vocab, s.d_model), "lm_head": (s.vocab, s.d_model),
        "attn_norm": (s.d_model,), "ffn_norm": (s.d_model,), "final_norm": (s.d_model,),
        "wq": (s.n_q_heads * s.d_head, s.d_model), "wk": (s.n_kv_heads * s.d_head, s.d_model),
        "wv": (s.n_kv_heads * s.d_head, s.d_model), "wo": (s.d_model, s.n_q_heads * s.d_head),
        "w_gate": (s.d_ffn, s.d_model), "w_up": (s.d_ffn, s.d_model), "w_down": (s.d_model, s.d_ffn),
    }[base]


def make_weights(shape: Shape, seed: int, dtype=torch.float32, device="cpu", std=0.02,
                 share=None):
    """Random-init weights: every matrix N(0, std^2) rounded to `dtype`, norm gains 1.
    Projections are [out_features, in_features].  `share` maps a name to an existing tensor
    (a draft reusing the target's embed / lm_head).  A CPU generator makes the values
    independent of the machine; pass a cuda device only where no oracle needs them."""
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    out = {}
    for name in weight_names(shape):
        if share and name in share:
            out[name] = share[name]
            continue
        shp = weight_shape(shape, name)
        if name.endswith("norm"):
            out[name] = torch.ones(shp, dtype=dtype, device=device)
        else:
            w = torch.empty(shp, dtype=torch.float32, device=device)
            w.normal_(0.0, std, generator=gen)
            out[name] = w.to(dtype)
    return out


def as_numpy(t: torch.Tensor):
    """Zero-copy numpy view for the oracle: fp32 as is, bf16 as uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def make_kv_fill(shape: Shape, batch: int, n_ctx: int, seed: int, dtype=torch.bfloat16,
                 device="cpu"):
    """KV contents for n_ctx past positions, N(0,1) rounded to `dtype`:
    two lists (K, V) of per-layer tensors [batch, n_kv_heads, n_ctx, d_head]."""
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    ks, vs = [], []
    for _ in range(shape.n_layers):
        for dst in (ks, vs):
            t = torch.empty((batch, shape.n_kv_heads, n_ctx, shape.d_head), dtype=torch.float32,
                            device=device)
            t.normal_(0.0, 1.0, generator=gen)
            dst.append(t.to(dtype))
    return ks, vs


def make_tokens(vocab: int, shape, seed: int):
    rng = np.random.Generator(np.random.Philox(key=seed))
    return rng.integers(0, vocab, size=shape, dtype=np.int64).astype(np.int32)


def make_accept_inputs(rows, gamma, vocab, seed, n_p_rows=None, p_std=2.0, noise_std=0.5,
                       dtype=torch.bfloat16, device="cpu"):
    """Workload 2: verifier logits N(0, p_std^2) rounded to `dtype`; drafter logits = the
    unrounded verifier logits + N(0, noise_std^2), rounded; draft tokens distributed as
    softmax(drafter logits) (drawn with the Gumbel-max trick, so no part of the acceptance
    rule is involved); uniforms fp32 in [0,1).
    Returns dict(p, q, tokens, uniforms) of torch tensors on `device`."""
    n_p_rows = gamma if n_p_rows is None else n_p_rows
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    p32 = torch.empty((rows, n_p_rows, vocab), dtype=torch.float32, device=device)
    p32.normal_(0.0, p_std, generator=gen)
    noise = torch.empty((rows, gamma, vocab), dtype=torch.float32, device=device)
    noise.normal_(0.0, noise_std, generator=gen)
    q = (p32[:, :gamma] + noise).to(dtype)
    del noise
    g = torch.empty((rows, gamma, vocab), dtype=torch.float32, device=device)
    g.exponential_(1.0, generator=gen)
    tokens = torch.argmax(q.float() - torch.log(g), dim=-1).to(torch.int32)
    del g
    u = torch.rand((rows, gamma + 1), dtype=torch.float32, device=device, generator=gen)
    u = torch.clamp(u, max=float(np.nextafter(np.float32(1.0), np.float32(0.0))))
    return {"p": p32.to(dtype), "q": q, "tokens": tokens, "uniforms": u}


def make_draft_from_target(p_logits: torch.Tensor, noise_std: float, seed: int):
    """Synthetic drafter for a verify step whose target logits p_logits [rows, gamma, V] (fp32)
    are already known: drafter logits = p + N(0, noise_std^2) and draft tokens distributed as
    softmax(drafter logits) (Gumbel-max).  Returns (q fp32 [rows, gamma, V], tokens int32)."""
    gen = torch.Generator(device=p_logits.device)
    gen.manual_seed(seed)
    noise = torch.empty_like(p_logits, dtype=torch.float32)
    noise.normal_(0.0, noise_std, generator=gen)
    q = p_logits.float() + noise
    g = torch.empty_like(q)
    g.exponential_(1.0, generator=gen)
    tokens = torch.argmax(q - torch.log(g), dim=-1).to(torch.int32)
    return q, tokens


def make_uniforms(shape, seed: int, device="cpu"):
    """fp32 uniforms in [0, 1)."""
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    u = torch.rand(shape, dtype=torch.float32, device=device, generator=gen)
    return torch.clamp(u, max=float(np.nextafter(np.float32(1.0), np.float32(0.0))))


def make_tape(seed: int, level: int, calls: int, width: int):
    """Uniform tape for one level of a chain: float32 [calls, width] in [0,1), counter-based
    (Philox keyed by seed and level) so both sides index the same numbers by (call, slot)."""
    rng = np.random.Generator(np.random.Philox(key=[seed, level]))
    return rng.random((calls, width), dtype=np.float32)


QUANT_WEIGHTS = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def quantize_w4(weights, group=128):
    """4-bit weight-only quantisation of every projection matrix by plain round-to-nearest per group of `group`
    input channels (asymmetric: scale = (max - min) / 15 rounded to bf16, zero = round(-min / scale) in 0..15),
    a stand-in for the calibrated quantiser the paper's intermediate model uses.  Returns (codes_and_rest, quant):
    the weight dict with each projection replaced by its codes, uint8 [n, K/2] (low nibble = even k), and
    quant[name] = (scale bf16 [n, K/group], zero uint8 [n, K/group])."""
    out, quant = dict(weights), {}
    for name, w in weights.items():
        if name.split(".")[-1] not in QUANT_WEIGHTS:
            continue
        n, K = w.shape
        g = w.float().reshape(n, K // group, group)
        lo, hi = g.amin(-1), g.amax(-1)
        scale = ((hi - lo) / 15.0).clamp_min(1e-8).to(torch.bfloat16)
        sf = scale.float()
        zero = torch.round(-lo / sf).clamp(0, 15)
        q = torch.round(g / sf[..., None] + zero[..., None]).clamp(0, 15).to(torch.uint8).reshape(n, K)
        out[name] = (q[:, 0::2] | (q[:, 1::2] << 4)).contiguous()
        quant[name] = (scale.contiguous(), zero.to(torch.uint8).contiguous())
    return out, quant
