"""CPU oracle (test infrastructure only): decoder-only transformer forward pass.

The paper treats a model as a black box, p_i(x | x_{<=t}) = M_i(x_{<=t})
(Problem Formulation, Sec. 3.1), whose single forward pass costs T_i (Eq. 2).
The architecture is the one its LLaMA-2 / LLaMA-3 / Qwen2 targets share:
pre-norm decoder, RMSNorm, rotary position embedding (rotate-half pairing),
grouped-query causal attention with a KV cache, SwiGLU MLP, untied lm_head.

Everything is numpy in fp64: weights and caches are widened to fp64 before
use and no intermediate is rounded to a narrower type.  numpy's matmul is the
only library primitive.  No blocking, fusion or reordering.

Weight dictionary (names are the boundary's weight order):
  embed [V, d]; per layer l: attn_norm [d], wq [h_q*d_h, d], wk [h_kv*d_h, d],
  wv [h_kv*d_h, d], wo [d, h_q*d_h], ffn_norm [d], w_gate [f, d], w_up [f, d],
  w_down [d, f]; final_norm [d]; lm_head [V, d].
Every projection is stored [out_features, in_features] and applied as x @ W.T.
"""
from dataclasses import dataclass

import numpy as np


@dataclass
class ModelConfig:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    d_head: int
    d_ffn: int
    vocab: int
    rope_theta: float = 10000.0
    rms_eps: float = 1e-5


def widen(a):
    """Any stored weight/cache array -> fp64.  uint16 arrays hold bfloat16 bit patterns; a CPU
    torch tensor (fp32 or bf16) is converted by torch, which does it on all cores."""
    if hasattr(a, "detach"):
        import torch
        return a.detach().to(torch.float64).numpy()
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def rmsnorm(x, gain, eps):
    """x * rsqrt(mean(x^2) + eps) * gain over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(x, positions, theta):
    """Rotary embedding, rotate-half pairing: element i pairs with i + d_h/2 and the
    pair is rotated by angle pos * theta^(-2i/d_h).  x [R, heads, d_h], positions [R]."""
    d_h = x.shape[-1]
    half = d_h // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / d_h)
    ang = positions.astype(np.float64)[:, None] * inv_freq[None, :]      # [R, half]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(z):
    return z / (1.0 + np.exp(-z))


class KVCache:
    """Per-model KV cache of the oracle: k[l], v[l] are [B, h_kv, max_len, d_h] arrays in
    `dtype` (fp64 by default; fp32 keeps the big configurations in memory and still holds
    bf16 inputs exactly), lens[b] the number of valid positions of sequence b."""

    def __init__(self, cfg: ModelConfig, batch: int, max_len: int, dtype=np.float64):
        shape = (batch, cfg.n_kv_heads, max_len, cfg.d_head)
        self.k = [np.zeros(shape, dtype) for _ in range(cfg.n_layers)]
        self.v = [np.zeros(shape, dtype) for _ in range(cfg.n_layers)]
        self.lens = np.zeros(batch, np.int64)
        self.max_len = max_len

    def truncate(self, new_lens):
        """Rollback to the accepted length (the 'partial rollback' of Sec. 3.3): only the
        length changes, stale rows are overwritten by the next append."""
        new_lens = np.broadcast_to(np.asarray(new_lens, np.int64), self.lens.shape)
        if np.any(new_lens > self.lens) or np.any(new_lens < 0):
            raise ValueError("truncate can only shorten")
        self.lens = new_lens.copy()


def attention(q, k, v, n_past):
    """Causal attention for one sequence.  q [R, h_q, d_h] are the R new rows at positions
    n_past..n_past+R-1; k, v [h_kv, n_past+R, d_h] hold every position up to the last new
    one.  Query head h reads KV head h // (h_q / h_kv).  Returns [R, h_q, d_h]."""
    R, h_q, d_h = q.shape
    h_kv = k.shape[0]
    group = h_q // h_kv
    out = np.empty_like(q)
    scale = 1.0 / np.sqrt(float(d_h))
    for h in range(h_q):
        kh, vh = k[h // group], v[h // group]
        for r in range(R):
            n_keys = n_past + r + 1
            s = (kh[:n_keys] @ q[r, h]) * scale
            w = np.exp(s - np.max(s))
            w = w / np.sum(w)
            out[r, h] = w @ vh[:n_keys]
    return out


def forward(cfg: ModelConfig, weights: dict, tokens, kv: KVCache):
    """One forward pass over tokens [B, R] appended at positions lens[b]..lens[b]+R-1.
    Appends their K/V, advances lens by R and returns fp64 logits [B, R, V]; row r is the
    distribution of the token that follows input token r."""
    tokens = np.asarray(tokens)
    B, R = tokens.shape
    if np.any(kv.lens + R > kv.max_len):
        raise ValueError("KV cache capacity exceeded")
    h_q, h_kv, d_h = cfg.n_q_heads, cfg.n_kv_heads, cfg.d_head
    x = widen(weights["embed"][tokens.reshape(-1).astype(np.int64)]).reshape(B, R, cfg.d_model)
    for l in range(cfg.n_layers):
        w = lambda name: widen(weights[f"l{l}.{name}"])
        n = rmsnorm(x, w("attn_norm"), cfg.rms_eps)
        q = (n @ w("wq").T).reshape(B, R, h_q, d_h)
        k = (n @ w("wk").T).reshape(B, R, h_kv, d_h)
        v = (n @ w("wv").T).reshape(B, R, h_kv, d_h)
        a = np.empty((B, R, h_q, d_h))
        for b in range(B):
            s0 = int(kv.lens[b])
            pos = np.arange(s0, s0 + R)
            qb = rope(q[b], pos, cfg.rope_theta)
            kb = rope(k[b], pos, cfg.rope_theta)
            kv.k[l][b, :, s0:s0 + R] = kb.transpose(1, 0, 2)
            kv.v[l][b, :, s0:s0 + R] = v[b].transpose(1, 0, 2)
            a[b] = attention(qb, widen(kv.k[l][b, :, :s0 + R]), widen(kv.v[l][b, :, :s0 + R]), s0)
        x = x + a.reshape(B, R, h_q * d_h) @ w("wo").T
        n = rmsnorm(x, w("ffn_norm"), cfg.rms_eps)
        x = x + (silu(n @ w("w_gate").T) * (n @ w("w_up").T)) @ w("w_down").T
    kv.lens = kv.lens + R
    n = rmsnorm(x, widen(weights["final_norm"]), cfg.rms_eps)
    return n @ widen(weights["lm_head"]).T


# ---------------------------------------------------------------------------------------------------------------
# Token trees (Related Work, "Verification Mechanisms"; Sec. 4.6): one forward pass over every node of a drafted
# tree.  Node 0 is the root (the last committed token); parents[i] < i is node i's parent.  A node sees the cache
# and its own ancestors (itself included), and sits at position lens[b] + depth(node): exactly what an ordinary
# forward pass over the root-to-node path would give it.

def tree_depths(parents):
    parents = list(parents)
    if not parents or parents[0] != -1:
        raise ValueError("node 0 is the root: parents[0] = -1")
    depth = [0] * len(parents)
    for i in range(1, len(parents)):
        if not 0 <= parents[i] < i:
            raise ValueError("parents must precede their children")
        depth[i] = depth[parents[i]] + 1
    return depth


def tree_ancestors(parents):
    """visible[i][j] = node j is node i or one of its ancestors."""
    n = len(parents)
    tree_depths(parents)
    visible = np.zeros((n, n), bool)
    for i in range(n):
        j = i
        while j >= 0:
            visible[i, j] = True
            j = parents[j]
    return visible


def attention_tree(q, k, v, n_past, visible):
    """Attention of the R tree nodes of one sequence: node r reads the n_past cached positions and the new rows j
    with visible[r][j].  q [R, h_q, d_h]; k, v [h_kv, n_past + R, d_h] with new row j at index n_past + j."""
    R, h_q, d_h = q.shape
    group = h_q // k.shape[0]
    out = np.empty_like(q)
    scale = 1.0 / np.sqrt(float(d_h))
    for h in range(h_q):
        kh, vh = k[h // group], v[h // group]
        for r in range(R):
            keys = np.concatenate([np.arange(n_past), n_past + np.nonzero(visible[r])[0]])
            s = (kh[keys] @ q[r, h]) * scale
            w = np.exp(s - np.max(s))
            w = w / np.sum(w)
            out[r, h] = w @ vh[keys]
    return out


def forward_tree(cfg: ModelConfig, weights: dict, tokens, parents, kv: KVCache):
    """One forward pass over the nodes tokens [B, R] of a tree with the same shape for every sequence.  Node r's
    K/V go to cache slot lens[b] + r (rotated for position lens[b] + depth(r)); lens advance by R; returns fp64
    logits [B, R, V].  KVCache.compact_tree then keeps an accepted path."""
    tokens = np.asarray(tokens)
    B, R = tokens.shape
    if len(parents) != R:
        raise ValueError("one parent per node")
    if np.any(kv.lens + R > kv.max_len):
        raise ValueError("KV cache capacity exceeded")
    depth = np.asarray(tree_depths(parents))
    visible = tree_ancestors(parents)
    h_q, h_kv, d_h = cfg.n_q_heads, cfg.n_kv_heads, cfg.d_head
    x = widen(weights["embed"][tokens.reshape(-1).astype(np.int64)]).reshape(B, R, cfg.d_model)
    for l in range(cfg.n_layers):
        w = lambda name: widen(weights[f"l{l}.{name}"])
        n = rmsnorm(x, w("attn_norm"), cfg.rms_eps)
        q = (n @ w("wq").T).reshape(B, R, h_q, d_h)
        k = (n @ w("wk").T).reshape(B, R, h_kv, d_h)
        v = (n @ w("wv").T).reshape(B, R, h_kv, d_h)
        a = np.empty((B, R, h_q, d_h))
        for b in range(B):
            s0 = int(kv.lens[b])
            pos = s0 + depth
            qb = rope(q[b], pos, cfg.rope_theta)
            kb = rope(k[b], pos, cfg.rope_theta)
            kv.k[l][b, :, s0:s0 + R] = kb.transpose(1, 0, 2)
            kv.v[l][b, :, s0:s0 + R] = v[b].transpose(1, 0, 2)
            a[b] = attention_tree(qb, widen(kv.k[l][b, :, :s0 + R]), widen(kv.v[l][b, :, :s0 + R]), s0, visible)
        x = x + a.reshape(B, R, h_q * d_h) @ w("wo").T
        n = rmsnorm(x, w("ffn_norm"), cfg.rms_eps)
        x = x + (silu(n @ w("w_gate").T) * (n @ w("w_up").T)) @ w("w_down").T
    kv.lens = kv.lens + R
    n = rmsnorm(x, widen(weights["final_norm"]), cfg.rms_eps)
    return n @ widen(weights["lm_head"]).T


def compact_tree(kv: KVCache, base_lens, paths):
    """After a tree forward that started at base_lens: keep the root and the accepted nodes paths[b] (root first,
    root excluded) of every sequence as consecutive positions, drop the rest.  lens[b] = base + 1 + len(path)."""
    base_lens = np.asarray(base_lens, np.int64)
    for b, path in enumerate(paths):
        s0 = int(base_lens[b])
        for j, node in enumerate(path):
            for l in range(len(kv.k)):
                kv.k[l][b, :, s0 + 1 + j] = kv.k[l][b, :, s0 + node]
                kv.v[l][b, :, s0 + 1 + j] = kv.v[l][b, :, s0 + node]
    kv.lens = base_lens + 1 + np.asarray([len(p) for p in paths], np.int64)
