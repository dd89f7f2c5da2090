"""psd_spec_accept_static, the entry point that allocates nothing (its scratch buffer is part of the library),
against psd_spec_accept on the same inputs: identical accepted lengths, tokens and flags, on two calls in a row,
the second smaller than the first (the buffer keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2510_26527_amd as psd
from paper_2510_26527_amd import runtime, synth


def test_sizes_beyond_the_built_in_buffer_are_refused_before_any_launch():
    L = psd.lib()
    rows, gamma, V = 4096, 8, 32000
    assert psd.psd_spec_accept_workspace_bytes(rows, gamma, gamma + 1, V) > psd.PSD_STATIC_SCRATCH_BYTES
    st = L.psd_spec_accept_static(0x1000, 0x2000, 0x3000, gamma, 0x4000, 1.0, 0x5000, 0x6000, rows, gamma + 1, V,
                                  psd.PSD_BF16, (gamma + 1) * V, gamma * V, 0, 0)
    assert st == psd.PSD_ERR_WORKSPACE
    assert psd.psd_spec_accept_workspace_bytes(64, 8, 9, 32000) <= psd.PSD_STATIC_SCRATCH_BYTES
    assert psd.psd_spec_accept_workspace_bytes(16, 16, 17, 152064) <= psd.PSD_STATIC_SCRATCH_BYTES
    # the other argument checks come first, as in psd_spec_accept
    assert L.psd_spec_accept_static(0, 0x2000, 0x3000, 2, 0x4000, 1.0, 0x5000, 0x6000, 1, 3, 16, psd.PSD_F32, 48, 32,
                                    0, 0) == psd.PSD_ERR_NULL
    assert L.psd_spec_accept_static(0x1000, 0x2000, 0x3000, 2, 0x4000, -1.0, 0x5000, 0x6000, 1, 3, 16, psd.PSD_F32, 48,
                                    32, 0, 0) == psd.PSD_ERR_TEMPERATURE


def _both(inp, temperature, dev):
    p, q, x, u = (inp[k].to(dev) for k in ("p", "q", "tokens", "uniforms"))
    rows, n_p_rows, V = p.shape
    gamma = q.shape[1]
    ref = runtime.Acceptor(dev)(p, q, x, u, temperature)
    ref = [t.clone() for t in ref]
    out = torch.full((3, rows), -7, dtype=torch.int32, device=dev)
    psd.psd_spec_accept_static(p, q, x, gamma, u, temperature, out[0], out[1], rows, n_p_rows, V,
                               psd.dtype_code(p.dtype), p.stride(0), q.stride(0), out[2])
    torch.cuda.synchronize()
    for name, a, b in zip(("accept_len", "token", "flags"), ref, out):
        assert torch.equal(a, b), f"{name}: workspace call {a.tolist()[:8]} static call {b.tolist()[:8]}"
    return ref[0].cpu().numpy()


@pytest.mark.gpu
def test_static_scratch_call_matches_the_workspace_call_twice_in_a_row():
    dev = torch.device("cuda")
    big = synth.make_accept_inputs(64, 8, 32000, seed=41, n_p_rows=9, dtype=torch.bfloat16)
    small = synth.make_accept_inputs(5, 3, 4100, seed=42, n_p_rows=3, dtype=torch.float32)
    n_big = _both(big, 1.0, dev)
    n_small = _both(small, 0.8, dev)             # smaller input on the buffer the first call left behind
    assert 0 < n_big.mean() < 8 and n_small.max() <= 3
    _both(big, 1.0, dev)                         # and back
    greedy = synth.make_accept_inputs(7, 4, 2048, seed=43, n_p_rows=5, dtype=torch.bfloat16)
    _both(greedy, 0.0, dev)                      # temperature 0 takes the same buffer
