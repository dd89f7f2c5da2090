"""CPU-side checks of the C boundary: the library loads without a GPU, exports every symbol
include/psd.h declares, and rejects bad arguments on the host before any launch."""
import ctypes
import os
import re

import pytest

import paper_2510_26527_amd as psd


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(psd.LIB_PATH):
        from paper_2510_26527_amd import build
        build.build()
    return psd.lib()


def _declared():
    text = open(psd.HEADER_PATH).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(psd_[a-z_0-9]+)\s*\(", text)))


def test_exports_every_declared_symbol(lib):
    names = _declared()
    assert {"psd_model_forward", "psd_spec_accept", "psd_kv_truncate"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(psd._SIGNATURES), "binding and header disagree"


def _desc(**kw):
    base = dict(n_layers=1, d_model=128, n_q_heads=2, n_kv_heads=2, d_head=64, d_ffn=256, vocab=512,
                rope_theta=1e4, rms_eps=1e-5, dtype=psd.PSD_BF16)
    base.update(kw)
    return psd.psd_model_desc(**base)


def _create(desc, n_ptrs=None, ptr=0x1000):
    n = 3 + 9 * desc.n_layers if n_ptrs is None else n_ptrs
    return psd.psd_model_create(desc, [ptr] * n)


def test_model_create_validation(lib):
    m = _create(_desc())
    psd.psd_model_destroy(m)
    for bad, code in ((dict(dtype=7), psd.PSD_ERR_DTYPE), (dict(d_head=48), psd.PSD_ERR_SHAPE),
                      (dict(n_q_heads=3), psd.PSD_ERR_SHAPE), (dict(d_model=96), psd.PSD_ERR_SHAPE),
                      (dict(vocab=0), psd.PSD_ERR_SHAPE), (dict(rope_theta=0.0), psd.PSD_ERR_SHAPE)):
        with pytest.raises(psd.PsdError) as e:
            _create(_desc(**bad))
        assert e.value.status == code, bad
    with pytest.raises(psd.PsdError) as e:
        _create(_desc(), n_ptrs=5)
    assert e.value.status == psd.PSD_ERR_SHAPE
    with pytest.raises(psd.PsdError) as e:
        _create(_desc(), ptr=0)
    assert e.value.status == psd.PSD_ERR_NULL
    with pytest.raises(psd.PsdError) as e:
        _create(_desc(), ptr=0x1004)          # not 16-byte aligned
    assert e.value.status == psd.PSD_ERR_SHAPE
    assert psd.status_string(psd.PSD_ERR_CAPACITY) == "KV cache capacity exceeded"


def test_w4_model_create_validation(lib):
    d = _desc()
    n, nq = 3 + 9 * d.n_layers, 7 * d.n_layers
    m = psd.psd_model_create_w4(d, [0x1000] * n, [0x2000] * nq, [0x3000] * nq)
    assert psd.psd_model_packed_bytes(m) > 0
    # steps of any row count have a workspace size: up to 16 rows on the packed 4-bit copy, the tiled kernel above
    assert 0 < psd.psd_model_workspace_bytes(m, 1, 7, 128) < psd.psd_model_workspace_bytes(m, 2, 20, 128)
    # a 4-bit model must be packed before its first forward; nothing is launched
    kv = ctypes.c_void_p()
    assert lib.psd_kv_create(m, 1, 128, 0x1000, 0x2000, 0x3000, 0, ctypes.byref(kv)) == psd.PSD_OK
    assert lib.psd_model_forward(m, 0x1000, 4, kv, 0x2000, 4, 0x4000, 1 << 30, 0) == psd.PSD_ERR_UNIMPLEMENTED
    psd.psd_kv_destroy(kv)
    psd.psd_model_destroy(m)
    for args, code in ((([0x1000] * n, [0x2000] * (nq - 1), [0x3000] * (nq - 1)), psd.PSD_ERR_SHAPE),
                       (([0x1000] * n, [0] * nq, [0x3000] * nq), psd.PSD_ERR_NULL),
                       (([0x1000] * n, [0x2001] * nq, [0x3000] * nq), psd.PSD_ERR_SHAPE)):
        with pytest.raises(psd.PsdError) as e:
            psd.psd_model_create_w4(d, *args)
        assert e.value.status == code
    with pytest.raises(psd.PsdError) as e:
        psd.psd_model_create_w4(_desc(dtype=psd.PSD_F32), [0x1000] * n, [0x2000] * nq, [0x3000] * nq)
    assert e.value.status == psd.PSD_ERR_DTYPE


def test_kv_and_forward_validation(lib):
    m = _create(_desc())
    assert psd.psd_kv_bytes(m, 2, 128) == 1 * 2 * 2 * 128 * 64 * 2
    assert psd.psd_kv_bytes(m, 2, 100) == 0                      # max_len must be a multiple of 64
    out = ctypes.c_void_p()
    L = lib
    assert L.psd_kv_create(m, 1, 100, 0x1000, 0x2000, 0x3000, 0, ctypes.byref(out)) == psd.PSD_ERR_SHAPE
    assert L.psd_kv_create(m, 1, 128, 0, 0x2000, 0x3000, 0, ctypes.byref(out)) == psd.PSD_ERR_NULL
    assert L.psd_kv_create(m, 1, 128, 0x1000, 0x2000, 0x3000, 129, ctypes.byref(out)) == psd.PSD_ERR_CAPACITY
    assert L.psd_kv_create(m, 1, 128, 0x1000, 0x2000, 0x3000, 120, ctypes.byref(out)) == psd.PSD_OK
    kv = out
    assert psd.psd_kv_len_upper_bound(kv) == 120
    need = psd.psd_model_workspace_bytes(m, 1, 9, 128)
    assert need > 0 and psd.psd_model_workspace_bytes(m, 0, 9, 128) == 0
    f = L.psd_model_forward
    assert f(m, 0, 4, kv, 0x5000, 4, 0x10000, need, 0) == psd.PSD_ERR_NULL            # no tokens
    assert f(m, 0x4000, 9, kv, 0x5000, 9, 0x10000, need, 0) == psd.PSD_ERR_CAPACITY   # 120 + 9 > 128
    assert f(m, 0x4000, 4, kv, 0x5000, 5, 0x10000, need, 0) == psd.PSD_ERR_SHAPE      # more logit rows than rows
    assert f(m, 0x4000, 4, kv, 0, 4, 0x10000, need, 0) == psd.PSD_ERR_NULL            # logits wanted, no buffer
    assert f(m, 0x4000, 4, kv, 0x5000, 4, 0x10000, 16, 0) == psd.PSD_ERR_WORKSPACE    # too small
    assert f(m, 0x4000, 4, kv, 0x5000, 4, 0x10010, need, 0) == psd.PSD_ERR_WORKSPACE  # misaligned
    assert f(m, 0x4000, 0, kv, 0x5000, 0, 0x10000, need, 0) == psd.PSD_ERR_SHAPE
    assert L.psd_kv_truncate(kv, 0, 0x1000, 1, -1, 0) == psd.PSD_ERR_NULL
    assert L.psd_kv_truncate_to(kv, -1, 0) == psd.PSD_ERR_SHAPE
    psd.psd_kv_destroy(kv)
    psd.psd_model_destroy(m)


def test_spec_accept_validation(lib):
    a = lib.psd_spec_accept
    ws = psd.psd_spec_accept_workspace_bytes(4, 8, 9, 32000)
    assert ws > 0 and psd.psd_spec_accept_workspace_bytes(4, 8, 7, 32000) == 0
    P, Q, X, U, N, T, W = 0x10000, 0x20000, 0x30000, 0x40000, 0x50000, 0x60000, 0x70000

    def call(gamma=8, temp=1.0, rows=4, n_p=9, V=32000, dtype=psd.PSD_BF16, ps=None, qs=None, p=P, q=Q, x=X, u=U,
             n=N, t=T, w=W, wb=ws):
        ps = n_p * V if ps is None else ps
        qs = gamma * V if qs is None else qs
        return a(p, q, x, gamma, u, temp, n, t, rows, n_p, V, dtype, ps, qs, 0, w, wb, 0)

    assert call(temp=-1.0) == psd.PSD_ERR_TEMPERATURE
    assert call(temp=0.0, x=0) == psd.PSD_ERR_NULL          # greedy mode still needs the draft tokens
    assert call(temp=float("nan")) == psd.PSD_ERR_TEMPERATURE
    assert call(temp=float("inf")) == psd.PSD_ERR_TEMPERATURE
    assert call(dtype=3) == psd.PSD_ERR_DTYPE
    assert call(gamma=65, n_p=65) == psd.PSD_ERR_SHAPE
    assert call(n_p=7) == psd.PSD_ERR_SHAPE
    assert call(V=0) == psd.PSD_ERR_SHAPE
    assert call(ps=100) == psd.PSD_ERR_SHAPE
    assert call(p=0) == psd.PSD_ERR_NULL
    assert call(q=0) == psd.PSD_ERR_NULL
    assert call(n=0) == psd.PSD_ERR_NULL
    assert call(w=0) == psd.PSD_ERR_WORKSPACE
    assert call(wb=8) == psd.PSD_ERR_WORKSPACE
    assert call(rows=0) == psd.PSD_OK                     # nothing to do, nothing launched


def test_tree_calls_validation(lib):
    """Malformed trees and arguments are refused on the host, before anything is launched."""
    def par(vals):
        return ctypes.cast((ctypes.c_int32 * len(vals))(*vals), ctypes.c_void_p)
    acc = lib.psd_tree_accept
    P, Q, X, U, LN, PA, TK = 0x10000, 0x20000, 0x30000, 0x40000, 0x50000, 0x60000, 0x70000

    def call(parents=(-1, 0, 0, 1), n=4, temp=1.0, rows=2, V=1000, dtype=psd.PSD_F32, p=P, q=Q, x=X, u=U, ps=None, qs=None,
             ln=LN, pa=PA, tk=TK):
        ps = n * V if ps is None else ps
        qs = n * V if qs is None else qs
        return acc(p, q, x, par(list(parents)), n, u, temp, ln, pa, tk, rows, V, dtype, ps, qs, 0, 0)

    assert call(parents=(0, 0, 0, 1)) == psd.PSD_ERR_SHAPE           # no root
    assert call(parents=(-1, 0, 3, 1)) == psd.PSD_ERR_SHAPE          # a parent after its child
    assert call(parents=(-1, 0, -1, 1)) == psd.PSD_ERR_SHAPE         # two roots
    assert call(parents=[-1] + [0] * 64, n=65) == psd.PSD_ERR_SHAPE  # more than 64 nodes
    assert call(n=0, parents=(-1,)) == psd.PSD_ERR_SHAPE
    assert call(temp=-0.5) == psd.PSD_ERR_TEMPERATURE
    assert call(dtype=9) == psd.PSD_ERR_DTYPE
    assert call(V=0) == psd.PSD_ERR_SHAPE
    assert call(ps=100) == psd.PSD_ERR_SHAPE
    assert call(q=0) == psd.PSD_ERR_NULL
    assert call(u=0) == psd.PSD_ERR_NULL
    assert call(pa=0) == psd.PSD_ERR_NULL
    assert call(rows=0) == psd.PSD_OK                                # nothing to do, nothing launched
    m = _create(_desc())
    kv = ctypes.c_void_p()
    assert lib.psd_kv_create(m, 1, 128, 0x1000, 0x2000, 0x3000, 100, ctypes.byref(kv)) == psd.PSD_OK
    need = psd.psd_model_workspace_bytes(m, 1, 8, 128)
    f = lib.psd_model_forward_tree
    assert f(m, 0x4000, 3, par([-1, 0, 2]), kv, 0x5000, 0x10000, need, 0) == psd.PSD_ERR_SHAPE       # parent == child
    assert f(m, 0x4000, 3, par([-1, 0, 0]), kv, 0, 0x10000, need, 0) == psd.PSD_ERR_NULL            # every node gets a row
    assert f(m, 0x4000, 33, par([-1] + [0] * 32), kv, 0x5000, 0x10000, need, 0) == psd.PSD_ERR_SHAPE   # more than 32 nodes
    assert f(m, 0x4000, 30, par([-1] + [0] * 29), kv, 0x5000, 0x10000, need, 0) == psd.PSD_ERR_CAPACITY  # 100 + 30 > 128
    assert f(m, 0x4000, 3, par([-1, 0, 0]), kv, 0x5000, 0x10000, 16, 0) == psd.PSD_ERR_WORKSPACE
    c = lib.psd_kv_compact_tree
    assert c(kv, 0, 0x2000, 0x3000, 8, 8, -1, 0) == psd.PSD_ERR_NULL
    assert c(kv, 0x1000, 0x2000, 0x3000, 3, 8, -1, 0) == psd.PSD_ERR_SHAPE       # path rows shorter than n_nodes - 1
    assert c(kv, 0x1000, 0x2000, 0x3000, 40, 40, -1, 0) == psd.PSD_ERR_SHAPE     # more than 32 nodes
    assert c(kv, 0x3000, 0x2000, 0x4000, 8, 8, -1, 0) == psd.PSD_ERR_SHAPE       # the cache's own length array as the base
    psd.psd_kv_destroy(kv)
    psd.psd_model_destroy(m)


def test_bench_refuses_more_than_one_gpu():
    """The build has no multi-GPU path: bench.py says so and exits before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
