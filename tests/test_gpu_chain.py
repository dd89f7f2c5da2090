"""Workload 1 end to end: the tiny fp32 three-level chain on the GPU against the CPU oracle.

Lockstep protocol: every forward the GPU chain made is recomputed by the oracle from the
same prefix and its logits compared (max-abs <= 1e-4); every acceptance and every draft
sample is re-decided by the oracle on the GPU's own logits with the same uniforms and must
agree bit for bit except at flagged near-ties; then a free-running oracle chain with its own
logits must emit the same text.  The chain's counters give Eq. (2) / Lemma 3.1."""
import numpy as np
import pytest
import torch

from oracle import accept as oacc
from oracle import chain as ochain
from oracle import forward as ofwd
from paper_2510_26527_amd import chain as gchain
from paper_2510_26527_amd import costmodel, runtime, synth

pytestmark = pytest.mark.gpu


class OracleLevel:
    def __init__(self, shape, weights, max_len):
        self.cfg = ofwd.ModelConfig(**shape.asdict())
        self.w = weights
        self.kv = ofwd.KVCache(self.cfg, 1, max_len)

    @property
    def kv_len(self):
        return int(self.kv.lens[0])

    def forward(self, tokens):
        return ofwd.forward(self.cfg, self.w, np.asarray([tokens], np.int32), self.kv)[0]

    def truncate(self, n):
        self.kv.truncate(n)


def _setup(shapes, seeds, dtype, max_len, gammas):
    ws = [synth.make_weights(s, sd, dtype) for s, sd in zip(shapes, seeds)]
    models = [runtime.Model(s, w) for s, w in zip(shapes, ws)]
    rows = [gammas[1] + 1] + [gammas[i] + 1 for i in range(1, len(shapes))]
    glevels = [gchain.Level(m, max_len, r) for m, r in zip(models, rows)]
    olevels = [OracleLevel(s, w, max_len) for s, w in zip(shapes, ws)]
    return glevels, olevels


def _lockstep(events, olevels, tol):
    worst, ties, n_accept = 0.0, 0, 0
    for ev in events:
        if ev[0] == "forward":
            _, i, start, toks, rows = ev
            lvl = olevels[i]
            if lvl.kv_len > start:
                lvl.truncate(start)
            assert lvl.kv_len == start
            ref = lvl.forward(toks)
            if rows is not None:
                got = rows.cpu().double().numpy()
                err = np.abs(got - ref[-got.shape[0]:]).max()
                worst = max(worst, err)
                assert err <= tol, f"level {i} forward at {start}: logits off by {err:.3e}"
        elif ev[0] == "accept":
            _, i, k, x, u, n, tok, flags, p, q = ev
            on, otok, ofl = oacc.spec_accept(p.double().numpy()[None], q.double().numpy()[None], x[None], u[None].astype(np.float64))
            n_accept += 1
            if ofl[0] & oacc.FLAG_NEAR_TIE:
                ties += 1
                continue
            assert (n, tok) == (int(on[0]), int(otok[0])), f"level {i} accept: gpu {(n, tok)} oracle {(on[0], otok[0])}"
        elif ev[0] == "sample":
            _, i, u, tok, row = ev
            assert tok == int(oacc.sample(row.double().numpy().reshape(1, -1), [u])[0])
    return worst, ties, n_accept


def test_workload1_tiny_three_level_chain():
    shapes = [synth.TINY_TARGET, synth.TINY_INTERMEDIATE, synth.TINY_DRAFT]
    gammas = [None, 8, 4]
    n_gen, max_len = 64, 192
    glevels, olevels = _setup(shapes, [101, 102, 103], torch.float32, max_len, gammas)
    prompt = synth.make_tokens(512, (32,), 7).tolist()
    tapes = [synth.make_tape(9, 0, 200, 16), synth.make_tape(9, 1, 400, 16), synth.make_tape(9, 2, 1000, 1)[:, 0]]
    g = gchain.Chain(glevels, gammas, tapes, 1.0, trace=True, timed=True)
    out = g.generate(prompt, n_gen)
    assert len(out) == n_gen and all(0 <= t < 512 for t in out)

    # lockstep: oracle prefill, then replay
    for lvl in olevels:
        lvl.forward(prompt[:-1])
    worst, ties, n_accept = _lockstep(g.events, olevels, 1e-4)
    print(f"lockstep: {len(g.events)} events, max abs logit err {worst:.2e}, accept calls {n_accept}, near-ties {ties}")

    # free-running oracle chain with its own logits and the same tapes
    _, olevels2 = _setup(shapes, [101, 102, 103], torch.float32, max_len, gammas)
    o = ochain.Chain(olevels2, gammas, [np.asarray(t, np.float64) for t in tapes], 1.0)
    ref = o.generate(prompt, n_gen)
    assert out == ref, f"first divergence at {next(i for i, (a, b) in enumerate(zip(out, ref)) if a != b)}"
    assert [lv.forwards for lv in glevels] == o.stats.forwards
    assert g.accept_lens[0] == o.stats.accept_lens[0] and g.accept_lens[1] == o.stats.accept_lens[1]

    # Eq. (2) / Lemma 3.1 from the measured run
    rep = costmodel.chain_report(n_gen, [lv.forwards for lv in glevels], [lv.time_ms for lv in glevels], g.accept_ms)
    assert rep["lemma31_ms"] == pytest.approx(rep["eq2_ms"], rel=1e-9)
    assert rep["F"][0] <= rep["F"][1] <= rep["F"][2]
    mean_tokens = np.mean([n + 1 for n in g.accept_lens[0]])
    print("chain report", {k: (round(v, 4) if isinstance(v, float) else v) for k, v in rep.items()}, "tokens per target forward", mean_tokens)
    for lv in glevels:
        lv.close()


def test_two_level_bf16_chain_lockstep():
    """A two-level bf16 chain (small GQA models, d_head 64 and 128): exercises the bf16 kernels
    inside the loop, catch-up rows of the draft and rollback; lockstep tolerance 2e-2 relative."""
    tgt = synth.Shape(2, 256, 2, 2, 128, 384, 1024, 1.0e4)
    drf = synth.Shape(1, 128, 2, 1, 64, 256, 1024, 1.0e4)
    gammas = [None, 5]
    max_len = 128
    ws = [synth.make_weights(tgt, 1, torch.bfloat16, std=0.05), synth.make_weights(drf, 2, torch.bfloat16, std=0.05)]
    models = [runtime.Model(tgt, ws[0]), runtime.Model(drf, ws[1])]
    glevels = [gchain.Level(models[0], max_len, 6), gchain.Level(models[1], max_len, 6)]
    olevels = [OracleLevel(tgt, ws[0], max_len), OracleLevel(drf, ws[1], max_len)]
    prompt = synth.make_tokens(1024, (9,), 3).tolist()
    tapes = [synth.make_tape(4, 0, 100, 8), synth.make_tape(4, 1, 400, 1)[:, 0]]
    g = gchain.Chain(glevels, gammas, tapes, 1.0, trace=True)
    out = g.generate(prompt, 40)
    for lvl in olevels:
        lvl.forward(prompt[:-1])
    # relative tolerance: compare row-wise
    worst = 0.0
    for ev in g.events:
        if ev[0] == "forward":
            _, i, start, toks, rows = ev
            lvl = olevels[i]
            if lvl.kv_len > start:
                lvl.truncate(start)
            ref = lvl.forward(toks)
            if rows is not None:
                got = rows.cpu().double().numpy()
                r = ref[-got.shape[0]:]
                rel = (np.abs(got - r).max(axis=1) / np.abs(r).max(axis=1)).max()
                worst = max(worst, rel)
                assert rel <= 2e-2
        elif ev[0] == "accept":
            _, i, k, x, u, n, tok, flags, p, q = ev
            on, otok, ofl = oacc.spec_accept(p.double().numpy()[None], q.double().numpy()[None], x[None], u[None].astype(np.float64))
            if not (ofl[0] & oacc.FLAG_NEAR_TIE):
                assert (n, tok) == (int(on[0]), int(otok[0]))
        elif ev[0] == "sample":
            _, i, u, tok, row = ev
            assert tok == int(oacc.sample(row.double().numpy().reshape(1, -1), [u])[0])
    print("bf16 chain lockstep worst rel err", worst, "accept lens", g.accept_lens[0])
    assert len(out) == 40
    for lv in glevels:
        lv.close()
