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


# ---------------------------------------------------------------- workload 4: full-size three-level chain
def _phi(x):
    from math import erf, sqrt
    return 0.5 * (1.0 + erf(x / sqrt(2.0)))


@pytest.fixture(scope="module")
def chain4_models():
    """LLaMA3-8B-shaped target, 16-layer half-width intermediate, one-layer draft sharing the
    target's embedding and lm_head; bf16 random init generated on the device (no oracle forward
    runs here: forward parity of these shapes is test_workload4_chain_models_full_size)."""
    tw = synth.make_weights(synth.LLAMA3_8B, 401, torch.bfloat16, device="cuda")
    mw = synth.make_weights(synth.CHAIN_INTERMEDIATE, 402, torch.bfloat16, device="cuda")
    dw = synth.make_weights(synth.CHAIN_DRAFT, 403, torch.bfloat16, device="cuda",
                            share={"embed": tw["embed"], "lm_head": tw["lm_head"]})
    models = [runtime.Model(synth.LLAMA3_8B, tw).pack(), runtime.Model(synth.CHAIN_INTERMEDIATE, mw).pack(),
              runtime.Model(synth.CHAIN_DRAFT, dw).pack()]
    assert models[2].weights["lm_head"].data_ptr() == models[0].weights["lm_head"].data_ptr()
    yield models
    for m in models:
        m.close()


@pytest.mark.parametrize("sigma", [0.25, 1.0])
def test_workload4_full_three_level_chain(chain4_models, sigma):
    """256-token prompt, 512 generated tokens, gamma_draft 6, gamma_intermediate 10, T = 1, with the
    agreement harness at noise sigma.  Every acceptance and every draft sample of the run is
    re-decided by the oracle on the GPU's own rows and uniforms (bit-exact except flagged
    near-ties); the per-token acceptance rates must land at 2 Phi(-sigma/2); Eq. (2) and
    Lemma 3.1 are recomputed from the measured counts and times."""
    from paper_2510_26527_amd import shim
    import json, os, time
    gammas = [None, 10, 6]
    n_gen, n_prompt, max_len = 512, 256, 896
    levels = [gchain.Level(chain4_models[0], max_len, 11), gchain.Level(chain4_models[1], max_len, 11),
              gchain.Level(chain4_models[2], max_len, 7)]
    prompt = synth.make_tokens(synth.LLAMA3_8B.vocab, (n_prompt,), 77).tolist()
    tapes = [synth.make_tape(14, 0, 3 * n_gen, 16), synth.make_tape(14, 1, 3 * n_gen, 16),
             synth.make_tape(14, 2, 12 * n_gen, 1)[:, 0]]
    st = {"accepts": [0, 0], "ties": 0, "samples": 0, "tested": [0, 0], "passed": [0, 0]}

    def sink(ev):
        if ev[0] == "accept":
            _, i, k, x, u, n, tok, flags, p, q = ev
            on, otok, ofl = oacc.spec_accept(p.double().numpy()[None], q.double().numpy()[None], x[None],
                                             u[None].astype(np.float64))
            st["accepts"][i] += 1
            st["tested"][i] += min(n + 1, k)
            st["passed"][i] += n
            if ofl[0] & oacc.FLAG_NEAR_TIE:
                st["ties"] += 1
                return
            assert (n, tok) == (int(on[0]), int(otok[0])), f"level {i} accept: gpu {(n, tok)} oracle {(on[0], otok[0])}"
        elif ev[0] == "sample":
            _, i, u, tok, row = ev
            st["samples"] += 1
            if st["samples"] % 8 == 0:            # every 8th draft sample: the draw is one fp64 pass over 128256 entries
                assert tok == int(oacc.sample(row.double().numpy().reshape(1, -1), [u])[0])

    g = shim.AgreementShimChain(levels, gammas, tapes, sigma, noise_seed=5, temperature=1.0, max_len=max_len,
                                trace=True, timed=True, sink=sink)
    t0 = time.time()
    out = g.generate(prompt, n_gen)
    wall_ms = (time.time() - t0) * 1e3
    assert len(out) == n_gen and all(0 <= t < synth.LLAMA3_8B.vocab for t in out)

    alpha = 2.0 * _phi(-sigma / 2.0)
    rates = [st["passed"][i] / st["tested"][i] for i in range(2)]
    for i in range(2):
        sd = (alpha * (1 - alpha) / st["tested"][i]) ** 0.5
        assert abs(rates[i] - alpha) < 5 * sd + 0.02, f"level {i}: acceptance rate {rates[i]:.3f}, expected {alpha:.3f}"
    rep = costmodel.chain_report(n_gen, [lv.forwards for lv in levels], [lv.time_ms for lv in levels], g.accept_ms)
    assert rep["lemma31_ms"] == pytest.approx(rep["eq2_ms"], rel=1e-9)
    tokens_per_target = float(np.mean([n + 1 for n in g.accept_lens[0]]))
    full = [n for n, k in zip(g.accept_lens[0], g.block_lens[0]) if k == 10]
    expect = (1 - alpha ** 11) / (1 - alpha)
    rep.update(sigma=sigma, alpha_expected=alpha, alpha_measured=rates, tokens_per_target_forward=tokens_per_target,
               tokens_per_target_forward_expected=expect, near_ties=st["ties"], accept_calls=st["accepts"],
               peeks=g.peeks, peek_ms=g.peek_ms, wall_ms_with_trace=wall_ms)
    # the same target decoding alone, one token per forward, on the same kernels and cache length
    tgt = levels[0]
    psd_len = n_prompt + n_gen // 2
    import paper_2510_26527_amd as psd
    psd.psd_kv_truncate_to(tgt.kv.handle, psd_len)
    tok1 = g.seq[psd_len:psd_len + 1]
    row = tgt.rows[0:1]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for it in range(40):
        if it == 8:
            e0.record()
        psd.psd_model_forward(tgt.model.handle, tok1, 1, tgt.kv.handle, row, 1, tgt.ws)
        psd.psd_kv_truncate_to(tgt.kv.handle, psd_len)
    e1.record()
    torch.cuda.synchronize()
    t_ar = e0.elapsed_time(e1) / 32
    rep.update(target_only_ms_per_token=t_ar, speedup_vs_target_only=t_ar * n_gen / (rep["eq2_ms"] + rep["accept_ms"]))
    rep.update(tokens_per_target_forward_var_full_blocks=float(np.var([n + 1 for n in full])),
               iid_var_at_expected_alpha=float(__import__("oracle.theory", fromlist=["x"]).variance_tokens(alpha, 11)))
    sd_tokens = np.std([n + 1 for n in full]) / max(len(full), 1) ** 0.5
    assert abs(np.mean([n + 1 for n in full]) - expect) < 5 * sd_tokens + 0.35
    os.makedirs("gpurun_out", exist_ok=True)
    with open(f"gpurun_out/chain4_sigma{sigma}.json", "w") as f:
        json.dump(rep, f, indent=1)
    print("workload 4 report", json.dumps({k: (round(v, 4) if isinstance(v, float) else v) for k, v in rep.items()}))
    for lv in levels:
        lv.close()


def test_greedy_three_level_chain_reproduces_target_greedy_decoding():
    """Temperature 0 at every level (greedy drafting, greedy verification): the chain must emit the
    target's own greedy continuation, which the oracle computes with one-token forwards and argmax.
    Steps where the oracle's top two logits are closer than 1e-3 end the comparison (none expected)."""
    shapes = [synth.TINY_TARGET, synth.TINY_INTERMEDIATE, synth.TINY_DRAFT]
    gammas = [None, 8, 4]
    n_gen, max_len = 48, 192
    glevels, olevels = _setup(shapes, [101, 102, 103], torch.float32, max_len, gammas)
    prompt = synth.make_tokens(512, (32,), 7).tolist()
    # the tapes are indexed but not read at temperature 0; disagreeing levels make many short blocks
    tapes = [synth.make_tape(9, 0, 400, 16), synth.make_tape(9, 1, 4000, 16), synth.make_tape(9, 2, 20000, 1)[:, 0]]
    g = gchain.Chain(glevels, gammas, tapes, 0.0)
    out = g.generate(prompt, n_gen)
    tgt = olevels[0]
    tgt.forward(prompt[:-1])
    ref, last = [], prompt[-1]
    for _ in range(n_gen):
        row = tgt.forward([last])[-1]
        top = np.sort(row)[-2:]
        if top[1] - top[0] < 1e-3:
            break
        last = int(np.argmax(row))
        ref.append(last)
    assert len(ref) >= n_gen // 2
    assert out[:len(ref)] == ref
    # random-init levels rarely agree on the argmax: most blocks end early, and the target still decides every token
    print("greedy chain: target forwards", glevels[0].forwards, "accept lens", g.accept_lens[0])
    for lv in glevels:
        lv.close()
    # a drafter that IS the target agrees everywhere: every block is accepted whole and the bonus token is used
    g2l, _ = _setup([synth.TINY_TARGET, synth.TINY_TARGET], [101, 101], torch.float32, max_len, [None, 5])
    g2 = gchain.Chain(g2l, [None, 5], [tapes[0], tapes[2]], 0.0)
    out2 = g2.generate(prompt, n_gen)
    assert out2[:len(ref)] == ref
    assert all(n == k for n, k in zip(g2.accept_lens[0], g2.block_lens[0]))
    assert g2l[0].forwards <= n_gen // 6 + 1
    for lv in g2l:
        lv.close()


def test_workload4_greedy_verification_block_length_variance(chain4_models):
    """The paper's ablation compares the acceptance-length variance of greedy verification and
    speculative sampling.  The same full-size chain and harness at sigma = 0.25, run at temperature 0
    (greedy drafting and greedy verification at every level): every decision is re-made by the oracle's
    greedy rule, and mean and variance of the tokens per target forward are set beside the truncated
    geometric law at the measured per-token match rate (Thm 3.3's i.i.d. reference)."""
    from oracle import theory
    from paper_2510_26527_amd import shim
    import json, os
    gammas, sigma = [None, 10, 6], 0.25
    n_gen, n_prompt, max_len = 256, 256, 896
    levels = [gchain.Level(chain4_models[0], max_len, 11), gchain.Level(chain4_models[1], max_len, 11),
              gchain.Level(chain4_models[2], max_len, 7)]
    prompt = synth.make_tokens(synth.LLAMA3_8B.vocab, (n_prompt,), 77).tolist()
    tapes = [synth.make_tape(14, 0, 3 * n_gen, 16), synth.make_tape(14, 1, 6 * n_gen, 16),
             synth.make_tape(14, 2, 30 * n_gen, 1)[:, 0]]
    st = {"tested": [0, 0], "passed": [0, 0]}

    def sink(ev):
        if ev[0] == "accept":
            _, i, k, x, u, n, tok, flags, p, q = ev
            on, otok = oacc.greedy_accept(p.numpy()[None], x[None])
            assert (n, tok) == (int(on[0]), int(otok[0])), f"level {i}: gpu {(n, tok)} oracle {(on[0], otok[0])}"
            st["tested"][i] += min(n + 1, k)
            st["passed"][i] += n
        elif ev[0] == "sample":
            assert ev[3] == int(np.argmax(ev[4].numpy()))

    g = shim.AgreementShimChain(levels, gammas, tapes, sigma, noise_seed=5, temperature=0.0, max_len=max_len,
                                trace=True, sink=sink)
    out = g.generate(prompt, n_gen)
    assert len(out) == n_gen
    full = np.array([n + 1 for n, k in zip(g.accept_lens[0], g.block_lens[0]) if k == 10])
    rate = st["passed"][0] / st["tested"][0]
    rep = {"sigma": sigma, "rule": "greedy", "match_rate": [st["passed"][i] / st["tested"][i] for i in range(2)],
           "target_forwards": levels[0].forwards, "tokens_per_target_forward_mean": float(full.mean()),
           "tokens_per_target_forward_var": float(full.var()),
           "iid_mean_at_rate": theory.expected_tokens(rate, 11), "iid_var_at_rate": theory.variance_tokens(rate, 11)}
    os.makedirs("gpurun_out", exist_ok=True)
    with open("gpurun_out/chain4_greedy_sigma0.25.json", "w") as f:
        json.dump(rep, f, indent=1)
    print("workload 4 greedy report", json.dumps(rep))
    assert abs(full.mean() - rep["iid_mean_at_rate"]) < 5 * (rep["iid_var_at_rate"] / len(full)) ** 0.5 + 0.5
    for lv in levels:
        lv.close()


def test_workload4_insertion_criterion_live(chain4_models):
    """Thm 3.2 on measured numbers: the same target and draft (the draft two sigma-steps away from the target)
    decoded as a two-level chain and as a three-level chain with the intermediate inserted.  Whether the
    insertion pays off is read from the measured Eq. (2) times, and compared with what the theorem's two
    conditions say when evaluated on the measured T and L."""
    from paper_2510_26527_amd import shim
    import json, os
    sigma, n_gen, n_prompt, max_len = 0.25, 256, 256, 896
    prompt = synth.make_tokens(synth.LLAMA3_8B.vocab, (n_prompt,), 77).tolist()

    def run(models, gammas, rows, noise_terms):
        levels = [gchain.Level(m, max_len, r) for m, r in zip(models, rows)]
        tapes = [synth.make_tape(15, i, 4 * n_gen, 16) for i in range(len(models) - 1)]
        tapes.append(synth.make_tape(15, 9, 12 * n_gen, 1)[:, 0])
        g = shim.AgreementShimChain(levels, gammas, tapes, sigma, noise_seed=6, noise_terms=noise_terms,
                                    temperature=1.0, max_len=max_len, timed=True)
        g.generate(prompt, n_gen)
        rep = costmodel.chain_report(n_gen, [lv.forwards for lv in levels], [lv.time_ms for lv in levels], g.accept_ms)
        for lv in levels:
            lv.close()
        return rep

    two = run([chain4_models[0], chain4_models[2]], [None, 6], [7, 7], [0, 2])
    three = run(chain4_models, [None, 10, 6], [11, 11, 7], [0, 1, 2])
    # notation of the theorem: M_i = target, M_{i+1} = draft, M_new = intermediate
    T_i, T_next, T_new = two["T_ms"][0], two["T_ms"][1], three["T_ms"][1]
    L_i, L_i_new, L_new = two["L"][0], three["L"][0], three["L"][1]
    c1, c2, helps = costmodel.insertion_criterion(T_new, T_i, T_next, L_new, L_i, L_i_new, two["beta"])
    measured_helps = three["eq2_ms"] + three["accept_ms"] < two["eq2_ms"] + two["accept_ms"]
    # the quantity the proof starts from, on the measured numbers: three-model minus two-model time by Lemma 3.1
    change = costmodel.insertion_time_change(n_gen, T_new, T_i, T_next, L_new, L_i, L_i_new, two["beta"])
    t_two, t_three = two["eq2_ms"] + two["accept_ms"], three["eq2_ms"] + three["accept_ms"]
    # Neither inequality near equality.  Thm 3.2 takes T_i and T_{i+1} as constants; here the target verifies 7 rows
    # per step in the two-level chain and 11 in the three-level one, and its measured step time differs between the two
    # (a few per cent), so the band around equality is 10 % plus how far the measured times depart from that assumption.
    drift = abs(three["T_ms"][0] - T_i) / T_i + abs(three["T_ms"][2] - T_next) / T_next
    clear = all(abs(l - r) > (0.1 + drift) * max(abs(l), abs(r)) for l, r in (c1, c2))
    rep = {"two_level": two, "three_level": three, "condition_1": c1, "condition_2": c2, "theorem_says_helps": helps,
           "measured_helps": measured_helps, "lemma31_predicted_change_ms": change,
           "measured_change_ms": t_three - t_two, "conditions_clear_of_equality": clear,
           "forward_time_drift_between_the_two_chains": drift}
    os.makedirs("gpurun_out", exist_ok=True)
    with open("gpurun_out/chain4_insertion.json", "w") as f:
        json.dump(rep, f, indent=1)
    print("insertion check", json.dumps(rep))
    assert two["L"][0] > 1 and three["L"][0] > two["L"][0]        # the intermediate raises the target's acceptance length
    # The conditions are sufficient, not necessary (tests/test_theory.py::test_neither_condition_is_necessary):
    # a clear "helps" must be seen in the measured times; a clear "does not" is checked through the full
    # three-term difference the proof starts from, which decides the matter either way.
    if clear and helps:
        assert measured_helps, rep
    if abs(change) > 0.1 * t_two:
        assert measured_helps == (change < 0), rep
    if clear and not helps and change > 0.1 * t_two:
        assert not measured_helps, rep


def test_four_level_tiny_chain():
    """The chain driver is n-level generic (the paper's conclusion names deeper chains as the next step): four
    fp32 models, block sizes 8 / 4 / 2, lockstep against the oracle and the same text from a free-running
    oracle chain."""
    extra = synth.Shape(1, 96, 3, 3, 32, 192, 512)
    shapes = [synth.TINY_TARGET, synth.TINY_INTERMEDIATE, synth.TINY_DRAFT, extra]
    gammas = [None, 8, 4, 2]
    n_gen, max_len = 48, 192
    seeds = [101, 102, 103, 104]
    glevels, olevels = _setup(shapes, seeds, torch.float32, max_len, gammas)
    prompt = synth.make_tokens(512, (20,), 17).tolist()
    tapes = [synth.make_tape(19, 0, 200, 16), synth.make_tape(19, 1, 400, 16), synth.make_tape(19, 2, 800, 16),
             synth.make_tape(19, 3, 2000, 1)[:, 0]]
    g = gchain.Chain(glevels, gammas, tapes, 1.0, trace=True)
    out = g.generate(prompt, n_gen)
    for lvl in olevels:
        lvl.forward(prompt[:-1])
    worst, ties, n_accept = _lockstep(g.events, olevels, 1e-4)
    _, olevels2 = _setup(shapes, seeds, torch.float32, max_len, gammas)
    o = ochain.Chain(olevels2, gammas, [np.asarray(t, np.float64) for t in tapes], 1.0)
    ref = o.generate(prompt, n_gen)
    assert out == ref
    assert [lv.forwards for lv in glevels] == o.stats.forwards
    F = [lv.forwards for lv in glevels]
    assert F[0] <= F[1] <= F[2] <= F[3]
    print(f"four levels: forwards {F}, lockstep max abs err {worst:.2e}, accept calls {n_accept}, near-ties {ties}")
    for lv in glevels:
        lv.close()


def test_workload4_quantised_target_as_intermediate(chain4_models):
    """The paper's own three-model system: the intermediate is a 4-bit weight-only quantised copy of the target
    (group size 128), here by round-to-nearest on the random-init LLaMA3-8B-shaped target.  Its forward pass is
    what is timed as T_2.  A random-init network does not survive quantisation the way a trained one does
    (measured: its logits decorrelate from the target's, 1 - TV = 0.50), so the agreement harness sets the
    acceptance rates here too.  Every acceptance is re-decided by the oracle; Thm 3.2's conditions are
    evaluated on the measured T and L and set beside the measured Eq. (2) times of the two-level and
    three-level chains."""
    from paper_2510_26527_amd import shim
    import json, os
    sigma, n_gen, n_prompt, max_len = 0.25, 256, 256, 896
    tgt, _, drf = chain4_models
    codes, quant = synth.quantize_w4(tgt.weights)
    mid = runtime.Model(synth.LLAMA3_8B, codes, quant=quant).pack()
    assert mid.weights["lm_head"].data_ptr() == tgt.weights["lm_head"].data_ptr()
    prompt = synth.make_tokens(synth.LLAMA3_8B.vocab, (n_prompt,), 77).tolist()
    st = {"tested": [0, 0], "passed": [0, 0], "ties": 0}

    def sink(ev):
        if ev[0] == "accept":
            _, i, k, x, u, n, tok, flags, p, q = ev
            on, otok, ofl = oacc.spec_accept(p.double().numpy()[None], q.double().numpy()[None], x[None],
                                             u[None].astype(np.float64))
            st["tested"][i] += min(n + 1, k)
            st["passed"][i] += n
            if ofl[0] & oacc.FLAG_NEAR_TIE:
                st["ties"] += 1
                return
            assert (n, tok) == (int(on[0]), int(otok[0])), f"level {i} accept: gpu {(n, tok)} oracle {(on[0], otok[0])}"

    def run(models, gammas, rows, noise_terms, trace):
        levels = [gchain.Level(m, max_len, r) for m, r in zip(models, rows)]
        tapes = [synth.make_tape(16, i, 4 * n_gen, 16) for i in range(len(models) - 1)]
        tapes.append(synth.make_tape(16, 9, 12 * n_gen, 1)[:, 0])
        g = shim.AgreementShimChain(levels, gammas, tapes, sigma, noise_seed=7, noise_terms=noise_terms, temperature=1.0,
                                    max_len=max_len, timed=True, trace=trace, sink=sink if trace else None)
        out = g.generate(prompt, n_gen)
        assert len(out) == n_gen
        rep = costmodel.chain_report(n_gen, [lv.forwards for lv in levels], [lv.time_ms for lv in levels], g.accept_ms)
        for lv in levels:
            lv.close()
        return rep

    three = run([tgt, mid, drf], [None, 10, 6], [11, 11, 7], [0, 1, 2], True)
    rates = [st["passed"][i] / max(st["tested"][i], 1) for i in range(2)]
    two = run([tgt, drf], [None, 6], [7, 7], [0, 2], False)
    T_i, T_next, T_new = two["T_ms"][0], two["T_ms"][1], three["T_ms"][1]
    L_i, L_i_new, L_new = two["L"][0], three["L"][0], three["L"][1]
    c1, c2, helps = costmodel.insertion_criterion(T_new, T_i, T_next, L_new, L_i, L_i_new, two["beta"])
    rep = {"two_level": two, "three_level": three, "acceptance_rate_target_vs_w4": rates[0],
           "acceptance_rate_w4_vs_draft": rates[1], "near_ties": st["ties"], "T_w4_over_T_target": T_new / T_i,
           "condition_1": c1, "condition_2": c2, "theorem_says_helps": helps,
           "measured_helps": three["eq2_ms"] + three["accept_ms"] < two["eq2_ms"] + two["accept_ms"]}
    os.makedirs("gpurun_out", exist_ok=True)
    with open("gpurun_out/chain4_w4_intermediate.json", "w") as f:
        json.dump(rep, f, indent=1)
    print("w4 intermediate", json.dumps(rep))
    assert three["T_ms"][1] < three["T_ms"][0]            # the 4-bit copy is cheaper per forward than the target
    mid.close()
