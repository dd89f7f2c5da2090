"""Pins for the greedy verification rule of the CPU oracle (oracle/accept.c, oracle_greedy_accept).

The paper lists greedy matching beside speculative sampling as a verification rule (Sec. 3.1)
and compares the two in its ablation on acceptance-length variance.  What fixes the rule:
it is the zero-temperature limit of the speculative-sampling rule; a chain that drafts and
verifies greedily reproduces the target's greedy decoding token for token; and its block
lengths under an i.i.d. match rate follow the truncated geometric law of Thm 3.3's proof.
"""
import numpy as np
import pytest
from scipy import stats

from oracle import accept, theory


def test_matches_library_argmax_and_first_mismatch():
    rng = np.random.default_rng(0)
    rows, gamma, V = 500, 6, 40
    lp = rng.normal(0, 2, (rows, gamma + 1, V))
    am = np.argmax(lp, axis=-1)
    x = am[:, :gamma].copy()
    flip = rng.random((rows, gamma)) < 0.2
    x[flip] = (x[flip] + 1 + rng.integers(0, V - 1, flip.sum())) % V
    n, tok = accept.greedy_accept(lp, x)
    mism = x != am[:, :gamma]
    n_ref = np.where(mism.any(1), mism.argmax(1), gamma)
    assert np.array_equal(n, n_ref)
    assert np.array_equal(tok, am[np.arange(rows), n_ref])
    # without the bonus row a fully matching block emits nothing
    n2, tok2 = accept.greedy_accept(lp[:, :gamma], x)
    assert np.array_equal(n2, n_ref)
    assert np.array_equal(tok2, np.where(n_ref == gamma, -1, am[np.arange(rows), np.minimum(n_ref, gamma - 1)]))


def test_worked_example_with_ties():
    lp = np.array([[[1.0, 3.0, 3.0], [0.0, 0.0, 0.0], [5.0, 1.0, 2.0], [-np.inf, -np.inf, -np.inf]]])
    # argmax rows: 1 (lowest of the tied 1, 2), 0, 0, 0
    assert [a.tolist() for a in accept.greedy_accept(lp, [[1, 0, 0]])] == [[3], [0]]
    assert [a.tolist() for a in accept.greedy_accept(lp, [[2, 0, 0]])] == [[0], [1]]
    assert [a.tolist() for a in accept.greedy_accept(lp, [[1, 0, 2]])] == [[2], [0]]
    assert [a.tolist() for a in accept.greedy_accept(lp[:, :3], [[1, 0, 0]])] == [[3], [-1]]
    assert [a.tolist() for a in accept.greedy_accept(lp[:, :1], np.empty((1, 0), np.int32))] == [[0], [1]]


def test_is_the_zero_temperature_limit_of_speculative_sampling():
    """At T -> 0 both softmaxes become one-hot at their argmax; with drafts x_j = argmax q_j the
    sampling rule accepts iff argmax p_j = x_j whatever the uniforms, and the residual is one-hot at
    argmax p_j."""
    rng = np.random.default_rng(1)
    rows, gamma, V = 400, 5, 30
    lp = rng.normal(0, 2, (rows, gamma + 1, V))
    lq = lp[:, :gamma] + rng.normal(0, 1.5, (rows, gamma, V))
    x = np.argmax(lq, axis=-1)
    u = rng.random((rows, gamma + 1))
    n_s, tok_s, _ = accept.spec_accept(lp, lq, x, u, temperature=1e-3)
    n_g, tok_g = accept.greedy_accept(lp, x)
    assert 0 < (n_g < gamma).mean() < 1
    assert np.array_equal(n_s, n_g) and np.array_equal(tok_s, tok_g)


def test_greedy_chain_reproduces_target_greedy_decoding():
    """Markov-table models: a drafter proposing argmax q(.|prev), verified greedily by the target,
    emits exactly the target's own greedy path."""
    V, gamma, n_tokens = 7, 4, 60
    seen = set()
    for seed in range(20):
        rng = np.random.default_rng(seed)
        P = np.log(rng.dirichlet(np.ones(V), V))          # P[prev] = target logits
        Q = P + rng.normal(0, 0.7, (V, V))                # a drafter that often agrees
        ref, prev = [], 3
        for _ in range(n_tokens):
            prev = int(np.argmax(P[prev]))
            ref.append(prev)
        out, last = [], 3
        while len(out) < n_tokens:
            x, t = [], last
            for _ in range(gamma):
                t = int(np.argmax(Q[t]))
                x.append(t)
            rows = np.stack([P[last]] + [P[t] for t in x])          # gamma + 1 verifier rows
            n, tok = accept.greedy_accept(rows[None], [x])
            out += x[:n[0]] + [int(tok[0])]
            seen.add(int(n[0]))
            last = out[-1]
        assert out[:n_tokens] == ref, seed
    assert {0, gamma} <= seen and len(seen) >= 3          # rejections, partial and full acceptances all occurred


def test_block_length_law_under_iid_match_rate():
    """If each position matches independently with probability alpha, tokens per verification are
    truncated geometric with gamma + 1 trials: the same law as for speculative sampling at equal
    alpha, so the two rules differ in acceptance-length variance only through alpha (Thm 3.3)."""
    rng = np.random.default_rng(4)
    rows, gamma, V, alpha = 200_000, 8, 5, 0.7
    lp = rng.normal(0, 1, (rows, gamma + 1, V))
    am = np.argmax(lp, -1)[:, :gamma]
    x = np.where(rng.random((rows, gamma)) < alpha, am, (am + 1) % V)
    n, tok = accept.greedy_accept(lp, x)
    N = n + 1
    mean, var = theory.expected_tokens(alpha, gamma + 1), theory.variance_tokens(alpha, gamma + 1)
    assert abs(N.mean() - mean) < 4 * np.sqrt(var / rows)
    assert N.var() == pytest.approx(var, rel=0.02)
    pmf = np.array(theory.tokens_per_verify_pmf(alpha, gamma + 1))
    assert stats.chisquare(np.bincount(N, minlength=gamma + 2)[1:], pmf * rows).pvalue > 1e-4
