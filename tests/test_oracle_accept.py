"""Pins for the CPU oracle of the acceptance test (oracle/accept.c).

The paper fixes one thing about the rule: the target's output distribution is preserved
(Abstract; Sec. 3.1; Conclusion).  Everything below follows from that and from textbook
facts, none of it from the oracle itself: the law implied by the code is *measured* by
bisection over its uniform inputs and compared with p; sampled laws are chi-square tested
at 10^6 draws; the acceptance probability is 1 - TV(p, q); the mean block length under an
i.i.d. acceptance rate is the truncated-geometric mean of Thm 3.3's proof.
"""
import numpy as np
import pytest
from scipy import stats

from oracle import accept, theory


def _rand_dist(rng, V, conc=1.0):
    return rng.dirichlet(np.full(V, conc))


def _logits(p):
    return np.log(p)


def _accept_threshold(lp, lq, x, lo=0.0, hi=1.0):
    """Largest u0 for which draft token x is accepted, found by bisection on the code."""
    def acc(u0):
        n, _, _ = accept.spec_accept(lp[None, None], lq[None, None], [[x]], [[u0, 0.5]])
        return n[0] == 1
    if acc(np.nextafter(1.0, 0.0)):
        return 1.0
    if not acc(0.0):
        return 0.0
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        if acc(mid):
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def _draw_law(lp, lq, x, V):
    """Lengths of the u1-intervals mapped to each token when x is rejected (u0 -> 1)."""
    u0 = np.nextafter(1.0, 0.0)
    # breakpoints by bisection: token index is non-decreasing in u1
    def tok(u1):
        n, t, _ = accept.spec_accept(lp[None, None], lq[None, None], [[x]], [[u0, u1]])
        assert n[0] == 0
        return int(t[0])
    edges = np.zeros(V + 1)
    edges[V] = 1.0
    for k in range(V - 1):                  # edge k+1 = sup{u1 : tok(u1) <= k}
        lo, hi = 0.0, 1.0
        if tok(0.0) > k:
            edges[k + 1] = 0.0
            continue
        if tok(np.nextafter(1.0, 0.0)) <= k:
            edges[k + 1] = 1.0
            continue
        for _ in range(60):
            mid = 0.5 * (lo + hi)
            if tok(mid) <= k:
                lo = mid
            else:
                hi = mid
        edges[k + 1] = 0.5 * (lo + hi)
    return np.diff(edges)


@pytest.mark.parametrize("V,seed", [(2, 0), (5, 1), (16, 2)])
def test_emitted_law_is_target_exact(V, seed):
    """Measure the law the code implies for one position and compare with p (to 1e-9):
    P(emit k) = sum_x q[x] (a_x [k = x] + (1 - a_x) len_x(k))."""
    rng = np.random.default_rng(seed)
    p, q = _rand_dist(rng, V), _rand_dist(rng, V)
    lp, lq = _logits(p), _logits(q)
    law = np.zeros(V)
    p_accept = 0.0
    for x in range(V):
        a = _accept_threshold(lp, lq, x)
        assert a == pytest.approx(min(1.0, p[x] / q[x]), abs=1e-12)
        p_accept += q[x] * a
        law[x] += q[x] * a
        if a < 1.0:
            law += q[x] * (1.0 - a) * _draw_law(lp, lq, x, V)
    np.testing.assert_allclose(law, p, atol=1e-9)
    assert p_accept == pytest.approx(1.0 - 0.5 * np.abs(p - q).sum(), abs=1e-10)


def _batch(rng, P, Q, rows, n_p_rows):
    """rows independent trials with per-position distributions P[j], Q[j]; drafts ~ Q[j]."""
    gamma, V = Q.shape
    lp = np.broadcast_to(np.log(P[:n_p_rows]), (rows, n_p_rows, V))
    lq = np.broadcast_to(np.log(Q), (rows, gamma, V))
    x = np.stack([rng.choice(V, size=rows, p=Q[j]) for j in range(gamma)], axis=1).astype(np.int32)
    u = rng.random((rows, gamma + 1))
    return lp, lq, x, u


def test_chi_square_and_acceptance_probability_1e6():
    """10^6 draws, V = 16: emitted token ~ p (chi-square) and P(accept) = 1 - TV (4 sigma)."""
    rng = np.random.default_rng(11)
    V, rows = 16, 1_000_000
    p, q = _rand_dist(rng, V, 0.7), _rand_dist(rng, V, 0.7)
    lp, lq, x, u = _batch(rng, p[None], q[None], rows, 1)
    n, tok, _ = accept.spec_accept(lp, lq, x, u)
    emitted = np.where(n == 1, x[:, 0], tok)
    counts = np.bincount(emitted, minlength=V)
    chi = stats.chisquare(counts, p * rows)
    assert chi.pvalue > 1e-4
    alpha = 1.0 - 0.5 * np.abs(p - q).sum()
    se = np.sqrt(alpha * (1 - alpha) / rows)
    assert abs(n.mean() - alpha) < 4 * se
    # the wrong residual (e.g. |p - q| or q - p) or a swapped ratio would fail the chi-square:
    wrong = np.maximum(q - p, 0); wrong /= wrong.sum()
    assert stats.chisquare(counts, (np.minimum(p, q) + (1 - alpha) * wrong) * rows).pvalue < 1e-10


def test_multi_position_joint_law_markov_tables():
    """gamma = 3, V = 4, first-order Markov 'models': the emitted block, extended to length
    gamma+1 with exact target samples, follows the target's autoregressive law (chi-square
    over all 256 sequences).  Catches wrong row indexing, a missing break, a wrong draw row."""
    rng = np.random.default_rng(5)
    V, gamma, rows = 4, 3, 1_000_000
    Pm = np.stack([_rand_dist(rng, V, 1.5) for _ in range(V)])      # target p(x | prev)
    Qm = np.stack([_rand_dist(rng, V, 1.5) for _ in range(V)])      # drafter q(x | prev)
    prev0 = 2
    # draft autoregressively from Q, build the rows both models would produce on that draft
    x = np.empty((rows, gamma), np.int32)
    lp = np.empty((rows, gamma + 1, V))
    lq = np.empty((rows, gamma, V))
    prev = np.full(rows, prev0)
    cdfQ = np.cumsum(Qm, axis=1)
    for j in range(gamma):
        lq[:, j] = np.log(Qm[prev])
        lp[:, j] = np.log(Pm[prev])
        x[:, j] = (rng.random(rows)[:, None] > cdfQ[prev]).sum(axis=1)
        prev = x[:, j]
    lp[:, gamma] = np.log(Pm[prev])
    u = rng.random((rows, gamma + 1))
    n, tok, _ = accept.spec_accept(lp, lq, x, u)
    seq = np.empty((rows, gamma + 1), np.int64)
    cdfP = np.cumsum(Pm, axis=1)
    for j in range(gamma + 1):
        from_draft = j < n
        is_tok = j == n
        prev = seq[:, j - 1] if j else np.full(rows, prev0)
        fresh = (rng.random(rows)[:, None] > cdfP[prev]).sum(axis=1)      # exact target samples
        seq[:, j] = np.where(from_draft, x[:, min(j, gamma - 1)], np.where(is_tok, tok, fresh))
    code = (seq * (V ** np.arange(gamma, -1, -1))).sum(axis=1)
    counts = np.bincount(code, minlength=V ** (gamma + 1))
    law = np.ones(V ** (gamma + 1))
    for c in range(law.size):
        digits = [(c // V ** (gamma - j)) % V for j in range(gamma + 1)]
        pr, pv = 1.0, prev0
        for d in digits:
            pr *= Pm[pv, d]
            pv = d
        law[c] = pr
    assert stats.chisquare(counts, law * rows).pvalue > 1e-4


def test_mean_and_variance_of_block_length_iid():
    """Same (p, q) at every position, gamma = 8, bonus row present: tokens per verification
    N = n + 1 is truncated geometric with n = gamma + 1 trials (proof of Thm 3.3):
    E[N] = (1 - alpha^(gamma+1)) / (1 - alpha)."""
    rng = np.random.default_rng(3)
    V, gamma, rows = 12, 8, 1_000_000
    p, q = _rand_dist(rng, V, 3.0), _rand_dist(rng, V, 3.0)
    alpha = np.minimum(p, q).sum()
    P = np.repeat(p[None], gamma + 1, 0)
    Q = np.repeat(q[None], gamma, 0)
    lp, lq, x, u = _batch(rng, P, Q, rows, gamma + 1)
    n, tok, _ = accept.spec_accept(lp, lq, x, u)
    N = n + 1
    mean, var = theory.expected_tokens(alpha, gamma + 1), theory.variance_tokens(alpha, gamma + 1)
    assert mean == pytest.approx((1 - alpha ** (gamma + 1)) / (1 - alpha), rel=1e-12)
    assert abs(N.mean() - mean) < 4 * np.sqrt(var / rows)
    assert N.var() == pytest.approx(var, rel=0.01)
    assert np.all(tok >= 0)
    # full pmf
    pmf = np.array(theory.tokens_per_verify_pmf(alpha, gamma + 1))
    assert stats.chisquare(np.bincount(N, minlength=gamma + 2)[1:], pmf * rows).pvalue > 1e-4


def test_special_cases():
    rng = np.random.default_rng(9)
    V, gamma, rows = 9, 5, 2000
    lp = rng.normal(0, 2, (rows, gamma + 1, V))
    x = rng.integers(0, V, (rows, gamma)).astype(np.int32)
    u = rng.random((rows, gamma + 1))
    # q == p: every token is accepted, the bonus token is the inverse-CDF draw from row gamma
    n, tok, fl = accept.spec_accept(lp, lp[:, :gamma], x, u)
    assert np.all(n == gamma) and np.all(fl & accept.FLAG_ZERO_RESIDUAL == 0)
    pg = np.exp(lp[:, gamma]); pg /= pg.sum(1, keepdims=True)
    ref = np.array([np.searchsorted(np.cumsum(pg[b]), u[b, gamma] * pg[b].sum(), side="right")
                    for b in range(rows)])
    assert np.array_equal(tok, np.minimum(ref, V - 1))
    # no bonus row: token is -1 when all are accepted
    n, tok, _ = accept.spec_accept(lp[:, :gamma], lp[:, :gamma], x, u)
    assert np.all(n == gamma) and np.all(tok == -1)
    # q one-hot on a token the target gives (almost) no mass: never accepted, residual = p
    lq = np.full((rows, gamma, V), -60.0)
    lq[:, :, 0] = 60.0
    lp0 = lp.copy()
    lp0[:, :, 0] = -1e9
    x0 = np.zeros((rows, gamma), np.int32)
    n, tok, _ = accept.spec_accept(lp0, lq, x0, u)
    assert np.all(n == 0)
    p0 = np.exp(lp0[:, 0]); p0 /= p0.sum(1, keepdims=True)
    ref = np.array([np.searchsorted(np.cumsum(p0[b]), u[b, gamma], side="right") for b in range(rows)])
    assert np.mean(tok == np.minimum(ref, V - 1)) > 0.999    # cumsum rounding may move an exact tie
    # very high temperature: both distributions become uniform, everything is accepted
    lq = lp[:, :gamma] + rng.normal(0, 1, (rows, gamma, V))
    n, _, _ = accept.spec_accept(lp, lq, x, u * 0.999, temperature=1e9)
    assert np.all(n == gamma)
    # gamma = 0 with a bonus row is plain inverse-CDF sampling
    t = accept.sample(lp[:, 0], u[:, 0])
    pp = np.exp(lp[:, 0]); pp /= pp.sum(1, keepdims=True)
    ref = np.array([np.searchsorted(np.cumsum(pp[b]), u[b, 0], side="right") for b in range(rows)])
    assert np.mean(t == np.minimum(ref, V - 1)) > 0.999


def test_temperature_is_logit_scaling():
    rng = np.random.default_rng(21)
    V, gamma, rows = 33, 4, 500
    lp = rng.normal(0, 3, (rows, gamma + 1, V))
    lq = lp[:, :gamma] + rng.normal(0, 1, (rows, gamma, V))
    x = rng.integers(0, V, (rows, gamma)).astype(np.int32)
    u = rng.random((rows, gamma + 1))
    a = accept.spec_accept(lp, lq, x, u, temperature=2.0)
    b = accept.spec_accept(lp / 2.0, lq / 2.0, x, u, temperature=1.0)
    assert all(np.array_equal(i, j) for i, j in zip(a[:2], b[:2]))
    c = accept.spec_accept(lp, lq, x, u, temperature=1.0)
    assert not np.array_equal(a[0], c[0])


def test_tie_break_and_flags():
    p = np.array([0.5, 0.3, 0.2]); q = np.array([0.2, 0.5, 0.3])
    lp, lq = np.log(p)[None, None], np.log(q)[None, None]
    rho = 0.3 / 0.5

    def run(x, u0, u1=0.5):
        n, t, f, r = accept.spec_accept(lp, lq, [[x]], [[u0, u1]], return_rho=True)
        return int(n[0]), int(t[0]), int(f[0]), r[0, 0]

    n, t, f, r = run(1, 0.59)
    assert (n, t) == (1, -1) and r == pytest.approx(rho, rel=1e-12)
    # rejected: residual max(0, p - q) = [0.3, 0, 0] -> always token 0, whatever u1
    for u1 in (0.0, 0.5, 0.999999):
        assert run(1, 0.61, u1)[:2] == (0, 0)
    # strict inequality: u == rho rejects, the next float below accepts
    exact = run(1, 0.5)[3]
    assert run(1, exact)[0] == 0 and run(1, np.nextafter(exact, 0))[0] == 1
    # rho >= 1 accepts any u < 1
    assert run(0, np.nextafter(1.0, 0))[0] == 1
    # near-tie flag: within 1e-5 of the ratio, on either side
    assert run(1, exact + 5e-6)[2] & accept.FLAG_NEAR_TIE
    assert run(1, exact - 5e-6)[2] & accept.FLAG_NEAR_TIE
    assert not run(1, exact + 1e-4)[2] & accept.FLAG_NEAR_TIE
    # zero target mass on the draft token never accepts, even at u = 0
    lpz = np.array([np.log(0.7), -np.inf, np.log(0.3)])[None, None]
    n, _, _ = accept.spec_accept(lpz, lq, [[1]], [[0.0, 0.5]])
    assert n[0] == 0


def test_stops_at_first_rejection():
    """Positions after the first rejection are not looked at (the break of Algorithm 1)."""
    rng = np.random.default_rng(2)
    V, gamma = 7, 6
    lp = rng.normal(0, 1, (1, gamma + 1, V)); lq = rng.normal(0, 1, (1, gamma, V))
    x = rng.integers(0, V, (1, gamma)).astype(np.int32)
    u = np.zeros((1, gamma + 1)); u[0, 2] = 0.999999999; u[0, gamma] = 0.3
    n, tok, _, rho = accept.spec_accept(lp, lq, x, u, return_rho=True)
    if rho[0, 2] < 1:
        assert n[0] == 2 and np.all(np.isnan(rho[0, 3:]))
        lp2, lq2 = lp.copy(), lq.copy()
        lp2[0, 3:] = 0; lq2[0, 3:] = 5            # garbage after the rejection changes nothing
        n2, tok2, _ = accept.spec_accept(lp2, lq2, x, u)
        assert (n2[0], tok2[0]) == (n[0], tok[0])


def test_rejects_bad_arguments():
    lp = np.zeros((1, 2, 4)); lq = np.zeros((1, 2, 4))
    with pytest.raises(ValueError):
        accept.spec_accept(lp, lq, [[0, 4]], [[0.1, 0.2, 0.3]])
    with pytest.raises(ValueError):
        accept.spec_accept(lp, lq, [[0, 1]], [[0.1, 0.2, 0.3]], temperature=0.0)
