"""Pins for oracle/theory.py: the paper's printed numbers (Table 1, Sec. 4.2), the
truncated-geometric expectation of Thm 3.3's proof, and the accounting identities."""
import math
import os

import numpy as np
import pytest

from oracle import theory

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table1_model_insertion.txt")


def _rows():
    out = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        out[f[0]] = [float(v) for v in f[1:]]
    return out


def test_table1_insertion_criterion():
    """Thm 3.2 first condition evaluated on Table 1's rows reproduces the ratios of Sec. 4.2."""
    rows = _rows()
    for case, (T_i, L_i_new, T_new, L_new, T_next, L_i, s0, s1, lhs_p, rhs_p) in rows.items():
        lhs, rhs = theory.insertion_gain(T_new, T_i, L_new, L_i, L_i_new)
        assert lhs == pytest.approx(lhs_p, abs=2e-3), case
        if case == "non_compliant":
            # the printed 0.117 is the magnitude: L_{i-new} < L_i makes the bracket negative
            assert rhs == pytest.approx(-rhs_p, abs=2e-3)
        else:
            assert rhs == pytest.approx(rhs_p, abs=2e-3), case
        # the criterion's verdict matches the measured change of speedup in every case
        assert (lhs < rhs) == (s1 > s0), case


def _three_terms(N, T1, T2new, T2, L1, L1p, L2p, beta):
    """The three terms of the difference (three-model time) - (two-model time) as the proof of Thm 3.2 writes
    them, with the proof's notation: T1 target, T2new the inserted model, T2 the drafter (= T_3' of the
    three-model chain), L1 the two-model acceptance length, L1p and L2p the three-model ones."""
    a = N * (1.0 / L1p - 1.0 / L1) * T1
    b = N / L2p * T2new
    c = beta * N * (1.0 / L2p - 1.0 / L1) * T2
    return a, b, c


def test_insertion_second_condition_is_the_proofs_condition_2():
    """Thm 3.2, second condition.  The proof subtracts the two-model time from the three-model time (both
    Lemma 3.1), gets three terms, and calls 'the last two terms sum to less than 0' Condition 2, which it
    rewrites as T_new/T_{i+1} < beta (L_new/L_i - 1).  Pinned here three ways: (1) the three terms really are
    the difference of the two Lemma 3.1 times, (2) the rewritten inequality holds exactly when the last two
    terms are negative, on random (T, L, beta), (3) a case worked by hand."""
    rng = np.random.default_rng(11)
    checked = 0
    for _ in range(4000):
        N = float(rng.integers(64, 4096))
        T1, T2new, T2 = rng.uniform(5, 50), rng.uniform(0.05, 30), rng.uniform(0.05, 10)
        L1 = rng.uniform(1.1, 8.0)
        L2p = rng.uniform(1.05, 12.0)
        L1p = rng.uniform(1.05, 14.0)
        beta = rng.uniform(0.2, 12.0)
        a, b, c = _three_terms(N, T1, T2new, T2, L1, L1p, L2p, beta)
        # (1) the difference of Lemma 3.1 for n = 3 and n = 2 (same beta, drafter unchanged)
        diff = theory.lemma31_time(N, [L1p, L2p], [T1, T2new, T2], beta) - theory.lemma31_time(N, [L1], [T1, T2], beta)
        assert a + b + c == pytest.approx(diff, rel=1e-9, abs=1e-9 * (abs(a) + abs(b) + abs(c)))
        lhs, rhs = theory.insertion_gain_lower(T2new, T2, L2p, L1, beta)
        lhs1, rhs1 = theory.insertion_gain(T2new, T1, L2p, L1, L1p)
        # (2) the printed inequalities are the proof's pair sums (skip knife-edge cases)
        if abs(b + c) > 1e-9 * (abs(b) + abs(c)):
            assert (lhs < rhs) == (b + c < 0)
            checked += 1
        if abs(a + b) > 1e-9 * (abs(a) + abs(b)):
            assert (lhs1 < rhs1) == (a + b < 0)
        # under the proof's premise L1' > L2' > L1 each condition alone makes the insertion pay off
        if L1p > L2p > L1 and (lhs < rhs or lhs1 < rhs1):
            assert diff < 0
    assert checked > 3500
    # (3) by hand: T_new = 7, T_{i+1} = 4, L_new = 4.67, L_i = 4.34, beta = 1.5:
    #     lhs = 7/4 = 1.75; rhs = 1.5 * (4.67/4.34 - 1) = 1.5 * 0.0760369 = 0.1140553
    lhs, rhs = theory.insertion_gain_lower(7.0, 4.0, 4.67, 4.34, 1.5)
    assert lhs == pytest.approx(1.75, abs=1e-12)
    assert rhs == pytest.approx(0.1140553, abs=1e-6)
    # and one where it holds: a cheap inserted model that lengthens the drafter-side blocks 3x, beta = 4
    lhs, rhs = theory.insertion_gain_lower(2.0, 1.0, 9.0, 3.0, 4.0)
    assert (lhs, rhs) == (2.0, 8.0)
    a, b, c = _three_terms(100.0, 20.0, 2.0, 1.0, 3.0, 10.0, 9.0, 4.0)
    assert b + c == pytest.approx(100 / 9 * 2 + 4 * 100 * (1 / 9 - 1 / 3) * 1) and b + c < 0


def test_neither_condition_is_necessary():
    """The theorem is worded 'if and only if' but its proof shows sufficiency only: all three terms together
    can be negative while neither pair is.  A worked counter-example (kept so that callers do not read a
    failed criterion as 'the insertion cannot pay off')."""
    # terms a = -3, b = 4, c = -3 (N = 1): 1/L1' - 1/L1 = -0.3 with T1 = 10; T2new/L2' = 4; beta (1/L2' - 1/L1) T2 = -3
    L1, L1p, L2p = 2.0, 5.0, 2.5
    T1, T2new, T2, beta = 10.0, 10.0, 30.0, 1.0
    a, b, c = _three_terms(1.0, T1, T2new, T2, L1, L1p, L2p, beta)
    assert (a, b, c) == pytest.approx((-3.0, 4.0, -3.0))
    lhs1, rhs1 = theory.insertion_gain(T2new, T1, L2p, L1, L1p)
    lhs2, rhs2 = theory.insertion_gain_lower(T2new, T2, L2p, L1, beta)
    assert not lhs1 < rhs1 and not lhs2 < rhs2
    assert theory.lemma31_time(1.0, [L1p, L2p], [T1, T2new, T2], beta) < theory.lemma31_time(1.0, [L1], [T1, T2], beta)


def test_expected_tokens_matches_pmf_sum():
    for alpha in (0.0, 0.3, 0.5, 0.8026, 0.9, 0.99):
        for n in (1, 2, 5, 9, 11, 17):
            pmf = theory.tokens_per_verify_pmf(alpha, n)
            assert sum(pmf) == pytest.approx(1.0, abs=1e-12)
            mean = sum(k * w for k, w in enumerate(pmf, start=1))
            assert theory.expected_tokens(alpha, n) == pytest.approx(mean, rel=1e-12)


def test_variance_special_cases():
    # a single trial has no spread; the untruncated geometric has alpha / (1-alpha)^2
    for alpha in (0.1, 0.5, 0.9):
        assert theory.variance_tokens(alpha, 1) == pytest.approx(0.0, abs=1e-15)
        assert theory.variance_tokens(alpha, 4000) == pytest.approx(alpha / (1 - alpha) ** 2, rel=1e-9)
    # closed form of the direct sum
    for alpha, n in ((0.8, 9), (0.5, 2), (0.3, 1), (0.9, 11)):
        closed = (alpha - (2 * n - 1) * alpha ** n + (2 * n - 1) * alpha ** (n + 1)
                  - alpha ** (2 * n)) / (1 - alpha) ** 2
        assert theory.variance_tokens(alpha, n) == pytest.approx(closed, abs=1e-12)


def test_lemma31_is_eq2_with_measured_lengths():
    """With L_i := N/F_i and beta := F_n L_{n-1}/N, Lemma 3.1 is Eq. (2) exactly."""
    N = 512
    F = [61, 140, 700]
    T = [2.1e-3, 0.4e-3, 0.2e-3]
    L = [N / F[0], N / F[1]]
    beta = F[2] * L[1] / N
    assert theory.lemma31_time(N, L, T, beta) == pytest.approx(theory.total_time(F, T), rel=1e-12)


def test_gaussian_noise_acceptance_rate():
    assert theory.acceptance_rate_gaussian_logit_noise(0.5) == pytest.approx(0.8026, abs=1e-4)
    assert theory.acceptance_rate_gaussian_logit_noise(0.25) == pytest.approx(0.9005, abs=1e-4)
    assert theory.acceptance_rate_gaussian_logit_noise(1.0) == pytest.approx(0.6171, abs=1e-4)
    # Monte-Carlo check of the limit itself at a large vocabulary
    rng = np.random.default_rng(7)
    lp = rng.normal(0, 2, 200000)
    lq = lp + rng.normal(0, 0.5, lp.size)
    p = np.exp(lp - lp.max()); p /= p.sum()
    q = np.exp(lq - lq.max()); q /= q.sum()
    assert 1 - 0.5 * np.abs(p - q).sum() == pytest.approx(0.8026, abs=0.01)
