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
