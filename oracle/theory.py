"""CPU oracle (test infrastructure only): the paper's cost model and stability formulas.

Plain closed forms and direct sums, each next to the passage it restates.
"""
import math


def total_time(F, T):
    """Eq. (2): T = sum_i F_i * T_i (forward-pass counts times per-forward costs)."""
    return sum(f * t for f, t in zip(F, T))


def lemma31_time(N, L, T, beta):
    """Lemma 3.1: T = sum_{i<n} (N / L_i) T_i + beta (N / L_{n-1}) T_n for an n-model chain;
    L has n-1 entries (verifying levels, target first), T has n."""
    n = len(T)
    assert len(L) == n - 1
    return sum(N / L[i] * T[i] for i in range(n - 1)) + beta * N / L[n - 2] * T[n - 1]


def insertion_gain(T_new, T_i, L_new, L_i, L_i_new):
    """Theorem 3.2, first condition.  Returns (lhs, rhs): inserting M_new between M_i and
    M_{i+1} is predicted to help when lhs = T_new/T_i < rhs = L_new (1/L_i - 1/L_{i-new})."""
    return T_new / T_i, L_new * (1.0 / L_i - 1.0 / L_i_new)


def insertion_gain_lower(T_new, T_next, L_new, L_i, beta):
    """Theorem 3.2, second condition, in the form its proof derives (Condition 2):
    T_new/T_{i+1} < beta (L_new / L_i - 1)."""
    return T_new / T_next, beta * (L_new / L_i - 1.0)


def tokens_per_verify_pmf(alpha, n):
    """Proof of Theorem 3.3: truncated geometric with at most n trials.  With per-token
    acceptance rate alpha (the proof's 1-p), N = k < n has probability (1-alpha) alpha^(k-1)
    and N = n has alpha^(n-1).  N counts tokens produced per verification (accepted + 1),
    n = gamma + 1."""
    pmf = [(1.0 - alpha) * alpha ** (k - 1) for k in range(1, n)]
    pmf.append(alpha ** (n - 1))
    return pmf


def expected_tokens(alpha, n):
    """E[N] = (1 - alpha^n) / (1 - alpha), the expectation printed in the proof of Thm 3.3."""
    if alpha == 1.0:
        return float(n)
    return (1.0 - alpha ** n) / (1.0 - alpha)


def variance_tokens(alpha, n):
    """Var(N) from the proof's definition E[N^2] = sum_{k<n} k^2 p (1-p)^(k-1) + n^2 (1-p)^(n-1),
    by direct summation.  (The closed forms the paper prints for S, E[N^2] and sigma^2 do not
    satisfy this sum - e.g. they give a non-zero variance at n = 1 - so they are not used.)"""
    pmf = tokens_per_verify_pmf(alpha, n)
    m1 = sum(k * w for k, w in enumerate(pmf, start=1))
    m2 = sum(k * k * w for k, w in enumerate(pmf, start=1))
    return m2 - m1 * m1


def acceptance_rate_gaussian_logit_noise(sigma):
    """Large-vocabulary limit of alpha = 1 - TV(p, q) when q's logits are p's plus
    independent N(0, sigma^2) noise: 2 * Phi(-sigma / 2)."""
    return math.erfc(sigma / (2.0 * math.sqrt(2.0)))
