"""The paper's cost model evaluated on measured runs (host arithmetic on a handful of numbers).

Eq. (2): T = sum_i F_i T_i.  Lemma 3.1: T = sum_{i<n} (N / L_i) T_i + beta (N / L_{n-1}) T_n, which is
Eq. (2) once L_i is read as tokens committed per forward pass of level i (L_i = N / F_i) and
beta as draft forwards per forward of the level above it (beta = F_n L_{n-1} / N).
Theorem 3.2 gives the conditions under which inserting a model between two levels pays off.
"""


def chain_report(n_tokens, forwards, level_ms, accept_ms=0.0, wall_ms=None):
    """forwards[i], level_ms[i]: forward-pass count and summed forward time of level i (target first)."""
    n = len(forwards)
    T = [level_ms[i] / forwards[i] if forwards[i] else 0.0 for i in range(n)]
    L = [n_tokens / forwards[i] if forwards[i] else float("inf") for i in range(n - 1)]
    eq2 = sum(f * t for f, t in zip(forwards, T))
    rep = {"N": n_tokens, "F": list(forwards), "T_ms": T, "L": L, "eq2_ms": eq2, "accept_ms": accept_ms}
    if n >= 2:
        beta = forwards[n - 1] * L[n - 2] / n_tokens
        lemma = sum(n_tokens / L[i] * T[i] for i in range(n - 1)) + beta * n_tokens / L[n - 2] * T[n - 1]
        rep.update(beta=beta, lemma31_ms=lemma)
    if wall_ms is not None:
        rep.update(wall_ms=wall_ms, other_ms=wall_ms - eq2 - accept_ms)
    return rep


def insertion_criterion(T_new, T_i, T_next, L_new, L_i, L_i_new, beta):
    """Theorem 3.2.  Inserting M_new between M_i and M_{i+1} is predicted to reduce the total time if
    T_new/T_i < L_new (1/L_i - 1/L_{i-new})   or   T_new/T_{i+1} < beta (L_new/L_i - 1).
    Returns ((lhs1, rhs1), (lhs2, rhs2), helps)."""
    c1 = (T_new / T_i, L_new * (1.0 / L_i - 1.0 / L_i_new))
    c2 = (T_new / T_next, beta * (L_new / L_i - 1.0))
    return c1, c2, (c1[0] < c1[1]) or (c2[0] < c2[1])


def insertion_time_change(N, T_new, T_i, T_next, L_new, L_i, L_i_new, beta):
    """The quantity the proof of Theorem 3.2 starts from: (three-model time) - (two-model time) by Lemma 3.1
    with the same beta and an unchanged drafter,
        N (1/L_{i-new} - 1/L_i) T_i + (N/L_new) T_new + beta N (1/L_new - 1/L_i) T_{i+1}.
    Negative: the insertion is predicted to pay off.  The theorem's two conditions say that the first two, or
    the last two, of these terms already sum to less than zero; each is sufficient when
    L_{i-new} > L_new > L_i, neither is necessary."""
    return (N * (1.0 / L_i_new - 1.0 / L_i) * T_i + N / L_new * T_new
            + beta * N * (1.0 / L_new - 1.0 / L_i) * T_next)
