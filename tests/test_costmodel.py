"""The product's cost-model helper against the oracle's closed forms and the paper's Table 1."""
import os

import pytest

from oracle import theory
from paper_2510_26527_amd import costmodel

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table1_model_insertion.txt")


def test_report_reproduces_eq2_and_lemma31():
    N, F, ms = 512, [61, 140, 700], [61 * 2.1, 140 * 0.4, 700 * 0.2]
    rep = costmodel.chain_report(N, F, ms, accept_ms=3.0, wall_ms=300.0)
    assert rep["eq2_ms"] == pytest.approx(theory.total_time(F, rep["T_ms"]))
    assert rep["lemma31_ms"] == pytest.approx(theory.lemma31_time(N, rep["L"], rep["T_ms"], rep["beta"]))
    assert rep["lemma31_ms"] == pytest.approx(rep["eq2_ms"])
    assert rep["other_ms"] == pytest.approx(300.0 - rep["eq2_ms"] - 3.0)


def test_insertion_criterion_on_table1():
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        T_i, L_i_new, T_new, L_new, T_next, L_i, s0, s1 = (float(v) for v in f[1:9])
        c1, c2, helps = costmodel.insertion_criterion(T_new, T_i, T_next, L_new, L_i, L_i_new, beta=1.0)
        assert c1 == pytest.approx(theory.insertion_gain(T_new, T_i, L_new, L_i, L_i_new))
        assert c2 == pytest.approx(theory.insertion_gain_lower(T_new, T_next, L_new, L_i, 1.0))
        assert (c1[0] < c1[1]) == (s1 > s0), f[0]


def test_insertion_criterion_matches_the_oracle_on_random_inputs():
    import numpy as np
    rng = np.random.default_rng(5)
    for _ in range(500):
        T_new, T_i, T_next = rng.uniform(0.1, 30, 3)
        L_new, L_i, L_i_new = rng.uniform(1.05, 12, 3)
        beta = rng.uniform(0.2, 10)
        c1, c2, helps = costmodel.insertion_criterion(T_new, T_i, T_next, L_new, L_i, L_i_new, beta)
        o1 = theory.insertion_gain(T_new, T_i, L_new, L_i, L_i_new)
        o2 = theory.insertion_gain_lower(T_new, T_next, L_new, L_i, beta)
        assert c1 == pytest.approx(o1, rel=1e-12) and c2 == pytest.approx(o2, rel=1e-12)
        assert helps == ((o1[0] < o1[1]) or (o2[0] < o2[1]))
        d = costmodel.insertion_time_change(1.0, T_new, T_i, T_next, L_new, L_i, L_i_new, beta)
        ref = theory.lemma31_time(1.0, [L_i_new, L_new], [T_i, T_new, T_next], beta) - \
            theory.lemma31_time(1.0, [L_i], [T_i, T_next], beta)
        assert d == pytest.approx(ref, rel=1e-9, abs=1e-12)
