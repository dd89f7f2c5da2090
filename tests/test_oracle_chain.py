"""Pins for the CPU oracle of the decoding loop (oracle/chain.py, Algorithm 1).

What the paper fixes is that the chain's output follows the target's distribution
(Abstract; Sec. 3.1; Conclusion).  Table-driven first-order Markov "models" make that
testable: the emitted stream must be a Markov chain with the target's transition matrix,
whatever the lower levels are.  Readings of Algorithm 1 that break the property (e.g. its
printed all-or-nothing top stage, or feeding the top stage the draft's rows as q) fail here.
"""
import numpy as np
import pytest
from scipy import stats

from oracle import chain as och
from oracle import theory


class TableLevel:
    """A 'model' whose next-token law depends on the previous token only."""

    def __init__(self, table):
        self.logits = np.log(table)
        self.hist = []

    @property
    def kv_len(self):
        return len(self.hist)

    def forward(self, tokens):
        self.hist += list(tokens)
        return self.logits[np.array(tokens, dtype=np.int64)]

    def truncate(self, n):
        assert n <= len(self.hist)
        del self.hist[n:]


def _tables(rng, n_levels, V, conc):
    return [np.stack([rng.dirichlet(np.full(V, conc)) for _ in range(V)]) for _ in range(n_levels)]


def _tapes(rng, n_levels, calls, width):
    return [rng.random((calls, width)) for _ in range(n_levels - 1)] + [rng.random(calls * width)]


def _transition_pvalue(seq, P, prev0):
    V = P.shape[0]
    prev = np.array([prev0] + list(seq[:-1]))
    cur = np.array(seq)
    pv = []
    for a in range(V):
        c = np.bincount(cur[prev == a], minlength=V)
        pv.append(stats.chisquare(c, P[a] * c.sum()).pvalue)
    return min(pv)


@pytest.mark.parametrize("n_levels,gammas", [(3, [None, 5, 3]), (2, [None, 4]), (4, [None, 6, 4, 2]),
                                             (1, [None])])
def test_stream_follows_target_markov_law(n_levels, gammas):
    rng = np.random.default_rng(100 + n_levels)
    V, N = 4, 60000
    tabs = _tables(rng, n_levels, V, 2.0)
    levels = [TableLevel(t) for t in tabs]
    ch = och.Chain(levels, gammas, _tapes(rng, n_levels, 3 * N, 8))
    out = ch.generate([1, 3], N)
    assert len(out) == N
    assert _transition_pvalue(out, tabs[0], 3) > 1e-4 / V
    # and it is distinguishable from the next level's law (the test has power)
    if n_levels > 1:
        assert _transition_pvalue(out, tabs[1], 3) < 1e-8
    # every level's cache ends consistent with the text
    full = [1, 3] + out
    for lvl in levels:
        assert lvl.hist == full[:len(lvl.hist)]


def test_printed_all_or_nothing_top_stage_would_be_biased():
    """Algorithm 1 as printed commits the whole block or samples one fresh token; simulate
    that rule on the same tables and see the transition test reject it - the reason the
    oracle commits the accepted prefix instead."""
    rng = np.random.default_rng(42)
    V, N, g = 4, 60000, 3
    P, Q = _tables(rng, 2, V, 2.0)
    out, prev = [], 3
    while len(out) < N:
        xs, pv, ok = [], prev, True
        for _ in range(g):
            x = rng.choice(V, p=Q[pv])
            ok = ok and rng.random() < min(1.0, P[pv, x] / Q[pv, x])
            xs.append(x); pv = x
        if ok:
            out += xs
        else:
            out.append(rng.choice(V, p=P[prev]))
        prev = out[-1]
    assert _transition_pvalue(out[:N], P, 3) < 1e-8


def test_counts_and_lemma31_identity():
    rng = np.random.default_rng(7)
    V, N = 6, 4000
    tabs = _tables(rng, 3, V, 3.0)
    levels = [TableLevel(t) for t in tabs]
    ch = och.Chain(levels, [None, 8, 4], _tapes(rng, 3, 3 * N, 10))
    out = ch.generate([0], N)
    F = ch.stats.forwards
    # one accept per verifying forward; block sizes never exceed gamma; accepted <= block
    for i in (0, 1):
        assert F[i] == len(ch.stats.accept_lens[i]) == len(ch.stats.block_lens[i])
        assert max(ch.stats.block_lens[i]) <= [8, 4][i]
        assert all(0 <= n <= k for n, k in zip(ch.stats.accept_lens[i], ch.stats.block_lens[i]))
    # the target commits accepted + 1 tokens per forward, except that the last block may be cut
    committed = sum(n + 1 for n in ch.stats.accept_lens[0])
    assert N <= committed <= N + 1
    # Lemma 3.1 with L_i = N / F_i and beta = F_n L_{n-1} / N reproduces Eq. (2)
    T = [3.0, 1.0, 0.1]
    L = [N / F[0], N / F[1]]
    assert theory.lemma31_time(N, L, T, F[2] * L[1] / N) == pytest.approx(theory.total_time(F, T))


def test_deterministic_given_tapes_and_trace_is_replayable():
    rng = np.random.default_rng(1)
    tabs = _tables(rng, 3, 5, 2.0)
    tapes = _tapes(rng, 3, 400, 8)
    runs = []
    for _ in range(2):
        ch = och.Chain([TableLevel(t) for t in tabs], [None, 4, 2], tapes, trace=True)
        runs.append((ch.generate([2, 2, 4], 100), ch.stats.events))
    assert runs[0][0] == runs[1][0]
    kinds = [e[0] for e in runs[0][1]]
    assert kinds.count("accept") == sum(1 for e in runs[0][1] if e[0] == "forward" and e[1] < 2)
