"""Pins for the CPU oracle of token-tree verification (oracle/tree.py).

What fixes the rule is that the verifier's distribution is preserved (Abstract; Sec. 3.1; Conclusion): the law of
the first committed token, measured from the code by bisection over its uniforms and summed over every tuple of
sibling tokens with the drafter's probabilities, must be the verifier's p exactly; a long stream decoded by
repeated tree steps from Markov-table models must follow the verifier's transition matrix (and not the
drafter's); and a tree with one child per node must decide exactly as the linear rule of oracle/accept.c."""
import itertools

import numpy as np
import pytest
from scipy import stats

from oracle import accept, tree


def _rand_dist(rng, V):
    return rng.dirichlet(np.full(V, 1.0))


def _bisect(pred):
    """sup{u in [0,1) : pred(u)} for a predicate that is true below a threshold."""
    if pred(np.nextafter(1.0, 0.0)):
        return 1.0
    if not pred(0.0):
        return 0.0
    lo, hi = 0.0, 1.0
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        if pred(mid):
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def _first_token_law(lp, lq, xs):
    """Law of the first committed token of a one-level tree whose k children carry the tokens xs, measured from the
    code: child i is reached with every earlier sibling refused (their uniforms just below 1)."""
    k, V = len(xs), lp.shape[0]
    n = k + 1
    P = np.tile(lp, (n, 1))
    Q = np.tile(lq, (n, 1))
    parents = [-1] + [0] * k
    tokens = [0] + list(xs)
    top = np.nextafter(1.0, 0.0)
    law, reach = np.zeros(V), 1.0
    for i in range(1, k + 1):
        def accepted(ui, i=i):
            u = np.full(n + 1, top)
            u[i] = ui
            path, _ = tree.tree_accept(P, Q, tokens, parents, u)
            return path[:1] == [i]
        a = _bisect(accepted)
        law[xs[i - 1]] += reach * a
        reach *= 1.0 - a
    if reach > 0.0:
        u = np.full(n + 1, top)
        edges = np.zeros(V + 1)
        edges[V] = 1.0
        for t in range(V - 1):
            def at_most(ud, t=t):
                u[n] = ud
                path, tok = tree.tree_accept(P, Q, tokens, parents, u)
                assert path == []
                return tok <= t
            edges[t + 1] = _bisect(at_most)
        law += reach * np.diff(edges)
    return law


@pytest.mark.parametrize("V,k,seed", [(2, 2, 0), (3, 2, 1), (3, 3, 2), (4, 2, 3)])
def test_first_token_law_is_the_verifiers_exactly(V, k, seed):
    rng = np.random.default_rng(seed)
    p, q = _rand_dist(rng, V), _rand_dist(rng, V)
    lp, lq = np.log(p), np.log(q)
    law = np.zeros(V)
    for xs in itertools.product(range(V), repeat=k):
        w = np.prod([q[x] for x in xs])
        law += w * _first_token_law(lp, lq, xs)
    np.testing.assert_allclose(law, p, atol=1e-9)


def test_second_sibling_is_tested_against_the_residual_not_against_p():
    """Worked by hand: p = (0.6, 0.4), q = (0.9, 0.1).  First child token 0: accepted with probability
    min(1, 0.6/0.9) = 2/3.  After its refusal the residual is norm(max(0, p - q)) = (0, 1); a second child with
    token 0 has ratio 0 (never accepted), one with token 1 has ratio 1/0.1 = 10 (always accepted)."""
    lp, lq = np.log([0.6, 0.4]), np.log([0.9, 0.1])
    P, Q = np.tile(lp, (3, 1)), np.tile(lq, (3, 1))
    top = np.nextafter(1.0, 0.0)
    assert tree.tree_accept(P, Q, [0, 0, 1], [-1, 0, 0], [0, 0.66, 0.5, 0.5]) == ([1], tree._draw([0.6, 0.4], 0.5))
    assert tree.tree_accept(P, Q, [0, 0, 1], [-1, 0, 0], [0, 0.67, top, 0.5])[0] == [2]
    assert tree.tree_accept(P, Q, [0, 0, 0], [-1, 0, 0], [0, 0.67, 0.0, 0.3]) == ([], 1)


def test_chain_shaped_tree_is_the_linear_rule():
    """One child per node: the same accepted length and emitted token as oracle/accept.c on the same uniforms."""
    rng = np.random.default_rng(5)
    V, gamma = 11, 5
    for _ in range(200):
        lp = rng.normal(0, 1.5, (gamma + 1, V))
        lq = lp[:gamma] + rng.normal(0, 0.7, (gamma, V))
        x = rng.integers(0, V, gamma)
        u = rng.random(gamma + 1)
        n, tok, _ = accept.spec_accept(lp[None], lq[None], x[None], u[None])
        Q = np.vstack([lq, np.zeros((1, V))])
        uu = np.concatenate([[0.0], u[:gamma], [u[gamma]]])
        path, t = tree.tree_accept(lp, Q, np.concatenate([[0], x]), [-1] + list(range(gamma)), uu)
        assert len(path) == n[0] and path == list(range(1, n[0] + 1)) and t == tok[0]


def test_stream_decoded_by_tree_steps_follows_the_verifiers_markov_law():
    """Repeated tree steps (depth 2, two children per node, tokens drawn i.i.d. from the drafter's table) with
    context-dependent tables: the transition counts of 60 000 emitted tokens fit the verifier's matrix (chi-square)
    and reject the drafter's."""
    rng = np.random.default_rng(11)
    V = 4
    Pm = np.stack([_rand_dist(rng, V) for _ in range(V)])
    Qm = np.stack([0.6 * Pm[a] + 0.4 * _rand_dist(rng, V) for a in range(V)])
    prev, counts, total = 0, np.zeros((V, V)), 0
    parents = [-1, 0, 0, 1, 1, 2, 2]
    while total < 60000:
        tokens = [prev, 0, 0, 0, 0, 0, 0]
        for i in range(1, 7):
            tokens[i] = int(rng.choice(V, p=Qm[tokens[parents[i]]]))
        lp = np.log(np.stack([Pm[tokens[i]] for i in range(7)]))
        lq = np.log(np.stack([Qm[tokens[i]] for i in range(7)]))
        path, tok = tree.tree_accept(lp, lq, tokens, parents, rng.random(8))
        for t in [tokens[c] for c in path] + [tok]:
            counts[prev, t] += 1
            prev = t
            total += 1
    chi_p = sum(((counts[a] - counts[a].sum() * Pm[a]) ** 2 / (counts[a].sum() * Pm[a])).sum() for a in range(V))
    chi_q = sum(((counts[a] - counts[a].sum() * Qm[a]) ** 2 / (counts[a].sum() * Qm[a])).sum() for a in range(V))
    df = V * (V - 1)
    assert stats.chi2.sf(chi_p, df) > 1e-4, chi_p
    assert stats.chi2.sf(chi_q, df) < 1e-6, chi_q


def test_greedy_tree_walk_is_greedy_decoding_and_reduces_to_the_linear_rule():
    """Every accepted node carries its parent's most likely token, the emitted token is the most likely one at the
    last node reached and no child there carries it; on a chain it is the linear greedy rule of oracle/accept.c."""
    rng = np.random.default_rng(21)
    V = 6
    parents = [-1, 0, 0, 1, 1, 2, 2, 3]
    for _ in range(300):
        lp = rng.normal(0, 1, (8, V))
        toks = rng.integers(0, V, 8)
        path, tok = tree.tree_greedy_accept(lp, toks, parents)
        node = 0
        for c in path:
            assert parents[c] == node and toks[c] == np.argmax(lp[node])
            assert all(toks[d] != np.argmax(lp[node]) for d in range(1, c) if parents[d] == node)   # the first such child
            node = c
        assert tok == np.argmax(lp[node])
        assert all(toks[d] != tok for d in range(1, 8) if parents[d] == node)
    gamma = 5
    for _ in range(200):
        lp = rng.normal(0, 1, (gamma + 1, V))
        x = rng.integers(0, V, gamma)
        n, tok = accept.greedy_accept(lp[None], x[None])
        path, t = tree.tree_greedy_accept(lp, np.concatenate([[0], x]), [-1] + list(range(gamma)))
        assert path == list(range(1, n[0] + 1)) and t == tok[0]
