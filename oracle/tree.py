"""CPU oracle (test infrastructure only): token-tree verification by multi-round speculative sampling.

The paper lists token-tree-based verification beside greedy matching and speculative sampling as a verification
mechanism (Related Work, "Verification Mechanisms") and names deeper / wider drafting as the next step
(Sec. 4.6); it prints no rule for it.  The rule below is the standard one for a tree whose sibling tokens are
independent draws from the drafter's distribution at their parent: try the children of a node one after the
other against the residual of the verifier's distribution there, descend into the first child that is accepted,
and when none is (or the node is a leaf) emit one token from what is left of the verifier's distribution.  With
one child per node it is the linear rule of oracle/accept.c; like that rule it must leave the verifier's
distribution unchanged (Abstract; Sec. 3.1), which is what tests/test_oracle_tree.py pins.

Plain numpy fp64, sequential loops, nothing blocked or reordered.
"""
import numpy as np


def _softmax(logits, temperature):
    s = np.asarray(logits, np.float64) / temperature
    e = np.exp(s - s.max())
    return e / e.sum()


def _draw(weights, u):
    """Smallest k with sum_{i<=k} w_i > u * sum(w); the last index with positive weight if rounding leaves none."""
    total = 0.0
    for w in weights:
        total += w
    t = u * total
    c, last = 0.0, -1
    for k, w in enumerate(weights):
        if w > 0.0:
            last = k
        c += w
        if c > t:
            return k
    return last


def tree_accept(p_logits, q_logits, tokens, parents, uniforms, temperature=1.0, tie_eps=1e-5, return_flags=False):
    """One verification of a drafted token tree.

    Nodes are numbered 0..n-1 in an order in which every parent precedes its children; node 0 is the root (the
    last committed token, which carries no drafted token).  parents[i] is the parent of node i (parents[0] = -1);
    the children of a node are tried in increasing index order.
      p_logits [n, V]  verifier's logits after the path ending in each node
      q_logits [n, V]  drafter's logits after the same path: the tokens of a node's children are independent
                       draws from softmax(q_logits[node] / T)
      tokens   [n]     drafted token of each node (tokens[0] is ignored)
      uniforms [n + 1] u[i] decides node i when it is tried (i >= 1; u[0] is unused), u[n] drives the one draw
    Returns (path, token): the accepted nodes from the root downwards (root excluded) and the token emitted after
    them.  The step commits tokens[path[0]], ..., tokens[path[-1]], token.  With return_flags a third value: bit 0
    set when some tested uniform lay within tie_eps of its acceptance probability (a decision rounding could flip)."""
    p_logits = np.asarray(p_logits, np.float64)
    q_logits = np.asarray(q_logits, np.float64)
    n = p_logits.shape[0]
    children = [[] for _ in range(n)]
    for i in range(1, n):
        if not 0 <= parents[i] < i:
            raise ValueError("parents must precede their children")
        children[parents[i]].append(i)
    path, node, flags = [], 0, 0
    while True:
        r = _softmax(p_logits[node], temperature)          # what is left of the verifier's distribution here
        q = _softmax(q_logits[node], temperature)
        descended = False
        for c in children[node]:
            x = int(tokens[c])
            ratio = np.inf if q[x] == 0.0 else r[x] / q[x]
            if abs(uniforms[c] - min(1.0, ratio)) < tie_eps:
                flags |= 1
            if uniforms[c] < min(1.0, ratio):
                path.append(c)
                node = c
                descended = True
                break
            rest = np.maximum(r - q, 0.0)                  # this sibling is refused: take the drafter's share out
            mass = rest.sum()
            if mass > 0.0:
                r = rest / mass                            # (mass 0 means r == q, where no refusal can happen)
        if not descended:
            token = _draw(r, uniforms[n])
            return (path, token, flags) if return_flags else (path, token)


def tree_greedy_accept(p_logits, tokens, parents):
    """Greedy matching on a tree (Related Work, "Verification Mechanisms"): at every node the verifier's most likely
    token (lowest index among equals) is compared with the children's tokens; the first child that carries it is
    descended into, and where none does that token is emitted.  Returns (path, token)."""
    p_logits = np.asarray(p_logits, np.float64)
    n = p_logits.shape[0]
    children = [[] for _ in range(n)]
    for i in range(1, n):
        if not 0 <= parents[i] < i:
            raise ValueError("parents must precede their children")
        children[parents[i]].append(i)
    path, node = [], 0
    while True:
        best = int(np.argmax(p_logits[node]))
        nxt = next((c for c in children[node] if int(tokens[c]) == best), None)
        if nxt is None:
            return path, best
        path.append(nxt)
        node = nxt
