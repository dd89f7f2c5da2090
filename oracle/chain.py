"""CPU oracle (test infrastructure only): the polybasic decoding loop.

Algorithm 1 (three models) made exact and written for an n-level chain
M_1 (target) ... M_n (draft), Sec. 3.1: the lowest level drafts, every level
above verifies the block handed up by the level below it "in ascending
order", and the target's output distribution is preserved.

Readings taken where Algorithm 1 is silent or inconsistent (each is pinned by
tests/test_oracle_chain.py through the distribution-preservation property):
  * drafting continues from the committed text plus the tokens already
    validated by the level above (Alg. 1 line 7 drafts from x_{<=t} although
    `accepted` has grown);
  * a verify forward is fed the last token that is not yet in that level's KV
    cache followed by the k proposed tokens, giving k+1 logits rows;
  * every stage applies full speculative sampling: accepted prefix plus one
    token drawn from the residual (or from the extra row if all k were
    accepted).  That token is an exact draw from the verifying level, so the
    proposal distribution seen by the next level up is the verifying level's
    own logits row at that position;
  * the top stage commits the accepted prefix (Sec. 3.3 "partial acceptance /
    partial rollback"), not all-or-nothing;
  * a level hands up exactly gamma tokens per block (the threshold mu of
    "Staged Verification"): the last inner round drafts
    min(gamma_below, room left) tokens and the extra token of a fully
    accepted block is dropped when there is no room for it.

A level is any object with
    forward(tokens: list[int]) -> float array [len(tokens), V]   (appends to its KV)
    kv_len: int                                                  (tokens in its KV)
    truncate(new_len: int)
Level 0 is the target.  gammas[i] (i >= 1) is the number of tokens level i hands
to level i-1 per verification.  tapes[i] supplies the uniforms: for a verifying
level a float array [calls, >= gamma+1] (row c serves that level's c-th accept
call: slots 0..k-1 the ratio tests, slot k the one draw); for the draft a flat
array, one uniform per sampled token.
"""
from dataclasses import dataclass, field

import numpy as np

from . import accept as _accept


@dataclass
class ChainStats:
    forwards: list                      # F_i, forward passes per level (prefill excluded)
    accept_lens: list                   # per verifying level: list of accepted counts n
    block_lens: list                    # per verifying level: list of block sizes k
    events: list = field(default_factory=list)   # optional trace, see generate(trace=True)


class Chain:
    def __init__(self, levels, gammas, tapes, temperature=1.0, trace=False):
        self.levels = levels
        self.n = len(levels)
        self.gammas = gammas
        self.tapes = tapes
        self.T = float(temperature)
        self.calls = [0] * self.n
        self.seq = []
        self.trace = trace
        self.stats = ChainStats([0] * self.n, [[] for _ in range(self.n)],
                                [[] for _ in range(self.n)])

    def _forward(self, i):
        """Feed level i every token of the sequence its KV does not hold yet."""
        lvl = self.levels[i]
        start = lvl.kv_len
        toks = self.seq[start:]
        rows = np.asarray(lvl.forward(list(toks)), dtype=np.float64)
        self.stats.forwards[i] += 1
        if self.trace:
            self.stats.events.append(("forward", i, start, list(toks), rows.copy()))
        return rows

    def _produce(self, i, want):
        """Append `want` tokens to the sequence, each an exact draw from level i given its
        prefix, and return [(token, level-i logits row it was drawn from / validated by)]."""
        out = []
        if i == self.n - 1:                                   # the draft: plain sampling
            for _ in range(want):
                row = self._forward(i)[-1]
                u = self.tapes[i][self.calls[i]]
                self.calls[i] += 1
                tok = int(_accept.sample(row[None, :], [u], self.T)[0])
                self.seq.append(tok)
                out.append((tok, row))
            return out
        while len(out) < want:
            k = min(self.gammas[i + 1], want - len(out))
            base = len(self.seq)
            block = self._produce(i + 1, k)
            rows = self._forward(i)
            p = rows[-(k + 1):]
            q = np.stack([r for (_, r) in block])
            x = np.array([t for (t, _) in block], np.int32)
            u = np.asarray(self.tapes[i][self.calls[i]][:k + 1], np.float64)
            self.calls[i] += 1
            n, tok, flags, rho = _accept.spec_accept(p[None], q[None], x[None], u[None], self.T,
                                                     return_rho=True)
            n, tok = int(n[0]), int(tok[0])
            self.stats.accept_lens[i].append(n)
            self.stats.block_lens[i].append(k)
            if self.trace:
                self.stats.events.append(("accept", i, k, x.copy(), u.copy(), n, tok, int(flags[0])))
            del self.seq[base + n:]
            for j in range(i, self.n):                        # roll every lower cache back too
                if self.levels[j].kv_len > base + n:
                    self.levels[j].truncate(base + n)
            out += [(int(x[j]), p[j]) for j in range(n)]
            if len(out) < want:
                self.seq.append(tok)
                out.append((tok, p[n]))
        return out

    def prefill(self, prompt):
        """Put prompt[:-1] into every level's KV; the last prompt token is the first x*."""
        self.seq = list(int(t) for t in prompt)
        for lvl in self.levels:
            if len(self.seq) > 1:
                lvl.forward(self.seq[:-1])

    def generate(self, prompt, n_generate):
        """Generate exactly n_generate tokens after the prompt; returns them as a list."""
        self.prefill(prompt)
        start = len(self.seq)
        self._produce(0, n_generate)
        return self.seq[start:start + n_generate]
