"""Synthetic-agreement harness for chains of random-init models (workload: full 3-level chain).

Independent random-init networks agree with each other at a fixed, low rate, so the acceptance
lengths of a chain built from them cannot be set.  This harness, which is outside the library,
sets them: every level below the target still runs its real forward (that is what gets timed
and counted as T_i in Eq. (2)), but the logits rows it hands on are replaced by

    l_i(prefix) = l_target(prefix) + sigma * (N_1[pos] + ... + N_i[pos]),        i >= 1,

where l_target(prefix) comes from an untimed extra forward of the target over the same prefix
(its KV length is restored afterwards) and N_j[pos] is a standard normal vector that depends
only on (seed, level j, absolute position).  Adjacent levels then differ by one sigma*N(0, I)
perturbation of the logits, for which the per-token acceptance rate 1 - TV tends, for a large
vocabulary, to 2*Phi(-sigma/2).  Tokens are still exact draws from the rows that later serve as
q, so the acceptance rule is exercised exactly as in a chain of trained models.
"""
import torch

import paper_2510_26527_amd as psd
from paper_2510_26527_amd.chain import Chain


class AgreementShimChain(Chain):
    def __init__(self, levels, gammas, tapes, sigma, noise_seed=0, noise_terms=None, **kw):
        """noise_terms[i]: how many of the N_j vectors level i's rows carry (default i: each level one more than
        the level above it; a two-level chain whose draft should sit as far from the target as the draft of a
        three-level chain passes [0, 2]; 0 for a level below the target leaves that level's own
        logits in place, e.g. a quantised copy of the target that needs no help to agree with it)."""
        super().__init__(levels, gammas, tapes, **kw)
        self.noise_terms = list(noise_terms) if noise_terms is not None else list(range(len(levels)))
        tgt = levels[0]
        self.sigma = float(sigma)
        self.noise_seed = int(noise_seed)
        self.vocab = tgt.model.shape.vocab
        self.peek_rows = torch.empty((tgt.max_rows + 2, self.vocab), dtype=torch.float32, device=self.dev)
        self._gen = torch.Generator(device=self.dev)
        self.peeks = 0
        self.peek_ms = 0.0
        self._peek_pending = []

    def _noise(self, level, pos):
        self._gen.manual_seed((self.noise_seed * 1000003 + level) * 1000003 + pos)
        return torch.randn(self.vocab, dtype=torch.float32, device=self.dev, generator=self._gen)

    def _rows_ready(self, i, dst, n_logit_rows):
        if i == 0 or dst is None or n_logit_rows == 0 or self.noise_terms[i] == 0:
            return             # the target, or a level that keeps its own logits (noise_terms 0)
        tgt = self.levels[0]
        keep = tgt.kv_len
        n_new = self.seq_len - keep
        assert n_logit_rows <= n_new <= self.peek_rows.shape[0]
        peek = self.peek_rows[:n_logit_rows]
        if self.timed:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
        psd.psd_model_forward(tgt.model.handle, self.seq[keep:self.seq_len], n_new, tgt.kv.handle, peek,
                              n_logit_rows, tgt.ws)
        psd.psd_kv_truncate_to(tgt.kv.handle, keep)
        if self.timed:
            e1.record()
            self._peek_pending.append((e0, e1))
        self.peeks += 1
        for r in range(n_logit_rows):
            pos = self.seq_len - n_logit_rows + r + 1            # index of the token row r predicts
            noise = self._noise(1, pos)
            for j in range(2, self.noise_terms[i] + 1):
                noise = noise + self._noise(j, pos)
            torch.add(peek[r], noise, alpha=self.sigma, out=dst[r])

    def generate(self, prompt, n_generate):
        out = super().generate(prompt, n_generate)
        if self.timed:
            self.peek_ms = sum(a.elapsed_time(b) for a, b in self._peek_pending)
            self._peek_pending = []
        return out
