"""Host loop of polybasic speculative decoding over the C boundary (Algorithm 1, n levels).

Only orchestration lives here: which model runs next, on which tokens, and where its
outputs land.  Every tensor stays on the GPU:
  * the token sequence is one device int32 buffer; a drafted token is written by
    psd_spec_accept (gamma = 0, plain sampling) straight into its slot, so drafting needs no
    host round trip;
  * a verifying level's forward writes its logits rows straight into that level's row buffer
    at the offset of the block being verified; those rows are, with no copy, the proposal
    rows q of the next level up (the verified tokens are exact draws from them);
  * per verification the host reads back two integers (accepted count and emitted token),
    which it needs to steer the loop, then rolls every cache at or below that level back with
    psd_kv_truncate_to.

Readings of Algorithm 1 used here: drafting continues after the tokens already validated; every
stage commits the accepted prefix plus one corrected or bonus token; a level hands up exactly
gamma tokens.  The per-level counters F_i and the event timers T_i feed the
cost model of Eq. (2) and Lemma 3.1 (costmodel.py).
"""
import numpy as np
import torch

import paper_2510_26527_amd as psd
from paper_2510_26527_amd import runtime


class Level:
    """One model of the chain with its batch-1 KV cache and logits row buffer."""

    def __init__(self, model: runtime.Model, max_len: int, max_rows: int):
        self.model = model
        self.kv = runtime.KVCache(model, 1, max_len)
        self.kv_len = 0
        self.rows = torch.empty((max_rows, model.shape.vocab), dtype=torch.float32, device=model.device)
        self.max_rows = max_rows
        self.ws = model.workspace_upto(1, max_rows + 2, max_len)
        self.forwards = 0
        self.time_ms = 0.0
        self._pending = []

    def close(self):
        self.kv.close()


class Chain:
    def __init__(self, levels, gammas, tapes, temperature=1.0, max_len=None, trace=False, timed=False, sink=None):
        """levels[0] is the target; gammas[i] (i >= 1) the block size level i hands to level i-1;
        tapes[i] float32 [calls, >= gamma+1] for verifying levels, flat for the draft.
        trace: record every forward / sample / accept with its tensors, into self.events or, if
        given, by calling sink(event) at once (a long run then keeps no copies)."""
        self.levels = levels
        self.n = len(levels)
        self.gammas = gammas
        self.dev = levels[0].model.device
        self.T = float(temperature)
        self.tapes = [torch.as_tensor(np.ascontiguousarray(t), dtype=torch.float32).to(self.dev) for t in tapes]
        self.calls = [0] * self.n
        self.max_len = max_len or levels[0].kv.max_len
        self.seq = torch.zeros(self.max_len + 64, dtype=torch.int32, device=self.dev)
        self.seq_len = 0
        self.acc = [runtime.Acceptor(self.dev) for _ in range(self.n)]
        self.out = torch.zeros((self.n, 4), dtype=torch.int32, device=self.dev)
        self.trace = trace
        self.timed = timed
        self.events = []
        self._emit = sink if sink is not None else self.events.append
        self.accept_lens = [[] for _ in range(self.n)]
        self.block_lens = [[] for _ in range(self.n)]
        self.accept_ms = 0.0
        self.forward_log = None       # a list: every forward is recorded there as (level, first position, tokens)

    # -------------------------------------------------------------- one forward of level i
    def _forward(self, i, n_logit_rows, out_row):
        """Feed level i every token its cache lacks; the last n_logit_rows logits rows land at
        rows[out_row:]."""
        lvl = self.levels[i]
        start, n_new = lvl.kv_len, self.seq_len - lvl.kv_len
        toks = self.seq[start:self.seq_len]
        dst = lvl.rows[out_row:out_row + n_logit_rows] if n_logit_rows else None
        if self.timed:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
        psd.psd_model_forward(lvl.model.handle, toks, n_new, lvl.kv.handle, dst, n_logit_rows, lvl.ws)
        if self.timed:
            e1.record()
            lvl._pending.append((e0, e1))
        lvl.kv_len = self.seq_len
        lvl.forwards += 1
        self._rows_ready(i, dst, n_logit_rows)
        if self.forward_log is not None:
            self.forward_log.append((i, start, toks.cpu().tolist()))
        if self.trace:
            self._emit(("forward", i, start, toks.cpu().tolist(),
                                None if dst is None else dst.detach().clone()))
        return dst

    def _rows_ready(self, i, dst, n_logit_rows):
        """Called after level i's forward has been enqueued, before anything reads its rows."""

    def _rollback(self, i, new_len):
        for j in range(i, self.n):
            lvl = self.levels[j]
            if lvl.kv_len > new_len:
                psd.psd_kv_truncate_to(lvl.kv.handle, new_len)
                lvl.kv_len = new_len

    # -------------------------------------------------------------- produce `want` tokens at level i
    def _produce(self, i, want, row0):
        """Append `want` tokens, each an exact draw from level i, to the device sequence; the
        level-i logits row of the j-th of them is rows[row0 + j]."""
        lvl = self.levels[i]
        if i == self.n - 1:                                     # the draft: plain sampling, no host sync
            for j in range(want):
                row = self._forward(i, 1, row0 + j)
                u = self.tapes[i][self.calls[i]:self.calls[i] + 1].view(1, 1)
                self.calls[i] += 1
                slot = self.seq[self.seq_len:self.seq_len + 1]
                ws_n = self.out[i, 0:1]
                a = self.acc[i]
                need = psd.psd_spec_accept_workspace_bytes(1, 0, 1, row.shape[-1])
                if a._ws is None or a._ws.numel() < need:
                    a._ws = torch.empty(max(need, 256), dtype=torch.uint8, device=self.dev)
                psd.psd_spec_accept(row, None, None, 0, u, self.T, ws_n, slot, 1, 1, row.shape[-1], psd.PSD_F32,
                                    row.shape[-1], 0, None, a._ws)
                self.seq_len += 1
                if self.trace:
                    self._emit(("sample", i, float(u.item()), int(slot.item()), row.detach().cpu().clone()))
            return
        have = 0
        below = self.levels[i + 1]
        while have < want:
            k = min(self.gammas[i + 1], want - have)
            base = self.seq_len
            self._produce(i + 1, k, 0)                          # k tokens at seq[base:base+k], q rows below.rows[0:k]
            # p rows for positions base-1 .. base+k-1; only a level with a parent keeps them as q rows
            p = self._forward(i, k + 1, row0 + have if i > 0 else 0)
            u = self.tapes[i][self.calls[i], :k + 1].contiguous().view(1, k + 1)
            self.calls[i] += 1
            x = self.seq[base:base + k].view(1, k)
            if self.timed:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
            n_t, tok_t, fl_t = self.acc[i](p.view(1, k + 1, -1), below.rows[0:k].view(1, k, -1), x, u, self.T)
            if self.timed:
                e1.record()
            res = torch.stack([n_t[0], tok_t[0], fl_t[0]]).cpu().tolist()      # the one host sync per stage
            if self.timed:
                self.accept_ms += e0.elapsed_time(e1)
            n, tok, flags = int(res[0]), int(res[1]), int(res[2])
            self.accept_lens[i].append(n)
            self.block_lens[i].append(k)
            if self.trace:
                self._emit(("accept", i, k, x.cpu().numpy()[0].copy(), u.cpu().numpy()[0].copy(), n, tok, flags,
                                    p.detach().cpu().clone(), below.rows[0:k].detach().cpu().clone()))
            self.seq_len = base + n
            self._rollback(i, base + n)
            have += n
            if have < want:
                self.seq[self.seq_len:self.seq_len + 1].copy_(tok_t[0:1])
                self.seq_len += 1
                have += 1

    # -------------------------------------------------------------- public
    def prefill(self, prompt):
        p = torch.as_tensor(np.asarray(prompt, dtype=np.int32)).to(self.dev)
        self.seq[:len(prompt)].copy_(p)
        self.seq_len = len(prompt) - 1
        if self.seq_len > 0:
            for i in range(self.n):
                self._forward_prefill(i)
        self.seq_len = len(prompt)

    def _forward_prefill(self, i):
        lvl = self.levels[i]
        n_new = self.seq_len - lvl.kv_len
        if n_new > 0:
            ws = lvl.model.workspace(1, n_new, lvl.kv.max_len)
            psd.psd_model_forward(lvl.model.handle, self.seq[lvl.kv_len:lvl.kv_len + n_new], n_new, lvl.kv.handle,
                                  None, 0, ws)
            lvl.kv_len += n_new
        lvl.ws = lvl.model.workspace_upto(1, lvl.max_rows + 2, lvl.kv.max_len)

    def generate(self, prompt, n_generate):
        self.prefill(prompt)
        start = self.seq_len
        for lvl in self.levels:
            lvl.forwards = 0
        self._produce(0, n_generate, 0)
        torch.cuda.synchronize()
        if self.timed:
            for lvl in self.levels:
                lvl.time_ms = sum(a.elapsed_time(b) for a, b in lvl._pending)
                lvl._pending = []
        return self.seq[start:start + n_generate].cpu().tolist()
