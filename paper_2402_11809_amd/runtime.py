"""Thin host loops of Algorithm 1 (greedy, and the printed sampling form) on top of the C ABI.

All arithmetic, the verification and the assembly of the next block run on the device; the
host only decides when to stop.  The block of iteration t+1 is written by iteration t into the
same token buffer it is read from, so a (step, commit) pair needs no host data at all.
"""
from __future__ import annotations

from typing import List, Tuple

import numpy as np

from .binding import SampleOut, KVCache, Model, StepOut
from .layout import first_step_layout, paper_layout, prefill_layout


class SpaceDecoder:
    def __init__(self, model: Model, k: int, batch: int = 1, capacity: int = 1024, prefill_chunk: int = 96,
                 want_logits: bool = False, emit_cap: int = 4096, eos_id: int = -1):
        import torch
        self.torch = torch
        self.model, self.k, self.batch = model, k, batch
        self.eos_id = int(eos_id)
        self.L = (k + 1) * (k + 1)
        max_rows = model.cfg.max_rows
        if self.L > max_rows:
            raise ValueError(f"(k+1)^2 = {self.L} rows exceed the model's max_rows {max_rows}")
        self.chunk = min(prefill_chunk, max_rows)
        self.kv = KVCache(model, batch, capacity)
        self.lay_step = model.layout(paper_layout(k))
        self.lay_first = model.layout(first_step_layout(k))
        self._prefill_layouts = {}
        self.out = StepOut(model, batch, self.L, k, next_rows=self.L, want_logits=want_logits, emit_cap=emit_cap,
                           eos_id=eos_id)
        self.out_first = StepOut(model, batch, k + 1, k, next_rows=self.L, want_logits=want_logits, emit_cap=emit_cap,
                                 eos_id=eos_id)
        # both step kinds append to one emit stream (and one finished flag) and write the same next-block buffer
        self.out_first.emit, self.out_first.emit_len = self.out.emit, self.out.emit_len
        self.out_first.c.emit, self.out_first.c.emit_len = self.out.c.emit, self.out.c.emit_len
        self.out_first.finished, self.out_first.c.finished = self.out.finished, self.out.c.finished
        self.out_first.next_tokens = self.out.next_tokens
        self.out_first.c.next_tokens = self.out.c.next_tokens
        self.committed = 0  # host mirror of len (all sequences advance alike during prefill)

    def _prefill_layout(self, n: int):
        if n not in self._prefill_layouts:
            self._prefill_layouts[n] = self.model.layout(prefill_layout(n))
        return self._prefill_layouts[n]

    def prefill(self, tokens: np.ndarray) -> None:
        """Commits tokens [batch, n] (x_1..x_{l-1}) to the cache, in chunks of up to `prefill_chunk` rows
        (at most the model's max_rows) through space_prefill: no LM head, no verification."""
        torch = self.torch
        t = torch.from_numpy(np.ascontiguousarray(tokens, dtype=np.int32)).to(self.model.device)
        n = t.shape[1]
        for c0 in range(0, n, self.chunk):
            c = min(self.chunk, n - c0)
            self.model.prefill(t[:, c0:c0 + c].contiguous(), self._prefill_layout(c), self.kv)
            self.model.kv_commit(self.kv, None, accepted_all=c - 1)
            self.committed += c

    def generate(self, prompt: np.ndarray, n_new: int) -> Tuple[np.ndarray, List[np.ndarray]]:
        """Greedy auto-correct decoding of n_new tokens after `prompt` [batch, n].  Returns the
        sequences [batch, n + n_new] and the accepted counts of every model invocation.  With an
        eos_id a sequence stops in front of that token; `self.lengths` holds the number of generated
        tokens per sequence (entries beyond it are padding)."""
        torch = self.torch
        prompt = np.ascontiguousarray(prompt, dtype=np.int32)
        assert prompt.shape[0] == self.batch
        n = prompt.shape[1]
        if n > 1:
            self.prefill(prompt[:, :-1])
        first = np.full((self.batch, self.k + 1), self.model.cfg.vocab, dtype=np.int32)
        first[:, 0] = prompt[:, -1]
        tok_first = torch.from_numpy(first).to(self.model.device)
        self.out.emit_len.zero_()
        self.out.finished.zero_()
        hist: List[np.ndarray] = []
        # first iteration: nothing to verify (Algorithm 1 starts from dummies that are always rejected)
        self.model.step(tok_first, self.lay_first, self.kv, self.out_first, next_layout=self.lay_step)
        self.model.kv_commit(self.kv, self.out_first.accepted_len)
        hist.append(self.out_first.accepted_len.cpu().numpy().copy())
        done = self.out.emit_len.cpu().numpy()
        fin = self.out.finished.cpu().numpy()
        steps = 1
        self.kv.set_len_bound(self.committed + steps * (self.k + 1))
        while not np.all((done >= n_new) | (fin != 0)):
            self.model.step(self.out.next_tokens, self.lay_step, self.kv, self.out, next_layout=self.lay_step)
            self.model.kv_commit(self.kv, self.out.accepted_len)
            hist.append(self.out.accepted_len.cpu().numpy().copy())
            done = self.out.emit_len.cpu().numpy()
            fin = self.out.finished.cpu().numpy()
            steps += 1
            self.kv.set_len_bound(self.committed + steps * (self.k + 1))
        emitted = self.out.emit.cpu().numpy()
        self.lengths = np.minimum(done, n_new)
        seqs = np.concatenate([prompt, emitted[:, :n_new]], axis=1)
        return seqs, hist

    def generate_sampled(self, prompt: np.ndarray, n_new: int, uniforms: np.ndarray, top_k: int = 10,
                         top_p: float = 0.95, residual: bool = False) -> Tuple[np.ndarray, List[np.ndarray]]:
        """Algorithm 1 with rejection sampling.  uniforms: float32 [iterations, batch, 2k+1], numbered as
        in space_sample_verify (test i at [i-1], extra token at [k], candidate j at [k+1+j]); the first
        iteration runs the block [x_l, M^k] (P_c = +inf in the paper: nothing can be accepted) and reads
        only [k:].  Tokens, P_c and the draft distributions stay on the device between iterations.  With an
        eos_id a sequence stops in front of that token (`self.lengths`, as in generate())."""
        torch = self.torch
        k, B, dev = self.k, self.batch, self.model.device
        prompt = np.ascontiguousarray(prompt, dtype=np.int32)
        assert prompt.shape[0] == B and uniforms.shape[1:] == (B, 2 * k + 1)
        u_dev = torch.from_numpy(np.ascontiguousarray(uniforms, dtype=np.float32)).to(dev)
        if prompt.shape[1] > 1:
            self.prefill(prompt[:, :-1])
        first = np.full((B, k + 1), self.model.cfg.vocab, dtype=np.int32)
        first[:, 0] = prompt[:, -1]
        tok = torch.from_numpy(first).to(dev)
        emit_cap = n_new + k + 1
        out_first = StepOut(self.model, B, k + 1, k, want_logits=True)
        out = StepOut(self.model, B, self.L, k, want_logits=True)
        souts = [SampleOut(self.model, B, k + 1, k, top_k, next_rows=self.L, emit_cap=emit_cap, eos_id=self.eos_id)
                 for _ in range(2)]
        souts[1].emit, souts[1].emit_len, souts[1].finished = souts[0].emit, souts[0].emit_len, souts[0].finished  # one output stream
        hist: List[np.ndarray] = []
        # iteration 0: one group, no candidates
        self.model.step(tok, self.lay_first, self.kv, out_first)
        pc0 = torch.full((B, k), float("inf"), device=dev)
        self.model.sample_verify(out_first.logits, tok, self.lay_first, pc0, u_dev[0, :, k:].contiguous(), souts[0],
                                 top_k=top_k, top_p=top_p, next_layout=self.lay_step)
        self.model.kv_commit(self.kv, souts[0].accepted_len)
        hist.append(souts[0].accepted_len.cpu().numpy().copy())
        it, cur = 1, 0
        done = souts[0].emit_len.cpu().numpy()
        fin = souts[0].finished.cpu().numpy()
        self.kv.set_len_bound(self.committed + 1)
        while not np.all((done >= n_new) | (fin != 0)):
            prev, nxt = souts[cur], souts[1 - cur]
            self.model.step(prev.next_tokens, self.lay_step, self.kv, out)
            self.model.sample_verify(out.logits, prev.next_tokens, self.lay_step, prev.new_pc, u_dev[it], nxt,
                                     top_k=top_k, top_p=top_p, residual=residual,
                                     draft_ids=prev.new_ids if residual else None,
                                     draft_probs=prev.new_probs if residual else None, next_layout=self.lay_step)
            self.model.kv_commit(self.kv, nxt.accepted_len)
            hist.append(nxt.accepted_len.cpu().numpy().copy())
            done = nxt.emit_len.cpu().numpy()
            fin = souts[0].finished.cpu().numpy()
            cur, it = 1 - cur, it + 1
            self.kv.set_len_bound(self.committed + 1 + (it - 1) * (k + 1))  # emitted counts stop at an EOS, len does not
        self.lengths = np.minimum(done, n_new)
        emitted = souts[0].emit.cpu().numpy()
        return np.concatenate([prompt, emitted[:, :n_new]], axis=1), hist
