"""Continuous batching over the paged cache form: requests join the running batch after their prompt
was prefilled and leave it when they are done, while the other sequences keep decoding
(the serving setting of the paper's section "Serving with SPACE": auto-correct decoding inside a
batching engine).  Host side only: page bookkeeping, admission, retirement; every token is computed
by space_prefill / space_step / space_kv_commit.

Layout of the state: the active sequences occupy rows 0 .. n-1 of a few device arrays (block table,
len, next-block tokens, emitted tokens); a sequence that leaves is replaced by the last active one
(its rows are copied, its pages stay where they are), so the batch of a step is always the contiguous
view [:n]."""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

from .binding import Model, PagePool, PagedKV, SpaceStepOut, _ptr
from .layout import paper_layout, prefill_layout

PAGE = 32  # positions per page


class PageAllocator:
    """Free list of page ids 0 .. n_pages-1.  alloc() is all-or-nothing."""

    def __init__(self, n_pages: int):
        if n_pages < 1:
            raise ValueError("n_pages < 1")
        self.n_pages = n_pages
        self._free = list(range(n_pages - 1, -1, -1))
        self._owned = [False] * n_pages

    @property
    def n_free(self) -> int:
        return len(self._free)

    def alloc(self, n: int) -> Optional[List[int]]:
        if n < 0:
            raise ValueError("negative page count")
        if n > len(self._free):
            return None
        got = [self._free.pop() for _ in range(n)]
        for p in got:
            self._owned[p] = True
        return got

    def free(self, pages: List[int]) -> None:
        for p in pages:
            if not (0 <= p < self.n_pages) or not self._owned[p]:
                raise ValueError(f"page {p} is not allocated")
            self._owned[p] = False
            self._free.append(p)


def pages_for(positions: int) -> int:
    return (positions + PAGE - 1) // PAGE


@dataclass
class Request:
    rid: int
    prompt: np.ndarray          # int32 [n], n >= 1
    n_new: int
    output: List[int] = field(default_factory=list)
    finished: bool = False      # stopped by the end-of-sequence token
    accepted: List[int] = field(default_factory=list)  # accepted candidates of every invocation
    uniforms: Optional[np.ndarray] = None  # sampling: float32 [iterations, 2k+1], one row per invocation


class _RowsOut:
    """space_step_out over rows [lo, hi) of the batcher's arrays (what Model.step needs: the struct, and
    the tensor views it points into kept alive).  verify=False: logits only, the verification is left to
    space_sample_verify."""

    def __init__(self, cb: "ContinuousBatcher", lo: int, hi: int, logits=None, verify: bool = True):
        self.keep = (cb.accepted[lo:hi], cb.bonus[lo:hi], cb.new_cands[lo:hi], cb.tokens[lo:hi], cb.emit[lo:hi],
                     cb.emit_len[lo:hi], cb.fin[lo:hi], logits)
        a, b, c, t, e, el, f, lg = self.keep
        if verify:
            self.c = SpaceStepOut(_ptr(lg), None, _ptr(a), _ptr(b), _ptr(c), cb.k, _ptr(t), _ptr(e), _ptr(el), cb.emit_cap,
                                  cb.eos_id, _ptr(f))
        else:
            self.c = SpaceStepOut(_ptr(lg), None, None, None, None, cb.k, None, None, None, 0, -1, None)


class _RowsSample:
    """The outputs of space_sample_verify over rows [0, n): accepted counts, next block, emitted tokens
    and finished flags land where the greedy path puts them; P_c and the draft distributions go to
    the set `nxt`."""

    def __init__(self, cb: "ContinuousBatcher", n: int, nxt: int):
        self.max_cands, self.top_k = cb.k, int(cb.sampling.get("top_k", 10))
        self.accepted_len, self.extra, self.new_cands = cb.accepted[:n], cb.bonus[:n], cb.new_cands[:n]
        self.new_pc, self.new_ids, self.new_probs = cb.pc[nxt][:n], cb.ids[nxt][:n], cb.probs[nxt][:n]
        self.next_tokens = cb.tokens_next[:n]
        self.emit, self.emit_len, self.emit_cap = cb.emit[:n], cb.emit_len[:n], cb.emit_cap
        self.ratios, self.eos_id, self.finished = cb.ratios[:n], cb.eos_id, cb.fin[:n]


class ContinuousBatcher:
    """Greedy auto-correct decoding of a stream of requests with at most `max_seqs` sequences in a step.

    submit() queues a request; run() admits requests while a row and enough pages for the prompt are
    free, runs steps over the active rows and retires sequences that have their n_new tokens or hit
    eos_id.  Pages for the positions a step may write (len + k + 1) are taken before the step; if the
    pool runs dry the youngest sequence is put back in the queue (its pages are freed, it starts over)."""

    def __init__(self, model: Model, k: int, max_seqs: int, n_pages: int, max_ctx: int, prefill_chunk: int = 96,
                 eos_id: int = -1, emit_cap: int = 64, sampling: Optional[dict] = None):
        """sampling: None for greedy verification inside space_step, or {"top_k": .., "top_p": ..,
        "residual": bool} for the rejection-sampling form (space_sample_verify on the step's logits);
        every request then brings its own uniforms, one row of 2k+1 numbers per invocation it takes
        part in (numbered as in space_sample_verify)."""
        import torch
        self.torch = torch
        self.model, self.k, self.S = model, k, max_seqs
        self.L = (k + 1) * (k + 1)
        if max_seqs > model.cfg.max_batch or self.L > model.cfg.max_rows:
            raise ValueError("model context too small for this batch / k")
        self.stride = pages_for(max_ctx)
        if PAGE * self.stride > model.cfg.max_ctx:
            raise ValueError("max_ctx beyond the model context's")
        self.chunk = min(prefill_chunk, model.cfg.max_rows)
        self.eos_id, self.emit_cap = eos_id, max(emit_cap, k + 1)
        self.pool = PagePool(model, n_pages)
        self.alloc = PageAllocator(n_pages)
        dev, i32 = model.device, torch.int32
        S = max_seqs
        self.table = torch.zeros(S, self.stride, dtype=i32, device=dev)
        self.len = torch.zeros(S, dtype=i32, device=dev)
        self.tokens = torch.zeros(S, self.L, dtype=i32, device=dev)
        self.accepted = torch.zeros(S, dtype=i32, device=dev)
        self.bonus = torch.zeros(S, dtype=i32, device=dev)
        self.new_cands = torch.zeros(S, k, dtype=i32, device=dev)
        self.emit = torch.zeros(S, self.emit_cap, dtype=i32, device=dev)
        self.emit_len = torch.zeros(S, dtype=i32, device=dev)
        self.fin = torch.zeros(S, dtype=i32, device=dev)
        self.lay_step = model.layout(paper_layout(k))
        self.sampling = dict(sampling) if sampling else None
        if self.sampling:
            f32 = torch.float32
            tk = int(self.sampling.get("top_k", 10))
            self.logits = torch.empty(S, self.L, model.cfg.vocab, dtype=f32, device=dev)
            # P_c and the draft distributions alternate between two sets: a call reads one and writes the other
            self.pc = [torch.full((S, k), float("inf"), dtype=f32, device=dev) for _ in range(2)]
            self.ids = [torch.full((S, k, tk), -1, dtype=i32, device=dev) for _ in range(2)]
            self.probs = [torch.zeros(S, k, tk, dtype=f32, device=dev) for _ in range(2)]
            self.ratios = torch.zeros(S, k, dtype=f32, device=dev)
            self.tokens_next = torch.zeros(S, self.L, dtype=i32, device=dev)
            self.cur = 0
        self._prefill_layouts: Dict[int, object] = {}
        self.queue: List[Request] = []
        self.rows: List[Request] = []        # request of every active row
        self.pages: List[List[int]] = []     # pages of every active row, in table order
        self.bound: List[int] = []           # committed positions of every active row (exact, read back)
        self.done: List[Request] = []
        self.steps = 0
        self.restarts = 0
        self._next_rid = 0

    # ---- views and structs over rows [lo, hi)
    def _kv(self, lo: int, hi: int, bound: int) -> PagedKV:
        kv = PagedKV(self.pool, self.table[lo:hi], self.len[lo:hi])
        kv.set_len_bound(bound)
        return kv

    def _out(self, lo: int, hi: int) -> "_RowsOut":
        return _RowsOut(self, lo, hi)

    def _prefill_layout(self, n: int):
        if n not in self._prefill_layouts:
            self._prefill_layouts[n] = self.model.layout(prefill_layout(n))
        return self._prefill_layouts[n]

    # ---- requests
    def submit(self, prompt, n_new: int, uniforms=None) -> int:
        prompt = np.ascontiguousarray(prompt, dtype=np.int32).reshape(-1)
        if prompt.size < 1 or n_new < 1:
            raise ValueError("empty prompt or n_new < 1")
        if self.sampling:
            if uniforms is None:
                raise ValueError("sampling needs the request's uniforms")
            uniforms = np.ascontiguousarray(uniforms, dtype=np.float32)
            if uniforms.ndim != 2 or uniforms.shape[1] != 2 * self.k + 1 or uniforms.shape[0] < n_new:
                raise ValueError("uniforms must be [>= n_new, 2k+1] (an invocation emits at least one token)")
        if prompt.size + n_new + self.k + 1 > PAGE * self.stride:
            raise ValueError("request longer than max_ctx")
        rid = self._next_rid
        self._next_rid += 1
        self.queue.append(Request(rid, prompt, int(n_new), uniforms=uniforms))
        return rid

    def _set_table(self, row: int, first: int, pages: List[int]) -> None:
        if pages:
            t = self.torch.tensor(pages, dtype=self.torch.int32)
            self.table[row, first:first + len(pages)].copy_(t, non_blocking=False)

    def _admit(self, req: Request) -> bool:
        """Prefill of x_1 .. x_{l-1}; the sequence becomes row n of the batch and takes part in the next
        invocation.  False if the pool cannot hold the prompt right now."""
        torch = self.torch
        n = len(self.rows)
        l = int(req.prompt.size)
        need = pages_for(l - 1 + self.k + 1)  # the prompt and the positions the first step may write
        pages = self.alloc.alloc(need)
        if pages is None:
            return False
        self._set_table(n, 0, pages)
        self.len[n:n + 1].zero_()
        self.emit_len[n:n + 1].zero_()
        self.fin[n:n + 1].zero_()
        kv = self._kv(n, n + 1, 0)
        toks = torch.from_numpy(req.prompt[None, :]).to(self.model.device)
        done = 0
        while done < l - 1:
            c = min(self.chunk, l - 1 - done)
            self.model.prefill(toks[:, done:done + c].contiguous(), self._prefill_layout(c), kv)
            self.model.kv_commit(kv, None, accepted_all=c - 1)
            done += c
        # The sequence joins the batch with the initial state Algorithm 1 prints: L_c = [0] * k.  A dummy
        # is accepted only if 0 happens to be the greedy token, so the output is the same as with the
        # one-group first block, and the invocation is shared with the running sequences.
        block = torch.full((self.k + 1, self.k + 1), self.model.shape.mask_id, dtype=torch.int32)
        block[:, 0] = 0
        block[0, 0] = int(req.prompt[-1])
        self.tokens[n].copy_(block.reshape(-1))
        if self.sampling:
            self.pc[self.cur][n].fill_(float("inf"))  # P_c = +inf: a dummy passes only if its uniform is 0
            self.ids[self.cur][n].fill_(-1)           # no draft distribution yet: the residual rule reduces to Q
            self.probs[self.cur][n].zero_()
        self.rows.append(req)
        self.pages.append(pages)
        self.bound.append(l - 1)
        return True

    def _retire(self, row: int) -> None:
        """Frees the row: the last active row moves into it (its pages stay where they are)."""
        last = len(self.rows) - 1
        self.alloc.free(self.pages[row])
        if row != last:
            moved = [self.table, self.len, self.tokens, self.emit, self.emit_len, self.fin]
            if self.sampling:
                moved += self.pc + self.ids + self.probs
            for t in moved:
                t[row].copy_(t[last])
            self.rows[row], self.pages[row], self.bound[row] = self.rows[last], self.pages[last], self.bound[last]
        self.rows.pop()
        self.pages.pop()
        self.bound.pop()

    def _collect(self) -> None:
        """Reads back what the last calls emitted and retires the sequences that are done."""
        n = len(self.rows)
        if n == 0:
            return
        elen = self.emit_len[:n].cpu().numpy()
        fin = self.fin[:n].cpu().numpy()
        emit = self.emit[:n].cpu().numpy()
        lens = self.len[:n].cpu().numpy()
        self.emit_len[:n].zero_()
        for row in range(n):
            req = self.rows[row]
            req.output.extend(int(t) for t in emit[row, :elen[row]])
            self.bound[row] = int(lens[row])
            if fin[row]:
                req.finished = True
        for row in range(n - 1, -1, -1):
            req = self.rows[row]
            if req.finished or len(req.output) >= req.n_new:
                req.output = req.output[:req.n_new]
                self.done.append(req)
                self._retire(row)

    def _grow(self) -> None:
        """Every active row gets the pages a step may write: positions len .. len + k.  When the pool is
        empty the youngest sequence (the last row, possibly the one that asks) goes back to the queue and
        starts over later; a single sequence that does not fit the pool is an error."""
        row = 0
        while row < len(self.rows):
            need = pages_for(self.bound[row] + self.k + 1) - len(self.pages[row])
            got = self.alloc.alloc(need) if need > 0 else []
            while got is None:
                victim = len(self.rows) - 1
                if victim == 0:
                    raise RuntimeError("page pool too small for a single sequence")
                req = self.rows[victim]
                req.output, req.accepted = [], []
                self.restarts += 1
                self.queue.insert(0, req)
                self._retire(victim)
                if victim == row:
                    break
                got = self.alloc.alloc(need)
            if got is None:
                continue  # the row itself went back to the queue
            if got:
                self._set_table(row, len(self.pages[row]), got)
                self.pages[row].extend(got)
            row += 1

    def step(self) -> None:
        """One model invocation over all active rows."""
        n = len(self.rows)
        kv = self._kv(0, n, max(self.bound))
        self.model.tune_rows(n * self.lay_step.n_rows)  # measured the first time this many rows come up
        if not self.sampling:
            self.model.step(self.tokens[:n], self.lay_step, kv, self._out(0, n), next_layout=self.lay_step)
        else:
            torch = self.torch
            out = _RowsOut(self, 0, n, logits=self.logits[:n], verify=False)
            self.model.step(self.tokens[:n], self.lay_step, kv, out)
            u = np.stack([r.uniforms[len(r.accepted)] for r in self.rows])
            cur, nxt = self.cur, 1 - self.cur
            sv = _RowsSample(self, n, nxt)
            res = bool(self.sampling.get("residual", False))
            self.model.sample_verify(self.logits[:n], self.tokens[:n], self.lay_step, self.pc[cur][:n],
                                     torch.from_numpy(u).to(self.model.device), sv,
                                     top_k=int(self.sampling.get("top_k", 10)), top_p=float(self.sampling.get("top_p", 0.95)),
                                     residual=res, draft_ids=self.ids[cur][:n] if res else None,
                                     draft_probs=self.probs[cur][:n] if res else None, next_layout=self.lay_step)
            self.tokens[:n].copy_(self.tokens_next[:n])
            self.cur = nxt
        self.model.kv_commit(kv, self.accepted[:n])
        acc = self.accepted[:n].cpu().numpy()
        for row in range(n):
            self.rows[row].accepted.append(int(acc[row]))
        self.steps += 1

    def run(self) -> List[Request]:
        """Runs until the queue and the batch are empty; returns the finished requests in order of id."""
        while self.queue or self.rows:
            while self.queue and len(self.rows) < self.S:
                if not self._admit(self.queue[0]):
                    break
                self.queue.pop(0)
            if not self.rows:
                raise RuntimeError("page pool too small for the next request")
            self._grow()
            self.step()
            self._collect()
        return sorted(self.done, key=lambda r: r.rid)
