"""Host loops of Algorithm 1 (greedy, and the printed sampling form) on top of the C ABI.

All arithmetic, the verification and the assembly of the next block run on the device: the block of
iteration t+1 is written by iteration t into the token buffer it is read from, so one iteration
(space_step + space_kv_commit, plus space_sample_verify in the sampling form) needs no host data.  It
is captured once into a HIP graph and replayed; the host only reads the emitted counts and the finished
flags now and then to decide when to stop -- after as many replays as the tokens still missing need at
the very least (every iteration emits at most k + 1), so no iteration runs that was not needed.
"""
from __future__ import annotations

import ctypes
from typing import Callable, List, Tuple

import numpy as np

from .binding import SampleOut, KVCache, Model, StepOut, _stream
from .layout import first_step_layout, paper_layout, prefill_layout


class SpaceDecoder:
    """One batch of sequences decoded with k mask tokens per group.  Reusable: generate() clears the cache.

    graph=False launches every iteration kernel by kernel from the host instead of replaying a captured
    graph (same kernels, same results)."""

    def __init__(self, model: Model, k: int, batch: int = 1, capacity: int = 1024, prefill_chunk: int = 96,
                 want_logits: bool = False, emit_cap: int = 4096, eos_id: int = -1, graph: bool = True):
        import torch
        self.torch = torch
        self.model, self.k, self.batch = model, k, batch
        self.eos_id = int(eos_id)
        self.use_graph = bool(graph)
        self.L = (k + 1) * (k + 1)
        max_rows = model.cfg.max_rows
        if self.L > max_rows:
            raise ValueError(f"(k+1)^2 = {self.L} rows exceed the model's max_rows {max_rows}")
        self.chunk = min(prefill_chunk, max_rows)
        self.capacity = capacity
        self.emit_cap = emit_cap
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
        self.iterations = 0  # model invocations since the last reset (the first one included)
        # accepted counts of every invocation, recorded on the device: row `_hist_pos` takes the next one
        self._hist_rows = 0
        self._hist = None
        self._hist_pos = torch.zeros(1, dtype=torch.int64, device=model.device)
        self._hist_idx = torch.zeros(1, dtype=torch.int64, device=model.device)
        self._graphs: List[object] = []  # captured iterations, replayed in turn
        self._eager: List[Callable[[], None]] = []
        self._turn = 0
        self._bound = 0
        self.lengths = np.zeros(batch, dtype=np.int64)

    # ---------------------------------------------------------------------------------------------
    def reset(self) -> None:
        """Empties the cache and the output stream: the decoder starts a new batch of sequences."""
        self.model._check(self.model.lib.space_kv_reset(self.model.ctx, ctypes.byref(self.kv.c), _stream()))
        self.out.emit_len.zero_()
        self.out.finished.zero_()
        self._hist_pos.zero_()
        self.committed = 0
        self.iterations = 0
        self._graphs, self._eager, self._turn = [], [], 0

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

    def tune(self, prompt_len: int = 0) -> None:
        """space_tune_rows for the row counts this decoder launches: the blocks of the iterations and, for
        a prompt of prompt_len tokens, its chunks.  Waits for the device (setup work, like the prefill)."""
        rows = {self.batch * self.L, self.batch * (self.k + 1)}
        if prompt_len > 0:
            rows.add(self.batch * min(self.chunk, prompt_len))
            if prompt_len > self.chunk and prompt_len % self.chunk:
                rows.add(self.batch * (prompt_len % self.chunk))
        for r in sorted(rows):
            self.model.tune_rows(r)

    def _ensure_hist(self, rows: int) -> None:
        torch = self.torch
        if self._hist is None or self._hist_rows < rows:
            keep = self._hist
            self._hist_rows = max(rows, 2 * self._hist_rows, 64)
            self._hist = torch.zeros(self._hist_rows, self.batch, dtype=torch.int32, device=self.model.device)
            if keep is not None:
                self._hist[: keep.shape[0]] = keep
            self._graphs, self._eager = [], []  # the captured iterations write into the old buffer

    def _record(self, accepted) -> None:
        """hist[pos] = accepted; pos += 1 -- on the device, so that it can be part of a captured iteration.
        Invocations beyond the rows the history was sized for overwrite its last row instead of running out
        of the buffer (callers that drive run() themselves may go on for longer than they announced)."""
        self.torch.clamp(self._hist_pos, max=self._hist_rows - 1, out=self._hist_idx)
        self._hist.index_copy_(0, self._hist_idx, accepted.view(1, -1))
        self._hist_pos.add_(1)

    def _capture(self, fn: Callable[[], None]):
        """fn captured into a HIP graph (after one rehearsal on a side stream, which also runs it once)."""
        torch = self.torch
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        return g

    def _set_bound(self, bound: int) -> None:
        """The cache lengths live on the device; the launches are shaped for this host-side bound of them.
        It is raised ahead of the iterations that can reach it (a captured iteration keeps the bound it was
        captured with, so a change drops the captured graphs)."""
        if bound + (self.k + 1) > self.capacity:
            raise ValueError(f"cache capacity {self.capacity} too small: up to {bound} positions and a block of "
                             f"{self.k + 1} groups would be needed")
        if bound != self._bound:
            self._graphs = []
        self._bound = bound
        self.kv.set_len_bound(bound)

    def rebound(self, n_iterations: int) -> int:
        """Reads the true cache lengths (synchronises) and sizes the launches for n_iterations more
        iterations from there; drops the captured graphs if the bound changes.  Returns the bound."""
        self.torch.cuda.synchronize()
        top = int(self.kv.len.cpu().numpy().max())
        self._set_bound(min(top + (self.k + 1) * n_iterations, self.capacity - (self.k + 1)))
        return self._bound

    def _hist_list(self) -> List[np.ndarray]:
        n = min(int(self._hist_pos.cpu()[0]), self._hist_rows)
        h = self._hist[:n].cpu().numpy()
        return [h[i].copy() for i in range(n)]

    # ---------------------------------------------------------------------------------------------
    def start(self, prompt: np.ndarray, n_new: int) -> None:
        """Clears the decoder, prefills prompt[:, :-1], runs the first iteration of Algorithm 1 (it starts
        from dummies that are always rejected: the block is [x_l, M^k], one token comes out) and prepares
        the iteration that run() repeats, sized for n_new generated tokens."""
        torch = self.torch
        prompt = np.ascontiguousarray(prompt, dtype=np.int32)
        assert prompt.shape[0] == self.batch
        k = self.k
        if self.emit_cap < n_new + k + 1:
            raise ValueError(f"emit_cap {self.emit_cap} below n_new + k + 1 = {n_new + k + 1}")
        self.reset()
        self._ensure_hist(n_new + 1)
        self.tune(prompt.shape[1] - 1)
        if prompt.shape[1] > 1:
            self.prefill(prompt[:, :-1])
        # every iteration commits at most k + 1 positions and a lone sequence stops once n_new tokens are
        # out: at most n_new + k positions on top of the prompt.  (In a batch a sequence keeps committing
        # while a slower one is still short; the loop raises the bound when that happens.)
        self._set_bound(self.committed + n_new + k + 1)
        first = np.full((self.batch, k + 1), self.model.cfg.vocab, dtype=np.int32)
        first[:, 0] = prompt[:, -1]
        tok_first = torch.from_numpy(first).to(self.model.device)
        self.model.step(tok_first, self.lay_first, self.kv, self.out_first, next_layout=self.lay_step)
        self.model.kv_commit(self.kv, self.out_first.accepted_len)
        self._record(self.out_first.accepted_len)
        self.iterations = 1
        self.kv.set_len_bound(self._bound)  # the commit advanced the library's own count; this is the bound that holds

        def iteration():
            self.model.step(self.out.next_tokens, self.lay_step, self.kv, self.out, next_layout=self.lay_step)
            self.model.kv_commit(self.kv, self.out.accepted_len)
            self._record(self.out.accepted_len)
            self.kv.set_len_bound(self._bound)

        self._eager = [iteration]
        self._graphs = []

    def prepare(self) -> int:
        """Captures the iteration into a HIP graph if that is wanted and not done yet.  The rehearsal in
        front of a capture runs the iteration once for real; returns the number of iterations that ran."""
        if not self.use_graph or self._graphs:
            return 0
        n = len(self._eager)
        graphs = [None] * n
        for i in range(n):  # in the order they would run from here, so that the state moves on correctly
            idx = (self._turn + i) % n
            graphs[idx] = self._capture(self._eager[idx])
        self._graphs = graphs
        self.iterations += n
        return n

    def run(self, n: int) -> None:
        """n more iterations without any host synchronisation (the capture, if it is still due, takes place
        first and counts for as many iterations as it ran)."""
        if n <= 0:
            return
        n -= self.prepare()
        for _ in range(max(n, 0)):
            if self.use_graph:
                self._graphs[self._turn].replay()
            else:
                self._eager[self._turn]()
            self._turn = (self._turn + 1) % len(self._eager)
            self.iterations += 1

    def _loop(self, n_new: int, emit_len, finished) -> None:
        """Runs iterations until every sequence has n_new tokens or is finished.  Between two looks at the
        counters it runs as many iterations as the missing tokens need at the very least."""
        per = self.k + 1
        setup = len(self._eager) if self.use_graph else 0  # iterations a capture costs
        while True:
            done = emit_len.cpu().numpy()
            fin = finished.cpu().numpy()
            live = (done < n_new) & (fin == 0)
            if not live.any():
                break
            need = int(-(-(n_new - int(done[live].min())) // per))  # ceil: the slowest live sequence decides
            reach = int(self.kv.len.cpu().numpy().max()) + need * per
            if reach > self._bound:  # a sequence of the batch ran ahead of (or past the end of) the others
                self._set_bound(min(max(reach, self._bound + 16 * per), self.capacity - per))
                if reach > self._bound:
                    raise ValueError(f"cache capacity {self.capacity} too small for {need} more iterations")
            if self.use_graph and not self._graphs and need < setup:
                # too few left to pay for a capture: launch them one by one
                for _ in range(need):
                    self._eager[self._turn]()
                    self._turn = (self._turn + 1) % len(self._eager)
                    self.iterations += 1
                continue
            self.run(need)
        self.lengths = np.minimum(emit_len.cpu().numpy(), n_new)

    def generate(self, prompt: np.ndarray, n_new: int) -> Tuple[np.ndarray, List[np.ndarray]]:
        """Greedy auto-correct decoding of n_new tokens after `prompt` [batch, n].  Returns the
        sequences [batch, n + n_new] and the accepted counts of every model invocation.  With an
        eos_id a sequence stops in front of that token; `self.lengths` holds the number of generated
        tokens per sequence (entries beyond it are padding)."""
        prompt = np.ascontiguousarray(prompt, dtype=np.int32)
        self.start(prompt, n_new)
        self._loop(n_new, self.out.emit_len, self.out.finished)
        emitted = self.out.emit.cpu().numpy()
        return np.concatenate([prompt, emitted[:, :n_new]], axis=1), self._hist_list()

    def generate_sampled(self, prompt: np.ndarray, n_new: int, uniforms: np.ndarray, top_k: int = 10,
                         top_p: float = 0.95, residual: bool = False) -> Tuple[np.ndarray, List[np.ndarray]]:
        """Algorithm 1 with rejection sampling.  uniforms: float32 [iterations, batch, 2k+1], numbered as
        in space_sample_verify (test i at [i-1], extra token at [k], candidate j at [k+1+j]); the first
        iteration runs the block [x_l, M^k] (P_c = +inf in the paper: nothing can be accepted) and reads
        only [k:].  Tokens, P_c, the draft distributions and the row of uniforms in use stay on the device
        between iterations.  With an eos_id a sequence stops in front of that token (`self.lengths`, as in
        generate())."""
        torch = self.torch
        k, B, dev = self.k, self.batch, self.model.device
        prompt = np.ascontiguousarray(prompt, dtype=np.int32)
        assert prompt.shape[0] == B and uniforms.shape[1:] == (B, 2 * k + 1)
        if uniforms.shape[0] < 2:
            raise ValueError("uniforms for at least two iterations are needed")
        u_dev = torch.from_numpy(np.ascontiguousarray(uniforms, dtype=np.float32)).to(dev)
        self.reset()
        self._ensure_hist(uniforms.shape[0] + 2)
        self.tune(prompt.shape[1] - 1)
        if prompt.shape[1] > 1:
            self.prefill(prompt[:, :-1])
        self._set_bound(self.committed + n_new + k + 1)
        first = np.full((B, k + 1), self.model.cfg.vocab, dtype=np.int32)
        first[:, 0] = prompt[:, -1]
        tok = torch.from_numpy(first).to(dev)
        emit_cap = n_new + k + 1
        out_first = StepOut(self.model, B, k + 1, k, want_logits=True)
        out = StepOut(self.model, B, self.L, k, want_logits=True)
        souts = [SampleOut(self.model, B, k + 1, k, top_k, next_rows=self.L, emit_cap=emit_cap, eos_id=self.eos_id)
                 for _ in range(2)]
        souts[1].emit, souts[1].emit_len, souts[1].finished = souts[0].emit, souts[0].emit_len, souts[0].finished  # one output stream
        # iteration 0: one group, no candidates
        self.model.step(tok, self.lay_first, self.kv, out_first)
        pc0 = torch.full((B, k), float("inf"), device=dev)
        self.model.sample_verify(out_first.logits, tok, self.lay_first, pc0, u_dev[0, :, k:].contiguous(), souts[0],
                                 top_k=top_k, top_p=top_p, next_layout=self.lay_step)
        self.model.kv_commit(self.kv, souts[0].accepted_len)
        self._record(souts[0].accepted_len)
        self.iterations = 1
        self.kv.set_len_bound(self._bound)
        # the uniforms of the iteration in turn: row `u_pos` of u_dev, fetched on the device (rows past the
        # end repeat the last one; the loop below never gets there unless the caller brought too few)
        u_pos = torch.ones(1, dtype=torch.int64, device=dev)
        u_now = torch.empty(B, 2 * k + 1, dtype=torch.float32, device=dev)
        u_last = uniforms.shape[0] - 1

        def make(prev: SampleOut, nxt: SampleOut) -> Callable[[], None]:
            def iteration():
                torch.index_select(u_dev, 0, u_pos, out=u_now.view(1, B, 2 * k + 1))
                u_pos.add_(1).clamp_(max=u_last)
                self.model.step(prev.next_tokens, self.lay_step, self.kv, out)
                self.model.sample_verify(out.logits, prev.next_tokens, self.lay_step, prev.new_pc, u_now, nxt,
                                         top_k=top_k, top_p=top_p, residual=residual,
                                         draft_ids=prev.new_ids if residual else None,
                                         draft_probs=prev.new_probs if residual else None, next_layout=self.lay_step)
                self.model.kv_commit(self.kv, nxt.accepted_len)
                self._record(nxt.accepted_len)
                self.kv.set_len_bound(self._bound)
            return iteration

        # the outputs of one iteration are the inputs of the next: two iterations that swap the buffers
        self._eager = [make(souts[0], souts[1]), make(souts[1], souts[0])]
        self._graphs, self._turn = [], 0
        self._loop(n_new, souts[0].emit_len, souts[0].finished)
        if self.iterations > uniforms.shape[0]:
            raise ValueError(f"{self.iterations} iterations ran but only {uniforms.shape[0]} rows of uniforms were given")
        emitted = souts[0].emit.cpu().numpy()
        return np.concatenate([prompt, emitted[:, :n_new]], axis=1), self._hist_list()
