"""ctypes binding of libspace_hip.so: the same calls as include/space.h, argument marshalling only.

PyTorch is used for device memory and streams.  There is no fallback: if the HIP library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

from .layout import BlockLayoutSpec

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libspace_hip.so")
_lib = None

SPACE_OK, SPACE_EINVAL, SPACE_ESHAPE, SPACE_ECAPACITY, SPACE_EHIP, SPACE_ENOMEM = 0, -1, -2, -3, -4, -5
STATUS_NAMES = {0: "SPACE_OK", -1: "SPACE_EINVAL", -2: "SPACE_ESHAPE", -3: "SPACE_ECAPACITY", -4: "SPACE_EHIP",
                -5: "SPACE_ENOMEM"}

EXPORTS = ["space_last_error", "space_init", "space_load_layer", "space_destroy", "space_layout_create", "space_layout_destroy",
           "space_kv_bytes", "space_kv_reset", "space_step", "space_kv_commit", "space_kv_rollback",
           "space_sample_verify", "space_sample_verify_static", "space_sar_loss", "space_sar_transform", "space_prefill", "space_kv_pool_bytes", "space_device_faults", "space_debug_buffer", "space_timing_enable",
           "space_timing_read", "space_tune_rows"]

KERNEL_CLASSES = ["embed", "norm", "qkv", "rope", "attn", "o", "gate_up", "down", "lm_head", "verify"]


class SpaceError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{STATUS_NAMES.get(code, code)}: {msg}")
        self.code = code


class SpaceConfig(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
                ("ffn", C.c_int32), ("vocab", C.c_int32), ("max_batch", C.c_int32), ("max_rows", C.c_int32),
                ("max_ctx", C.c_int32), ("rms_eps", C.c_float), ("rope_base", C.c_float), ("n_kv_heads", C.c_int32)]


class SpaceLayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]


class SpaceWeights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("layers", C.POINTER(SpaceLayerWeights))]


class SpaceKV(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("len", C.c_void_p), ("batch", C.c_int32),
                ("capacity", C.c_int32), ("host_len_bound", C.c_int32), ("block_table", C.c_void_p),
                ("table_stride", C.c_int32), ("n_pages", C.c_int32)]


class SpaceStepOut(C.Structure):
    _fields_ = [("logits", C.c_void_p), ("argmax", C.c_void_p), ("accepted_len", C.c_void_p), ("bonus", C.c_void_p),
                ("new_cands", C.c_void_p), ("max_cands", C.c_int32), ("next_tokens", C.c_void_p),
                ("emit", C.c_void_p), ("emit_len", C.c_void_p), ("emit_cap", C.c_int32), ("eos_id", C.c_int32),
                ("finished", C.c_void_p)]


class SpaceSampleParams(C.Structure):
    _fields_ = [("top_k", C.c_int32), ("top_p", C.c_float), ("residual", C.c_int32)]


class SpaceSampleIO(C.Structure):
    _fields_ = [("logits", C.c_void_p), ("tokens", C.c_void_p), ("p_c", C.c_void_p), ("uniforms", C.c_void_p),
                ("draft_ids", C.c_void_p), ("draft_probs", C.c_void_p), ("accepted_len", C.c_void_p),
                ("extra", C.c_void_p), ("new_cands", C.c_void_p), ("new_pc", C.c_void_p), ("max_cands", C.c_int32),
                ("new_ids", C.c_void_p), ("new_probs", C.c_void_p), ("next_tokens", C.c_void_p), ("emit", C.c_void_p),
                ("emit_len", C.c_void_p), ("emit_cap", C.c_int32), ("ratios", C.c_void_p), ("eos_id", C.c_int32),
                ("finished", C.c_void_p)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libspace_hip.so (built in-tree by paper_2402_11809_amd.build); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(f"{_LIB_PATH} not built: run `python -m paper_2402_11809_amd.build`")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    lib.space_last_error.restype = C.c_char_p
    lib.space_last_error.argtypes = [vp]
    lib.space_init.restype = C.c_int
    lib.space_init.argtypes = [C.POINTER(SpaceConfig), C.POINTER(SpaceWeights), C.POINTER(vp)]
    lib.space_load_layer.restype = C.c_int
    lib.space_load_layer.argtypes = [vp, i32, C.POINTER(SpaceLayerWeights)]
    lib.space_destroy.restype = None
    lib.space_destroy.argtypes = [vp]
    lib.space_layout_create.restype = C.c_int
    lib.space_layout_create.argtypes = [vp, i32, C.POINTER(C.c_uint8), C.POINTER(C.c_int32), C.POINTER(vp)]
    lib.space_layout_destroy.restype = None
    lib.space_layout_destroy.argtypes = [vp, vp]
    lib.space_kv_bytes.restype = sz
    lib.space_kv_bytes.argtypes = [C.POINTER(SpaceConfig), i32, i32]
    lib.space_kv_pool_bytes.restype = sz
    lib.space_kv_pool_bytes.argtypes = [C.POINTER(SpaceConfig), i32]
    lib.space_kv_reset.restype = C.c_int
    lib.space_kv_reset.argtypes = [vp, C.POINTER(SpaceKV), vp]
    lib.space_prefill.restype = C.c_int
    lib.space_prefill.argtypes = [vp, vp, vp, C.POINTER(SpaceKV), vp]
    lib.space_step.restype = C.c_int
    lib.space_step.argtypes = [vp, vp, vp, vp, C.POINTER(SpaceKV), C.POINTER(SpaceStepOut), vp]
    lib.space_kv_commit.restype = C.c_int
    lib.space_kv_commit.argtypes = [vp, C.POINTER(SpaceKV), vp, i32, vp]
    lib.space_kv_rollback.restype = C.c_int
    lib.space_kv_rollback.argtypes = [vp, C.POINTER(SpaceKV), vp, i32, vp]
    lib.space_sample_verify.restype = C.c_int
    lib.space_sample_verify.argtypes = [vp, i32, vp, vp, C.POINTER(SpaceSampleParams), C.POINTER(SpaceSampleIO), vp]
    lib.space_sample_verify_static.restype = C.c_int
    lib.space_sample_verify_static.argtypes = lib.space_sample_verify.argtypes
    lib.space_tune_rows.restype = C.c_int
    lib.space_tune_rows.argtypes = [vp, i32, vp]
    lib.space_sar_loss.restype = C.c_int
    lib.space_sar_loss.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp]
    i32p = C.POINTER(C.c_int32)
    lib.space_sar_transform.restype = C.c_int
    lib.space_sar_transform.argtypes = [i32p, i32, i32, i32, i32, C.c_float, C.c_float, C.c_float, i32p, i32p, i32p, i32p, i32p]
    lib.space_device_faults.restype = C.c_int
    lib.space_device_faults.argtypes = [vp, vp]
    lib.space_timing_enable.restype = C.c_int
    lib.space_timing_enable.argtypes = [vp, C.c_uint32, i32]
    lib.space_timing_read.restype = C.c_int
    lib.space_timing_read.argtypes = [vp, vp, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.space_debug_buffer.restype = C.c_int
    lib.space_debug_buffer.argtypes = [vp, C.c_char_p, C.POINTER(vp), C.POINTER(sz)]
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream(stream=None) -> Optional[int]:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream) or None


class Layout:
    def __init__(self, model: "Model", spec: BlockLayoutSpec):
        self.model, self.spec = model, spec
        im = np.ascontiguousarray(spec.is_mask, dtype=np.uint8)
        gr = np.ascontiguousarray(spec.group, dtype=np.int32)
        h = C.c_void_p()
        rc = model.lib.space_layout_create(model.ctx, len(im), im.ctypes.data_as(C.POINTER(C.c_uint8)),
                                           gr.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(h))
        model._check(rc)
        self.handle = h
        self.n_rows, self.n_groups = spec.n_rows, spec.n_groups


class KVCache:
    """Caller-owned cache memory (torch tensors) plus the space_kv struct describing it."""

    def __init__(self, model: "Model", batch: int, capacity: int, stream=None):
        import torch
        self.model = model
        nbytes = model.lib.space_kv_bytes(C.byref(model.cfg), batch, capacity)
        if nbytes == 0:
            raise SpaceError(SPACE_EINVAL, f"bad kv shape batch={batch} capacity={capacity}")
        dev = model.device
        self.k = torch.empty(nbytes // 2, dtype=torch.bfloat16, device=dev)
        self.v = torch.empty(nbytes // 2, dtype=torch.bfloat16, device=dev)
        self.len = torch.empty(batch, dtype=torch.int32, device=dev)
        self.c = SpaceKV(_ptr(self.k), _ptr(self.v), _ptr(self.len), batch, capacity, 0, None, 0, 0)
        self.batch, self.capacity = batch, capacity
        self.kv_heads = model.cfg.n_kv_heads if model.cfg.n_kv_heads > 0 else model.cfg.n_heads
        model._check(model.lib.space_kv_reset(model.ctx, C.byref(self.c), _stream(stream)))

    # views in the documented layouts (for tests and tools)
    def k_view(self):
        m = self.model.cfg
        return self.k.view(m.n_layers, self.batch, self.kv_heads, self.capacity, m.head_dim)

    def v_view(self):
        m = self.model.cfg
        return self.v.view(m.n_layers, self.batch, self.kv_heads, self.capacity // 32, m.head_dim, 32)

    def v_rows(self):
        """V as [layers, batch, heads, capacity, head_dim] (a copy)."""
        m = self.model.cfg
        return self.v_view().permute(0, 1, 2, 3, 5, 4).reshape(m.n_layers, self.batch, self.kv_heads, self.capacity,
                                                                m.head_dim)

    def set_len_bound(self, n: int) -> None:
        self.c.host_len_bound = int(n)


class PagePool:
    """Caller-owned k and v pools of the paged cache form: n_pages pages of 32 positions."""

    def __init__(self, model: "Model", n_pages: int):
        import torch
        self.model, self.n_pages = model, int(n_pages)
        nbytes = model.lib.space_kv_pool_bytes(C.byref(model.cfg), self.n_pages)
        if nbytes == 0:
            raise SpaceError(SPACE_EINVAL, f"bad pool size n_pages={n_pages}")
        self.k = torch.zeros(nbytes // 2, dtype=torch.bfloat16, device=model.device)
        self.v = torch.zeros(nbytes // 2, dtype=torch.bfloat16, device=model.device)
        self.kv_heads = model.cfg.n_kv_heads if model.cfg.n_kv_heads > 0 else model.cfg.n_heads

    def k_view(self):
        m = self.model.cfg
        return self.k.view(m.n_layers, self.n_pages, self.kv_heads, 32, m.head_dim)

    def v_view(self):
        m = self.model.cfg
        return self.v.view(m.n_layers, self.n_pages, self.kv_heads, m.head_dim, 32)


class PagedKV:
    """space_kv in the paged form: `batch` sequences over a pool.  `table` is a CUDA int32 tensor
    [batch, table_stride] (a view of a larger table is fine as long as it is contiguous), `len` a CUDA
    int32 tensor [batch]; both stay owned by the caller, who fills the table."""

    def __init__(self, pool: PagePool, table, len_):
        assert table.is_cuda and table.is_contiguous() and table.element_size() == 4 and table.dim() == 2
        assert len_.is_cuda and len_.is_contiguous() and len_.element_size() == 4 and len_.numel() == table.shape[0]
        self.pool, self.table, self.len = pool, table, len_
        self.model = pool.model
        self.batch, self.table_stride = int(table.shape[0]), int(table.shape[1])
        self.capacity = 32 * self.table_stride
        self.kv_heads = pool.kv_heads
        self.c = SpaceKV(_ptr(pool.k), _ptr(pool.v), _ptr(len_), self.batch, self.capacity, 0, _ptr(table),
                         self.table_stride, pool.n_pages)

    def set_len_bound(self, n: int) -> None:
        self.c.host_len_bound = int(n)


class StepOut:
    """Device buffers for the outputs of space_step, allocated once and reused."""

    def __init__(self, model: "Model", batch: int, n_rows: int, max_cands: int, next_rows: int = 0,
                 want_logits: bool = True, emit_cap: int = 0, eos_id: int = -1):
        import torch
        dev, i32 = model.device, torch.int32
        self.logits = torch.empty(batch, n_rows, model.cfg.vocab, dtype=torch.float32, device=dev) if want_logits else None
        self.argmax = torch.empty(batch, n_rows, dtype=i32, device=dev)
        self.accepted_len = torch.empty(batch, dtype=i32, device=dev)
        self.bonus = torch.empty(batch, dtype=i32, device=dev)
        self.new_cands = torch.empty(batch, max(max_cands, 1), dtype=i32, device=dev)
        self.next_tokens = torch.empty(batch, next_rows, dtype=i32, device=dev) if next_rows else None
        self.emit = torch.zeros(batch, emit_cap, dtype=i32, device=dev) if emit_cap else None
        self.emit_len = torch.zeros(batch, dtype=i32, device=dev) if emit_cap else None
        self.finished = torch.zeros(batch, dtype=i32, device=dev) if emit_cap else None
        self.c = SpaceStepOut(_ptr(self.logits), _ptr(self.argmax), _ptr(self.accepted_len), _ptr(self.bonus),
                              _ptr(self.new_cands), max(max_cands, 1), _ptr(self.next_tokens), _ptr(self.emit),
                              _ptr(self.emit_len), emit_cap, int(eos_id) if emit_cap else -1, _ptr(self.finished))


class SampleOut:
    """Device buffers for the outputs of space_sample_verify, allocated once and reused."""

    def __init__(self, model: "Model", batch: int, n_groups: int, max_cands: int, top_k: int, next_rows: int = 0,
                 emit_cap: int = 0, eos_id: int = -1):
        import torch
        dev, i32, f32 = model.device, torch.int32, torch.float32
        self.max_cands, self.top_k = max_cands, top_k
        self.accepted_len = torch.empty(batch, dtype=i32, device=dev)
        self.extra = torch.empty(batch, dtype=i32, device=dev)
        self.new_cands = torch.empty(batch, max_cands, dtype=i32, device=dev)
        self.new_pc = torch.empty(batch, max_cands, dtype=f32, device=dev)
        self.new_ids = torch.empty(batch, max_cands, top_k, dtype=i32, device=dev)
        self.new_probs = torch.empty(batch, max_cands, top_k, dtype=f32, device=dev)
        self.next_tokens = torch.empty(batch, next_rows, dtype=i32, device=dev) if next_rows else None
        self.emit = torch.zeros(batch, emit_cap, dtype=i32, device=dev) if emit_cap else None
        self.emit_len = torch.zeros(batch, dtype=i32, device=dev) if emit_cap else None
        self.emit_cap = emit_cap
        self.eos_id = int(eos_id) if emit_cap else -1
        self.finished = torch.zeros(batch, dtype=i32, device=dev) if emit_cap else None
        self.ratios = torch.empty(batch, max(n_groups - 1, 1), dtype=f32, device=dev)


class Model:
    """space_ctx of one model.  `weights` maps tensor names to CUDA bf16 tensors:
    embed [V+1, d], final_norm [d], lm_head [V, d], layers: list of dicts with attn_norm wq wk wv wo
    ffn_norm w_gate w_up w_down."""

    def __init__(self, shape, weights: Dict[str, object], max_batch: int = 1, max_rows: int = 36,
                 max_ctx: int = 4096):
        import torch
        self.lib = load_library()
        self.shape = shape
        self.cfg = SpaceConfig(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.ffn, shape.vocab,
                               max_batch, max_rows, max_ctx, shape.rms_eps, shape.rope_base,
                               int(getattr(shape, "n_kv_heads", 0)))
        layers = weights["layers"]
        arr = (SpaceLayerWeights * shape.n_layers)()
        for l, lw in enumerate(layers):
            if lw is None:  # handed over later with load_layer()
                continue
            for name, _ in SpaceLayerWeights._fields_:
                t = lw[name]
                assert t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous(), name
                setattr(arr[l], name, _ptr(t))
        for name in ("embed", "final_norm", "lm_head"):
            t = weights[name]
            assert t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous(), name
        self.device = weights["embed"].device
        w = SpaceWeights(_ptr(weights["embed"]), _ptr(weights["final_norm"]), _ptr(weights["lm_head"]), arr)
        h = C.c_void_p()
        torch.cuda.synchronize()
        rc = self.lib.space_init(C.byref(self.cfg), C.byref(w), C.byref(h))
        if rc != SPACE_OK:
            raise SpaceError(rc, (self.lib.space_last_error(None) or b"").decode())
        self.ctx = h
        self._layouts: List[Layout] = []

    def _check(self, rc: int) -> None:
        if rc != SPACE_OK:
            raise SpaceError(rc, (self.lib.space_last_error(self.ctx) or b"").decode())

    def close(self) -> None:
        if getattr(self, "ctx", None):
            self.lib.space_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def layout(self, spec: BlockLayoutSpec) -> Layout:
        lay = Layout(self, spec)
        self._layouts.append(lay)
        return lay

    def kv_cache(self, batch: int, capacity: int) -> KVCache:
        return KVCache(self, batch, capacity)

    def step(self, tokens, layout: Layout, kv: KVCache, out: StepOut, next_layout: Optional[Layout] = None,
             stream=None) -> None:
        """space_step: tokens is a CUDA int32 tensor [batch, layout.n_rows]."""
        assert tokens.is_cuda and tokens.dtype.is_floating_point is False and tokens.element_size() == 4
        assert tokens.numel() == kv.batch * layout.n_rows and tokens.is_contiguous()
        rc = self.lib.space_step(self.ctx, _ptr(tokens), layout.handle,
                                 next_layout.handle if next_layout is not None else None,
                                 C.byref(kv.c), C.byref(out.c), _stream(stream))
        self._check(rc)

    def prefill(self, tokens, layout: Layout, kv: KVCache, stream=None) -> None:
        """space_prefill: the forward without LM head and verification; commit with kv_commit(kv, None, G - 1)."""
        assert tokens.is_cuda and tokens.dtype.is_floating_point is False and tokens.element_size() == 4
        assert tokens.numel() == kv.batch * layout.n_rows and tokens.is_contiguous()
        self._check(self.lib.space_prefill(self.ctx, _ptr(tokens), layout.handle, C.byref(kv.c), _stream(stream)))

    def load_layer(self, l: int, lw: Dict[str, object]) -> None:
        """space_load_layer: hands over a layer that was None in `weights["layers"]`."""
        import torch
        one = SpaceLayerWeights()
        for name, _ in SpaceLayerWeights._fields_:
            t = lw[name]
            assert t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous(), name
            setattr(one, name, _ptr(t))
        torch.cuda.synchronize()
        self._check(self.lib.space_load_layer(self.ctx, int(l), C.byref(one)))

    def sample_verify(self, logits, tokens, layout: Layout, p_c, uniforms, out: SampleOut, top_k: int = 10,
                      top_p: float = 0.95, residual: bool = False, draft_ids=None, draft_probs=None,
                      next_layout: Optional[Layout] = None, stream=None, static: bool = False) -> None:
        """space_sample_verify (static=True: space_sample_verify_static, same arguments): logits float32 [batch, L, vocab], tokens int32 [batch, L], p_c float32
        [batch, max_cands], uniforms float32 [batch, G + max_cands], all CUDA and contiguous."""
        import torch
        batch = tokens.shape[0]
        for t, dt in ((logits, torch.float32), (tokens, torch.int32), (p_c, torch.float32), (uniforms, torch.float32)):
            assert t.is_cuda and t.dtype == dt and t.is_contiguous()
        assert p_c.shape == (batch, out.max_cands) and uniforms.shape == (batch, layout.spec.n_groups + out.max_cands)
        assert logits.shape == (batch, layout.n_rows, self.cfg.vocab)
        params = SpaceSampleParams(int(top_k), float(top_p), int(bool(residual)))
        io = SpaceSampleIO(_ptr(logits), _ptr(tokens), _ptr(p_c), _ptr(uniforms), _ptr(draft_ids), _ptr(draft_probs),
                           _ptr(out.accepted_len), _ptr(out.extra), _ptr(out.new_cands), _ptr(out.new_pc),
                           out.max_cands, _ptr(out.new_ids), _ptr(out.new_probs), _ptr(out.next_tokens), _ptr(out.emit),
                           _ptr(out.emit_len), out.emit_cap, _ptr(out.ratios), out.eos_id, _ptr(out.finished))
        fn = self.lib.space_sample_verify_static if static else self.lib.space_sample_verify
        rc = fn(self.ctx, batch, layout.handle, next_layout.handle if next_layout is not None else None,
                C.byref(params), C.byref(io), _stream(stream))
        self._check(rc)

    def sar_loss(self, logits, labels, row_loss=None, stream=None):
        """space_sar_loss: logits float32 [rows, vocab], labels int32 [rows] (CUDA).  Returns (loss_sum, n_terms)
        as one-element CUDA tensors."""
        import torch
        assert logits.is_cuda and logits.dtype == torch.float32 and logits.is_contiguous()
        assert labels.is_cuda and labels.dtype == torch.int32 and labels.is_contiguous()
        rows = labels.numel()
        assert logits.numel() == rows * self.cfg.vocab
        loss = torch.empty(1, dtype=torch.float32, device=self.device)
        n = torch.empty(1, dtype=torch.int32, device=self.device)
        self._check(self.lib.space_sar_loss(self.ctx, _ptr(logits), _ptr(labels), rows, _ptr(row_loss), _ptr(loss), _ptr(n),
                                            _stream(stream)))
        return loss, n

    def kv_commit(self, kv: KVCache, accepted_len=None, accepted_all: int = 0, stream=None) -> None:
        rc = self.lib.space_kv_commit(self.ctx, C.byref(kv.c), _ptr(accepted_len), int(accepted_all), _stream(stream))
        self._check(rc)

    def kv_rollback(self, kv: KVCache, n=None, n_all: int = 0, stream=None) -> None:
        rc = self.lib.space_kv_rollback(self.ctx, C.byref(kv.c), _ptr(n), int(n_all), _stream(stream))
        self._check(rc)

    def tune_rows(self, rows: int, stream=None) -> None:
        """space_tune_rows: measures how the many-row projection kernel should cut `rows` rows (waits for
        the stream; never changes a result).  A row count measured before is not measured again."""
        done = self.__dict__.setdefault("_tuned_rows", set())
        if int(rows) in done:
            return
        self._check(self.lib.space_tune_rows(self.ctx, int(rows), _stream(stream)))
        done.add(int(rows))

    def timing_enable(self, classes: Sequence[str], max_records: int = 4096) -> None:
        mask = 0
        for c in classes:
            mask |= 1 << KERNEL_CLASSES.index(c)
        self._check(self.lib.space_timing_enable(self.ctx, mask, max_records))

    def timing_read(self, stream=None) -> Dict[str, tuple]:
        """{class: (total_ms, launches)} since the last read."""
        n = len(KERNEL_CLASSES)
        ms, cnt = (C.c_double * n)(), (C.c_int64 * n)()
        self._check(self.lib.space_timing_read(self.ctx, _stream(stream), ms, cnt))
        return {KERNEL_CLASSES[i]: (ms[i], cnt[i]) for i in range(n) if cnt[i]}

    def debug_buffer(self, name: str) -> np.ndarray:
        """Copy of a scratch buffer (test hook) as a flat numpy array of its element type."""
        import torch
        ptr, nbytes = C.c_void_p(), C.c_size_t()
        self._check(self.lib.space_debug_buffer(self.ctx, name.encode(), C.byref(ptr), C.byref(nbytes)))
        torch.cuda.synchronize()
        host = np.empty(nbytes.value, dtype=np.uint8)
        hip = C.CDLL("libamdhip64.so")
        hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
        rc = hip.hipMemcpy(host.ctypes.data, ptr, nbytes.value, 2)
        if rc != 0:
            raise SpaceError(SPACE_EHIP, f"hipMemcpy failed with {rc}")
        dt = {"x": np.float32, "pos": np.int32}.get(name, np.uint16)
        return host.view(dt)

    def device_faults(self, stream=None) -> int:
        rc = self.lib.space_device_faults(self.ctx, _stream(stream))
        if rc < 0:
            self._check(rc)
        return rc


def weights_to_device(weights_bits: Dict[str, object], device="cuda:0") -> Dict[str, object]:
    """uint16 bf16 bit patterns (numpy) -> CUDA bf16 tensors with the same structure."""
    import torch

    def up(a: np.ndarray):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(device).view(torch.bfloat16)

    out: Dict[str, object] = {k: up(v) for k, v in weights_bits.items() if k != "layers"}
    out["layers"] = [{k: up(v) for k, v in lw.items()} for lw in weights_bits["layers"]]
    return out


def sar_transform(tokens: Sequence[int], n_prompt: int, k: int, mask_id: int, p_ar: float, u_keep: float, u_pos: float):
    """space_sar_transform (host side, no GPU needed): returns (input_ids, labels, m); m = 0 for an untouched sample."""
    lib = load_library()
    toks = np.ascontiguousarray(tokens, dtype=np.int32)
    n = len(toks)
    ids, lab = np.zeros(n, dtype=np.int32), np.zeros(n, dtype=np.int32)
    n_in, n_lab, m = C.c_int32(), C.c_int32(), C.c_int32()
    p = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    rc = lib.space_sar_transform(p(toks), int(n_prompt), n - int(n_prompt), int(k), int(mask_id), float(p_ar), float(u_keep),
                                 float(u_pos), p(ids), p(lab), C.byref(n_in), C.byref(n_lab), C.byref(m))
    if rc != SPACE_OK:
        raise SpaceError(rc, "space_sar_transform")
    return ids[: n_in.value].tolist(), lab[: n_lab.value].tolist(), m.value
