"""space_sample_verify_static (the entry point for callers that cannot allocate: its scratch is a fixed
array inside the library's device image) against space_sample_verify on the same inputs, through the
C ABI: every output equal bit for bit, on two calls in a row, the second one with a smaller input, so
that what the first call left in the shared array cannot leak into the second."""
import dataclasses

import numpy as np
import pytest

from oracle import space_oracle as so
from space_inputs import SHAPES, all_weights
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu


def _inputs(rng, spec, V, k, B, mask_id):
    L = spec.n_rows
    P = (rng.standard_normal((B, L, V)) * 2.5).astype(np.float32)
    toks = np.zeros((B, L), dtype=np.int32)
    p_c = rng.uniform(0.02, 0.3, size=(B, k)).astype(np.float32)   # small P_c: acceptance is common
    u = rng.uniform(0.0, 1.0, size=(B, 2 * k + 1)).astype(np.float32)
    for b in range(B):
        # candidates that the verifier finds plausible, so that accepted counts above 0 occur
        cands = [int(np.argmax(P[b, g * (k + 1)])) if rng.uniform() < 0.85 else int(rng.integers(0, V)) for g in range(k)]
        toks[b], _ = so.extended_input([int(rng.integers(0, V))], cands, k, mask_id)
    return P, toks, p_c, u


def _run(torch, gm, binding, lay, spec, k, top_k, top_p, B, inputs, static):
    P, toks, p_c, u = inputs
    out = binding.SampleOut(gm, B, spec.n_groups, k, top_k, next_rows=spec.n_rows, emit_cap=16)
    gm.sample_verify(torch.from_numpy(P).cuda(), torch.from_numpy(toks).cuda(), lay, torch.from_numpy(p_c).cuda(),
                     torch.from_numpy(u).cuda(), out, top_k=top_k, top_p=top_p, next_layout=lay, static=static)
    torch.cuda.synchronize()
    return {n: getattr(out, n).cpu().numpy().copy() for n in
            ("accepted_len", "extra", "new_cands", "new_pc", "new_ids", "new_probs", "next_tokens", "emit", "emit_len",
             "ratios", "finished")}


def test_static_scratch_entry_point_equals_the_allocating_one():
    torch = gc.require_gpu()
    from paper_2402_11809_amd import binding, layout as lo
    V = 5000
    shape = dataclasses.replace(SHAPES["tiny"], vocab=V, n_layers=1)
    gm = gc.make_gpu_model(shape, all_weights(shape, seed=0), max_batch=6, max_rows=36, max_ctx=64)
    rng = np.random.default_rng(2024)
    # first call: 6 sequences of 36 rows, 10 kept tokens; second call: 2 sequences of 16 rows, 4 kept tokens
    seen_accept = 0
    for k, B, top_k, top_p in ((5, 6, 10, 0.95), (3, 2, 4, 0.8)):
        spec = lo.paper_layout(k)
        lay = gm.layout(spec)
        inputs = _inputs(rng, spec, V, k, B, shape.mask_id)
        ref = _run(torch, gm, binding, lay, spec, k, top_k, top_p, B, inputs, static=False)
        got = _run(torch, gm, binding, lay, spec, k, top_k, top_p, B, inputs, static=True)
        for name, r in ref.items():
            g = got[name]
            assert g.dtype == r.dtype and g.shape == r.shape, name
            assert np.array_equal(g.view(np.uint8), r.view(np.uint8)), (k, name)
        seen_accept += int((ref["accepted_len"] > 0).sum())
        assert gm.device_faults() == 0
    assert seen_accept >= 1


def test_static_scratch_entry_point_rejects_oversized_input():
    gc.require_gpu()
    from paper_2402_11809_amd import binding, layout as lo
    shape = dataclasses.replace(SHAPES["tiny"], n_layers=1)
    gm = gc.make_gpu_model(shape, all_weights(shape, seed=0), max_batch=32, max_rows=36, max_ctx=64)
    lay = gm.layout(lo.paper_layout(5))  # 36 rows: 29 sequences are 1044 rows > 1024
    params = binding.SpaceSampleParams(10, 0.95, 0)
    io = binding.SpaceSampleIO()
    import ctypes as C
    rc = gm.lib.space_sample_verify_static(gm.ctx, 29, lay.handle, None, C.byref(params), C.byref(io), None)
    assert rc == binding.SPACE_ECAPACITY
    assert b"SPACE_STATIC_MAX_ROWS" in gm.lib.space_last_error(gm.ctx)
