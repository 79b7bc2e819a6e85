"""Seeded random configurations of one step against the oracle, through the C ABI: model shape (with
and without grouped-query attention, head sizes 64 and 128), batch 1..4, any grouped layout of up to 96
rows, ragged contexts from empty to 150 positions, either attention path or the library's choice, the
many-row projection kernel forced or not, contiguous or paged cache."""
import numpy as np
import pytest

from oracle import space_oracle as so
from space_inputs import SHAPES, all_weights
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu

NAMES = ("tiny", "small128", "gqa-small", "gqa128")
TUNES = (None, "attn=0", "attn=1000000", "wide=1", "wide=1,attn=0", "wide=1,wideks=2")


@pytest.fixture(scope="module")
def models():
    torch = gc.require_gpu()
    w = {n: all_weights(SHAPES[n], seed=1) for n in NAMES}
    return torch, w, {n: gc.oracle_model(SHAPES[n], w[n]) for n in NAMES}


@pytest.mark.parametrize("case", range(24))
def test_random_step_configuration(models, case):
    torch, weights, oracles = models
    from paper_2402_11809_amd import binding, layout as lo
    rng = np.random.default_rng(5000 + case)
    name = NAMES[int(rng.integers(0, 4))]
    shape, om = SHAPES[name], oracles[name]
    B = int(rng.integers(1, 5))
    while True:
        G, m = int(rng.integers(1, 10)), int(rng.integers(0, 9))
        if G * (1 + m) <= 96:
            break
    spec = lo.grouped_layout(G, m)
    L = spec.n_rows
    tune = TUNES[int(rng.integers(0, len(TUNES)))]
    paged = bool(rng.integers(0, 2))
    ctxs = [int(rng.integers(0, 150)) for _ in range(B)]
    gm = gc.make_gpu_model(shape, weights[name], max_batch=B, max_rows=L, max_ctx=256, tune=tune)
    cont = binding.KVCache(gm, B, 256)
    okvs = []
    for b, c in enumerate(ctxs):
        okv = gc.synthetic_oracle_kv(om, seed=case * 10 + b, ctx=c, std=0.5) if c > 0 else so.OracleKV(om)
        if c > 0:
            gc.upload_oracle_kv(torch, cont, b, okv)
        else:
            cont.len[b] = 0
        okvs.append(okv)
    cache = cont
    if paged:  # the same positions in pages scattered over a pool
        pool = binding.PagePool(gm, B * 8 + 3)
        perm = rng.permutation(B * 8 + 3)[: B * 8].reshape(B, 8).astype(np.int32)
        kp, vp, kc, vc = pool.k_view(), pool.v_view(), cont.k_view(), cont.v_view()
        for b in range(B):
            for j in range(8):
                kp[:, perm[b, j]] = kc[:, b, :, 32 * j:32 * j + 32]
                vp[:, perm[b, j]] = vc[:, b, :, j]
        cache = binding.PagedKV(pool, torch.from_numpy(perm).cuda(), cont.len.clone())
    cache.set_len_bound(max(ctxs))
    toks = rng.integers(0, shape.vocab, size=(B, L)).astype(np.int32)
    toks[:, spec.is_mask == 1] = shape.mask_id
    out = binding.StepOut(gm, B, L, max(1, m))
    gm.step(torch.from_numpy(toks).cuda(), gm.layout(spec), cache, out)
    torch.cuda.synchronize()
    what = dict(shape=name, B=B, G=G, m=m, tune=tune, paged=paged, ctxs=ctxs)
    assert gm.device_faults() == 0, what
    for b in range(B):
        ref, _, _, _ = so.block_forward_cached(om, okvs[b], toks[b], spec.is_mask.astype(bool))
        err = np.abs(out.logits.cpu().numpy()[b] - ref).max()
        assert err < gc.LOGIT_TIGHT, (what, b, err)
        gc.check_ids(out.argmax.cpu().numpy()[b], ref, f"{what} seq {b}")
