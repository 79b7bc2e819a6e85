"""Helpers shared by the GPU parity tests: build the HIP model and the oracle from the same
seeded weights, move oracle caches into the device layout, compare with the stated bars."""
from __future__ import annotations

import numpy as np

from oracle import space_oracle as so
from space_inputs import bf16_bits_to_f32, f32_to_bf16_bits, normal_bf16

LOGIT_TOL = 2e-2      # absolute bar stated for the build (bf16 weights and cache)
LOGIT_TIGHT = 2e-3    # what the split-bf16 activation path keeps on models of a few layers
LOGIT_DEEP = 5e-3     # ... and at 32 layers (measured 2.0e-3)
TIE_GAP = 1e-3        # an id may differ only where the oracle's top-2 logits are this close


def require_gpu():
    import pytest
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2402_11809_amd import binding
    binding.load_library()  # fail loudly if the HIP library is not built
    return torch


def make_gpu_model(shape, weights_bits, max_batch=1, max_rows=36, max_ctx=4096, attn=None, tune=None):
    """attn: None (the library picks the attention kernel), "head" (one workgroup per head and query
    tile whenever the block has at most 48 rows) or "split" (always the split over the key axis).
    tune: a raw SPACE_TUNE string instead (e.g. "wide=1": the many-row projection kernel for every
    row count).  The library reads the override once, when the model is created."""
    import os
    from paper_2402_11809_amd import binding
    dev_w = binding.weights_to_device(weights_bits)
    old = os.environ.get("SPACE_TUNE")
    if tune is not None:
        attn = tune
        os.environ["SPACE_TUNE"] = tune
    elif attn is not None:
        os.environ["SPACE_TUNE"] = {"head": "attn=1000000", "split": "attn=0"}[attn]
    try:
        return binding.Model(shape, dev_w, max_batch=max_batch, max_rows=max_rows, max_ctx=max_ctx)
    finally:
        if attn is not None:
            if old is None:
                del os.environ["SPACE_TUNE"]
            else:
                os.environ["SPACE_TUNE"] = old


def oracle_model(shape, weights_bits, precision="bf16_kv"):
    return so.model_from_weights(shape, weights_bits, precision)


def bits_to_f64(bits):
    return bf16_bits_to_f32(bits).astype(np.float64)


def synthetic_oracle_kv(model, seed, ctx, std=1.0):
    """OracleKV filled with N(0, std) bf16 keys / values (single-layer micro-benchmark recipe)."""
    kv = so.OracleKV(model)
    for l in range(model.n_layers):
        kv.k[l] = bits_to_f64(normal_bf16(seed, l, "kv_k", (ctx, model.kv_heads, model.head_dim), std))
        kv.v[l] = bits_to_f64(normal_bf16(seed, l, "kv_v", (ctx, model.kv_heads, model.head_dim), std))
    return kv


def upload_oracle_kv(torch, cache, b, okv):
    """Writes an OracleKV (values must be bf16-representable) into sequence b of a device cache."""
    ctx = okv.length
    kview, vview = cache.k_view(), cache.v_view()
    H, dh = kview.shape[2], kview.shape[4]
    pad = (-ctx) % 32
    for l in range(len(okv.k)):
        kb = torch.from_numpy(f32_to_bf16_bits(okv.k[l].astype(np.float32)).view(np.int16)).to(kview.device)
        vb = torch.from_numpy(f32_to_bf16_bits(okv.v[l].astype(np.float32)).view(np.int16)).to(kview.device)
        kview[l, b, :, :ctx, :] = kb.view(torch.bfloat16).permute(1, 0, 2)
        v = vb.view(torch.bfloat16).permute(1, 0, 2)  # [H, ctx, dh]
        if pad:
            v = torch.cat([v, torch.zeros(H, pad, dh, dtype=v.dtype, device=v.device)], dim=1)
        nb = (ctx + pad) // 32
        vview[l, b, :, :nb] = v.reshape(H, nb, 32, dh).permute(0, 1, 3, 2)
    lens = cache.len.cpu()
    lens[b] = ctx
    cache.len.copy_(lens)
    cache.set_len_bound(int(lens.max()))


def download_kv_rows(cache, l, b, lo, hi):
    """K and V rows [lo, hi) of layer l, sequence b as float64 [rows, H, dh]."""
    k = cache.k_view()[l, b, :, lo:hi, :].float().permute(1, 0, 2).cpu().numpy().astype(np.float64)
    v = cache.v_rows()[l, b, :, lo:hi, :].float().permute(1, 0, 2).cpu().numpy().astype(np.float64)
    return k, v


def decode_planes(buf_u16, rows, cols):
    """hi + lo operand planes in tile order -> float64 [rows, cols].  The last row tile stores only
    its real rows ([plane][4 column groups][last rows][8])."""
    row_tiles = (rows + 15) // 16
    last = rows - 16 * (row_tiles - 1)
    k_tiles = (cols + 31) // 32
    kstride = (row_tiles - 1) * 1024 + 64 * last
    a = bf16_bits_to_f32(buf_u16[: k_tiles * kstride]).astype(np.float64).reshape(k_tiles, kstride)
    out = np.zeros((rows, k_tiles * 32))
    for t in range(row_tiles):
        c = last if t == row_tiles - 1 else 16
        tile = a[:, t * 1024: t * 1024 + 64 * c].reshape(k_tiles, 2, 4, c, 8)   # kt, plane, kc, row, j
        tile = tile[:, 0] + tile[:, 1]
        out[t * 16: t * 16 + c] = tile.transpose(2, 0, 1, 3).reshape(c, k_tiles * 32)
    return out[:, :cols]


def top2_gap(logits_row):
    part = np.partition(logits_row, -2)[-2:]
    return float(part[1] - part[0])


def check_ids(gpu_ids, oracle_logits, what=""):
    """ids must equal the oracle argmax except where the oracle's top-2 gap is below TIE_GAP, in
    which case the GPU id must be one of those two.  Returns the number of tolerated ties."""
    ties = 0
    ref = np.argmax(oracle_logits, axis=-1)
    for r, (g, o) in enumerate(zip(gpu_ids, ref)):
        if int(g) != int(o):
            gap = top2_gap(oracle_logits[r])
            second = int(np.argsort(oracle_logits[r])[-2])
            assert gap < TIE_GAP and int(g) == second, f"{what} row {r}: gpu {g} oracle {o} gap {gap}"
            ties += 1
    return ties


def assert_bf16_close(got, ref, what="", min_same=0.97):
    """Stored bf16 values.  Both sides round the same quantity to bf16, computed in fp32 on the
    GPU and in fp64 by the oracle, so almost all values are identical and the rest differ by a
    rounding step of the value or of one of the (larger) terms it was summed from."""
    diff = np.abs(got - ref)
    rms = float(np.sqrt(np.mean(ref * ref)))
    bound = np.abs(ref) * 2.0 ** -7 + rms * 2.0 ** -6
    same = float(np.mean(got == ref))
    assert np.all(diff <= bound), f"{what}: max abs diff {diff.max():.3e} (rms {rms:.3e}), identical {same:.4f}"
    assert same > min_same, f"{what}: only {same:.4f} identical"


def real_rows(spec):
    """Rows of the non-mask tokens of a block (x_l, then the candidates), in order."""
    return [int(i) for i in np.nonzero(np.asarray(spec.is_mask) == 0)[0]]


def rel_pos(spec):
    """Position offset of each row relative to the committed length, counted the slow way: the number
    of in-block keys the row sees under Eq. 3 (non-mask keys up to itself, mask keys of its own group
    up to itself) minus one (sentence after Eq. 3)."""
    n = spec.n_rows
    out = np.zeros(n, dtype=np.int32)
    for i in range(n):
        seen = 0
        for j in range(i + 1):
            if not spec.is_mask[j] or (spec.is_mask[i] and spec.group[j] == spec.group[i]):
                seen += 1
        out[i] = seen - 1
    return out
