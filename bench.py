#!/usr/bin/env python3
"""Benchmark of the SPACE auto-correct decoding step on one MI355X.

Workload (benchmark configs[1]): LLaMA-7B-shaped decoder, random-init N(0, 0.02) bf16
weights, batch 1, prompt of 512 uniform-random ids (511 cached positions after prefill), k = 5,
i.e. step blocks of (k+1)^2 = 36 rows.  One "step" is one pass of the whole hot path: space_step
(forward under the semi-autoregressive mask + LM head + argmax + greedy verification + assembly
of the next block) followed by space_kv_commit, with every input resident in HBM.

Prints ONE JSON line: step latency (the metric), tokens/s, achieved HBM GB/s of the whole step,
a roofline object for the dominant kernel (the gate/up projection of the SwiGLU FFN, timed with
HIP events on the step's stream in a second, instrumented pass) and the CPU oracle timed on a
bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(shape, rows, ctx):
    """Bytes one step must move once: all weights, the cached K/V, the staged block K/V."""
    d, hd, f, V, nl = shape.d_model, shape.n_heads * shape.head_dim, shape.ffn, shape.vocab, shape.n_layers
    hkv = shape.kv_heads * shape.head_dim
    per_layer = {"qkv": (hd + 2 * hkv) * d * 2, "o": d * hd * 2, "gate_up": 2 * f * d * 2, "down": d * f * 2}
    w_layers = nl * sum(per_layer.values())
    w_lm = V * d * 2
    kv_tok = nl * 2 * hkv * 2
    total = w_layers + w_lm + ctx * kv_tok + rows * kv_tok + rows * 2
    return total, per_layer, w_lm


def device_weights(shape, seed, threads):
    """Generates the seeded weights layer by layer on host threads and uploads them."""
    import torch
    from space_inputs import head_weights, layer_weights

    def up(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)

    out = {k: up(v) for k, v in head_weights(shape, seed).items()}
    layers = [None] * shape.n_layers
    with ThreadPoolExecutor(max(1, threads)) as ex:
        for l, lw in enumerate(ex.map(lambda i: layer_weights(shape, seed, i), range(shape.n_layers))):
            layers[l] = {k: up(v) for k, v in lw.items()}
    out["layers"] = layers
    return out


def streamed_model(binding, shape, seed, threads, **model_kw):
    """Model whose layers are generated, uploaded, packed (space_load_layer) and freed a few at a time:
    for shapes whose canonical and packed copies do not fit the device together."""
    import torch
    from space_inputs import head_weights, layer_weights

    def up(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)

    w = {k: up(v) for k, v in head_weights(shape, seed).items()}
    w["layers"] = [None] * shape.n_layers
    model = binding.Model(shape, w, **model_kw)
    del w
    window = max(1, min(threads, 8))
    with ThreadPoolExecutor(window) as ex:
        for l0 in range(0, shape.n_layers, window):
            ls = list(range(l0, min(l0 + window, shape.n_layers)))
            for l, lw in zip(ls, ex.map(lambda i: layer_weights(shape, seed, i), ls)):
                dev = {k: up(v) for k, v in lw.items()}
                model.load_layer(l, dev)
                del dev, lw
    torch.cuda.empty_cache()
    return model


def cpu_baseline(shape, k, ctx, seed, n_layers_sample, reps):
    """The oracle's cached step (float64) on the host cores, on the first n_layers_sample layers +
    the LM head of the same workload, extrapolated linearly to all layers."""
    from oracle import space_oracle as so
    from space_inputs import head_weights, layer_weights, normal_bf16, bf16_bits_to_f32
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    sub = shape.with_layers(n_layers_sample)
    w = dict(head_weights(shape, seed))
    with ThreadPoolExecutor(8) as ex:
        w["layers"] = list(ex.map(lambda l: layer_weights(shape, seed, l), range(n_layers_sample)))
    m = so.model_from_weights(sub, w, precision="bf16_kv")
    for l in range(n_layers_sample):
        m.layer(l)
    m.head()
    kv = so.OracleKV(m)
    for l in range(n_layers_sample):
        kv.k[l] = bf16_bits_to_f32(normal_bf16(seed, l, "kv_k", (ctx, shape.kv_heads, shape.head_dim))).astype(np.float64)
        kv.v[l] = bf16_bits_to_f32(normal_bf16(seed, l, "kv_v", (ctx, shape.kv_heads, shape.head_dim))).astype(np.float64)
    rng = np.random.default_rng(seed)
    cands = [int(t) for t in rng.integers(0, shape.vocab, size=k)]

    def layers_only():
        toks, is_mask = so.extended_input([1], cands, k, m.mask_id)
        t0 = time.perf_counter()
        A = so.sar_attention_mask(is_mask, k)
        vis = np.concatenate([np.ones((len(toks), ctx), dtype=np.int64), A], axis=1)
        pos = so.position_ids(vis)
        x = m.head()["embed"][toks]
        for l in range(n_layers_sample):
            x, _, _ = so._layer_forward(m, m.layer(l), x, pos, kv.k[l], kv.v[l], vis)
        t1 = time.perf_counter()
        P = so._logits(m, x)
        so.verify_greedy(P, k, cands)
        t2 = time.perf_counter()
        return t1 - t0, t2 - t1

    layers_only()
    tl, th = [], []
    for _ in range(reps):
        a, b = layers_only()
        tl.append(a)
        th.append(b)
    per_layer = float(np.median(tl)) / n_layers_sample
    head = float(np.median(th))
    ms = (per_layer * shape.n_layers + head) * 1e3
    return {"value": round(ms, 1), "unit": "ms/step", "cores": int(cores), "kind": "oracle",
            "sample": f"oracle cached step (float64 numpy), {n_layers_sample} of {shape.n_layers} layers + LM head + "
                      f"verification at the same shape (36 rows, ctx {ctx}, synthetic N(0,1) bf16 K/V), median of "
                      f"{reps}; layer time scaled to {shape.n_layers} layers"}


def layer_microbench(args):
    """Benchmark configs[2]: one 7B-shaped layer, blocks of L rows under the semi-autoregressive
    mask against 4096 cached positions of N(0,1) K/V; attention, the four projections and the LM head
    + verification are timed separately with the per-class HIP-event hook."""
    import torch
    from paper_2402_11809_amd import binding
    from paper_2402_11809_amd.layout import grouped_layout
    from space_inputs import SHAPES, normal_bf16
    shape = SHAPES[args.shape].with_layers(1)
    w = device_weights(shape, args.seed, 8)
    model = binding.Model(shape, w, max_batch=1, max_rows=36, max_ctx=4224)
    cache = binding.KVCache(model, 1, 4224)
    ctx = 4096

    def up(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    kb = up(normal_bf16(args.seed, 0, "kv_k", (ctx, shape.kv_heads, shape.head_dim)))
    vb = up(normal_bf16(args.seed, 0, "kv_v", (ctx, shape.kv_heads, shape.head_dim)))
    cache.k_view()[0, 0, :, :ctx] = kb.permute(1, 0, 2)
    cache.v_view()[0, 0, :, :ctx // 32] = vb.permute(1, 0, 2).reshape(shape.kv_heads, ctx // 32, 32, shape.head_dim).permute(0, 1, 3, 2)
    cache.len.fill_(ctx)
    classes = ["qkv", "attn", "o", "gate_up", "down", "lm_head", "verify", "norm", "rope"]
    rows = {}
    for groups, masks in [(2, 1), (2, 3), (4, 3), (4, 7), (6, 5)]:
        spec = grouped_layout(groups, masks)
        lay = model.layout(spec)
        out = binding.StepOut(model, 1, spec.n_rows, max(1, masks), want_logits=False)
        toks = torch.randint(0, shape.vocab, (1, spec.n_rows), dtype=torch.int32, device="cuda")
        cache.set_len_bound(ctx)
        for _ in range(5):
            model.step(toks, lay, cache, out)
        model.timing_enable(classes, max_records=16 * args.steps)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            model.step(toks, lay, cache, out)
        tm = model.timing_read()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        model.timing_enable([], 0)
        rows[f"L={spec.n_rows} ({groups}x(1+{masks}))"] = dict(
            {c: round(tm[c][0] * 1e3 / tm[c][1], 2) for c in tm}, step_us_instrumented=round(ms * 1e3, 1))
    print(json.dumps({"metric": "per-kernel-class time of one 7B-shaped layer + LM head, ctx 4096 (us per launch)",
                      "unit": "us", "n_gpus": 1, "data": "synthetic", "dtype": "bf16", "rows": rows}), flush=True)


def batched_bench(args):
    """Benchmark configs[4]: 8 sequences with ragged contexts (uniform 256..4096, seeded), blocks of
    (k+1)^2 rows each, accepted lengths drawn from a geometric law (failure probability 0.4) and passed
    to the commit explicitly.  The caches hold N(0,1) bf16 K/V (no prompt is run: 8 x 4096 positions of
    prefill are not what this mode measures).  Reported against both roofs: the bytes that have to move
    once (weights + the K/V of every sequence) and the MFMA work of B*L rows (split-bf16 operands: two
    MFMAs per product)."""
    import torch
    from paper_2402_11809_amd import binding
    from paper_2402_11809_amd.layout import paper_layout
    from space_inputs import SHAPES, geometric_accept_lengths, ragged_context_lengths
    shape = SHAPES[args.shape] if not args.layers else SHAPES[args.shape].with_layers(args.layers)
    B, k = args.batch, args.k
    spec = paper_layout(k)
    L = spec.n_rows
    w = device_weights(shape, args.seed, args.gen_threads)
    cap = 4096 + 32 * ((args.steps + args.warmup + 2) * (k + 1) // 32 + 2)
    model = binding.Model(shape, w, max_batch=B, max_rows=L, max_ctx=cap)
    del w
    model.tune_rows(B * L)  # how the many-row projection kernel cuts these rows (measured once, results unchanged)
    if args.paged:  # the same positions in pages of 32, scattered over the pool by a seeded permutation
        pool = binding.PagePool(model, B * cap // 32)
        perm = np.random.default_rng(args.seed).permutation(B * cap // 32).astype(np.int32).reshape(B, cap // 32)
        cache = binding.PagedKV(pool, torch.from_numpy(perm).cuda(), torch.zeros(B, dtype=torch.int32, device="cuda"))
        cache.k, cache.v = pool.k, pool.v
    else:
        cache = binding.KVCache(model, B, cap)
    ctxs = [int(c) for c in ragged_context_lengths(seed=args.seed, batch=B, lo=256, hi=4096)]
    g = torch.Generator(device="cuda").manual_seed(args.seed)
    for kv in (cache.k, cache.v):      # N(0, 1) bf16 everywhere; only the first ctx_b slots of a sequence are read
        for c0 in range(0, kv.numel(), 1 << 28):
            n = min(1 << 28, kv.numel() - c0)
            kv[c0:c0 + n] = torch.randn(n, device="cuda", generator=g, dtype=torch.float32).to(torch.bfloat16)
    cache.len.copy_(torch.tensor(ctxs, dtype=torch.int32))
    lay = model.layout(spec)
    out = binding.StepOut(model, B, L, k, next_rows=L, want_logits=False)
    toks = torch.randint(0, shape.vocab, (B, L), dtype=torch.int32, device="cuda", generator=g)
    toks[:, torch.from_numpy(spec.is_mask.astype(bool))] = shape.mask_id
    n_total = args.steps + args.warmup
    acc = torch.from_numpy(np.stack([geometric_accept_lengths(seed=args.seed, batch=B, k=k, p_fail=0.4, step=i)
                                     for i in range(n_total)]).astype(np.int32)).cuda()
    bound = max(ctxs)

    def one(i):
        nonlocal bound
        cache.set_len_bound(bound)
        model.step(toks, lay, cache, out, next_layout=lay)
        model.kv_commit(cache, acc[i])
        bound += k + 1
        toks.copy_(out.next_tokens)

    for i in range(args.warmup):
        one(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.warmup, n_total):
        one(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    assert model.device_faults() == 0
    lens = cache.len.cpu().numpy()
    expect = np.array(ctxs) + (acc.cpu().numpy() + 1).sum(axis=0)
    assert np.array_equal(lens, expect), (lens, expect)
    ctx_mid = (np.array(ctxs) + lens) / 2
    # one more step with every kernel class bracketed by HIP events: where the time goes (the step above is
    # the measurement; this one only apportions it).  The commit is rolled back so that the lengths stay.
    classes = ["norm", "qkv", "rope", "attn", "o", "gate_up", "down", "lm_head"]
    model.timing_enable(classes, max_records=8 * shape.n_layers + 8)
    cache.set_len_bound(int(lens.max()))
    model.step(toks, lay, cache, out, next_layout=lay)
    timing = model.timing_read()
    model.kv_rollback(cache, None, n_all=0)
    model.timing_enable([], 0)
    per_layer_us = {c: round(timing[c][0] * 1e3 / shape.n_layers, 1) for c in timing if c != "lm_head"}
    if "lm_head" in timing:
        per_layer_us["lm_head_per_step"] = round(timing["lm_head"][0] * 1e3, 1)
    w_bytes = algorithmic_bytes(shape, 0, 0)[0]
    kv_tok = 2 * shape.n_layers * shape.kv_heads * shape.head_dim * 2
    bytes_step = int(w_bytes + kv_tok * (ctx_mid.sum() + B * L))
    n_params = w_bytes / 2
    flops = 2.0 * 2.0 * B * L * n_params       # hi and lo plane: two MFMAs per product
    t_hbm, t_mfma = bytes_step / (HBM_PEAK_GBPS * 1e9) * 1e3, flops / 2.5e15 * 1e3
    print(json.dumps({
        "metric": f"batched auto-correct step latency, {args.shape}-shape bf16, batch {B}, k={k}" + (", paged cache" if args.paged else ""),
        "value": round(ms, 3),
        "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 3),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"configs[4]: {B} sequences, contexts {ctxs}, k={k}, {B * L} rows per step, accepted "
                               f"lengths geometric (p_fail 0.4), synthetic N(0,1) K/V", "batch": B, "k": k, "rows": B * L},
        "tokens_per_s": round(float((acc[args.warmup:].sum().item() + B * args.steps) / (ms * 1e-3 * args.steps)), 1),
        "algorithmic_bytes_per_step": bytes_step, "ms_at_hbm_peak": round(t_hbm, 3),
        "mfma_flops_per_step": flops, "ms_at_mfma_peak": round(t_mfma, 3),
        "frac_of_binding_roof": round(max(t_hbm, t_mfma) / ms, 4),
        "kernel_us_per_layer": per_layer_us}), flush=True)


def prefill_bench(args):
    """Prompt of --prompt tokens through space_prefill in chunks of --prefill-chunk rows (Algorithm 1
    needs the keys and values of x_1 .. x_{l-1} before its loop starts).  Reported against the MFMA
    roof: 2 flops x 2 products (hi and lo activation plane) per weight element and row, plus the causal
    attention products."""
    import torch
    from paper_2402_11809_amd import binding
    from paper_2402_11809_amd.runtime import SpaceDecoder
    from space_inputs import SHAPES, prompt_tokens
    shape = SHAPES[args.shape] if not args.layers else SHAPES[args.shape].with_layers(args.layers)
    n, chunk = args.prompt, args.prefill_chunk
    w = device_weights(shape, args.seed, args.gen_threads)
    model = binding.Model(shape, w, max_batch=1, max_rows=max(chunk, 36), max_ctx=(n + 64 + 31) // 32 * 32)
    del w
    dec = SpaceDecoder(model, args.k, capacity=(n + 64 + 31) // 32 * 32, prefill_chunk=chunk)
    dec.tune(n)
    prompt = prompt_tokens(shape, seed=args.seed, n=n + 1)
    times = []
    for rep in range(args.warmup + args.steps):
        dec.kv.len.zero_()
        dec.kv.set_len_bound(0)
        dec.committed = 0
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        dec.prefill(prompt[:, :-1])
        torch.cuda.synchronize()
        if rep >= args.warmup:
            times.append(time.perf_counter() - t0)
    assert model.device_faults() == 0 and int(dec.kv.len.cpu()[0]) == n
    ms = float(np.mean(times)) * 1e3
    w_bytes = algorithmic_bytes(shape, 0, 0)[0]
    lm = shape.vocab * shape.d_model
    n_params = w_bytes / 2 - lm
    attn_flops = shape.n_layers * 2 * 2.0 * 2.0 * shape.n_heads * shape.head_dim * n * n / 2   # QK^T and PV, both split
    flops = 2.0 * 2.0 * n * n_params + attn_flops
    print(json.dumps({
        "metric": f"prompt prefill, {args.shape}-shape bf16, {n} tokens in chunks of {chunk}", "value": round(n / ms * 1e3, 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"prefill of {n} uniform-random ids, chunk {chunk}", "prompt": n, "chunk": chunk},
        "mfma_flops": flops, "ms_at_mfma_peak": round(flops / 2.5e15 * 1e3, 3),
        "frac_of_mfma_peak": round(flops / 2.5e15 / (ms * 1e-3), 4)}), flush=True)


def serve_bench(args):
    """Continuous batching over the paged cache (the paper's serving setting in small): --serve requests
    with seeded prompt lengths (64..1024) and budgets (32..160 new tokens), at most --batch sequences
    in a step, greedy auto-correct decoding with k candidates.  Wall time includes the prefills.  With
    random weights hardly any candidate is accepted, so a step yields about one token per sequence:
    the line measures the machinery, not the method's speed-up."""
    import torch
    from paper_2402_11809_amd import binding
    from paper_2402_11809_amd.serving import ContinuousBatcher, pages_for
    from space_inputs import SHAPES, prompt_tokens
    shape = SHAPES[args.shape] if not args.layers else SHAPES[args.shape].with_layers(args.layers)
    S, k = max(args.batch, 2), args.k
    rng = np.random.default_rng(args.seed)
    reqs = [(int(rng.integers(64, 1025)), int(rng.integers(32, 161))) for _ in range(args.serve)]
    max_ctx = 32 * pages_for(max(p + n for p, n in reqs) + 2 * (k + 1))
    w = device_weights(shape, args.seed, args.gen_threads)
    chunk = 512
    model = binding.Model(shape, w, max_batch=S, max_rows=max(chunk, (k + 1) ** 2) // 1, max_ctx=max_ctx)
    del w
    cb = ContinuousBatcher(model, k, max_seqs=S, n_pages=S * pages_for(max_ctx), max_ctx=max_ctx, prefill_chunk=chunk)
    for i, (p, n) in enumerate(reqs):
        cb.submit(prompt_tokens(shape, seed=args.seed + 100 + i, n=p)[0], n)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    done = cb.run()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    assert model.device_faults() == 0 and len(done) == len(reqs)
    new = sum(len(r.output) for r in done)
    acc = [a for r in done for a in r.accepted]
    print(json.dumps({
        "metric": f"continuous batching, {args.shape}-shape bf16, {len(reqs)} requests, at most {S} sequences, k={k}",
        "value": round(new / dt, 1), "unit": "generated tokens/s", "n_gpus": 1, "steps": cb.steps, "warmup": 0,
        "ms_per_step": round(dt * 1e3 / max(cb.steps, 1), 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{len(reqs)} requests, prompts 64..1024 ({sum(p for p, _ in reqs)} tokens), "
                               f"{new} new tokens, paged cache, prefill chunk {chunk}", "max_seqs": S, "k": k},
        "wall_s": round(dt, 3), "prompt_tokens_per_s_overall": round(sum(p for p, _ in reqs) / dt, 1),
        "mean_accepted": round(float(np.mean(acc)), 3), "restarts": cb.restarts}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--shape", default="7b")
    ap.add_argument("--layers", type=int, default=0, help="run only the first N layers of the shape (0: all)")
    ap.add_argument("--stream-layers", action="store_true",
                    help="hand the layers over one by one (automatic when two copies of the weights exceed the device)")
    ap.add_argument("--k", type=int, default=5)
    ap.add_argument("--prompt", type=int, default=512)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--layer-microbench", action="store_true",
                    help="time the kernel classes of one layer at ctx 4096 for L in {4, 8, 16, 32, 36} instead")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run three plain 256 MiB device copies, the known-size kernel the HBM counters "
                         "of a rocprofv3 --pmc run are scaled by")
    ap.add_argument("--batch", type=int, default=1,
                    help="> 1: the batched configuration (ragged contexts 256..4096, synthetic K/V, forced commits)")
    ap.add_argument("--serve", type=int, default=0, help="continuous batching over this many synthetic requests")
    ap.add_argument("--paged", action="store_true", help="with --batch: the cache in pages of 32 positions behind a block table")
    ap.add_argument("--prefill-chunk", type=int, default=0,
                    help="time the prefill of --prompt tokens in chunks of this many rows instead of the step")
    ap.add_argument("--cpu-layers", type=int, default=8)
    ap.add_argument("--gen-threads", type=int, default=16)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.stderr.write("bench.py: this build measures one GPU only (the step of one sequence group lives on one "
                         "MI355X: batches shard by sequence, larger models by rows / contraction of the projections). "
                         "Run with --gpus 1.\n")
        sys.exit(2)

    if args.layer_microbench:
        layer_microbench(args)
        return
    if args.serve > 0:
        serve_bench(args)
        return
    if args.prefill_chunk > 0:
        prefill_bench(args)
        return
    if args.batch > 1:
        batched_bench(args)
        return

    import torch
    from paper_2402_11809_amd import binding
    from paper_2402_11809_amd import layout as lo
    from paper_2402_11809_amd.runtime import SpaceDecoder
    from space_inputs import SHAPES, prompt_tokens

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    shape = SHAPES[args.shape] if not args.layers else SHAPES[args.shape].with_layers(args.layers)
    k, L = args.k, (args.k + 1) ** 2
    t0 = time.time()
    weight_bytes = algorithmic_bytes(shape, 0, 0)[0]
    if args.stream_layers or 2 * weight_bytes > 240e9:  # canonical + packed would not fit 288 GB
        model = streamed_model(binding, shape, args.seed, args.gen_threads, max_batch=1, max_rows=max(L, 96))
        log(f"weights generated, uploaded and packed layer by layer in {time.time() - t0:.1f}s")
    else:
        w = device_weights(shape, args.seed, args.gen_threads)
        log(f"weights generated and uploaded in {time.time() - t0:.1f}s")
        model = binding.Model(shape, w, max_batch=1, max_rows=max(L, 96))
        del w
    torch.cuda.empty_cache()
    log(f"space_init done at {time.time() - t0:.1f}s")

    total_steps = args.warmup + 3 * args.steps + 16
    capacity = ((args.prompt + 6 * total_steps + 64 + 31) // 32) * 32
    # The product's own loop (runtime.SpaceDecoder): prefill, the first iteration of Algorithm 1, then the
    # iteration (space_step + space_kv_commit) captured once into a HIP graph and replayed.  It reads and
    # writes device memory only; the cache-length bound the launches are shaped for covers every replay.
    n_new = (k + 1) * (args.warmup + args.steps + 3)  # what the capture, the warm-up and the timed replays can emit
    dec = SpaceDecoder(model, k, batch=1, capacity=capacity, prefill_chunk=96, want_logits=False,
                       emit_cap=(k + 1) * (total_steps + 1), graph=not args.no_graph)
    prompt = prompt_tokens(shape, args.seed, args.prompt)
    dec.start(prompt, n_new)
    torch.cuda.synchronize()
    log(f"prefill done at {time.time() - t0:.1f}s, len = {int(dec.kv.len.cpu()[0])}")
    dec.prepare()  # the capture (and its rehearsal), outside the timed region
    graph = dec._graphs[0] if dec._graphs else None
    eager_dec = dec._eager[0]

    def run_step():
        dec.run(1)

    def one_step():
        eager_dec()

    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    len0 = int(dec.kv.len.cpu()[0])
    emit0 = int(dec.out.emit_len.cpu()[0])
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    ms_per_step = (t_end - t_start) * 1e3 / args.steps
    emit1 = int(dec.out.emit_len.cpu()[0])
    assert int(dec.kv.len.cpu()[0]) - len0 == emit1 - emit0 and model.device_faults() == 0
    # the same steps launched one kernel at a time from the host, for comparison (the launches are sized
    # anew from the true length, read here outside every timed region)
    dec.rebound(min(args.steps, 32) + 1)
    t_e0 = time.perf_counter()
    for _ in range(min(args.steps, 32)):
        one_step()
    torch.cuda.synchronize()
    ms_eager = (time.perf_counter() - t_e0) * 1e3 / min(args.steps, 32)
    tokens = emit1 - emit0
    len1 = len0 + tokens
    ctx_mid = (len0 + len1) // 2
    bytes_step, per_layer_bytes, lm_bytes = algorithmic_bytes(shape, L, ctx_mid)
    gbps = bytes_step / (ms_per_step * 1e-3) / 1e9

    # second pass: the same steps with the projection launches bracketed by HIP events
    classes = ["qkv", "o", "gate_up", "down", "lm_head", "attn"]
    steps_instr = min(args.steps, 32)
    model.timing_enable(classes, max_records=(5 * shape.n_layers + 1) * steps_instr)
    dec.rebound(steps_instr + 1)
    t2 = time.perf_counter()
    for _ in range(steps_instr):
        one_step()
    timing = model.timing_read()
    ms_instr = (time.perf_counter() - t2) * 1e3 / steps_instr
    model.timing_enable([], 0)
    kernel_us = {c: timing[c][0] * 1e3 / timing[c][1] for c in timing}
    class_bytes_all = dict(per_layer_bytes, lm_head=lm_bytes)
    # the dominant kernel: the class with the largest share of the measured step among those that move weights
    dom = max((c for c in kernel_us if c in class_bytes_all), key=lambda c: timing[c][0])
    dom_names = {"gate_up": "gemm_skinny_kernel, SwiGLU epilogue (gate/up projection)",
                 "qkv": "gemm_skinny_kernel, fp32 partial sums (QKV projection)",
                 "down": "gemm_skinny_kernel, fp32 partial sums (down projection)",
                 "o": "gemm_skinny_kernel, fp32 partial sums (output projection)",
                 "lm_head": "gemm_skinny_kernel, argmax epilogue (LM head)"}
    dom_bytes = class_bytes_all[dom]
    dom_s = kernel_us[dom] * 1e-6
    achieved = dom_bytes / dom_s / 1e9
    class_bytes = dict(per_layer_bytes, lm_head=lm_bytes)
    per_class = {c: {"us": round(kernel_us[c], 2),
                     "GBps": round(class_bytes[c] / (kernel_us[c] * 1e-6) / 1e9, 1) if c in class_bytes else None}
                 for c in kernel_us}

    # HBM bytes per launch of that kernel come from hardware counters, which this process cannot read: they
    # are taken from the committed rocprofv3 --pmc summary of this very command (FETCH_SIZE and WRITE_SIZE
    # in runs of their own) and labelled as such; null when that summary does not cover this workload.
    traffic, traffic_source = None, "not measured in this run (needs rocprofv3 --pmc)"
    tpath = os.path.join(ROOT, "profiles", "gate_up_7b_k5_hbm_traffic.txt")
    if dom == "gate_up" and args.shape == "7b" and k == 5 and not args.layers and os.path.exists(tpath):
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch="):
                traffic = float(line.split("=", 1)[1])
                traffic_source = ("stored: profiles/gate_up_7b_k5_hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE, "
                                  "of this command on an earlier run; not measured in this run)")

    result = {
        "metric": "auto-correct step latency, 7B-shape bf16, k=5" if args.shape == "7b" and k == 5 and not args.layers
                  else f"auto-correct step latency, {shape.name}-shape bf16, k={k}",
        "value": round(ms_per_step, 4), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{ {'7b': 'configs[1]', '13b': 'configs[3]'}.get(args.shape, 'extra shape') }: LLaMA-{shape.name}-shaped decoder, random init N(0,0.02) bf16, batch 1, "
                               f"prompt {args.prompt}, k={k}, block {L} rows, ctx {len0}->{len1}",
                   "shape": args.shape, "k": k, "block_rows": L, "batch": 1, "ctx_start": len0, "ctx_end": len1},
        "achieved_hbm_GBps": round(gbps, 1), "hbm_frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4),
        "algorithmic_bytes_per_step": bytes_step,
        "tokens_per_s": round(tokens / (t_end - t_start), 1), "tokens_per_step": round(tokens / args.steps, 3),
        "launch": "eager" if graph is None else "hip_graph_replay", "ms_per_step_eager": round(ms_eager, 4),
        "ms_per_step_instrumented": round(ms_instr, 4),
        "kernels": per_class,
        "roofline": {"bound": "hbm", "kernel": dom_names[dom],
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic, "traffic_source": traffic_source,
                     "bytes_per_launch": dom_bytes, "avg_us_per_launch": round(kernel_us[dom], 2),
                     "launches_timed": int(timing[dom][1]),
                     "share_of_step": round(timing[dom][0] / steps_instr / sum(v[0] / steps_instr for v in timing.values()), 3),
                     "whole_step_frac": round(gbps / HBM_PEAK_GBPS, 4)},
    }
    # the rejection-sampling form of the verification (top-k 10, top-p 0.95) on one block of logits:
    # two small launches that would replace the greedy scan; reported next to the step, not part of it
    if not args.pmc_calibration:
        spec = lo.paper_layout(k)
        lay = model.layout(spec)
        g = torch.Generator(device="cuda").manual_seed(args.seed)
        logits = torch.randn(1, L, shape.vocab, device="cuda", generator=g) * 2.5
        toks = torch.randint(0, shape.vocab, (1, L), device="cuda", generator=g, dtype=torch.int32)
        sout = binding.SampleOut(model, 1, spec.n_groups, k, 10, next_rows=L)
        p_c = torch.ones(1, k, device="cuda")
        uni = torch.rand(1, spec.n_groups + k, device="cuda", generator=g)
        def sv():
            model.sample_verify(logits, toks, lay, p_c, uni, sout, top_k=10, top_p=0.95, next_layout=lay)
        sv()
        torch.cuda.synchronize()
        if args.no_graph:
            run_sv, per = sv, 1
        else:  # ten calls per replay, so that the host's marshalling is not what gets timed
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                sv()
            torch.cuda.current_stream().wait_stream(side)
            sg = torch.cuda.CUDAGraph()
            with torch.cuda.graph(sg):
                for _ in range(10):
                    sv()
            run_sv, per = sg.replay, 10
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        run_sv()
        ev0.record()
        for _ in range(10):
            run_sv()
        ev1.record()
        torch.cuda.synchronize()
        result["sample_verify_us"] = round(ev0.elapsed_time(ev1) * 1e3 / (10 * per), 2)
        del logits
    if not args.pmc_calibration:
        # two reference points beside the vendor peak: what a plain 1 GiB device copy moves on this machine
        # (read + write), and what the measured latency would give at the mean tokens per step the paper
        # reports for its fine-tuned models (Table 1: 2.23 on XSum, 3.54 on HumanEval-X) -- a labelled
        # projection: random weights accept nothing, the acceptance itself is not measured here
        src = torch.empty(256 << 20, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for _ in range(10):
            dst.copy_(src)
        ev1.record()
        torch.cuda.synchronize()
        copy_gbps = 10 * 2 * src.numel() * 4 / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
        del src, dst
        result["device_copy_GBps"] = round(copy_gbps, 1)
        result["hbm_frac_of_device_copy"] = round(gbps / copy_gbps, 4)
        result["projected_tokens_per_s"] = {"kind": "projection, not a measurement", "at_2.23_tokens_per_step": round(2.23e3 / ms_per_step, 1),
                                            "at_3.54_tokens_per_step": round(3.54e3 / ms_per_step, 1)}
    if args.pmc_calibration:
        src = torch.full((64 << 20,), 1.0, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(shape, k, ctx_mid, args.seed, min(args.cpu_layers, shape.n_layers), reps=5)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
