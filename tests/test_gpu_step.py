"""GPU parity of the auto-correct step against the CPU oracle, through the C ABI.

The oracle runs in float64 with the one rounding the implementation's storage format imposes
(k after rotary and v are cached in bf16).  Bar: logits within 2e-2 absolute (in practice within
2e-3: activations feed the matrix units as split bf16 hi + lo planes); token ids, accepted
lengths and new candidates identical except where the oracle's top-2 logits are closer than
1e-3; cache rows identical except for values that sit on a bf16 rounding boundary.
"""
import numpy as np
import pytest

from oracle import space_oracle as so
from space_inputs import SHAPES, all_weights, prompt_tokens
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_mod():
    return gc.require_gpu()


def _setup(shape_name, max_batch=1, max_rows=64, seed=0, attn=None):
    shape = SHAPES[shape_name]
    w = all_weights(shape, seed=seed)
    gm = gc.make_gpu_model(shape, w, max_batch=max_batch, max_rows=max_rows, attn=attn)
    om = gc.oracle_model(shape, w)
    return shape, gm, om


def _run_step(torch, gm, cache, spec, tokens_np, next_spec=None, batch=1):
    from paper_2402_11809_amd import binding
    lay = gm.layout(spec)
    nxt = gm.layout(next_spec) if next_spec is not None else None
    max_c = max(1, int(spec.is_mask.sum()))
    out = binding.StepOut(gm, batch, spec.n_rows, max_c, next_rows=next_spec.n_rows if next_spec else 0)
    t = torch.from_numpy(np.ascontiguousarray(tokens_np, dtype=np.int32)).cuda()
    gm.step(t, lay, cache, out, next_layout=nxt)
    torch.cuda.synchronize()
    assert gm.device_faults() == 0
    return out


@pytest.mark.parametrize("shape_name,k,attn", [("tiny", 1, None), ("tiny", 3, None), ("tiny", 4, None),
                                               ("tiny", 5, None), ("small128", 2, None), ("small128", 5, None),
                                               ("small128", 6, None), ("tiny", 3, "split"), ("small128", 5, "split"),
                                               ("tiny", 1, "split"), ("gqa-small", 3, None), ("gqa-small", 5, "split"),
                                               ("gqa128", 5, None), ("gqa128", 6, None)])
def test_step_matches_oracle(torch_mod, shape_name, k, attn):
    """One step after a real prefill: logits, ids, verification outputs, staged and committed K/V.
    Blocks of at most 48 rows run the one-workgroup-per-head attention kernel unless attn says
    otherwise; k = 6 (49 rows) and the 16-row prefill chunks of the "split" cases run the other one.
    The gqa shapes have fewer key/value heads than query heads (grouped-query attention)."""
    torch = torch_mod
    from paper_2402_11809_amd import layout as lo
    from paper_2402_11809_amd.runtime import SpaceDecoder
    shape, gm, om = _setup(shape_name, max_rows=64, attn=attn)
    n_prompt = 45
    prompt = prompt_tokens(shape, seed=1, n=n_prompt)
    dec = SpaceDecoder(gm, k, batch=1, capacity=128, prefill_chunk=16)
    dec.prefill(prompt[:, :-1])
    okv = so.OracleKV(om)
    so.prefill(om, okv, prompt[0, :-1])
    # committed prompt rows agree
    torch.cuda.synchronize()
    assert int(dec.kv.len.cpu()[0]) == n_prompt - 1 == okv.length
    for l in range(shape.n_layers):
        gk, gv = gc.download_kv_rows(dec.kv, l, 0, 0, n_prompt - 1)
        gc.assert_bf16_close(gk, okv.k[l], f"prefill K layer {l}", min_same=0.97 if l == 0 else 0.9)
        gc.assert_bf16_close(gv, okv.v[l], f"prefill V layer {l}", min_same=0.97 if l == 0 else 0.9)
    # candidates: the oracle's own greedy continuation with the last one corrupted
    truth = so.ar_greedy(om, prompt[0], k + 1)[n_prompt:]
    cands = list(truth[:k])
    if k >= 2:
        cands[k - 1] = (cands[k - 1] + 1) % shape.vocab
    spec = lo.paper_layout(k)
    toks, is_mask = so.extended_input([int(prompt[0, -1])], cands, k, shape.mask_id)
    assert np.array_equal(is_mask.astype(np.uint8), spec.is_mask)
    out = _run_step(torch, gm, dec.kv, spec, toks[None], next_spec=spec)
    ref, ks, vs, pos = so.space_step_cached(om, okv, int(prompt[0, -1]), cands, k, commit=False)
    g_logits = out.logits.cpu().numpy()[0].astype(np.float64)
    err = np.abs(g_logits - ref.logits).max()
    print(f"{shape_name} k={k}: max |logit diff| = {err:.3e}")
    assert err < gc.LOGIT_TIGHT < gc.LOGIT_TOL
    g_arg = out.argmax.cpu().numpy()[0]
    ties = gc.check_ids(g_arg, ref.logits, "argmax")
    if ties == 0:
        assert int(out.accepted_len.cpu()[0]) == ref.accepted == (k - 1 if k >= 2 else k)
        assert int(out.bonus.cpu()[0]) == ref.emitted[-1]
        assert list(out.new_cands.cpu().numpy()[0][:k]) == ref.new_cands
        nxt, _ = so.extended_input([ref.emitted[-1]], ref.new_cands, k, shape.mask_id)
        assert list(out.next_tokens.cpu().numpy()[0]) == list(nxt)
    # K/V of the accepted rows sit at their final slots; commit makes them visible
    a = int(out.accepted_len.cpu()[0])
    gm.kv_commit(dec.kv, out.accepted_len)
    torch.cuda.synchronize()
    assert int(dec.kv.len.cpu()[0]) == n_prompt - 1 + a + 1
    rows = [g * (k + 1) for g in range(a + 1)]
    for l in range(shape.n_layers):
        gk, gv = gc.download_kv_rows(dec.kv, l, 0, n_prompt - 1, n_prompt + a)
        gc.assert_bf16_close(gk, ks[l][rows], f"committed K layer {l}", min_same=0.97 if l == 0 else 0.9)
        gc.assert_bf16_close(gv, vs[l][rows], f"committed V layer {l}", min_same=0.97 if l == 0 else 0.9)
    # rollback takes them away again
    gm.kv_rollback(dec.kv, None, n_all=a + 1)
    torch.cuda.synchronize()
    assert int(dec.kv.len.cpu()[0]) == n_prompt - 1


@pytest.mark.parametrize("k", [3, 5])
def test_forced_acceptance_lengths(torch_mod, k):
    """Every acceptance length 0..k (closed form: longest prefix equal to the greedy continuation)."""
    torch = torch_mod
    from paper_2402_11809_amd import layout as lo
    from paper_2402_11809_amd.runtime import SpaceDecoder
    shape, gm, om = _setup("tiny")
    prompt = prompt_tokens(shape, seed=2, n=30)
    truth = so.ar_greedy(om, prompt[0], k + 1)[30:]
    dec = SpaceDecoder(gm, k, capacity=96, prefill_chunk=32)
    dec.prefill(prompt[:, :-1])
    spec = lo.paper_layout(k)
    for j in range(k + 1):
        cands = list(truth[:k])
        if j < k:
            cands[j] = (cands[j] + 7) % shape.vocab
        toks, _ = so.extended_input([int(prompt[0, -1])], cands, k, shape.mask_id)
        out = _run_step(torch, gm, dec.kv, spec, toks[None])
        assert int(out.accepted_len.cpu()[0]) == j
        assert int(out.bonus.cpu()[0]) == truth[j]
        # nothing committed: the next variant sees the same cache
        gm.kv_rollback(dec.kv, None, n_all=0)


@pytest.mark.parametrize("shape_name,k,n_new", [("tiny", 4, 32), ("tiny", 2, 24), ("small128", 5, 24),
                                                ("gqa-small", 4, 24)])
def test_generate_is_lossless(torch_mod, shape_name, k, n_new):
    """Config 1: greedy SPACE on the GPU == plain greedy AR decoding (oracle) == GPU one-token
    decoding, token for token."""
    torch = torch_mod
    from paper_2402_11809_amd.runtime import SpaceDecoder
    shape, gm, om = _setup(shape_name)
    prompt = prompt_tokens(shape, seed=0, n=64)
    dec = SpaceDecoder(gm, k, capacity=256, prefill_chunk=64)
    seqs, hist = dec.generate(prompt, n_new)
    assert all(0 <= int(h[0]) <= k for h in hist) and int(hist[0][0]) == 0
    ref = so.ar_greedy(om, prompt[0], n_new)
    got = [int(t) for t in seqs[0]]
    if got != ref:
        # tolerated only at a near tie of the oracle's logits
        first = next(i for i, (a, b) in enumerate(zip(got, ref)) if a != b)
        logits = so.causal_forward(om, ref[:first])[-1]
        assert gc.top2_gap(logits) < gc.TIE_GAP, f"diverged at {first} with gap {gc.top2_gap(logits)}"
    # GPU autoregressive decoding through the same ABI (k = 0 blocks of one row)
    gm2 = gc.make_gpu_model(shape, all_weights(shape, seed=0), max_rows=64)
    dec0 = SpaceDecoder(gm2, 0, capacity=256, prefill_chunk=64)
    seq0, _ = dec0.generate(prompt, n_new)
    assert [int(t) for t in seq0[0]] == got
    print(f"{shape_name} k={k}: {n_new} tokens in {len(hist)} invocations")


def test_graph_replayed_loop_equals_the_host_driven_loop(torch_mod):
    """Algorithm 1's while loop as the product runs it: one iteration (step + commit) captured into a HIP
    graph and replayed, the host looking at the counters only after as many replays as the missing tokens
    need at least.  It must emit what the kernel-by-kernel loop emits, invocation by invocation, which in
    turn is the oracle's greedy sequence; a decoder can be used again; a batch works the same way."""
    torch = torch_mod
    from paper_2402_11809_amd.runtime import SpaceDecoder
    shape, gm, om = _setup("small128", max_batch=3)
    k, n_new = 3, 30
    prompt = prompt_tokens(shape, seed=5, n=48, batch=3)
    outs = []
    for graph in (True, False):
        dec = SpaceDecoder(gm, k, batch=3, capacity=256, prefill_chunk=32, graph=graph)
        seqs, hist = dec.generate(prompt, n_new)
        outs.append((seqs.copy(), [h.copy() for h in hist], dec.iterations, dec.kv.len.cpu().numpy().copy()))
        if graph:  # again on the same decoder (and its captured graphs are dropped with the old state)
            seqs2, hist2 = dec.generate(prompt, n_new)
            assert np.array_equal(seqs, seqs2) and len(hist) == len(hist2)
            assert all(np.array_equal(a, b) for a, b in zip(hist, hist2))
    (sa, ha, ia, la), (sb, hb, ib, lb) = outs
    assert np.array_equal(sa, sb) and ia == ib == len(ha) == len(hb)
    assert all(np.array_equal(a, b) for a, b in zip(ha, hb)) and np.array_equal(la, lb)
    assert np.array_equal(la, 47 + np.sum([h + 1 for h in ha], axis=0))
    # no invocation ran that was not needed: before the last one some sequence was still short
    short = np.sum([h + 1 for h in ha[:-1]], axis=0)
    assert (short < n_new).any()
    for b in range(3):
        ref = so.ar_greedy(om, prompt[b], n_new)
        got = [int(t) for t in sa[b]]
        if got != ref:
            first = next(i for i, (x, y) in enumerate(zip(got, ref)) if x != y)
            assert gc.top2_gap(so.causal_forward(om, ref[:first])[-1]) < gc.TIE_GAP
    assert gm.device_faults() == 0


def test_eos_stops_the_sequence(torch_mod):
    """EOS check of Algorithm 1 on the device: the output ends in front of the first EOS token, also
    when it falls in the middle of a step's accepted run; the flag is sticky."""
    torch = torch_mod
    from paper_2402_11809_amd.runtime import SpaceDecoder
    shape, gm, om = _setup("tiny")
    prompt = prompt_tokens(shape, seed=0, n=40)
    ref = so.ar_greedy(om, prompt[0], 20)
    gen = ref[40:]
    for pos in (0, 2, 9):
        eos = gen[pos]
        first = gen.index(eos)
        for k in (2, 4):
            dec = SpaceDecoder(gm, k, capacity=128, prefill_chunk=32, eos_id=eos)
            seqs, hist = dec.generate(prompt, 20)
            oracle_out, _ = so.space_generate(om, [int(t) for t in prompt[0]], k, 20, eos_id=eos)
            n = int(dec.lengths[0])
            assert n == first == len(oracle_out) - 40
            assert [int(t) for t in seqs[0][: 40 + n]] == oracle_out
            assert int(dec.out.finished.cpu()[0]) == 1
            # one more step appends nothing
            gm.step(dec.out.next_tokens, dec.lay_step, dec.kv, dec.out, next_layout=dec.lay_step)
            torch.cuda.synchronize()
            assert int(dec.out.emit_len.cpu()[0]) == n


def test_first_step_layout_and_prefill_chunking(torch_mod):
    """[x_l, M^k] alone gives the same extra token / candidates as the full block with dummies, and
    the cache does not depend on how the prompt was chunked."""
    torch = torch_mod
    from paper_2402_11809_amd import layout as lo
    from paper_2402_11809_amd.runtime import SpaceDecoder
    shape, gm, om = _setup("tiny")
    k = 4
    prompt = prompt_tokens(shape, seed=3, n=41)
    d1 = SpaceDecoder(gm, k, capacity=96, prefill_chunk=7)
    d2 = SpaceDecoder(gm, k, capacity=96, prefill_chunk=40)
    d1.prefill(prompt[:, :-1])
    d2.prefill(prompt[:, :-1])
    torch.cuda.synchronize()
    k1 = d1.kv.k_view()[:, 0, :, :40].float().cpu().numpy()
    k2 = d2.kv.k_view()[:, 0, :, :40].float().cpu().numpy()
    assert np.mean(k1 == k2) > 0.995 and np.abs(k1 - k2).max() < 0.05
    first = np.array([[int(prompt[0, -1])] + [shape.mask_id] * k])
    o1 = _run_step(torch, gm, d1.kv, lo.first_step_layout(k), first)
    full, _ = so.extended_input([int(prompt[0, -1])], [0] * k, k, shape.mask_id)
    o2 = _run_step(torch, gm, d1.kv, lo.paper_layout(k), full[None])
    assert int(o1.accepted_len.cpu()[0]) == 0
    assert int(o1.bonus.cpu()[0]) == int(o2.argmax.cpu()[0, 0])
    assert list(o1.new_cands.cpu().numpy()[0]) == list(o2.argmax.cpu().numpy()[0, 1:k + 1])
    assert np.abs(o1.logits.cpu().numpy()[0] - o2.logits.cpu().numpy()[0, :k + 1]).max() < 1e-4


@pytest.mark.parametrize("shape_name,n_prompt,chunk", [("small128", 411, 410), ("small128", 411, 200), ("gqa-small", 300, 299),
                                                        ("tiny", 1001, 1000)])
def test_long_prompt_chunks_match_oracle(torch_mod, shape_name, n_prompt, chunk):
    """Prompt chunks of hundreds of rows through space_prefill (no LM head, last layer stops after its
    keys and values; projections in 96- and 128-row passes, attention over a long causal block): the
    cache they leave equals the oracle's, and so does the auto-correct step that follows."""
    torch = torch_mod
    from paper_2402_11809_amd import binding, layout as lo
    from paper_2402_11809_amd.runtime import SpaceDecoder
    shape, gm, om = _setup(shape_name, max_rows=chunk)
    k = 3
    prompt = prompt_tokens(shape, seed=5, n=n_prompt)
    dec = SpaceDecoder(gm, k, capacity=(n_prompt + 64 + 31) // 32 * 32, prefill_chunk=chunk)
    dec.prefill(prompt[:, :-1])
    torch.cuda.synchronize()
    assert gm.device_faults() == 0 and int(dec.kv.len.cpu()[0]) == n_prompt - 1
    okv = so.OracleKV(om)
    so.prefill(om, okv, prompt[0, :-1])
    n = n_prompt - 1
    for l in range(shape.n_layers):      # keys and values of every layer, bf16 on both sides
        kd = dec.kv.k_view()[l, 0, :, :n].float().cpu().numpy()                  # [Hkv, n, dh]
        ko = np.transpose(okv.k[l][:n], (1, 0, 2))
        vd = dec.kv.v_rows()[l, 0, :, :n].float().cpu().numpy()
        vo = np.transpose(okv.v[l][:n], (1, 0, 2))
        for got, want in ((kd, ko), (vd, vo)):
            # both are bf16 roundings of values that differ by the fp32 path's error (bounded like the
            # logits' tight bar): one bf16 step where they fall on different sides, plus that error
            ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 2.0 ** -10))) - 7)
            assert np.all(np.abs(got - want) <= 1.001 * ulp + gc.LOGIT_TIGHT) and np.mean(got != want) < 0.15
    truth = so.ar_greedy(om, prompt[0], k)[n_prompt:]
    cands = truth[:2] + [(truth[2] + 1) % shape.vocab]
    toks, _ = so.extended_input([int(prompt[0, -1])], cands, k, shape.mask_id)
    out = _run_step(torch, gm, dec.kv, lo.paper_layout(k), toks[None])
    ref, _, _, _ = so.space_step_cached(om, okv, int(prompt[0, -1]), cands, k)
    assert np.abs(out.logits.cpu().numpy()[0] - ref.logits).max() < gc.LOGIT_TOL
    assert int(out.accepted_len.cpu()[0]) == ref.accepted == 2
    assert int(out.bonus.cpu()[0]) == ref.emitted[-1]
    # a block that long cannot be verified: space_step says so
    if chunk > 96:
        with pytest.raises(binding.SpaceError) as e:
            _run_step(torch, gm, dec.kv, lo.prefill_layout(chunk), prompt[:, :chunk])
        assert e.value.code == binding.SPACE_ESHAPE


def _batched_step_vs_oracle(torch, shape, w, B, k, tune, tol, threads=1, ctxs=None, capacity=160):
    from paper_2402_11809_amd import binding, layout as lo
    spec = lo.paper_layout(k)
    L = spec.n_rows
    gm = gc.make_gpu_model(shape, w, max_batch=B, max_rows=L, tune=tune)
    om = gc.oracle_model(shape, w)
    if ctxs is None:
        ctxs = [(17 * (b + 1)) % 90 + 3 for b in range(B)]
    cache = binding.KVCache(gm, B, capacity)
    okvs = []
    for b, c in enumerate(ctxs):
        okv = gc.synthetic_oracle_kv(om, seed=20 + b, ctx=c, std=0.5)
        gc.upload_oracle_kv(torch, cache, b, okv)
        okvs.append(okv)
    rng = np.random.default_rng(9)
    toks = np.zeros((B, L), dtype=np.int32)
    cands = []
    for b in range(B):
        c = [int(t) for t in rng.integers(0, shape.vocab, size=k)]
        cands.append(c)
        toks[b], _ = so.extended_input([int(rng.integers(0, shape.vocab))], c, k, shape.mask_id)
    out = _run_step(torch, gm, cache, spec, toks, batch=B)
    worst = 0.0
    for b in range(B):
        ref, _, _, _ = so.space_step_cached(om, okvs[b], int(toks[b, 0]), cands[b], k, commit=False)
        err = np.abs(out.logits.cpu().numpy()[b] - ref.logits).max()
        worst = max(worst, err)
        assert err < tol, (b, err)
        gc.check_ids(out.argmax.cpu().numpy()[b], ref.logits, f"seq {b}")
        assert int(out.accepted_len.cpu()[b]) == ref.accepted
    return worst


@pytest.mark.parametrize("shape_name,B,k,ks", [("small128", 1, 5, 0), ("small128", 4, 5, 0), ("gqa-small", 5, 4, 0), ("gqa128", 2, 8, 0),
                                                ("tiny", 7, 3, 0), ("small128", 4, 5, 1), ("small128", 6, 5, 2), ("gqa128", 2, 8, 4),
                                                ("tiny", 7, 3, 2)])
def test_many_row_projection_kernel_on_small_blocks(torch_mod, shape_name, B, k, ks):
    """The projection kernel for many rows (activation planes shared through LDS, 128-row passes), forced
    for every row count: a single ragged tile, exactly one pass, a pass plus a few rows, odd numbers of
    contraction tiles, all three epilogues; with the number of partial sums over the contraction its cost
    model picks (ks = 0) and with 1, 2 and 4 forced (what space_tune_rows may choose between).  Every
    sequence against its own oracle step."""
    shape = SHAPES[shape_name]
    tune = "wide=1" + (f",wideks={ks}" if ks else "")
    _batched_step_vs_oracle(torch_mod, shape, all_weights(shape, seed=2), B, k, tune, gc.LOGIT_TIGHT)


@pytest.mark.parametrize("shape_name,B,k", [("small128", 3, 5), ("small128", 6, 5), ("gqa128", 2, 8), ("small128", 8, 5)])
def test_library_switches_between_the_projection_kernels_by_itself(torch_mod, shape_name, B, k):
    """Row counts on both sides of the library's own switch points, nothing forced: 108 and 162 rows (only
    the QKV projection takes the many-row kernel, the others run as two skinny passes), 216 rows (two
    passes of the many-row kernel, the second short) and 288 rows (three, the last of two row tiles)."""
    shape = SHAPES[shape_name]
    _batched_step_vs_oracle(torch_mod, shape, all_weights(shape, seed=3), B, k, None, gc.LOGIT_TIGHT)


@pytest.mark.parametrize("shape_name,B,k,ctxs,tune", [
    ("gqa-small", 17, 5, "ragged", None), ("gqa-small", 17, 5, "uniform", "attn=0"),
    ("gqa-small", 17, 5, "one-long", "attn=1000000"), ("gqa128", 9, 8, "ragged", None), ("small128", 12, 5, "ragged", None),
    ("small128", 3, 5, "one-long", "attn=0"), ("gqa-small", 33, 3, "ragged", "attn=0")])
def test_batches_with_long_ragged_contexts(torch_mod, shape_name, B, k, ctxs, tune):
    """Batches whose contexts run to several hundred positions, with the attention kernel the library picks
    by itself (for these workgroup counts the one with a workgroup per (sequence, head) that sums, rotates
    and stores the block in its prologue: two partial sums of the projection, three items per thread) and
    with either one forced: ragged lengths, equal lengths, one long sequence among short ones, and a block of
    two query groups (rotary and store in a pass of their own); up to 33 sequences x 8 heads (more
    workgroups than CUs).  Every sequence against its own oracle step."""
    shape = SHAPES[shape_name]
    lens = {"ragged": [40 + (211 * b) % 700 for b in range(B)], "uniform": [544] * B,
            "one-long": [33 + b for b in range(B - 1)] + [760]}[ctxs]
    _batched_step_vs_oracle(torch_mod, shape, all_weights(shape, seed=5), B, k, tune, gc.LOGIT_TIGHT, ctxs=lens, capacity=800)


@pytest.mark.parametrize("B,k", [(6, 5), (2, 8), (8, 5)])
def test_measured_cut_and_split_stay_within_rounding(torch_mod, B, k):
    """space_tune_rows picks how the many-row kernel cuts the rows into workgroups (pieces of 128, 96, 64
    or 32 rows) and in how many parts the plain-sum projections add up the contraction.  The cut changes
    no bit (next test); the number of partial sums reorders fp32 additions, so whatever it picks, the
    logits stay within 1e-3 of the untuned step's (a reordered sum can move a key or value across a bf16
    rounding boundary, which shows downstream), and indices and accepted counts are the same wherever
    the untuned step's top two logits are more than 1e-3 apart.  216 rows (all projections), 162 rows (QKV
    only) and 288 rows; also the call's error paths."""
    torch = torch_mod
    from paper_2402_11809_amd import binding, layout as lo
    shape = SHAPES["small128"]
    w = all_weights(shape, seed=4)
    spec = lo.paper_layout(k)
    L = spec.n_rows
    rng = np.random.default_rng(12)
    toks = rng.integers(0, shape.vocab, size=(B, L)).astype(np.int32)
    results = []
    for tuned in (False, True):
        gm = gc.make_gpu_model(shape, w, max_batch=B, max_rows=L)
        if tuned:
            gm.tune_rows(B * L)
            gm.tune_rows(B * L)  # a second request for the same count is a no-op
            with pytest.raises(binding.SpaceError) as e:
                gm._check(gm.lib.space_tune_rows(gm.ctx, B * L + 1, None))
            assert e.value.code == binding.SPACE_ESHAPE
            with pytest.raises(binding.SpaceError) as e:
                gm._check(gm.lib.space_tune_rows(gm.ctx, 0, None))
            assert e.value.code == binding.SPACE_ESHAPE
        cache = binding.KVCache(gm, B, 160)
        om = gc.oracle_model(shape, w)
        for b in range(B):
            gc.upload_oracle_kv(torch, cache, b, gc.synthetic_oracle_kv(om, seed=40 + b, ctx=11 * b + 5, std=0.5))
        out = _run_step(torch, gm, cache, spec, toks, batch=B)
        results.append((out.logits.cpu().numpy().copy(), out.argmax.cpu().numpy().copy(), out.accepted_len.cpu().numpy().copy()))
    (l0, a0, n0), (l1, a1, n1) = results
    assert np.abs(l0 - l1).max() < 1e-3
    top2 = np.sort(l0, axis=-1)[..., -2:]
    clear = (top2[..., 1] - top2[..., 0]) > 1e-3
    assert np.array_equal(a0[clear], a1[clear])
    if clear.all():
        assert np.array_equal(n0, n1)


def test_every_row_cut_gives_the_same_bits(torch_mod):
    """288 rows = 9 groups of 32 rows, cut in every piece size and both launch orders (forced through
    SPACE_TUNE widecut=): logits, indices and accepted counts equal the default cut's bit for bit."""
    torch = torch_mod
    from paper_2402_11809_amd import binding, layout as lo
    shape = SHAPES["small128"]
    w = all_weights(shape, seed=5)
    B, k = 8, 5
    spec = lo.paper_layout(k)
    L = spec.n_rows
    toks = np.random.default_rng(13).integers(0, shape.vocab, size=(B, L)).astype(np.int32)
    om = gc.oracle_model(shape, w)
    okvs = [gc.synthetic_oracle_kv(om, seed=60 + b, ctx=9 * b + 4, std=0.5) for b in range(B)]
    ref = None
    for cut in (None, "2:0:0:1:0", "0:3:0:0:0", "0:3:0:0:1", "0:1:3:0:1", "0:0:4:1:0", "1:0:2:1:1", "0:0:0:9:1", "1:1:1:0:0"):
        gm = gc.make_gpu_model(shape, w, max_batch=B, max_rows=L, tune=None if cut is None else "widecut=" + cut)
        cache = binding.KVCache(gm, B, 160)
        for b in range(B):
            gc.upload_oracle_kv(torch, cache, b, okvs[b])
        out = _run_step(torch, gm, cache, spec, toks, batch=B)
        got = (out.logits.cpu().numpy().copy(), out.argmax.cpu().numpy().copy(), out.accepted_len.cpu().numpy().copy())
        if ref is None:
            ref = got
        else:
            for x, y in zip(ref, got):
                assert np.array_equal(x, y), cut


@pytest.mark.parametrize("shape_name,B,k,ctxs", [("small128", 1, 5, [300]), ("small128", 3, 5, [5, 700, 33]), ("gqa-small", 2, 8, [500, 64]),
                                                 ("tiny", 1, 3, [790]), ("gqa128", 4, 2, [31, 32, 33, 650])])
def test_key_split_with_more_workgroups_than_chunks(torch_mod, shape_name, B, k, ctxs):
    """The key-split attention with several workgroups along the keys, sized for the longest sequence of
    the batch: sequences with fewer chunks than workgroups (those workgroups only leave the empty marker
    for the merge kernel), a nearly empty cache next to a long one, blocks of 36 rows (rotary fused), 81
    rows (two query groups), 16 and 9 rows.  Against the oracle's step, and three steps in a row on the
    same context give the same bits."""
    torch = torch_mod
    from paper_2402_11809_amd import binding, layout as lo
    shape = SHAPES[shape_name]
    w = all_weights(shape, seed=6)
    spec = lo.paper_layout(k)
    L = spec.n_rows
    om = gc.oracle_model(shape, w)
    okvs = [gc.synthetic_oracle_kv(om, seed=70 + b, ctx=c, std=0.5) for b, c in enumerate(ctxs)]
    rng = np.random.default_rng(14)
    toks = np.zeros((B, L), dtype=np.int32)
    cands = []
    for b in range(B):
        c = [int(t) for t in rng.integers(0, shape.vocab, size=k)]
        cands.append(c)
        toks[b], _ = so.extended_input([int(rng.integers(0, shape.vocab))], c, k, shape.mask_id)
    gm = gc.make_gpu_model(shape, w, max_batch=B, max_rows=L, tune="attn=0")
    cache = binding.KVCache(gm, B, 800)
    for b in range(B):
        gc.upload_oracle_kv(torch, cache, b, okvs[b])
    ref = None
    for rep in range(3):
        out = _run_step(torch, gm, cache, spec, toks, batch=B)
        got = (out.logits.cpu().numpy().copy(), out.argmax.cpu().numpy().copy(), out.accepted_len.cpu().numpy().copy())
        if ref is None:
            ref = got
            for b in range(B):
                o, _, _, _ = so.space_step_cached(om, okvs[b], int(toks[b, 0]), cands[b], k, commit=False)
                assert np.abs(got[0][b] - o.logits).max() < gc.LOGIT_TIGHT, b
                gc.check_ids(got[1][b], o.logits, f"seq {b}")
        else:
            for x, y in zip(ref, got):
                assert np.array_equal(x, y), rep


@pytest.mark.parametrize("shape_name", ["7b", "13b", "70b"])
def test_many_row_projection_kernel_at_full_width(torch_mod, shape_name):
    """One layer + LM head at the width of the 7B, 13B and 70B members of the family, 5 sequences x 81
    rows = 405 rows: the library picks the many-row kernel by itself (4 passes, the last of 21 rows;
    contraction splits; 2000 LM-head tiles).  Against the stated bar, not the tight one: in a one-layer
    random model of this width the attention output is ~30x the embedding, and with contexts of 3..88
    positions every key or value that rounds to the other bf16 neighbour (both sides round, from fp32
    and from fp64) shows in it.  Measured over the 13 M logits: 4.7e-3 at the 7B width, 1.1e-2 at the
    70B width (median row 2e-3, mean 5e-4), the same to three digits with either projection kernel."""
    shape = SHAPES[shape_name].with_layers(1)
    worst = _batched_step_vs_oracle(torch_mod, shape, all_weights(shape, seed=0, threads=8), 5, 8, None, gc.LOGIT_TOL)
    print(f"{shape_name} layer, 405 rows: max |logit diff| = {worst:.3e}")


def test_ragged_batch_matches_oracle(torch_mod):
    """Batch of sequences with different context lengths and candidates (config 5 in small):
    every sequence must match its own oracle step; explicit commit counts land in len."""
    torch = torch_mod
    from paper_2402_11809_amd import binding, layout as lo
    shape, gm, om = _setup("small128", max_batch=3, max_rows=36)
    k, B = 5, 3
    ctxs = [37, 100, 64]
    cache = binding.KVCache(gm, B, 160)
    okvs = []
    for b, c in enumerate(ctxs):
        okv = gc.synthetic_oracle_kv(om, seed=10 + b, ctx=c, std=0.5)
        gc.upload_oracle_kv(torch, cache, b, okv)
        okvs.append(okv)
    rng = np.random.default_rng(5)
    toks = np.zeros((B, 36), dtype=np.int32)
    cands = []
    for b in range(B):
        c = [int(t) for t in rng.integers(0, shape.vocab, size=k)]
        cands.append(c)
        toks[b], _ = so.extended_input([int(rng.integers(0, shape.vocab))], c, k, shape.mask_id)
    spec = lo.paper_layout(k)
    out = _run_step(torch, gm, cache, spec, toks, batch=B)
    for b in range(B):
        ref, ks, vs, pos = so.space_step_cached(om, okvs[b], int(toks[b, 0]), cands[b], k, commit=False)
        err = np.abs(out.logits.cpu().numpy()[b] - ref.logits).max()
        assert err < gc.LOGIT_TOL, (b, err)
        gc.check_ids(out.argmax.cpu().numpy()[b], ref.logits, f"seq {b}")
    forced = torch.tensor([0, 5, 2], dtype=torch.int32, device="cuda")
    gm.kv_commit(cache, forced)
    torch.cuda.synchronize()
    assert list(cache.len.cpu().numpy()) == [ctxs[0] + 1, ctxs[1] + 6, ctxs[2] + 3]
    ref, ks, vs, pos = so.space_step_cached(om, okvs[1], int(toks[1, 0]), cands[1], k, commit=False)
    gk, gv = gc.download_kv_rows(cache, 2, 1, ctxs[1], ctxs[1] + 6)
    gc.assert_bf16_close(gk, ks[2][[g * 6 for g in range(6)]], "forced commit K", min_same=0.9)
    gc.assert_bf16_close(gv, vs[2][[g * 6 for g in range(6)]], "forced commit V", min_same=0.9)


@pytest.mark.parametrize("attn", [None, "split"])
def test_empty_cache_and_mixed_lengths(torch_mod, attn):
    """Degenerate contexts: decoding from a one-token prompt (the first blocks run against an empty
    or nearly empty cache), and a batch in which one sequence has nothing cached while another has
    several chunks."""
    torch = torch_mod
    from paper_2402_11809_amd import binding, layout as lo
    from paper_2402_11809_amd.runtime import SpaceDecoder
    shape, gm, om = _setup("tiny", max_batch=2, attn=attn)
    k = 3
    prompt = prompt_tokens(shape, seed=9, n=1)
    dec = SpaceDecoder(gm, k, batch=1, capacity=64, prefill_chunk=16)
    seq, hist = dec.generate(prompt, 10)
    ref = so.ar_greedy(om, prompt[0], 10)
    got = [int(t) for t in seq[0]]
    if got != ref:
        first = next(i for i, (a, b) in enumerate(zip(got, ref)) if a != b)
        assert gc.top2_gap(so.causal_forward(om, ref[:first])[-1]) < gc.TIE_GAP
    # batch of two: sequence 0 empty, sequence 1 with 70 cached positions
    cache = binding.KVCache(gm, 2, 128)
    okv0 = so.OracleKV(om)
    okv1 = gc.synthetic_oracle_kv(om, seed=8, ctx=70, std=0.5)
    gc.upload_oracle_kv(torch, cache, 1, okv1)
    spec = lo.paper_layout(k)
    rng = np.random.default_rng(3)
    toks = np.zeros((2, spec.n_rows), dtype=np.int32)
    for b in range(2):
        toks[b], _ = so.extended_input([int(rng.integers(0, shape.vocab))], [int(t) for t in rng.integers(0, shape.vocab, size=k)],
                                       k, shape.mask_id)
    out = _run_step(torch, gm, cache, spec, toks, batch=2)
    for b, okv in enumerate((okv0, okv1)):
        ref_logits, _, _, _ = so.block_forward_cached(om, okv, toks[b], spec.is_mask.astype(bool), k)
        err = np.abs(out.logits.cpu().numpy()[b] - ref_logits).max()
        assert err < gc.LOGIT_TIGHT, (b, err)
        gc.check_ids(out.argmax.cpu().numpy()[b], ref_logits, f"sequence {b}")


def test_layers_handed_over_one_by_one(torch_mod):
    """space_load_layer: a model whose layers arrive after space_init gives bit-identical outputs; a step
    before the last layer arrived is refused."""
    torch = torch_mod
    from paper_2402_11809_amd import binding, layout as lo
    shape = SHAPES["tiny"]
    w = all_weights(shape, seed=0)
    gm = gc.make_gpu_model(shape, w, max_rows=16)
    dev_w = binding.weights_to_device(w)
    layers = dev_w["layers"]
    gm2 = binding.Model(shape, dict(dev_w, layers=[None] * shape.n_layers), max_batch=1, max_rows=16)
    spec = lo.paper_layout(3)
    toks = np.random.default_rng(0).integers(0, shape.vocab, size=(1, spec.n_rows)).astype(np.int32)
    toks[0, spec.is_mask == 1] = shape.mask_id
    c1, c2 = binding.KVCache(gm, 1, 64), binding.KVCache(gm2, 1, 64)
    gm2.load_layer(1, layers[1])
    with pytest.raises(binding.SpaceError) as e:
        _run_step(torch, gm2, c2, spec, toks)
    assert e.value.code == binding.SPACE_EINVAL
    gm2.load_layer(0, layers[0])
    with pytest.raises(binding.SpaceError):
        gm2.load_layer(0, layers[0])
    a = _run_step(torch, gm, c1, spec, toks)
    b = _run_step(torch, gm2, c2, spec, toks)
    assert torch.equal(a.logits, b.logits) and torch.equal(a.argmax, b.argmax)


def test_error_paths(torch_mod):
    torch = torch_mod
    from paper_2402_11809_amd import binding, layout as lo
    shape, gm, om = _setup("tiny", max_rows=25)
    with pytest.raises(binding.SpaceError) as e:
        gm.layout(lo.paper_layout(5))  # 36 rows > max_rows
    assert e.value.code == binding.SPACE_ECAPACITY
    bad = lo.BlockLayoutSpec(np.array([1, 0], dtype=np.uint8), np.array([0, 0], dtype=np.int32))
    with pytest.raises(binding.SpaceError) as e:
        gm.layout(bad)
    assert e.value.code == binding.SPACE_EINVAL
    cache = binding.KVCache(gm, 1, 32)
    cache.set_len_bound(30)
    spec = lo.paper_layout(4)
    out = binding.StepOut(gm, 1, 25, 4)
    t = torch.zeros(1, 25, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.SpaceError) as e:
        gm.step(t, gm.layout(spec), cache, out)
    assert e.value.code == binding.SPACE_ECAPACITY
    with pytest.raises(binding.SpaceError) as e:
        gm.kv_commit(cache, None, accepted_all=0)  # nothing staged
    assert e.value.code == binding.SPACE_EINVAL
    # the verification assembles next blocks of at most 96 rows: a longer next_layout is refused on the host
    gm_long = gc.make_gpu_model(shape, all_weights(shape, seed=0), max_batch=1, max_rows=128)
    c_long = binding.KVCache(gm_long, 1, 256)
    out_long = binding.StepOut(gm_long, 1, 25, 4, next_rows=112)
    with pytest.raises(binding.SpaceError) as e:
        gm_long.step(t, gm_long.layout(spec), c_long, out_long, next_layout=gm_long.layout(lo.prefill_layout(112)))
    assert e.value.code == binding.SPACE_ESHAPE
    # an out-of-range token id is clamped and counted, not a fault of the GPU
    cache.set_len_bound(0)
    t[0, 0] = shape.vocab + 5
    gm.step(t, gm.layout(spec), cache, out)
    assert gm.device_faults() == 1
    assert gm.device_faults() == 0
    # space_prefill: same capacity checks as the step; more sequences than the scratch was sized for
    cache.set_len_bound(30)
    with pytest.raises(binding.SpaceError) as e:
        gm.prefill(t, gm.layout(spec), cache)
    assert e.value.code == binding.SPACE_ECAPACITY
    gm1 = gc.make_gpu_model(shape, all_weights(shape, seed=0), max_batch=2, max_rows=16)
    two = binding.KVCache(gm1, 2, 64)
    lay25 = lo.prefill_layout(16)
    gm1.prefill(torch.zeros(2, 16, dtype=torch.int32, device="cuda"), gm1.layout(lay25), two)   # 32 rows: fits
    gm1.kv_commit(two, None, accepted_all=15)
    assert two.len.cpu().tolist() == [16, 16]
    # a paged view with more pages per sequence than the context allows
    pool = binding.PagePool(gm1, 8)
    with pytest.raises(binding.SpaceError) as e:
        big = binding.PagedKV(pool, torch.zeros(1, 200, dtype=torch.int32, device="cuda"), torch.zeros(1, dtype=torch.int32, device="cuda"))
        gm1.prefill(torch.zeros(1, 16, dtype=torch.int32, device="cuda"), gm1.layout(lay25), big)
    assert e.value.code == binding.SPACE_ECAPACITY


@pytest.mark.parametrize("groups,masks,attn,shape_name", [
    (2, 1, None, "7b"), (2, 3, None, "7b"), (4, 3, None, "7b"), (4, 7, None, "7b"), (6, 5, None, "7b"),
    (2, 1, "head", "7b"), (6, 5, "head", "7b"), (6, 5, None, "70b"), (6, 5, "head", "70b"), (6, 5, None, "13b")])
def test_single_7b_layer_long_cache(torch_mod, groups, masks, attn, shape_name):
    """Config 3: one LLaMA-7B-shaped layer, block of L = groups * (1 + masks) rows under the
    semi-autoregressive mask against a cache of 4096 positions of N(0, 1) K/V.  Also at the 13B
    width and at the 70B width (grouped-query attention, 64 query heads over 8 key/value heads)."""
    torch = torch_mod
    from paper_2402_11809_amd import binding, layout as lo
    shape = SHAPES[shape_name].with_layers(1)
    w = all_weights(shape, seed=0, threads=8)
    gm = gc.make_gpu_model(shape, w, max_batch=1, max_rows=36, max_ctx=4224, attn=attn)
    om = gc.oracle_model(shape, w)
    ctx = 4096
    okv = gc.synthetic_oracle_kv(om, seed=3, ctx=ctx, std=1.0)
    cache = binding.KVCache(gm, 1, 4224)
    gc.upload_oracle_kv(torch, cache, 0, okv)
    spec = lo.grouped_layout(groups, masks)
    rng = np.random.default_rng(groups * 10 + masks)
    toks = rng.integers(0, shape.vocab, size=spec.n_rows).astype(np.int32)
    toks[spec.is_mask == 1] = shape.mask_id
    out = _run_step(torch, gm, cache, spec, toks[None])
    ref_logits, ks, vs, pos = so.block_forward_cached(om, okv, toks, spec.is_mask.astype(bool))
    assert list(pos) == [ctx + int(p) for p in gc.rel_pos(spec)]
    err = np.abs(out.logits.cpu().numpy()[0] - ref_logits).max()
    print(f"{shape_name} layer, L={spec.n_rows} ({groups}x(1+{masks})), ctx 4096: max |logit diff| = {err:.3e}")
    assert err < gc.LOGIT_TIGHT
    gc.check_ids(out.argmax.cpu().numpy()[0], ref_logits, "argmax")
    # greedy verification on these rows, closed form
    am = np.argmax(ref_logits, axis=-1)
    real = gc.real_rows(spec)
    acc = 0
    while acc < groups - 1 and toks[real[acc + 1]] == am[real[acc]]:
        acc += 1
    assert int(out.accepted_len.cpu()[0]) == acc
    assert int(out.bonus.cpu()[0]) == am[real[acc]]


@pytest.mark.parametrize("k,attn", [(3, None), (8, None), (3, "split"), (5, "head")])
def test_ragged_batch_of_eight_with_forced_commits(torch_mod, k, attn):
    """Config 5 in small: 8 sequences, ragged context lengths, blocks of (k+1)^2 rows (up to 648 rows in
    total, i.e. several projection passes), accepted lengths drawn from a geometric law and passed to
    the commit explicitly; afterwards len and the committed rows are checked."""
    torch = torch_mod
    from paper_2402_11809_amd import binding, layout as lo
    from space_inputs import geometric_accept_lengths, ragged_context_lengths
    L = (k + 1) ** 2
    shape, gm, om = _setup("small128", max_batch=8, max_rows=L, attn=attn)
    B = 8
    ctxs = [int(c) for c in ragged_context_lengths(seed=4, batch=B, lo=16, hi=300)]
    cache = binding.KVCache(gm, B, 352)
    okvs = []
    for b, c in enumerate(ctxs):
        okv = gc.synthetic_oracle_kv(om, seed=20 + b, ctx=c, std=0.5)
        gc.upload_oracle_kv(torch, cache, b, okv)
        okvs.append(okv)
    rng = np.random.default_rng(k)
    toks = np.zeros((B, L), dtype=np.int32)
    cands = []
    for b in range(B):
        c = [int(t) for t in rng.integers(0, shape.vocab, size=k)]
        cands.append(c)
        toks[b], _ = so.extended_input([int(rng.integers(0, shape.vocab))], c, k, shape.mask_id)
    out = _run_step(torch, gm, cache, lo.paper_layout(k), toks, batch=B)
    refs = []
    for b in range(B):
        ref, ks, vs, pos = so.space_step_cached(om, okvs[b], int(toks[b, 0]), cands[b], k, commit=False)
        refs.append((ref, ks, vs))
        err = np.abs(out.logits.cpu().numpy()[b] - ref.logits).max()
        assert err < gc.LOGIT_TIGHT, (b, err)
        ties = gc.check_ids(out.argmax.cpu().numpy()[b], ref.logits, f"seq {b}")
        if ties == 0:
            assert int(out.accepted_len.cpu()[b]) == ref.accepted
    forced_np = geometric_accept_lengths(seed=4, batch=B, k=k)
    assert forced_np.min() >= 0 and forced_np.max() <= k
    forced = torch.from_numpy(forced_np).cuda()
    gm.kv_commit(cache, forced)
    torch.cuda.synchronize()
    assert list(cache.len.cpu().numpy()) == [c + int(a) + 1 for c, a in zip(ctxs, forced_np)]
    for b in (0, B - 1):
        a = int(forced_np[b])
        rows = [g * (k + 1) for g in range(a + 1)]
        gk, gv = gc.download_kv_rows(cache, 1, b, ctxs[b], ctxs[b] + a + 1)
        gc.assert_bf16_close(gk, refs[b][1][1][rows], f"seq {b} K", min_same=0.9)
        gc.assert_bf16_close(gv, refs[b][2][1][rows], f"seq {b} V", min_same=0.9)
    # a per-sequence rollback undoes the commit
    gm.kv_rollback(cache, forced + 1)
    torch.cuda.synchronize()
    assert list(cache.len.cpu().numpy()) == ctxs
