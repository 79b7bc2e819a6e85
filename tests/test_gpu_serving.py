"""GPU tests of the paged cache form and of continuous batching on top of it, through the C ABI.
A page is read exactly as a 32-position run of the contiguous form, so the two forms must agree bit
for bit; the batcher's outputs are checked against plain greedy decoding of the oracle (auto-correct
decoding is lossless, whatever the company a sequence keeps in its batch)."""
import numpy as np
import pytest

from oracle import space_oracle as so
from space_inputs import SHAPES, all_weights, prompt_tokens
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_mod():
    return gc.require_gpu()


@pytest.mark.parametrize("shape_name,attn,chunk", [("small128", None, 32), ("gqa-small", "split", 69), ("tiny", "head", 32)])
def test_paged_cache_equals_contiguous_cache(torch_mod, shape_name, attn, chunk):
    torch = torch_mod
    from paper_2402_11809_amd import binding, layout as lo
    shape = SHAPES[shape_name]
    w = all_weights(shape, seed=1)
    k, B = 3, 3
    spec = lo.paper_layout(k)
    L = spec.n_rows
    gm = gc.make_gpu_model(shape, w, max_batch=B, max_rows=max(48, chunk), max_ctx=256, attn=attn)
    om = gc.oracle_model(shape, w)
    n_prompt = [45, 70, 9]
    prompts = [prompt_tokens(shape, seed=30 + b, n=n_prompt[b])[0] for b in range(B)]
    rng = np.random.default_rng(3)
    # every sequence is prefilled twice, on a contiguous cache of its own and through a one-row view of the pool
    stride = 6                                            # 192 positions per sequence
    n_pages = 40
    pool = binding.PagePool(gm, n_pages)
    perm = rng.permutation(n_pages)[: B * stride].reshape(B, stride).astype(np.int32)
    table = torch.from_numpy(perm).cuda()
    lens = torch.zeros(B, dtype=torch.int32, device="cuda")
    caches = [binding.KVCache(gm, 1, 32 * stride) for _ in range(B)]
    for b in range(B):
        toks = torch.from_numpy(prompts[b][None, :-1].astype(np.int32)).cuda()
        n = toks.shape[1]
        view = binding.PagedKV(pool, table[b:b + 1], lens[b:b + 1])
        for kv in (caches[b], view):
            for c0 in range(0, n, chunk):                   # chunks of 64 rows and more take the row-chunk K/V store
                c = min(chunk, n - c0)
                gm.prefill(toks[:, c0:c0 + c].contiguous(), gm.layout(lo.prefill_layout(c)), kv)
                gm.kv_commit(kv, None, accepted_all=c - 1)
    torch.cuda.synchronize()
    assert lens.cpu().tolist() == [n - 1 for n in n_prompt]
    # the pages hold what the contiguous rows hold
    for b in range(B):
        n = n_prompt[b] - 1
        kc = caches[b].k_view()[:, 0, :, :n]                                    # [layers, Hkv, n, dh]
        kp = pool.k_view()[:, table[b].long()].permute(0, 2, 1, 3, 4).reshape(shape.n_layers, pool.kv_heads, -1, shape.head_dim)[:, :, :n]
        assert torch.equal(kc, kp)
        vc = caches[b].v_rows()[:, 0, :, :n]
        vp = pool.v_view()[:, table[b].long()].permute(0, 2, 1, 4, 3).reshape(shape.n_layers, pool.kv_heads, -1, shape.head_dim)[:, :, :n]
        assert torch.equal(vc, vp)
    # one batched step over the three paged sequences against three single steps on the contiguous caches
    toks = np.zeros((B, L), dtype=np.int32)
    cands = []
    for b in range(B):
        truth = so.ar_greedy(om, prompts[b], k)[n_prompt[b]:]
        c = truth[:b % (k + 1)] + [int(t) for t in rng.integers(0, shape.vocab, size=k - b % (k + 1))]
        cands.append(c)
        toks[b], _ = so.extended_input([int(prompts[b][-1])], c, k, shape.mask_id)
    batch_kv = binding.PagedKV(pool, table, lens)
    batch_kv.set_len_bound(max(n_prompt))
    out = binding.StepOut(gm, B, L, k, next_rows=L)
    gm.step(torch.from_numpy(toks).cuda(), gm.layout(spec), batch_kv, out, next_layout=gm.layout(spec))
    gm.kv_commit(batch_kv, out.accepted_len)
    torch.cuda.synchronize()
    assert gm.device_faults() == 0
    # the same launch shapes on a contiguous cache of three sequences: identical bits are expected
    cc = binding.KVCache(gm, B, 32 * stride)
    for b in range(B):
        cc.k_view()[:, b] = caches[b].k_view()[:, 0]
        cc.v_view()[:, b] = caches[b].v_view()[:, 0]
    cc.len.copy_(torch.tensor([n - 1 for n in n_prompt], dtype=torch.int32))
    cc.set_len_bound(max(n_prompt))
    ref_out = binding.StepOut(gm, B, L, k, next_rows=L)
    gm.step(torch.from_numpy(toks).cuda(), gm.layout(spec), cc, ref_out, next_layout=gm.layout(spec))
    gm.kv_commit(cc, ref_out.accepted_len)
    torch.cuda.synchronize()
    assert torch.equal(ref_out.logits, out.logits)                                # bit for bit
    assert torch.equal(ref_out.accepted_len, out.accepted_len) and torch.equal(ref_out.next_tokens, out.next_tokens)
    assert torch.equal(cc.len, lens)
    for b in range(B):
        okv = so.OracleKV(om)
        so.prefill(om, okv, prompts[b][:-1])
        ref, _, _, _ = so.space_step_cached(om, okv, int(prompts[b][-1]), cands[b], k)
        assert np.abs(out.logits[b].cpu().numpy() - ref.logits).max() < gc.LOGIT_TIGHT
        assert int(out.accepted_len[b]) == ref.accepted
    assert lens.cpu().tolist() == [n_prompt[b] - 1 + int(out.accepted_len[b]) + 1 for b in range(B)]


def test_bad_table_entries_are_clamped_and_counted(torch_mod):
    torch = torch_mod
    from paper_2402_11809_amd import binding, layout as lo
    shape = SHAPES["tiny"]
    gm = gc.make_gpu_model(shape, all_weights(shape, seed=0), max_batch=1, max_rows=16, max_ctx=128)
    pool = binding.PagePool(gm, 4)
    table = torch.tensor([[0, 9, -3, 1]], dtype=torch.int32, device="cuda")       # entries 1 and 2 outside the pool
    lens = torch.tensor([40], dtype=torch.int32, device="cuda")                   # the step writes into page entry 1
    kv = binding.PagedKV(pool, table, lens)
    kv.set_len_bound(40)
    spec = lo.paper_layout(2)
    out = binding.StepOut(gm, 1, spec.n_rows, 2)
    before = gm.device_faults()
    gm.step(torch.zeros(1, spec.n_rows, dtype=torch.int32, device="cuda"), gm.layout(spec), kv, out)
    torch.cuda.synchronize()
    assert gm.device_faults() > before
    assert bool(torch.isfinite(out.logits).all())
    bad = binding.PagedKV(pool, table, lens)
    bad.c.capacity = 64                                                            # not 32 * table_stride
    with pytest.raises(binding.SpaceError) as e:
        gm.step(torch.zeros(1, spec.n_rows, dtype=torch.int32, device="cuda"), gm.layout(spec), bad, out)
    assert e.value.code == binding.SPACE_EINVAL


@pytest.mark.parametrize("shape_name,k,max_seqs,n_pages", [("tiny", 3, 3, 40), ("small128", 4, 4, 64), ("tiny", 2, 2, 4)])
def test_continuous_batching_is_lossless(torch_mod, shape_name, k, max_seqs, n_pages):
    """Requests of different prompt lengths and budgets join and leave the running batch; every output
    equals plain greedy decoding of that prompt alone.  The last case has so few pages that sequences
    are put back in the queue and start over."""
    torch = torch_mod
    from paper_2402_11809_amd.serving import ContinuousBatcher
    shape = SHAPES[shape_name]
    w = all_weights(shape, seed=4)
    gm = gc.make_gpu_model(shape, w, max_batch=max_seqs, max_rows=max(32, (k + 1) ** 2), max_ctx=160)
    om = gc.oracle_model(shape, w)
    rng = np.random.default_rng(11)
    reqs = []
    for i in range(7):
        n = int(rng.integers(1, 70))
        reqs.append((prompt_tokens(shape, seed=50 + i, n=n)[0], int(rng.integers(3, 28))))
    eos = None
    cb = ContinuousBatcher(gm, k, max_seqs=max_seqs, n_pages=n_pages, max_ctx=160, prefill_chunk=32)
    for p, n_new in reqs:
        cb.submit(p, n_new)
    done = cb.run()
    torch.cuda.synchronize()
    assert gm.device_faults() == 0 and len(done) == len(reqs) and cb.alloc.n_free == n_pages
    assert cb.steps < sum(n for _, n in reqs)             # batched and more than one token per invocation
    assert (cb.restarts > 0) == (n_pages == 4)            # only the starved pool has to put sequences back
    for r, (p, n_new) in zip(done, reqs):
        ref = so.ar_greedy(om, p, n_new)[len(p):]
        assert r.output == [int(t) for t in ref], r.rid
    # the same stream with an end-of-sequence id taken from the middle of one continuation
    ref3 = so.ar_greedy(om, reqs[3][0], reqs[3][1])[len(reqs[3][0]):]
    eos = int(ref3[len(ref3) // 2])
    cb = ContinuousBatcher(gm, k, max_seqs=max_seqs, n_pages=n_pages, max_ctx=160, prefill_chunk=32, eos_id=eos)
    for p, n_new in reqs:
        cb.submit(p, n_new)
    done = cb.run()
    for r, (p, n_new) in zip(done, reqs):
        ref = [int(t) for t in so.ar_greedy(om, p, n_new)[len(p):]]
        want = ref[: ref.index(eos)] if eos in ref else ref
        assert r.output == want and r.finished == (eos in ref), r.rid
    assert cb.alloc.n_free == n_pages


def test_continuous_batching_with_rejection_sampling(torch_mod):
    """The batcher with space_sample_verify instead of the greedy scan.  top_k = 1 makes sampling
    deterministic: every output must equal plain greedy decoding.  With top-k 10 / top-p 0.95 every
    request must follow the oracle's own sampling loop on its own uniforms token for token while the
    oracle's uniforms keep 5e-4 clear of their thresholds (as in the single-sequence test)."""
    torch = torch_mod
    from oracle import space_sampling as sp
    from paper_2402_11809_amd import layout as lo
    from paper_2402_11809_amd.serving import ContinuousBatcher
    from tests.test_gpu_sampling import _fragile
    shape = SHAPES["tiny"]
    w = all_weights(shape, seed=0)
    k, S = 3, 3
    gm = gc.make_gpu_model(shape, w, max_batch=S, max_rows=32, max_ctx=160)
    om = gc.oracle_model(shape, w)
    rng = np.random.default_rng(21)
    reqs = []
    for i in range(6):
        n, n_new = int(rng.integers(2, 50)), int(rng.integers(5, 20))
        reqs.append((prompt_tokens(shape, seed=70 + i, n=n)[0], n_new,
                     rng.uniform(0.001, 0.999, size=(n_new + 2, 2 * k + 1)).astype(np.float32)))
    for top_k, residual in ((1, False), (10, False), (10, True)):
        cb = ContinuousBatcher(gm, k, max_seqs=S, n_pages=30, max_ctx=160, prefill_chunk=32,
                               sampling={"top_k": top_k, "top_p": 0.95, "residual": residual})
        for p, n_new, u in reqs:
            cb.submit(p, n_new, uniforms=u)
        done = cb.run()
        torch.cuda.synchronize()
        assert gm.device_faults() == 0 and len(done) == len(reqs) and cb.alloc.n_free == 30
        compared = 0
        for r, (p, n_new, u) in zip(done, reqs):
            if top_k == 1:
                ref = [int(t) for t in so.ar_greedy(om, p, n_new)[len(p):]]
                if r.output != ref:
                    first = next(i for i, (a, b) in enumerate(zip(r.output, ref)) if a != b)
                    assert gc.top2_gap(so.causal_forward(om, list(p) + ref[:first])[-1]) < gc.TIE_GAP
                continue
            trace = []
            oseq, ohist = sp.space_generate_sampling(om, [int(t) for t in p], k, n_new, u, top_k=10, top_p=0.95,
                                                     extra="residual" if residual else "printed", trace=trace)
            spec = lo.paper_layout(k)
            n_ok, steps_ok = 0, 0
            for (P32, cands, p_c, uu), acc in zip(trace, ohist):
                if _fragile(P32, spec, cands, p_c, uu, 10, 0.95, MARGIN=5e-4):
                    break
                n_ok += acc + 1
                steps_ok += 1
            n_ok = min(n_ok, n_new)
            assert r.output[:n_ok] == oseq[len(p):len(p) + n_ok], (r.rid, residual, steps_ok)
            assert r.accepted[:steps_ok] == ohist[:steps_ok]
            compared += n_ok
        if top_k > 1:
            assert compared >= 20, compared
