"""GPU parity of space_sample_verify (rejection-sampling form of Algorithm 1) against
oracle/space_sampling.py, through the C ABI.  Integer outputs (accepted count, tokens) must be
equal; a case is only excused when the oracle itself shows that a uniform sits within 1e-5 of
the threshold it is compared with (both sides decide in float32, whose exp may differ in the
last bit)."""
import numpy as np
import pytest

from oracle import space_oracle as so
from oracle import space_sampling as sp
from space_inputs import SHAPES, all_weights, prompt_tokens
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu

MARGIN = 1e-5


@pytest.fixture(scope="module")
def torch_mod():
    return gc.require_gpu()


def _fragile(P, spec, cands, p_c, u, top_k, top_p, MARGIN=MARGIN):
    """True if some uniform of this case is within MARGIN of the value it is compared with."""
    k = len(cands)
    real = gc.real_rows(spec)
    q_ids, q_probs = sp.warp(P[real[0]], top_k, top_p)
    acc = 0
    for i in range(1, k + 1):
        with np.errstate(divide="ignore", invalid="ignore"):
            ratio = float(sp.prob_of(q_ids, q_probs, cands[i - 1]) / np.float32(p_c[i - 1]))
        if abs(u[i - 1] - ratio) < MARGIN:
            return True
        if u[i - 1] <= ratio:
            acc += 1
            q_ids, q_probs = sp.warp(P[real[i]], top_k, top_p)
        else:
            break
    rows = [real[acc]] + [real[acc] + 1 + j for j in range(k)]
    for row, uu in zip(rows, [u[k]] + list(u[k + 1:])):
        _, probs = sp.warp(P[row], top_k, top_p)
        if np.any(np.abs(np.cumsum(probs.astype(np.float64)) - uu) < MARGIN):
            return True
    return False


def _case(rng, spec, V, k, mode):
    """Logits, candidates, P_c and uniforms of one sequence; `mode` steers how many candidates pass."""
    L = spec.n_rows
    P = (rng.standard_normal((L, V)) * 2.5).astype(np.float32)
    real = gc.real_rows(spec)
    cands, p_c = [], []
    for i in range(1, k + 1):
        ids, probs = sp.warp(P[real[i - 1]], 10, 0.95)
        if mode == "likely":
            c = int(ids[0]); pc = float(probs[0]) * rng.uniform(0.5, 1.5)
        elif mode == "mixed":
            j = int(rng.integers(0, len(ids))); c = int(ids[j]); pc = float(rng.uniform(0.05, 1.0))
        else:
            c = int(rng.integers(0, V)); pc = float(rng.uniform(0.05, 1.0))
        cands.append(c); p_c.append(pc)
    u = rng.uniform(0.0, 1.0, size=2 * k + 1).astype(np.float32)
    return P, cands, p_c, u


@pytest.mark.parametrize("V,k,top_k,top_p", [(32000, 5, 10, 0.95), (32000, 3, 10, 0.95), (1000, 5, 4, 0.8),
                                             (40000, 2, 64, 1.0), (1000, 5, 1, 0.95)])
def test_sample_verify_matches_oracle(torch_mod, V, k, top_k, top_p):
    torch = torch_mod
    from paper_2402_11809_amd import binding, layout as lo
    shape = SHAPES["tiny"]
    import dataclasses
    shape = dataclasses.replace(shape, vocab=V, n_layers=1)
    w = all_weights(shape, seed=0)
    B = 4
    spec = lo.paper_layout(k)
    L = spec.n_rows
    gm = gc.make_gpu_model(shape, w, max_batch=B, max_rows=L, max_ctx=64)
    lay = gm.layout(spec)
    rng = np.random.default_rng(100 * k + top_k)
    n_checked = 0
    for rep, mode in enumerate(["likely", "mixed", "random", "likely"]):
        P = np.zeros((B, L, V), dtype=np.float32)
        toks = np.zeros((B, L), dtype=np.int32)
        p_c = np.ones((B, k), dtype=np.float32)
        u = np.zeros((B, 2 * k + 1), dtype=np.float32)
        cands = []
        for b in range(B):
            P[b], c, pc, u[b] = _case(rng, spec, V, k, mode)
            cands.append(c)
            p_c[b] = pc
            t, _ = so.extended_input([int(rng.integers(0, V))], c, k, shape.mask_id)
            toks[b] = t
        if rep == 3:
            p_c[0, :] = np.inf                                   # first iteration: dummies are rejected
        out = binding.SampleOut(gm, B, spec.n_groups, k, top_k, next_rows=L, emit_cap=16)
        gm.sample_verify(torch.from_numpy(P).cuda(), torch.from_numpy(toks).cuda(), lay, torch.from_numpy(p_c).cuda(),
                         torch.from_numpy(u).cuda(), out, top_k=top_k, top_p=top_p, next_layout=lay)
        torch.cuda.synchronize()
        assert gm.device_faults() == 0
        for b in range(B):
            if _fragile(P[b], spec, cands[b], p_c[b], u[b], top_k, top_p):
                continue
            ref = sp.verify_sampling(P[b], k, cands[b], p_c[b], u[b], top_k=top_k, top_p=top_p)
            n_checked += 1
            assert int(out.accepted_len.cpu()[b]) == ref.accepted
            assert int(out.extra.cpu()[b]) == ref.emitted[-1]
            assert out.new_cands.cpu().numpy()[b].tolist() == ref.new_cands
            np.testing.assert_allclose(out.new_pc.cpu().numpy()[b], np.array(ref.new_pc), rtol=2e-6)
            got_r = out.ratios.cpu().numpy()[b]
            np.testing.assert_allclose(got_r[: len(ref.ratios)], np.array(ref.ratios), rtol=2e-6, atol=1e-30)
            assert np.all(got_r[len(ref.ratios):] == -1.0)
            n = int(out.emit_len.cpu()[b])
            assert out.emit.cpu().numpy()[b, :n].tolist() == ref.emitted
            nxt, _ = so.extended_input([ref.emitted[-1]], ref.new_cands, k, shape.mask_id)
            assert out.next_tokens.cpu().numpy()[b].tolist() == list(nxt)
            idx = 1 + ref.accepted * (k + 1)
            for j in range(k):                                    # the distributions the drafts came from
                ids, probs = sp.warp(P[b, idx + j], top_k, top_p)
                g_ids = out.new_ids.cpu().numpy()[b, j]
                g_pr = out.new_probs.cpu().numpy()[b, j]
                assert g_ids[: len(ids)].tolist() == ids.tolist() and np.all(g_ids[len(ids):] == -1)
                np.testing.assert_allclose(g_pr[: len(ids)], probs, rtol=2e-6)
    assert n_checked >= 12


def test_residual_rule_matches_oracle(torch_mod):
    torch = torch_mod
    from paper_2402_11809_amd import binding, layout as lo
    import dataclasses
    V, k, top_k, top_p = 2000, 4, 8, 0.9
    shape = dataclasses.replace(SHAPES["tiny"], vocab=V, n_layers=1)
    gm = gc.make_gpu_model(shape, all_weights(shape, seed=0), max_batch=6, max_rows=25, max_ctx=64)
    spec = lo.paper_layout(k)
    lay = gm.layout(spec)
    L, B = spec.n_rows, 6
    rng = np.random.default_rng(5)
    P = (rng.standard_normal((B, L, V)) * 2.0).astype(np.float32)
    D = (rng.standard_normal((B, k, V)) * 2.0).astype(np.float32)      # logits the drafts were drawn from
    toks = np.zeros((B, L), dtype=np.int32)
    p_c = np.zeros((B, k), dtype=np.float32)
    d_ids = -np.ones((B, k, top_k), dtype=np.int32)
    d_pr = np.zeros((B, k, top_k), dtype=np.float32)
    u = rng.uniform(0, 1, size=(B, 2 * k + 1)).astype(np.float32)
    cands, dists = [], []
    for b in range(B):
        cs, ds = [], []
        for i in range(k):
            ids, probs = sp.warp(D[b, i], top_k, top_p)
            c, pc = sp.draw(ids, probs, float(rng.uniform()))
            cs.append(c); ds.append((ids, probs))
            p_c[b, i] = pc
            d_ids[b, i, : len(ids)] = ids
            d_pr[b, i, : len(ids)] = probs
            # make the draft plausible for the verifier too
            P[b, gc.real_rows(spec)[i], c] += 3.0
        cands.append(cs); dists.append(ds)
        toks[b], _ = so.extended_input([1], cs, k, shape.mask_id)
    out = binding.SampleOut(gm, B, spec.n_groups, k, top_k)
    gm.sample_verify(torch.from_numpy(P).cuda(), torch.from_numpy(toks).cuda(), lay, torch.from_numpy(p_c).cuda(),
                     torch.from_numpy(u).cuda(), out, top_k=top_k, top_p=top_p, residual=True,
                     draft_ids=torch.from_numpy(d_ids).cuda(), draft_probs=torch.from_numpy(d_pr).cuda())
    torch.cuda.synchronize()
    seen_rejection = 0
    for b in range(B):
        ref = sp.verify_sampling(P[b], k, cands[b], p_c[b], u[b], top_k=top_k, top_p=top_p, extra="residual",
                                 draft_dists=dists[b])
        plain = sp.verify_sampling(P[b], k, cands[b], p_c[b], u[b], top_k=top_k, top_p=top_p)
        seen_rejection += ref.accepted < k
        assert int(out.accepted_len.cpu()[b]) == ref.accepted
        assert int(out.extra.cpu()[b]) == ref.emitted[-1], (b, ref.emitted, plain.emitted)
        assert out.new_cands.cpu().numpy()[b].tolist() == ref.new_cands
    assert seen_rejection >= 2


def test_top_k_one_equals_the_greedy_step(torch_mod):
    """Greedy limit on the device: with top_k = 1 and P_c = 1 the sampling verification of the logits of a
    real step returns what the step's own greedy verification returned."""
    torch = torch_mod
    from paper_2402_11809_amd import binding, layout as lo
    from paper_2402_11809_amd.runtime import SpaceDecoder
    shape = SHAPES["tiny"]
    w = all_weights(shape, seed=0)
    gm = gc.make_gpu_model(shape, w, max_batch=1, max_rows=64)
    om = gc.oracle_model(shape, w)
    k = 4
    prompt = prompt_tokens(shape, seed=2, n=30)
    dec = SpaceDecoder(gm, k, batch=1, capacity=128, prefill_chunk=16)
    dec.prefill(prompt[:, :-1])
    truth = so.ar_greedy(om, prompt[0], k + 1)[30:]
    spec = lo.paper_layout(k)
    lay = gm.layout(spec)
    for n_ok in (0, 2, 4):
        cands = list(truth[:k])
        if n_ok < k:
            cands[n_ok] = (cands[n_ok] + 7) % shape.vocab
        toks, _ = so.extended_input([int(prompt[0, -1])], cands, k, shape.mask_id)
        t = torch.from_numpy(toks[None].astype(np.int32)).cuda()
        out = binding.StepOut(gm, 1, spec.n_rows, k, next_rows=spec.n_rows)
        gm.step(t, lay, dec.kv, out, next_layout=lay)
        sout = binding.SampleOut(gm, 1, spec.n_groups, k, 1, next_rows=spec.n_rows)
        u = torch.full((1, 2 * k + 1), 0.37, dtype=torch.float32, device="cuda")
        gm.sample_verify(out.logits, t, lay, torch.ones(1, k, device="cuda"), u, sout, top_k=1, top_p=0.95,
                         next_layout=lay)
        torch.cuda.synchronize()
        assert int(sout.accepted_len.cpu()[0]) == int(out.accepted_len.cpu()[0])
        assert int(sout.extra.cpu()[0]) == int(out.bonus.cpu()[0])
        assert sout.new_cands.cpu().tolist() == out.new_cands.cpu().tolist()
        assert sout.next_tokens.cpu().tolist() == out.next_tokens.cpu().tolist()
        gm.kv_rollback(dec.kv, None, n_all=0)


def test_sampling_loop_on_model_logits_teacher_forced(torch_mod):
    """Several consecutive steps of Algorithm 1 in the sampling setting on a real (tiny) model: each
    side computes its own logits from the same tokens; decisions are compared wherever the oracle's
    uniforms keep 2e-3 clear of their thresholds (the logits agree to ~2e-4); the next step's tokens
    and P_c always come from the oracle, and both caches commit the oracle's accepted count."""
    torch = torch_mod
    from paper_2402_11809_amd import binding, layout as lo
    from paper_2402_11809_amd.runtime import SpaceDecoder
    shape = SHAPES["tiny"]
    w = all_weights(shape, seed=0)
    gm = gc.make_gpu_model(shape, w, max_batch=1, max_rows=64)
    om = gc.oracle_model(shape, w)
    k, top_k, top_p = 3, 10, 0.95
    prompt = prompt_tokens(shape, seed=4, n=24)
    dec = SpaceDecoder(gm, k, batch=1, capacity=128, prefill_chunk=16)
    dec.prefill(prompt[:, :-1])
    okv = so.OracleKV(om)
    so.prefill(om, okv, prompt[0, :-1])
    spec = lo.paper_layout(k)
    lay = gm.layout(spec)
    rng = np.random.default_rng(11)
    last = int(prompt[0, -1])
    cands, p_c = [0] * k, [np.inf] * k                       # first iteration of Algorithm 1
    compared = accepted_total = 0
    for step in range(8):
        u = rng.uniform(0, 1, size=2 * k + 1).astype(np.float32)
        toks, is_mask = so.extended_input([last], cands, k, shape.mask_id)
        P, ks, vs, pos = so.block_forward_cached(om, okv, toks, is_mask, k)
        P32 = P.astype(np.float32)
        ref = sp.verify_sampling(P32, k, cands, p_c, u, top_k=top_k, top_p=top_p)
        t = torch.from_numpy(toks[None].astype(np.int32)).cuda()
        out = binding.StepOut(gm, 1, spec.n_rows, k)
        gm.step(t, lay, dec.kv, out)
        sout = binding.SampleOut(gm, 1, spec.n_groups, k, top_k, next_rows=spec.n_rows)
        pc_t = torch.from_numpy(np.array([p_c], dtype=np.float32)).cuda()
        gm.sample_verify(out.logits, t, lay, pc_t, torch.from_numpy(u[None]).cuda(), sout, top_k=top_k, top_p=top_p,
                         next_layout=lay)
        torch.cuda.synchronize()
        assert np.abs(out.logits.cpu().numpy()[0] - P).max() < gc.LOGIT_TIGHT
        if not _fragile(P32, spec, cands, p_c, u, top_k, top_p, MARGIN=2e-3):
            compared += 1
            assert int(sout.accepted_len.cpu()[0]) == ref.accepted
            assert int(sout.extra.cpu()[0]) == ref.emitted[-1]
            assert sout.new_cands.cpu().numpy()[0].tolist() == ref.new_cands
            np.testing.assert_allclose(sout.new_pc.cpu().numpy()[0], np.array(ref.new_pc), rtol=5e-3)
            nxt, _ = so.extended_input([ref.emitted[-1]], ref.new_cands, k, shape.mask_id)
            assert sout.next_tokens.cpu().numpy()[0].tolist() == list(nxt)
        okv.append(ks, vs, [g * (k + 1) for g in range(ref.accepted + 1)])
        gm.kv_commit(dec.kv, None, accepted_all=ref.accepted)
        accepted_total += ref.accepted
        last, cands, p_c = ref.emitted[-1], ref.new_cands, [float(x) for x in ref.new_pc]
    torch.cuda.synchronize()
    assert int(dec.kv.len.cpu()[0]) == okv.length
    assert compared >= 5
    print(f"sampling loop: {compared} of 8 steps compared, {accepted_total} candidates accepted")


def test_device_resident_sampling_loop(torch_mod):
    """SpaceDecoder.generate_sampled keeps tokens, P_c and draft distributions on the device between
    iterations.  With top_k = 1 it must equal plain greedy decoding exactly; with top-k 10 / top-p 0.95
    it must follow the oracle's loop token for token as long as the oracle's uniforms keep 5e-4 clear of
    their thresholds (afterwards the two runs are allowed to part)."""
    torch = torch_mod
    from paper_2402_11809_amd import layout as lo
    from paper_2402_11809_amd.runtime import SpaceDecoder
    shape = SHAPES["tiny"]
    w = all_weights(shape, seed=0)
    gm = gc.make_gpu_model(shape, w, max_batch=1, max_rows=64)
    om = gc.oracle_model(shape, w)
    k, n_new = 3, 20
    prompt = prompt_tokens(shape, seed=6, n=20)
    u = np.random.default_rng(2).uniform(0.001, 0.999, size=(n_new + 2, 1, 2 * k + 1)).astype(np.float32)
    dec = SpaceDecoder(gm, k, batch=1, capacity=128, prefill_chunk=16)
    seq, hist = dec.generate_sampled(prompt, n_new, u, top_k=1, top_p=0.95)
    ref = so.ar_greedy(om, prompt[0], n_new)
    got = [int(t) for t in seq[0]]
    if got != ref:
        first = next(i for i, (a, b) in enumerate(zip(got, ref)) if a != b)
        assert gc.top2_gap(so.causal_forward(om, ref[:first])[-1]) < gc.TIE_GAP
    assert int(hist[0][0]) == 0
    # end-of-sequence stop in the sampling loop (top_k = 1, so the continuation is the greedy one)
    gen = ref[len(prompt[0]):]
    eos = gen[7]
    dec = SpaceDecoder(gm, k, batch=1, capacity=128, prefill_chunk=16, eos_id=eos)
    seq, _ = dec.generate_sampled(prompt, n_new, u, top_k=1, top_p=0.95)
    oseq, _ = sp.space_generate_sampling(om, prompt[0], k, n_new, u[:, 0], top_k=1, top_p=0.95, eos_id=eos)
    n = int(dec.lengths[0])
    assert n == gen.index(eos) == len(oseq) - len(prompt[0])
    assert [int(t) for t in seq[0][: len(prompt[0]) + n]] == oseq
    # real sampling against the oracle's own loop
    for residual in (False, True):
        dec = SpaceDecoder(gm, k, batch=1, capacity=128, prefill_chunk=16)
        seq, hist = dec.generate_sampled(prompt, n_new, u, top_k=10, top_p=0.95, residual=residual)
        trace = []
        oseq, ohist = sp.space_generate_sampling(om, prompt[0], k, n_new, u[:, 0], top_k=10, top_p=0.95,
                                                 extra="residual" if residual else "printed", trace=trace)
        spec = lo.paper_layout(k)
        n_ok = len(prompt[0])
        steps_ok = 0
        for (P32, cands, p_c, uu), acc in zip(trace, ohist):
            if _fragile(P32, spec, cands, p_c, uu, 10, 0.95, MARGIN=5e-4):
                break
            n_ok += acc + 1
            steps_ok += 1
        n_ok = min(n_ok, len(oseq))
        assert [int(t) for t in seq[0][:n_ok]] == oseq[:n_ok], (residual, steps_ok)
        assert [int(h[0]) for h in hist[:steps_ok]] == ohist[:steps_ok]
        assert steps_ok >= 4, steps_ok
        print(f"sampling loop (residual={residual}): {steps_ok} of {len(ohist)} iterations compared, {n_ok - len(prompt[0])} tokens")


def test_sample_verify_eos_stop(torch_mod):
    """EOS check of Algorithm 1 in the sampling form: the emitted run ends in front of the first EOS
    token, the flag is set and stays set, sequences without the token are untouched."""
    torch = torch_mod
    import dataclasses
    from paper_2402_11809_amd import binding, layout as lo
    V, k, B = 1000, 4, 6
    shape = dataclasses.replace(SHAPES["tiny"], vocab=V, n_layers=1)
    spec = lo.paper_layout(k)
    L = spec.n_rows
    gm = gc.make_gpu_model(shape, all_weights(shape, seed=0), max_batch=B, max_rows=L, max_ctx=64)
    lay = gm.layout(spec)
    rng = np.random.default_rng(77)
    P = np.zeros((B, L, V), dtype=np.float32)
    toks = np.zeros((B, L), dtype=np.int32)
    p_c = np.ones((B, k), dtype=np.float32)
    u = np.zeros((B, 2 * k + 1), dtype=np.float32)
    cands = []
    for b in range(B):
        P[b], c, p_c[b], u[b] = _case(rng, spec, V, k, "likely")
        cands.append(c)
        toks[b], _ = so.extended_input([int(rng.integers(0, V))], c, k, shape.mask_id)
    refs = [sp.verify_sampling(P[b], k, cands[b], p_c[b], u[b]) for b in range(B)]
    checked = 0
    for pick in range(k + 1):
        usable = [b for b in range(B) if not _fragile(P[b], spec, cands[b], p_c[b], u[b], 10, 0.95)
                  and len(refs[b].emitted) > pick]
        if not usable:
            continue
        eos = refs[usable[0]].emitted[pick]
        out = binding.SampleOut(gm, B, spec.n_groups, k, 10, next_rows=L, emit_cap=16, eos_id=eos)
        args = (torch.from_numpy(P).cuda(), torch.from_numpy(toks).cuda(), lay, torch.from_numpy(p_c).cuda(),
                torch.from_numpy(u).cuda(), out)
        gm.sample_verify(*args, next_layout=lay)
        torch.cuda.synchronize()
        fin = out.finished.cpu().numpy()
        n = out.emit_len.cpu().numpy()
        for b in usable:
            em = refs[b].emitted
            want = em[: em.index(eos)] if eos in em else em
            assert out.emit.cpu().numpy()[b, : n[b]].tolist() == want
            assert int(fin[b]) == int(eos in em)
            checked += 1
        gm.sample_verify(*args, next_layout=lay)                 # second call: finished ones stay as they are
        torch.cuda.synchronize()
        n2 = out.emit_len.cpu().numpy()
        for b in usable:
            em = refs[b].emitted
            if eos in em:
                assert n2[b] == n[b] and int(out.finished.cpu()[b]) == 1
            else:
                assert n2[b] == 2 * n[b]
    assert checked >= 8
    out = binding.SampleOut(gm, B, spec.n_groups, k, 10, next_rows=L, emit_cap=16, eos_id=3)
    out.finished = None
    with pytest.raises(binding.SpaceError) as e:
        gm.sample_verify(*args[:5], out, next_layout=lay)
    assert e.value.code == binding.SPACE_EINVAL


def test_sample_verify_error_paths(torch_mod):
    torch = torch_mod
    from paper_2402_11809_amd import binding, layout as lo
    shape = SHAPES["tiny"]
    gm = gc.make_gpu_model(shape, all_weights(shape, seed=0), max_batch=1, max_rows=16)
    spec = lo.paper_layout(3)
    lay = gm.layout(spec)
    P = torch.zeros(1, 16, shape.vocab, device="cuda")
    t = torch.zeros(1, 16, dtype=torch.int32, device="cuda")
    pc = torch.ones(1, 3, device="cuda")
    u = torch.zeros(1, 7, device="cuda")
    out = binding.SampleOut(gm, 1, spec.n_groups, 3, 10)
    for kw in (dict(top_k=0), dict(top_k=65), dict(top_p=0.0), dict(top_p=1.5), dict(residual=True)):
        with pytest.raises(binding.SpaceError) as e:
            gm.sample_verify(P, t, lay, pc, u, out, **kw)
        assert e.value.code == binding.SPACE_EINVAL
