"""Pins of the sampling oracle (oracle/space_sampling.py) against things other than itself:
the library warpers, the greedy limit (itself pinned by brute force in test_oracle_pins.py),
closed forms of the acceptance law, the speculative-sampling identity, planted row markers."""
import numpy as np
import pytest

from oracle import space_oracle as so
from oracle import space_sampling as sp


def _rows(seed, n, V, scale=2.0):
    return (np.random.default_rng(seed).standard_normal((n, V)) * scale).astype(np.float32)


@pytest.mark.parametrize("top_k,top_p", [(10, 0.95), (10, 0.5), (3, 0.99), (50, 0.9), (1, 0.95)])
def test_warp_matches_library_warpers(top_k, top_p):
    """top-k then top-p as chained by the transformers logits processors (Appendix, Random
    Sampling: top-p = 0.95, top-k = 10)."""
    torch = pytest.importorskip("torch")
    lp = pytest.importorskip("transformers.generation.logits_process")
    rows = _rows(1, 12, 500)
    for r in rows:
        s = torch.from_numpy(r)[None]
        s = lp.TopKLogitsWarper(top_k=top_k)(None, s)
        s = lp.TopPLogitsWarper(top_p=top_p)(None, s)
        ref = torch.softmax(s, dim=-1)[0].numpy()
        ids, probs = sp.warp(r, top_k, top_p)
        assert set(ids.tolist()) == set(np.nonzero(ref > 0)[0].tolist())
        np.testing.assert_allclose(probs, ref[ids], rtol=2e-6, atol=1e-7)
        assert np.all(np.diff(probs) <= 0)              # descending order
        assert abs(float(probs.sum()) - 1.0) < 1e-6


def test_warp_ties_take_lowest_id_and_nucleus_is_shortest_prefix():
    x = np.zeros(8, dtype=np.float32)
    x[[5, 2, 7]] = 3.0                                  # three equal maxima
    ids, probs = sp.warp(x, top_k=2, top_p=1.0)
    assert ids.tolist() == [2, 5]
    np.testing.assert_allclose(probs, [0.5, 0.5], rtol=1e-6)
    # probabilities 0.5, 0.25, 0.125, ...: top_p = 0.75 is reached exactly by two tokens
    y = np.log(np.array([0.5, 0.25, 0.125, 0.0625, 0.0625], dtype=np.float64)).astype(np.float32)
    ids, probs = sp.warp(y, top_k=5, top_p=0.74)
    assert ids.tolist() == [0, 1]
    ids, probs = sp.warp(y, top_k=5, top_p=0.76)
    assert ids.tolist() == [0, 1, 2]
    np.testing.assert_allclose(probs, np.array([0.5, 0.25, 0.125]) / 0.875, rtol=1e-5)


def test_draw_is_inverse_cdf():
    ids = np.array([7, 3, 9]); probs = np.array([0.6, 0.3, 0.1], dtype=np.float32)
    N = 20000
    hits = {7: 0, 3: 0, 9: 0}
    for j in range(N):
        t, p = sp.draw(ids, probs, (j + 0.5) / N)
        hits[t] += 1
        assert p == probs[list(ids).index(t)]
    for t, p in zip(ids, probs):
        assert abs(hits[int(t)] / N - float(p)) < 2.0 / N + 1e-6
    assert sp.draw(ids, probs, 0.0)[0] == 7 and sp.draw(ids, probs, 0.9999999)[0] == 9


@pytest.mark.parametrize("k", [1, 3, 5])
def test_greedy_limit_equals_greedy_verification(k):
    """top_k = 1 makes every distribution one-hot: the rule r <= Q(c)/P_c accepts exactly the
    candidates that equal the argmax, whatever the uniforms are."""
    V, L = 50, (k + 1) ** 2
    rng = np.random.default_rng(k)
    P = _rows(10 + k, L, V)
    am = np.argmax(P, axis=-1)
    for j in range(k + 1):                               # j correct candidates, then a wrong one
        cands = [int(am[i * (k + 1)]) for i in range(k)]
        if j < k:
            cands[j] = (cands[j] + 1) % V
        ref = so.verify_greedy(P.astype(np.float64), k, cands)
        u = rng.uniform(0.01, 0.99, size=2 * k + 1)
        got = sp.verify_sampling(P, k, cands, [1.0] * k, u, top_k=1, top_p=0.95)
        assert got.accepted == ref.accepted == j
        assert got.emitted == ref.emitted and got.new_cands == ref.new_cands
        assert all(float(p) == 1.0 for p in got.new_pc)


def test_acceptance_threshold_and_first_iteration():
    k, V = 2, 6
    L = (k + 1) ** 2
    P = np.full((L, V), -30.0, dtype=np.float32)
    P[:, 0] = 0.0
    P[0, :3] = np.log(np.array([0.5, 0.3, 0.2]))        # Q of the first test
    ids, probs = sp.warp(P[0], 10, 1.0)
    q1 = float(probs[list(ids).index(1)])
    assert abs(q1 - 0.3) < 1e-6
    u = [0.0] * (2 * k + 1)
    for pc, thr in ((0.6, q1 / 0.6), (0.3, 1.0), (0.1, 1.0)):   # min(1, Q/P_c)
        for r, expect in ((thr - 1e-4, True), (min(thr + 1e-4, 0.9999), thr >= 1.0)):
            u[0] = r
            u[1] = 0.99999                               # second candidate (token 5, prob ~0) is rejected
            res = sp.verify_sampling(P, k, [1, 5], [pc, 1.0], u, top_k=10, top_p=1.0)
            assert (res.accepted >= 1) == expect, (pc, r)
    # P_c = +inf: the dummies of the first iteration are rejected for every r > 0
    u[0] = 1e-6
    res = sp.verify_sampling(P, k, [0, 0], [np.inf, np.inf], u, top_k=10, top_p=1.0)
    assert res.accepted == 0 and float(res.ratios[0]) == 0.0


def test_speculative_sampling_identity_for_the_residual_rule():
    """sum_c P(c) min(1, Q(c)/P(c)) [t = c] + (1 - beta) norm(max(0, Q - P))(t) = Q(t)."""
    rng = np.random.default_rng(3)
    for _ in range(20):
        V = 9
        q = rng.dirichlet(np.ones(V)).astype(np.float32)
        p = rng.dirichlet(np.ones(V)).astype(np.float32)
        ids = np.arange(V)
        _, res = sp.residual(ids, q, ids, p)
        acc = np.minimum(q, p)                            # P(c) min(1, Q(c)/P(c))
        beta = acc.sum()
        law = acc + (1.0 - beta) * res
        np.testing.assert_allclose(law, q, atol=2e-6)


@pytest.mark.parametrize("extra", ["printed", "residual"])
def test_law_of_the_first_emitted_token(extra):
    """k = 1, candidate c fixed: the first emitted token is c with probability beta = min(1, Q(c)/P_c)
    and otherwise a draw from Q (as printed) or from the residual (cited rule).  Checked on a
    grid of (r, u) pairs, i.e. by integration, not by a random experiment."""
    V, k = 5, 1
    q = np.array([0.4, 0.3, 0.15, 0.1, 0.05]); pd = np.array([0.1, 0.6, 0.1, 0.1, 0.1])
    P = np.zeros((4, V), dtype=np.float32)
    P[0] = np.log(q)
    c = 1
    N = 150
    counts = np.zeros(V)
    d_ids = np.argsort(-pd, kind="stable"); d_probs = pd[d_ids].astype(np.float32)
    for a in range(N):
        for b in range(N):
            u = [(a + 0.5) / N, (b + 0.5) / N, 0.5]
            res = sp.verify_sampling(P, k, [c], [pd[c]], u, top_k=V, top_p=1.0, extra=extra,
                                     draft_dists=[(d_ids, d_probs)])
            counts[res.emitted[0]] += 1
    beta = min(1.0, q[c] / pd[c])
    tail = q if extra == "printed" else np.maximum(0, q - pd) / np.maximum(0, q - pd).sum()
    law = (1 - beta) * tail
    law[c] += beta
    np.testing.assert_allclose(counts / N ** 2, law, atol=2.5 / N)


@pytest.mark.parametrize("k", [2, 5])
def test_candidate_refresh_reads_the_mask_group_behind_the_last_accepted_token(k):
    """Every block row gets a marker token of its own (probability ~1): the new candidates must be
    the markers of rows idx .. idx+k-1 with idx = 1 + accepted (k+1) (block-relative form of
    idx = l+1+i(k+1) in Algorithm 1), the extra token the marker of row accepted (k+1)."""
    L = (k + 1) ** 2
    V = L + 3
    P = np.full((L, V), -40.0, dtype=np.float32)
    for r in range(L):
        P[r, r] = 0.0
    for acc in range(k + 1):
        # candidate i is accepted iff it equals the marker of row (i-1)(k+1)
        cands = [(i - 1) * (k + 1) for i in range(1, k + 1)]
        if acc < k:
            cands[acc] = V - 1
        u = [0.5] * (2 * k + 1)
        res = sp.verify_sampling(P, k, cands, [1.0] * k, u, top_k=10, top_p=0.95)
        assert res.accepted == acc
        assert res.emitted == cands[:acc] + [acc * (k + 1)]
        idx = 1 + acc * (k + 1)
        assert res.new_cands == list(range(idx, idx + k))
        assert all(abs(float(p) - 1.0) < 1e-6 for p in res.new_pc)


def test_each_draw_uses_its_own_uniform():
    """uniforms[i-1] decides the i-th test, uniforms[k] the extra token, uniforms[k+1+j] the j-th
    new candidate: every row offers two tokens with probabilities 0.6 / 0.4, so the position of a
    uniform relative to 0.6 shows up in exactly one output."""
    k = 3
    L = (k + 1) ** 2
    V = 2 * L
    P = np.full((L, V), -40.0, dtype=np.float32)
    for r in range(L):
        P[r, 2 * r] = np.log(0.6)
        P[r, 2 * r + 1] = np.log(0.4)
    cands = [0, 2 * (k + 1), 2 * 2 * (k + 1)]          # the likelier token of rows 0, k+1, 2(k+1)
    base = [0.3] * (2 * k + 1)                           # all tests pass (0.3 <= 0.6 / 1), all draws take the 0.6 token
    ref = sp.verify_sampling(P, k, cands, [1.0] * k, base, top_k=10, top_p=1.0)
    assert ref.accepted == k and ref.emitted[-1] == 2 * k * (k + 1)
    idx = 1 + k * (k + 1)
    assert ref.new_cands == [2 * (idx + j) for j in range(k)]
    for pos in range(2 * k + 1):
        u = list(base)
        u[pos] = 0.7
        res = sp.verify_sampling(P, k, cands, [1.0] * k, u, top_k=10, top_p=1.0)
        if pos < k:                                      # the (pos+1)-th test now fails
            assert res.accepted == pos
        elif pos == k:
            assert res.accepted == k and res.emitted[-1] == 2 * k * (k + 1) + 1 and res.new_cands == ref.new_cands
        else:
            j = pos - k - 1
            expect = list(ref.new_cands)
            expect[j] += 1
            assert res.accepted == k and res.emitted == ref.emitted and res.new_cands == expect
            assert abs(float(res.new_pc[j]) - 0.4) < 1e-6


def test_sampling_loop_at_top_k_one_is_plain_greedy_decoding():
    """The decoding loop of Algorithm 1 in the sampling setting, with every distribution one-hot
    (top_k = 1), must reproduce plain greedy autoregressive decoding token for token."""
    from space_inputs import SHAPES, all_weights, prompt_tokens
    shape = SHAPES["tiny"]
    m = so.model_from_weights(shape, all_weights(shape, seed=0))
    prompt = [int(t) for t in prompt_tokens(shape, seed=5, n=12)[0]]
    k, n_new = 3, 14
    u = np.random.default_rng(1).uniform(0.01, 0.99, size=(n_new + 1, 2 * k + 1)).astype(np.float32)
    seq, hist = sp.space_generate_sampling(m, prompt, k, n_new, u, top_k=1, top_p=0.95)
    assert seq == so.ar_greedy(m, prompt, n_new)
    assert hist[0] == 0 and all(0 <= a <= k for a in hist)
    # and with real sampling every emitted token lies in the warped support of its own causal forward
    seq2, _ = sp.space_generate_sampling(m, prompt, k, 8, u, top_k=4, top_p=0.9)
    for i in range(len(prompt), len(seq2)):
        ids, _ = sp.warp(so.causal_forward(m, seq2[:i])[-1].astype(np.float32), 4, 0.9)
        assert seq2[i] in ids.tolist()


def test_sampling_loop_eos_stop_equals_truncated_greedy_at_top_k_one():
    """With top_k = 1 the sampling loop is greedy decoding; an eos_id cuts it in front of that token."""
    from space_inputs import SHAPES, all_weights, prompt_tokens
    shape = SHAPES["tiny"]
    om = so.model_from_weights(shape, all_weights(shape, seed=0), "exact")
    prompt = [int(t) for t in prompt_tokens(shape, seed=8, n=12)[0]]
    k, n_new = 3, 14
    u = np.random.default_rng(0).uniform(0.01, 0.99, size=(n_new + 2, 2 * k + 1)).astype(np.float32)
    ref = so.ar_greedy(om, prompt, n_new)
    gen = ref[len(prompt):]
    for pos in (0, 5, len(gen) - 1):
        eos = gen[pos]
        seq, _ = sp.space_generate_sampling(om, prompt, k, n_new, u, top_k=1, top_p=0.9, eos_id=eos)
        assert seq == ref[: len(prompt) + gen.index(eos)]
    seq, _ = sp.space_generate_sampling(om, prompt, k, n_new, u, top_k=1, top_p=0.9, eos_id=shape.vocab + 5)
    assert seq == ref
