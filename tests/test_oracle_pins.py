"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test names the passage it pins.  A mistake planted in the oracle (a dropped term, a
wrong index, a transposed operand) is meant to fail at least one of them.
"""
import os

import numpy as np
import pytest

from oracle import space_oracle as so
from space_inputs import SHAPES, all_weights, prompt_tokens

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def model(tiny_shape, tiny_weights):
    return so.model_from_weights(tiny_shape, tiny_weights)


@pytest.fixture(scope="module")
def prompt(tiny_shape):
    return [int(t) for t in prompt_tokens(tiny_shape, seed=0, n=64)[0]]


@pytest.fixture(scope="module")
def ar_sequence(model, prompt):
    return so.ar_greedy(model, prompt, 40)


# ---------------------------------------------------------------- structure (Eq. 2, Eq. 3)


def _read_golden():
    rows = []
    with open(os.path.join(GOLDEN, "sar_mask_k2_l2.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            r, kind, pos, vis = line.split()
            rows.append((int(r), kind, int(pos), [int(v) for v in vis.split(",")]))
    return rows


@pytest.mark.parametrize("reading", ["group", "literal"])
def test_worked_example_k2(reading):
    """Eq. 2 / Eq. 3 / position ids for k=2, l=2 (appendix figure caption: 8 extra tokens)."""
    rows = _read_golden()
    toks, is_mask = so.extended_input([11, 12], [21, 22], 2, mask_id=99)
    assert len(toks) == 2 + 8 == len(rows)
    assert ["M" if m else "t" for m in is_mask] == ["M" if k == "M" else "t" for _, k, _, _ in rows]
    assert list(toks) == [11, 12, 99, 99, 21, 99, 99, 22, 99, 99]
    A = so.sar_attention_mask(is_mask, 2, reading)
    for r, _, pos, vis in rows:
        assert [j + 1 for j in np.nonzero(A[r - 1])[0]] == vis
    assert list(so.position_ids(A)) == [p for _, _, p, _ in rows]


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5, 8])
@pytest.mark.parametrize("l", [1, 2, 7])
def test_extended_input_identities(k, l):
    """|I| = l + k(k+2); k+1 mask groups of k; closed-form positions (Eq. 2, text after Eq. 3)."""
    toks, is_mask = so.extended_input(list(range(l)), list(range(100, 100 + k)), k, mask_id=-1)
    assert len(toks) == l + k * (k + 2)
    assert is_mask.sum() == k * (k + 1)
    grp = so.mask_group_ids(is_mask)
    assert grp.max() == k
    A = so.sar_attention_mask(is_mask, k)
    pos = so.position_ids(A)
    # prompt rows: 0..l-1; block row (g, t'): candidate at l-1+g, mask t' at l-1+g+t'
    expect = list(range(l))
    for g in range(k + 1):
        if g > 0:
            expect.append(l - 1 + g)
        expect += [l - 1 + g + t for t in range(1, k + 1)]
    assert list(pos) == expect
    # non-mask rows never see a mask key; every row sees itself
    assert np.all(A[np.ix_(~is_mask, is_mask)] == 0)
    assert np.all(np.diag(A) == 1)
    assert np.all(np.triu(A, 1) == 0)


def test_literal_reading_differs_from_k3():
    """The printed clause "i-j<k" leaks across groups from k = 3 on; the prose does not."""
    for k in (1, 2):
        _, im = so.extended_input([0], list(range(k)), k, -1)
        assert np.array_equal(so.sar_attention_mask(im, k, "group"), so.sar_attention_mask(im, k, "literal"))
    _, im = so.extended_input([0], [1, 2, 3], 3, -1)
    G, L = so.sar_attention_mask(im, 3, "group"), so.sar_attention_mask(im, 3, "literal")
    assert not np.array_equal(G, L)
    # rows: 0 x | 1 2 3 M | 4 c | 5 6 7 M ...: literal lets row 5 see mask 3 (5-3 = 2 < 3)
    assert L[5, 3] == 1 and G[5, 3] == 0
    assert np.all(L >= G)


# ---------------------------------------------------------------- numeric building blocks


def test_bf16_round_matches_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(4000) * 3, rng.standard_normal(1000) * 1e-3,
                        np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 0.0, 3.3895314e38 / 4])])
    ref = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(so.bf16_round(x), ref)
    # exact ties go to the even mantissa
    assert so.bf16_round(np.array([1.00390625]))[0] == 1.0
    assert so.bf16_round(np.array([1.01171875]))[0] == 1.015625


def test_widen_bits_matches_torch():
    torch = pytest.importorskip("torch")
    bits = np.arange(0, 0x7F80, 37, dtype=np.uint16)
    ref = torch.from_numpy(bits.astype(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(so.widen_bf16_bits(bits), ref)


def test_rmsnorm_invariants():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((5, 64))
    y = so.rmsnorm(x, np.ones(64), 0.0)
    assert np.allclose(np.mean(y * y, axis=-1), 1.0, atol=1e-12)
    w = rng.standard_normal(64)
    assert np.allclose(so.rmsnorm(3.7 * x, w, 0.0), so.rmsnorm(x, w, 0.0), atol=1e-12)
    # eps sits inside the root: a zero row maps to zero, and a tiny row is damped by sqrt(eps)
    assert np.all(so.rmsnorm(np.zeros((1, 8)), np.ones(8), 1e-5) == 0)
    t = np.full((1, 8), 1e-8)
    assert np.allclose(so.rmsnorm(t, np.ones(8), 1e-5), 1e-8 / np.sqrt(1e-16 + 1e-5))


def test_rope_properties():
    rng = np.random.default_rng(3)
    q = rng.standard_normal((6, 2, 64))
    k = rng.standard_normal((6, 2, 64))
    pos = np.array([0, 1, 5, 17, 300, 4095])
    rq = so.rope(q, pos, 10000.0)
    assert np.array_equal(rq[0], q[0])                      # position 0 is the identity
    assert np.allclose(np.linalg.norm(rq, axis=-1), np.linalg.norm(q, axis=-1))
    # scores depend on the position difference only
    a = so.rope(q[:1], np.array([40]), 1e4)[0, 0] @ so.rope(k[:1], np.array([33]), 1e4)[0, 0]
    b = so.rope(q[:1], np.array([1007]), 1e4)[0, 0] @ so.rope(k[:1], np.array([1000]), 1e4)[0, 0]
    assert abs(a - b) < 1e-9
    # pair (i, i + dh/2) rotates by pos * base^(-2i/dh): check one pair by hand
    x = np.zeros((1, 1, 64)); x[0, 0, 3] = 1.0
    y = so.rope(x, np.array([7]), 10000.0)[0, 0]
    ang = 7 * 10000.0 ** (-6 / 64)
    assert np.isclose(y[3], np.cos(ang)) and np.isclose(y[35], np.sin(ang))
    assert np.count_nonzero(np.abs(y) > 1e-15) == 2


def test_attention_all_non_mask_is_causal_sdpa():
    """With no mask tokens Eq. 3 is the causal mask: compare with torch's causal SDPA."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(4)
    R, H, dh = 9, 3, 16
    q, k, v = (rng.standard_normal((R, H, dh)) for _ in range(3))
    A = so.sar_attention_mask(np.zeros(R, dtype=bool))
    out = so._attention(q, k, v, A, 1.0 / np.sqrt(dh)).reshape(R, H, dh)
    tq, tk, tv = (torch.from_numpy(t).permute(1, 0, 2)[None] for t in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.allclose(out, ref, atol=1e-12)


# ---------------------------------------------------------------- forward vs a library decoder


def _hf_llama(shape, weights):
    torch = pytest.importorskip("torch")
    tr = pytest.importorskip("transformers")
    cfg = tr.LlamaConfig(
        vocab_size=shape.vocab + 1, hidden_size=shape.d_model, intermediate_size=shape.ffn,
        num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_heads,
        num_key_value_heads=shape.kv_heads, head_dim=shape.head_dim, rms_norm_eps=shape.rms_eps,
        rope_theta=shape.rope_base, attention_bias=False, mlp_bias=False, tie_word_embeddings=False,
        max_position_embeddings=8192, attn_implementation="eager")
    net = tr.LlamaForCausalLM(cfg).double().eval()
    W = lambda b: torch.from_numpy(so.widen_bf16_bits(b))
    sd = {"model.embed_tokens.weight": W(weights["embed"]), "model.norm.weight": W(weights["final_norm"])}
    lm = torch.zeros(shape.vocab + 1, shape.d_model, dtype=torch.float64)
    lm[: shape.vocab] = W(weights["lm_head"])
    sd["lm_head.weight"] = lm
    names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj",
             "wo": "self_attn.o_proj", "w_gate": "mlp.gate_proj", "w_up": "mlp.up_proj",
             "w_down": "mlp.down_proj", "attn_norm": "input_layernorm", "ffn_norm": "post_attention_layernorm"}
    for l, lw in enumerate(weights["layers"]):
        for k, n in names.items():
            sd[f"model.layers.{l}.{n}.weight"] = W(lw[k])
    missing, unexpected = net.load_state_dict(sd, strict=False)
    assert not [m for m in missing if "rotary" not in m] and not unexpected
    return net


def test_grouped_query_forward_matches_library_llama():
    """Grouped-query attention (the 70B member of the LLaMA-2 family the paper evaluates): the same
    comparison on a shape with 8 query heads over 2 key/value heads, plus the lossless invariant."""
    torch = pytest.importorskip("torch")
    from space_inputs import SHAPES, all_weights, prompt_tokens
    shape = SHAPES["gqa-small"]
    weights = all_weights(shape, seed=0)
    m = so.model_from_weights(shape, weights)
    assert m.kv_heads == 2 and weights["layers"][0]["wk"].shape == (2 * shape.head_dim, shape.d_model)
    net = _hf_llama(shape, weights)
    k = 3
    seq = [int(t) for t in prompt_tokens(shape, seed=3, n=9)[0]]
    toks, is_mask = so.extended_input(seq, [5, 6, 7], k, m.mask_id)
    A = so.sar_attention_mask(is_mask, k)
    pos = so.position_ids(A)
    mine = so.forward_dense(m, toks, A, pos)
    add = torch.zeros(A.shape, dtype=torch.float64)
    add[torch.from_numpy(A == 0)] = torch.finfo(torch.float64).min
    with torch.no_grad():
        ref = net(input_ids=torch.from_numpy(toks)[None], attention_mask=add[None, None],
                  position_ids=torch.from_numpy(pos)[None]).logits[0, :, : shape.vocab].numpy()
    assert np.abs(mine - ref).max() < 1e-6
    # cached form == dense form, and SPACE == plain greedy decoding
    out, _ = so.space_generate(m, seq, k=3, n_new=10, form="cached")
    assert out == so.ar_greedy(m, seq, 10)


def test_dense_forward_matches_library_llama(tiny_shape, tiny_weights, model, prompt):
    """The LLaMA decoder the paper builds on (Experimental Settings) is a library model:
    the oracle's forward under Eq. 3 masks and the paper's position ids must equal the
    transformers implementation fed the same 4-D mask and position ids."""
    torch = pytest.importorskip("torch")
    net = _hf_llama(tiny_shape, tiny_weights)
    k = 3
    seq = prompt[:10]
    toks, is_mask = so.extended_input(seq, [5, 6, 7], k, model.mask_id)
    A = so.sar_attention_mask(is_mask, k)
    pos = so.position_ids(A)
    mine = so.forward_dense(model, toks, A, pos)
    add = torch.zeros(A.shape, dtype=torch.float64)
    add[torch.from_numpy(A == 0)] = torch.finfo(torch.float64).min
    with torch.no_grad():
        ref = net(input_ids=torch.from_numpy(toks)[None], attention_mask=add[None, None],
                  position_ids=torch.from_numpy(pos)[None]).logits[0, :, : tiny_shape.vocab].numpy()
    # the library keeps its rotary cos/sin tables in float32, hence 1e-6 and not 1e-12;
    # any structural slip (pairing, eps placement, scale, mask) shows at 1e-3 or more
    assert np.abs(mine - ref).max() < 1e-6
    # and the plain causal forward
    with torch.no_grad():
        ref2 = net(input_ids=torch.tensor([seq])).logits[0, :, : tiny_shape.vocab].numpy()
    assert np.abs(so.causal_forward(model, seq) - ref2).max() < 1e-6


# ---------------------------------------------------------------- Algorithm 1


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_lossless_cached(model, prompt, ar_sequence, k):
    """Greedy SPACE equals plain greedy AR decoding token for token (the paper's lossless
    claim, end of the Auto-Correct Decoding section), tiny decoder, 32 new tokens."""
    seq, hist = so.space_generate(model, prompt, k, 32, form="cached")
    assert seq == ar_sequence[: 64 + 32]
    assert all(0 <= a <= k for a in hist)
    assert hist[0] == 0


@pytest.mark.parametrize("k", [2, 4])
def test_lossless_dense(model, prompt, ar_sequence, k):
    """Same through the definition-level form (full I, full A-bar, no cache)."""
    seq, _ = so.space_generate(model, prompt[:24], k, 10, form="dense")
    ref = so.ar_greedy(model, prompt[:24], 10)
    assert seq == ref


@pytest.mark.parametrize("k", [3, 4])
def test_forced_acceptance_lengths(model, prompt, ar_sequence, k):
    """accepted = longest prefix of the candidates equal to the greedy continuation; the extra
    token is the next greedy token; every acceptance length 0..k is forced by corrupting the
    true continuation at one place (Algorithm 1, verification loop)."""
    l = 64 + 5
    seq = ar_sequence[:l]
    truth = ar_sequence[l: l + k + 1]
    for j in range(k + 1):
        cands = list(truth[:k])
        if j < k:
            cands[j] = (cands[j] + 1) % model.vocab
        res = so.space_step_dense(model, seq, cands, k)
        assert res.accepted == j
        assert res.emitted == truth[: j + 1]
        # the new candidates are what the mask group behind the last accepted token predicts: mask t of
        # that group is, by Eq. 3, the last row of a plain causal forward over [x, c_1..c_j, M * t]
        expect = [int(np.argmax(so.causal_forward(model, seq + cands[:j] + [model.mask_id] * t)[-1]))
                  for t in range(1, k + 1)]
        assert res.new_cands == expect
        kv = so.OracleKV(model)
        so.prefill(model, kv, seq[:-1])
        res2, _, _, _ = so.space_step_cached(model, kv, seq[-1], cands, k)
        assert res2.accepted == j and res2.emitted == res.emitted and res2.new_cands == res.new_cands
        assert kv.length == l - 1 + j + 1


def test_first_iteration_rejects_dummies(model, prompt):
    """P_c = +inf on the first iteration: nothing is accepted even if a dummy equals the
    greedy token (Algorithm 1, line 1)."""
    truth = so.ar_greedy(model, prompt[:20], 3)[20:]
    res = so.space_step_dense(model, prompt[:20], truth[:3], 3, candidates_valid=False)
    assert res.accepted == 0 and res.emitted == [truth[0]]
    res = so.space_step_dense(model, prompt[:20], truth[:3], 3, candidates_valid=True)
    assert res.accepted == 3


def test_block_rows_reduce_to_causal_forwards(model, prompt):
    """Brute force: under the same-group reading, block row (g, t') must equal the last row of a
    plain causal forward over [x_1..x_l, c_1..c_g, M * t'] with positions 0..n-1."""
    k = 3
    seq = prompt[:12]
    cands = [3, 1, 4]
    toks, is_mask = so.extended_input(seq, cands, k, model.mask_id)
    A = so.sar_attention_mask(is_mask, k)
    P = so.forward_dense(model, toks, A, so.position_ids(A))
    l = len(seq)
    for g in range(k + 1):
        for t in range(k + 1):
            row = l - 1 + g * (k + 1) + t
            plain = list(seq) + cands[:g] + [model.mask_id] * t
            ref = so.causal_forward(model, plain)[-1]
            assert np.abs(P[row] - ref).max() < 1e-9, (g, t)
    # the literal reading breaks this from k = 3 on (first mask of group 1 sees a foreign mask)
    AL = so.sar_attention_mask(is_mask, k, "literal")
    PL = so.forward_dense(model, toks, AL, so.position_ids(AL))
    assert np.abs(PL - P).max() > 1e-6


def test_dense_equals_cached_and_cache_equals_prefill(model, prompt):
    """The cached form is the dense form: same logits, and after the commit the cache holds
    what a fresh prefill of the committed sequence produces."""
    k = 4
    seq = prompt[:20]
    truth = so.ar_greedy(model, seq, k)[20:]
    cands = truth[:2] + [(truth[2] + 1) % model.vocab, 17]
    dense = so.space_step_dense(model, seq, cands, k)
    kv = so.OracleKV(model)
    so.prefill(model, kv, seq[:-1])
    res, ks, vs, pos = so.space_step_cached(model, kv, seq[-1], cands, k)
    assert np.abs(res.logits - dense.logits).max() < 1e-9
    assert res.accepted == dense.accepted == 2
    committed = seq + cands[:2]
    fresh = so.OracleKV(model)
    so.prefill(model, fresh, committed)
    assert kv.length == fresh.length == len(committed)
    for l in range(model.n_layers):
        assert np.abs(kv.k[l] - fresh.k[l]).max() < 1e-9
        assert np.abs(kv.v[l] - fresh.v[l]).max() < 1e-9
    kv.truncate(2)
    assert kv.length == len(seq)


def test_mask_and_later_rows_do_not_influence_earlier_real_rows(model, prompt):
    """Changing a later candidate (or the mask embedding) leaves earlier non-mask rows bit-identical."""
    k = 3
    kv = so.OracleKV(model)
    so.prefill(model, kv, prompt[:15])
    a, _, _, _ = so.space_step_cached(model, kv, prompt[15], [1, 2, 3], k, commit=False)
    b, _, _, _ = so.space_step_cached(model, kv, prompt[15], [1, 2, 9], k, commit=False)
    rows_before_c3 = 3 * (k + 1)
    assert np.array_equal(a.logits[:rows_before_c3], b.logits[:rows_before_c3])
    assert not np.array_equal(a.logits[rows_before_c3], b.logits[rows_before_c3])
    saved = model.head()["embed"][model.mask_id].copy()
    try:
        model.head()["embed"][model.mask_id] = saved * -2.0
        c, _, _, _ = so.space_step_cached(model, kv, prompt[15], [1, 2, 3], k, commit=False)
    finally:
        model.head()["embed"][model.mask_id] = saved
    real = [g * (k + 1) for g in range(k + 1)]
    assert np.array_equal(a.logits[real], c.logits[real])
    assert not np.array_equal(a.logits[1], c.logits[1])


def test_first_step_short_block_is_equivalent(model, prompt):
    """The first iteration may run on [x_l, M^k] alone: group 0 and row 0 never see later groups."""
    k = 4
    kv = so.OracleKV(model)
    so.prefill(model, kv, prompt[:30])
    full, _, _, _ = so.space_step_cached(model, kv, prompt[30], [0] * k, k, candidates_valid=False, commit=False)
    toks = np.array([prompt[30]] + [model.mask_id] * k)
    im = np.array([False] + [True] * k)
    P, _, _, pos = so.block_forward_cached(model, kv, toks, im)
    assert np.abs(P - full.logits[: k + 1]).max() < 1e-12   # row count changes BLAS blocking only
    assert list(pos) == [30 + i for i in range(k + 1)]


@pytest.mark.parametrize("mode,bound", [("bf16_kv", 5e-3), ("bf16_points", 2e-2)])
def test_rounding_modes_are_close_and_round(tiny_shape, tiny_weights, prompt, mode, bound):
    """The bf16 precision modes only add roundings: logits stay close to the exact ones on the
    tiny decoder (the cache-only mode much closer than the all-operands mode), and staged K/V
    are bf16-representable."""
    exact = so.model_from_weights(tiny_shape, tiny_weights)
    rounded = so.model_from_weights(tiny_shape, tiny_weights, precision=mode)
    kv_e, kv_r = so.OracleKV(exact), so.OracleKV(rounded)
    so.prefill(exact, kv_e, prompt[:20])
    so.prefill(rounded, kv_r, prompt[:20])
    a, _, _, _ = so.space_step_cached(exact, kv_e, prompt[20], [1, 2, 3], 3, commit=False)
    b, ks, vs, _ = so.space_step_cached(rounded, kv_r, prompt[20], [1, 2, 3], 3, commit=False)
    assert 0 < np.abs(a.logits - b.logits).max() < bound
    assert np.array_equal(so.bf16_round(ks[0]), ks[0]) and np.array_equal(so.bf16_round(vs[1]), vs[1])


def test_unknown_precision_is_refused(tiny_shape, tiny_weights):
    with pytest.raises(ValueError):
        so.model_from_weights(tiny_shape, tiny_weights, precision="fp64")
    with pytest.raises(ValueError):
        so.model_from_weights(tiny_shape, tiny_weights, precision="bf16")


@pytest.mark.parametrize("shape_name", ["tiny", "gqa-small"])
def test_cache_rounding_mode_rounds_exactly_the_cached_quantities(shape_name):
    """What ``precision="bf16_kv"`` may change (readings: precision): the keys after the rotary
    embedding and the values, i.e. what a bf16 KV cache stores, and nothing else.  Layer by layer,
    the exact-mode layer is run on the inputs the rounding mode's layer saw (its x and its cache):
      * normalised rows and rotated queries are bit-equal to the exact mode's (not rounded);
      * stored k and v are the nearest-even bf16 roundings of the exact mode's rotated k and of v;
      * k was not rounded in front of the rotation (that gives other values), and q is not
        bf16-representable;
      * the attention output is what the exact mode computes from the unrounded q and the rounded k, v,
        and the rest of the layer (output projection, FFN) adds no rounding."""
    shape = SHAPES[shape_name]
    w = all_weights(shape, seed=3)
    exact = so.model_from_weights(shape, w, precision="exact")
    rounded = so.model_from_weights(shape, w, precision="bf16_kv")
    prompt = [int(t) for t in prompt_tokens(shape, seed=1, n=20)[0]]
    kv = so.OracleKV(rounded)
    so.prefill(rounded, kv, prompt[:-1])
    k = 3
    toks, is_mask = so.extended_input([prompt[-1]], [5, 6, 7], k, shape.mask_id)
    trace = []
    _, ks, vs, pos = so.block_forward_cached(rounded, kv, toks, is_mask, k, trace=trace)
    R, ctx = len(toks), kv.length
    vis = np.concatenate([np.ones((R, ctx), dtype=np.int64), so.sar_attention_mask(is_mask, k)], axis=1)
    x_in = exact.head()["embed"][toks]
    for l in range(shape.n_layers):
        wl = exact.layer(l)
        # the exact-mode layer on the same inputs, but WITHOUT the cache of this layer's own rows, so that
        # its k and v come back unrounded
        tr_e = {}
        _, k_e, v_e = so._layer_forward(exact, wl, x_in, pos, kv.k[l], kv.v[l], vis, tr_e)
        tr = trace[l]
        assert np.array_equal(tr["xn1"], tr_e["xn1"])
        assert np.array_equal(tr["q"], tr_e["q"])
        assert not np.array_equal(so.bf16_round(tr["q"]), tr["q"])
        assert np.array_equal(ks[l], so.bf16_round(k_e)) and np.array_equal(vs[l], so.bf16_round(v_e))
        assert not np.array_equal(ks[l], k_e) and not np.array_equal(vs[l], v_e)
        # rounding in front of the rotation is a different thing
        Hkv, dh = exact.kv_heads, shape.head_dim
        k_pre = (tr_e["xn1"] @ wl["wk"].T).reshape(R, Hkv, dh)
        assert not np.array_equal(ks[l], so.rope(so.bf16_round(k_pre), pos, shape.rope_base))
        # attention: unrounded q against [cache ; rounded k], [cache ; rounded v]
        o = so._attention(tr_e["q"], np.concatenate([kv.k[l], ks[l]], axis=0), np.concatenate([kv.v[l], vs[l]], axis=0),
                          vis, 1.0 / np.sqrt(dh))
        assert np.array_equal(tr["attn_out"], o)
        assert not np.array_equal(tr["attn_out"], tr_e["attn_out"])
        # the rest of the layer adds no rounding: exact arithmetic from this attention output
        x_mid = x_in + o @ wl["wo"].T
        n2 = so.rmsnorm(x_mid, wl["ffn_norm"], shape.rms_eps)
        assert np.array_equal(tr["xn2"], n2)
        x_out = x_mid + (so.silu(n2 @ wl["w_gate"].T) * (n2 @ wl["w_up"].T)) @ wl["w_down"].T
        assert np.array_equal(tr["x"], x_out)
        x_in = tr["x"]
    # every cached row of the prefill is bf16-representable as well
    assert all(np.array_equal(so.bf16_round(a), a) for a in kv.k + kv.v)


def test_eos_stop_truncates_in_front_of_the_token(model, prompt):
    """Algorithm 1 returns O[:eos_index]: with the EOS id set to a token the greedy continuation
    contains, the output is that continuation up to (not including) its first occurrence, whatever
    k is and wherever inside a step the token falls."""
    seq = prompt[:12]
    ref = so.ar_greedy(model, seq, 16)
    gen = ref[len(seq):]
    for pos in (0, 3, 7):
        eos = gen[pos]
        first = gen.index(eos)
        for k in (1, 3, 5):
            out, _ = so.space_generate(model, seq, k, 16, eos_id=eos)
            assert out == ref[: len(seq) + first], (pos, k)
    out, _ = so.space_generate(model, seq, 3, 16, eos_id=model.vocab + 5)   # never generated
    assert out == ref
