"""Pins of the SAR-SFT oracle (oracle/space_sft.py) against what the paper and the mathematics fix.
No GPU."""
import math
import os

import numpy as np
import pytest

from oracle import space_oracle as so
from oracle import space_sft as sf
from space_inputs import SHAPES, all_weights, prompt_tokens

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "sar_sft_k2_n5.txt")


def _golden():
    rows = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        pos, kind, w, label, _ = line.split()
        rows.append((int(pos), kind, [float(v) for v in w.split(",")], int(label)))
    return rows


def test_worked_example():
    """Transform and loss of the hand-worked case (second and third equation of the section)."""
    rows = _golden()
    s = sf.sar_transform([7], [1, 2, 3, 0, 2], k=2, mask_id=4, p_ar=0.3, u_keep=0.9, u_pos=0.7)
    assert s.m == 3                                      # 1 + floor(0.7 * (5 - 2))
    assert s.input_ids == [7, 1, 2, 4, 4] and s.labels == [7, 1, 2, 3, 0, 2]
    assert ["M" if t == 4 else "t" for t in s.input_ids[1:]] == ["M" if k == "M" else "t" for _, k, _, _ in rows[1:]]
    logits = np.log(np.array([w for _, _, w, _ in rows]))
    assert [s.labels[p + 1] for p, _, _, _ in rows] == [lab for _, _, _, lab in rows]
    want = math.log(4.0 * (8 / 3) * (8 / 5) * (10 / 6) * (10 / 4))
    assert abs(sf.loss_sar(logits, s) - want) < 1e-12 and abs(want - 4.264243) < 1e-6
    terms = sf.next_token_terms(logits, s)
    assert np.allclose(terms, [math.log(4), math.log(8 / 3), math.log(8 / 5), math.log(10 / 6), math.log(10 / 4)])
    # a constant added to a row of logits changes nothing (probabilities are normalised per row)
    assert abs(sf.loss_sar(logits + np.arange(5)[:, None], s) - want) < 1e-12


@pytest.mark.parametrize("k", [1, 2, 5])
def test_transform_structure(k):
    """The input keeps m - 1 answer tokens and k masks, the labels are the untouched original tokens
    through y_{m+k}; every m of {1..N-k} is reachable and nothing outside; p_ar decides by u_keep."""
    rng = np.random.default_rng(k)
    x = [int(t) for t in rng.integers(0, 50, size=4)]
    y = [int(t) for t in rng.integers(0, 50, size=12)]
    n, seen = len(y), set()
    for u in np.linspace(0.0, 0.999999, 400):
        s = sf.sar_transform(x, y, k, mask_id=99, p_ar=0.5, u_keep=0.5, u_pos=float(u))
        assert 1 <= s.m <= n - k
        seen.add(s.m)
        assert s.input_ids == x + y[: s.m - 1] + [99] * k
        assert s.labels == x + y[: s.m + k] and 99 not in s.labels
        assert len(s.labels) == len(s.input_ids) + 1
    assert seen == set(range(1, n - k + 1))
    keep = sf.sar_transform(x, y, k, 99, p_ar=0.5, u_keep=0.49, u_pos=0.3)
    assert keep.m is None and keep.input_ids == keep.labels == x + y
    assert sf.sar_transform(x, y, k, 99, p_ar=1.0, u_keep=0.999999, u_pos=0.3).m is None     # p_ar = 1: always untouched
    assert sf.sar_transform(x, y, k, 99, p_ar=0.0, u_keep=0.0, u_pos=0.3).m is not None
    with pytest.raises(ValueError):
        sf.sar_transform(x, y[:k], k, 99, 0.0, 0.5, 0.5)


def test_losses_against_the_library_cross_entropy():
    """L_AR is the summed next-token cross entropy over the answer tokens (first equation): the library's
    cross_entropy on the same logits.  L_SAR's first sum is L_AR of the prefix y_1..y_{m-1}; its second sum
    has exactly k + 1 terms."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(3)
    V, k = 17, 3
    x = [int(t) for t in rng.integers(0, V, size=5)]
    y = [int(t) for t in rng.integers(0, V, size=9)]
    s = sf.sar_transform(x, y, k, V, p_ar=1.0, u_keep=0.2, u_pos=0.0)
    logits = rng.standard_normal((len(s.input_ids), V)) * 3
    ce = torch.nn.functional.cross_entropy(torch.from_numpy(logits[len(x) - 1: -1]), torch.tensor(y), reduction="sum")
    assert abs(sf.loss_ar(logits, s) - float(ce)) < 1e-10
    t = sf.sar_transform(x, y, k, V, p_ar=0.0, u_keep=0.2, u_pos=0.55)
    lg = rng.standard_normal((len(t.input_ids), V)) * 3
    terms = sf.next_token_terms(lg, t)
    assert len(terms) == (t.m - 1) + (k + 1)
    prefix = sf.SftSample(x + y[: t.m - 1], x + y[: t.m - 1], len(x), None, k)
    assert abs(terms[: t.m - 1].sum() - sf.loss_ar(lg[: len(prefix.input_ids)], prefix)) < 1e-12
    ce2 = torch.nn.functional.cross_entropy(torch.from_numpy(lg[len(x) - 1:]), torch.tensor(y[: t.m + k]), reduction="sum")
    assert abs(sf.loss_sar(lg, t) - float(ce2)) < 1e-10
    # the tail alone, from the rows of the last real token and the masks
    tail = sf.sar_tail_terms(lg[len(x) + t.m - 2:], y[t.m - 1: t.m + k])
    assert np.allclose(tail, terms[t.m - 1:], rtol=0, atol=1e-12)


def test_sar_loss_on_a_model_matches_the_decoding_block(tiny_shape, tiny_weights):
    """The second sum of L_SAR uses the very predictions the decoding step makes: a causal forward over
    X ++ y_<m ++ M^k (training view) and the cached one-group block [y_{m-1}, M^k] (inference view,
    Algorithm 1's first iteration) give the same k + 1 rows of logits, hence the same loss terms."""
    om = so.model_from_weights(tiny_shape, tiny_weights)
    k = 4
    toks = [int(t) for t in prompt_tokens(tiny_shape, seed=5, n=30)[0]]
    x, y = toks[:12], toks[12:]
    s = sf.sar_transform(x, y, k, tiny_shape.mask_id, p_ar=0.0, u_keep=0.5, u_pos=0.4)
    logits = so.causal_forward(om, s.input_ids)
    full = sf.next_token_terms(logits, s)
    kv = so.OracleKV(om)
    so.prefill(om, kv, s.input_ids[: len(x) + s.m - 2])
    blk, _ = so.extended_input([s.input_ids[len(x) + s.m - 2]], [], 0, tiny_shape.mask_id)
    blk = np.concatenate([blk, np.full(k, tiny_shape.mask_id)])
    P, _, _, _ = so.block_forward_cached(om, kv, blk, np.array([False] + [True] * k))
    tail = sf.sar_tail_terms(P, y[s.m - 1: s.m + k])
    assert np.abs(tail - full[s.m - 1:]).max() < 1e-9
    assert abs(sf.loss_sar(logits, s) - (full[: s.m - 1].sum() + tail.sum())) < 1e-9
