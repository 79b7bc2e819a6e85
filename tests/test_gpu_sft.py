"""GPU parity of the SAR-SFT loss reduction (space_sar_loss; Methods, "Semi-Autoregressive Finetuning")
against oracle/space_sft.py, through the C ABI."""
import numpy as np
import pytest

from oracle import space_oracle as so
from oracle import space_sft as sf
from space_inputs import SHAPES, all_weights, prompt_tokens
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("V,rows", [(32000, 36), (1000, 7), (40001, 96)])
def test_loss_terms_on_given_logits(V, rows):
    """-log softmax(row)[label] per row and their sum, float32 on the device against float64: every term
    within 2e-5 (the logits are a few units wide), rows with a negative label left out, same bits twice."""
    torch = gc.require_gpu()
    import dataclasses
    from paper_2402_11809_amd import binding
    shape = dataclasses.replace(SHAPES["tiny"], vocab=V, n_layers=1)
    gm = gc.make_gpu_model(shape, all_weights(shape, seed=0), max_batch=1, max_rows=96)
    rng = np.random.default_rng(V)
    logits = (rng.standard_normal((rows, V)) * 3.0).astype(np.float32)
    labels = rng.integers(0, V, size=rows).astype(np.int32)
    labels[rng.integers(0, rows, size=max(1, rows // 5))] = -1
    labels[0] = int(np.argmax(logits[0]))          # a likely token and an unlikely one
    labels[1] = int(np.argmin(logits[1]))
    lg, lb = torch.from_numpy(logits).cuda(), torch.from_numpy(labels).cuda()
    row_loss = torch.empty(rows, dtype=torch.float32, device="cuda")
    loss, n = gm.sar_loss(lg, lb, row_loss)
    loss2, _ = gm.sar_loss(lg, lb)                  # terms kept inside the library
    torch.cuda.synchronize()
    lp = sf.log_softmax_rows(logits)
    want = np.array([-lp[r, labels[r]] if labels[r] >= 0 else 0.0 for r in range(rows)])
    got = row_loss.cpu().numpy().astype(np.float64)
    assert np.abs(got - want).max() < 2e-5
    assert int(n.cpu()[0]) == int((labels >= 0).sum())
    assert abs(float(loss.cpu()[0]) - want.sum()) < 2e-5 * rows
    assert loss.cpu().numpy().tobytes() == loss2.cpu().numpy().tobytes()
    assert gm.device_faults() == 0


@pytest.mark.parametrize("shape_name,k", [("tiny", 4), ("small128", 5), ("gqa-small", 3)])
def test_sar_loss_of_a_sample_matches_oracle(shape_name, k):
    """One transformed sample end to end: the product's dataloader transform, one space_step over the block
    [last prompt token, y_1 .. y_{m-1}, M^k] (every real token a group of its own, the masks behind the last
    one: under Eq. 3 that is the causal training view), space_sar_loss over its logits with the labels
    y_1 .. y_{m+k}; against L_SAR of the oracle's own causal forward over the transformed input."""
    torch = gc.require_gpu()
    from paper_2402_11809_amd import binding, layout as lo
    from paper_2402_11809_amd.runtime import SpaceDecoder
    shape = SHAPES[shape_name]
    w = all_weights(shape, seed=1)
    gm = gc.make_gpu_model(shape, w, max_batch=1, max_rows=64)
    om = gc.oracle_model(shape, w, precision="exact")
    toks = [int(t) for t in prompt_tokens(shape, seed=9, n=44)[0]]
    n_prompt = 20
    for u_pos in (0.0, 0.37, 0.97):
        ids, labels, m = binding.sar_transform(toks, n_prompt, k, shape.mask_id, 0.0, 0.5, u_pos)
        ref = sf.sar_transform(toks[:n_prompt], toks[n_prompt:], k, shape.mask_id, 0.0, 0.5, u_pos)
        assert ids == ref.input_ids and labels == ref.labels and m == ref.m
        dec = SpaceDecoder(gm, k, capacity=128, prefill_chunk=32)
        dec.prefill(np.asarray([ids[: n_prompt - 1]], dtype=np.int32))
        block = ids[n_prompt - 1:]                          # x_P, y_1 .. y_{m-1}, M x k
        spec = lo.BlockLayoutSpec(np.array([0] * m + [1] * k, dtype=np.uint8),
                                  np.array(list(range(m)) + [m - 1] * k, dtype=np.int32))
        out = binding.StepOut(gm, 1, spec.n_rows, k)
        gm.step(torch.tensor([block], dtype=torch.int32, device="cuda"), gm.layout(spec), dec.kv, out)
        lab = torch.tensor(labels[n_prompt:], dtype=torch.int32, device="cuda")
        assert lab.numel() == spec.n_rows == (m - 1) + (k + 1)
        row_loss = torch.empty(spec.n_rows, dtype=torch.float32, device="cuda")
        loss, n = gm.sar_loss(out.logits[0], lab, row_loss)
        torch.cuda.synchronize()
        o_logits = so.causal_forward(om, ids)
        terms = sf.next_token_terms(o_logits, ref)
        got = row_loss.cpu().numpy().astype(np.float64)
        # logits agree to 2e-3 (bf16 cache against the exact oracle): a term moves by at most twice that
        assert np.abs(got - terms).max() < 2 * gc.LOGIT_TIGHT, (u_pos, np.abs(got - terms).max())
        assert int(n.cpu()[0]) == len(terms)
        assert abs(float(loss.cpu()[0]) - sf.loss_sar(o_logits, ref)) < 2 * gc.LOGIT_TIGHT * len(terms)
        assert gm.device_faults() == 0
