"""CPU oracle for the training half of SPACE (arxiv 2402.11809, Methods, "Semi-Autoregressive
Finetuning"): the dataloader transform and the two losses L_AR and L_SAR.

TEST INFRASTRUCTURE ONLY, like the rest of this package: only tests may import it, it imports
nothing of the product and shares no code with it.  Plain numpy float64, one log-softmax per row.

Notation (1-based, as in the paper): prompt X, answer Y = {y_1..y_N}, k mask tokens [M].
  * L_AR  = - sum_{t=1..N} log P(y_t | y_<t, X)                                   (first loss equation)
  * transform: with probability p_ar the sample stays as it is; otherwise a position m is drawn, the
    input becomes X ++ {y_1..y_{m-1}, [M] x k} (second equation: y^k_<m) and the labels stay the
    original tokens, cut behind y_{m+k}
  * L_SAR = - sum_{t=1..m-1} log P(y_t | y_<t, X) - sum_{t=m..m+k} log P(y_t | y^k_<m, X)
                                                                                  (third equation)
All probabilities of one sample come from ONE causal forward over its input: the token in front of
y_t predicts y_t (t <= m: a real token; the last real token y_{m-1} -- the last prompt token when
m = 1 -- predicts y_m), and the j-th mask token predicts y_{m+j}, j = 1..k.  That is k + 1 terms in
the second sum, the same k + 1 predictions one row group of the decoding step makes (the extra
token and k candidates).

Readings of the paper taken here
  * Range of m.  The text draws m from {0, 1, .., N-k}; the equations index y from 1 and need
    y_{m+k} to exist and y_{m-1} (or the prompt) to stand in front of the masks.  Taken: m is drawn
    uniformly from {1, .., N-k}, the positions for which all k + 1 labels of the second sum exist
    (the printed set read 1-based, without the value 0 that has no token y_0 to predict).  Needs
    N > k.
  * "Truncate the input and label sequences to keep the first m + k tokens" (appendix, training
    details): the input keeps m - 1 real answer tokens and k masks; the labels are kept through
    y_{m+k}, the last token the second sum asks for.
  * The random numbers (keep or transform; which m) are inputs, so neither side needs a generator:
    keep iff u_keep < p_ar; m = 1 + floor(u_pos * (N - k)).
  * Sums, not means, as printed.

Pins live in tests/test_oracle_sft.py.  Unpinned: anything about what training with this loss
does to a model (needs the datasets and checkpoints): "parity unpinned".
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np


@dataclass
class SftSample:
    input_ids: List[int]      # X ++ answer part (real tokens, then k mask ids when transformed)
    labels: List[int]         # X ++ the original answer tokens the losses refer to (never a mask id)
    n_prompt: int
    m: Optional[int]          # None: untouched sample (L_AR); else the drawn position, 1-based
    k: int


def sar_transform(x: Sequence[int], y: Sequence[int], k: int, mask_id: int, p_ar: float, u_keep: float,
                  u_pos: float) -> SftSample:
    """The modified dataloader: one sample in, one sample out."""
    x, y = [int(t) for t in x], [int(t) for t in y]
    n = len(y)
    if u_keep < p_ar:
        return SftSample(x + y, x + y, len(x), None, k)
    if n <= k:
        raise ValueError(f"answer of {n} tokens is too short for k = {k}")
    m = 1 + int(np.floor(u_pos * (n - k)))
    m = min(max(m, 1), n - k)
    return SftSample(x + y[: m - 1] + [mask_id] * k, x + y[: m + k], len(x), m, k)


def log_softmax_rows(logits: np.ndarray) -> np.ndarray:
    z = np.asarray(logits, dtype=np.float64)
    z = z - z.max(axis=-1, keepdims=True)
    return z - np.log(np.exp(z).sum(axis=-1, keepdims=True))


def next_token_terms(logits: np.ndarray, sample: SftSample) -> np.ndarray:
    """-log P of every answer token of the sample's labels, in order: entry t-1 belongs to y_t.  Row i
    of `logits` ([len(input_ids), vocab], one causal forward over input_ids) predicts label i + 1."""
    lp = log_softmax_rows(logits)
    p, n_lab = sample.n_prompt, len(sample.labels)
    if p < 1:
        raise ValueError("an empty prompt leaves nothing in front of y_1")
    assert lp.shape[0] == len(sample.input_ids) and n_lab - 1 <= lp.shape[0]
    return np.array([-lp[i - 1, sample.labels[i]] for i in range(p, n_lab)])


def loss_ar(logits: np.ndarray, sample: SftSample) -> float:
    """L_AR of an untouched sample."""
    assert sample.m is None
    return float(next_token_terms(logits, sample).sum())


def loss_sar(logits: np.ndarray, sample: SftSample) -> float:
    """L_SAR of a transformed sample: m - 1 autoregressive terms and k + 1 terms read off the last
    real token and the k mask tokens."""
    assert sample.m is not None
    terms = next_token_terms(logits, sample)
    assert len(terms) == (sample.m - 1) + (sample.k + 1)
    return float(terms[: sample.m - 1].sum() + terms[sample.m - 1:].sum())


def sar_tail_terms(block_logits: np.ndarray, labels: Sequence[int]) -> np.ndarray:
    """The second sum of L_SAR from the logits of the k + 1 rows [y_{m-1}, M^k] alone (the one-group block
    of the decoding step): row j predicts labels[j] = y_{m+j}, j = 0..k."""
    lp = log_softmax_rows(block_logits)
    assert lp.shape[0] == len(labels)
    return np.array([-lp[j, int(t)] for j, t in enumerate(labels)])
