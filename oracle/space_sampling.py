"""CPU oracle for the rejection-sampling form of the SPACE verification (arxiv 2402.11809,
Algorithm 1 as printed, with the sampling settings of the appendix "Random Sampling":
top-k = 10, top-p = 0.95).

TEST INFRASTRUCTURE ONLY, like the rest of this package: only tests may import it, it imports
nothing of the product and shares no code with it.

Precision.  Every decision here is an integer (accept / reject, which token is drawn) taken
from floating point, so both sides have to take it in one precision.  The paper fixes none;
the implementation under test works in float32, hence this file does too: every quantity
below is numpy float32 and every sum runs in the stated order.  The random numbers the
method draws are *inputs* (one uniform per acceptance test, one for the extra token, one per
new candidate), so neither side needs a generator.

Readings of the paper taken here
  * "normalized output logits P" (text before Eq. 4): P[row] is the softmax of the row's logits
    after the warping below; Q in Algorithm 1 is one such row.
  * Warping: the appendix names top-p = 0.95 and top-k = 10 but not how they combine.  Taken:
    first the top_k largest logits (ties: lowest token id first), softmax over those, then the
    nucleus: the shortest prefix of that descending order whose mass reaches top_p,
    renormalised.  This is also what the common library warpers produce when chained in
    their default order (pinned against them in the tests).
  * Acceptance: "r <= Q(L_c[i]) / P_c[i]" is evaluated as printed, as a float32 quotient.
    P_c = +inf (first iteration) gives quotient 0, so a dummy is rejected unless r = 0.
  * Extra token: Algorithm 1 prints "a ~ Q", the plain distribution of the last accepted row,
    also after a rejection.  The speculative-sampling papers it cites draw from
    norm(max(0, Q - P)) after a rejection, which is what makes the output distribution equal
    Q exactly.  ``extra="printed"`` (default) follows Algorithm 1; ``extra="residual"``
    implements the cited rule and needs the full draft distribution of the rejected slot.
  * Drawing from a distribution: inverse CDF over the kept tokens in descending order of
    probability, i.e. the first token whose running sum exceeds the uniform; the last kept
    token if rounding leaves the sum short.

Pins live in tests/test_oracle_sampling.py.  Unpinned: acceptance *rates* (they need the
fine-tuned weights): "parity unpinned".
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

F32 = np.float32


def warp(logits_row: np.ndarray, top_k: int, top_p: float) -> Tuple[np.ndarray, np.ndarray]:
    """Kept token ids (descending probability, ties by lowest id) and their probabilities
    (float32, summing to one up to rounding) of one row after top-k and top-p warping."""
    x = np.asarray(logits_row, dtype=F32)
    V = x.shape[0]
    kk = max(1, min(int(top_k), V))
    # the kk largest, lowest id first among equals: stable sort of the negated values
    order = np.argsort(-x, kind="stable")[:kk]
    top = x[order]
    e = np.exp((top - top[0]).astype(F32)).astype(F32)
    total = F32(0.0)
    for v in e:                      # sequential float32 sum in descending order
        total = F32(total + v)
    p = (e / total).astype(F32)
    keep = kk
    run = F32(0.0)
    for j in range(kk):              # shortest prefix whose mass reaches top_p
        run = F32(run + p[j])
        if run >= F32(top_p):
            keep = j + 1
            break
    kept = p[:keep]
    mass = F32(0.0)
    for v in kept:
        mass = F32(mass + v)
    return order[:keep].astype(np.int64), (kept / mass).astype(F32)


def prob_of(ids: np.ndarray, probs: np.ndarray, token: int) -> np.float32:
    hit = np.nonzero(ids == int(token))[0]
    return F32(probs[hit[0]]) if hit.size else F32(0.0)


def draw(ids: np.ndarray, probs: np.ndarray, u: float) -> Tuple[int, np.float32]:
    """Inverse CDF: first kept token whose running float32 sum exceeds u."""
    run = F32(0.0)
    for j in range(len(ids)):
        run = F32(run + probs[j])
        if F32(u) < run:
            return int(ids[j]), F32(probs[j])
    return int(ids[-1]), F32(probs[-1])


def residual(q_ids, q_probs, p_ids, p_probs) -> Tuple[np.ndarray, np.ndarray]:
    """norm(max(0, Q - P)) over the tokens Q keeps, in Q's order (speculative sampling)."""
    r = np.array([max(F32(0.0), F32(q_probs[j] - prob_of(p_ids, p_probs, int(q_ids[j])))) for j in range(len(q_ids))],
                 dtype=F32)
    s = F32(0.0)
    for v in r:
        s = F32(s + v)
    if s <= 0:
        return q_ids, q_probs
    return q_ids, (r / s).astype(F32)


@dataclass
class SampleStepResult:
    accepted: int                 # i*
    emitted: List[int]            # accepted candidates + the extra token
    new_cands: List[int]          # L_c of the next step
    new_pc: List[np.float32]      # P_c of the next step
    ratios: List[np.float32]      # Q(L_c[i]) / P_c[i] of every test that was made
    new_dists: List[Tuple[np.ndarray, np.ndarray]]  # (ids, probs) each new candidate was drawn from


def verify_sampling(P_blk: np.ndarray, k: int, cands: Sequence[int], p_c: Sequence[float], uniforms: Sequence[float],
                    top_k: int = 10, top_p: float = 0.95, extra: str = "printed",
                    draft_dists: Optional[Sequence[Tuple[np.ndarray, np.ndarray]]] = None) -> SampleStepResult:
    """Lines 6-22 of Algorithm 1 on the logits of the block rows (row 0 = the paper's P[l]).

    uniforms: 2k+1 numbers in [0, 1): r of the i-th acceptance test at [i-1], the extra
    token's at [k], the j-th new candidate's at [k+1+j].  ``draft_dists[i-1]`` (ids, probs)
    is the distribution c_i was drawn from, needed by extra="residual" only."""
    assert len(uniforms) == 2 * k + 1 and len(cands) == k and len(p_c) == k
    idx = 1
    q_ids, q_probs = warp(P_blk[0], top_k, top_p)
    emitted: List[int] = []
    ratios: List[np.float32] = []
    acc = 0
    rejected_slot = None
    for i in range(1, k + 1):
        r = F32(uniforms[i - 1])
        with np.errstate(divide="ignore", invalid="ignore"):
            ratio = F32(prob_of(q_ids, q_probs, cands[i - 1]) / F32(p_c[i - 1]))
        ratios.append(ratio)
        if r <= ratio:
            emitted.append(int(cands[i - 1]))
            idx += k + 1
            q_ids, q_probs = warp(P_blk[i * (k + 1)], top_k, top_p)
            acc += 1
        else:
            rejected_slot = i
            break
    if extra == "residual" and rejected_slot is not None and draft_dists is not None:
        d_ids, d_probs = draft_dists[rejected_slot - 1]
        x_ids, x_probs = residual(q_ids, q_probs, d_ids, d_probs)
    else:
        x_ids, x_probs = q_ids, q_probs
    a, _ = draw(x_ids, x_probs, uniforms[k])
    emitted.append(a)
    new_cands: List[int] = []
    new_pc: List[np.float32] = []
    new_dists: List[Tuple[np.ndarray, np.ndarray]] = []
    for j in range(k):
        ids, probs = warp(P_blk[idx + j], top_k, top_p)
        t, pt = draw(ids, probs, uniforms[k + 1 + j])
        new_cands.append(t)
        new_pc.append(pt)
        new_dists.append((ids, probs))
    return SampleStepResult(acc, emitted, new_cands, new_pc, ratios, new_dists)


def space_generate_sampling(m, prompt: Sequence[int], k: int, n_new: int, uniforms: np.ndarray, top_k: int = 10,
                            top_p: float = 0.95, extra: str = "printed", trace: Optional[list] = None,
                            eos_id: Optional[int] = None):
    """Algorithm 1 in the sampling setting with a KV cache of x_1..x_{l-1}: uniforms[step] holds the
    2k+1 numbers of that iteration.  Starts from L_c = [0]*k, P_c = [+inf]*k as printed.  Stops once
    n_new tokens are out (overshoot truncated), or, with an eos_id, in front of the first such token
    among the emitted ones (the end-of-sequence check of Algorithm 1).  Returns (sequence, accepted
    counts).  ``trace`` collects (logits, candidates, P_c, uniforms) of every iteration for the tests."""
    from . import space_oracle as so
    seq = [int(t) for t in prompt]
    target = len(seq) + n_new
    kv = so.OracleKV(m)
    if len(seq) > 1:
        so.prefill(m, kv, seq[:-1])
    cands: List[int] = [0] * k
    p_c: List[float] = [np.inf] * k
    drafts = None
    hist: List[int] = []
    step = 0
    while len(seq) < target:
        toks, is_mask = so.extended_input([seq[-1]], cands, k, m.mask_id)
        P, ks, vs, _ = so.block_forward_cached(m, kv, toks, is_mask, k)
        P32 = P.astype(F32)
        if trace is not None:
            trace.append((P32, list(cands), list(p_c), np.array(uniforms[step], dtype=F32)))
        res = verify_sampling(P32, k, cands, p_c, uniforms[step], top_k=top_k, top_p=top_p, extra=extra,
                              draft_dists=drafts)
        kv.append(ks, vs, [g * (k + 1) for g in range(res.accepted + 1)])
        hist.append(res.accepted)
        if eos_id is not None and eos_id in res.emitted:
            seq.extend(res.emitted[: res.emitted.index(eos_id)])
            return seq[:target], hist
        seq.extend(res.emitted)
        cands, p_c, drafts = res.new_cands, [float(x) for x in res.new_pc], res.new_dists
        step += 1
    return seq[:target], hist
