"""CPU oracle for the SPACE auto-correct decoding step (arxiv 2402.11809).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP path is checked
against.  Only tests, the smoke check and the CPU-baseline leg of the benchmark may import
it; the product never does, and it imports nothing of the product.  It shares no code with
the HIP path (only the seeded input generators in ``space_inputs`` feed both).

Everything is numpy float64 with one library primitive (matrix product) per step and no
blocking, fusion or reordering beyond what the paper's equations state.

What follows the paper directly
  * extended input I = {x_1..x_l, M^k, c_1, M^k, ..., c_k, M^k}        (Methods, Eq. 2)
  * attention mask A-bar                                                (Methods, Eq. 3)
  * position ids = row sums of A-bar minus one                          (text after Eq. 3)
  * the decoding loop, verification and candidate refresh               (Algorithm 1)
What the paper leaves to the model family (LLaMA, Experimental Settings) and is fixed here
  * pre-norm decoder, RMSNorm (eps inside the root), rotary embedding with half-split
    pairing and base 10000, SwiGLU FFN, softmax scale 1/sqrt(head_dim), no biases,
    untied embedding / LM head; optionally grouped-query attention (the 70B member of the
    family: n_kv_heads key/value heads, query head h reads head h // (n_heads / n_kv_heads)).

Readings of the paper taken here (each also listed in the design notes of the repo)
  * Eq. 3, second clause: the printed condition "i-j<k" would let the first masks of one
    group see the last masks of the previous group once k >= 3; the prose (Algorithm
    description and the appendix on the attention mask) says masks see only masks of their
    own group.  ``reading="group"`` (default) follows the prose; ``reading="literal"``
    evaluates the printed condition so that tests can show where the two part.
  * Greedy verification: Algorithm 1 is printed for sampling; the greedy limit accepts c_i
    iff it equals argmax of the current Q, and "sample a ~ Q" becomes argmax Q.  Ties take
    the lowest token id.
  * Algorithm 1 starts with L_c = [0]*k and P_c = +inf, i.e. the dummies of the first
    iteration are always rejected; ``candidates_valid=False`` encodes P_c = +inf.
  * The paper never mentions a KV cache.  The cached form keeps K/V of x_1..x_{l-1}; the
    step block is x_l followed by the k(k+2) extension tokens, (k+1)^2 rows.
  * Precision is not stated in the paper.  ``precision="exact"`` is float64 throughout.
    ``precision="bf16_kv"`` additionally rounds (nearest-even) the cached quantities, k after
    rotary and v, to bfloat16: a bf16 KV cache is a storage format of the implementation
    under test, and an argmax can only be compared when both sides hold the same cache.
    ``precision="bf16_points"`` rounds, on top of that, every activation that a plain bf16
    pipeline would feed to a matrix unit (normalised rows entering each projection, q after
    rotary, attention output, SwiGLU product); kept to show how far such a pipeline drifts.

Parity pins live in tests/test_oracle_*.py.  Unpinned: the numeric values of mask-row
logits beyond the per-row causal reduction (the paper prints no worked numeric example)
-- "parity unpinned" for acceptance *rates*, which need the fine-tuned weights.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np

# --------------------------------------------------------------------------------------
# number formats
# --------------------------------------------------------------------------------------


def bf16_round(x: np.ndarray) -> np.ndarray:
    """float64 -> float32 -> bfloat16 (round to nearest even) -> float64."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = ((u + 0x7FFF + lsb) >> 16) << 16
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(x))


def widen_bf16_bits(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 storage -> float64, exactly."""
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    return u.view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------------------
# model
# --------------------------------------------------------------------------------------


@dataclass
class OracleModel:
    """LLaMA-shaped decoder with weights widened to float64 on demand.

    ``layer_bits(l)`` returns the bf16 bit patterns of layer l (dict with wq wk wv wo
    w_gate w_up w_down attn_norm ffn_norm, matrices [out, in]); ``head_bits`` holds embed
    ([vocab+1, d], last row is the mask token), final_norm, lm_head.
    """

    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rms_eps: float
    rope_base: float
    head_bits: Dict[str, np.ndarray]
    layer_bits: Callable[[int], Dict[str, np.ndarray]]
    precision: str = "exact"  # or "bf16_kv", "bf16_points"
    cache_layers: bool = True
    n_kv_heads: int = 0  # 0: as many key/value heads as query heads; else query head h uses head h // (H / n_kv_heads)
    _layers: Dict[int, Dict[str, np.ndarray]] = field(default_factory=dict)
    _head: Optional[Dict[str, np.ndarray]] = None

    @property
    def mask_id(self) -> int:
        return self.vocab

    @property
    def kv_heads(self) -> int:
        return self.n_kv_heads if self.n_kv_heads > 0 else self.n_heads

    def __post_init__(self) -> None:
        if self.precision not in ("exact", "bf16_kv", "bf16_points"):
            raise ValueError(f"unknown precision {self.precision!r}")

    def rnd(self, x: np.ndarray) -> np.ndarray:
        """Rounding of an activation operand."""
        return bf16_round(x) if self.precision == "bf16_points" else x

    def rnd_kv(self, x: np.ndarray) -> np.ndarray:
        """Rounding of a value that is stored in the KV cache."""
        return bf16_round(x) if self.precision in ("bf16_kv", "bf16_points") else x

    def head(self) -> Dict[str, np.ndarray]:
        if self._head is None:
            self._head = {k: widen_bf16_bits(v) for k, v in self.head_bits.items()}
        return self._head

    def layer(self, l: int) -> Dict[str, np.ndarray]:
        if l in self._layers:
            return self._layers[l]
        w = {k: widen_bf16_bits(v) for k, v in self.layer_bits(l).items()}
        if self.cache_layers:
            self._layers[l] = w
        return w


PRECISIONS = ("exact", "bf16_kv", "bf16_points")


def model_from_weights(shape, weights: Dict[str, object], precision: str = "exact") -> OracleModel:
    if precision not in PRECISIONS:
        raise ValueError(f"unknown precision {precision!r}: one of {PRECISIONS}")
    layers = weights["layers"]
    head = {k: weights[k] for k in ("embed", "final_norm", "lm_head")}
    return OracleModel(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.ffn,
                       shape.vocab, shape.rms_eps, shape.rope_base, head,
                       lambda l: layers[l], precision, n_kv_heads=getattr(shape, "n_kv_heads", 0))


def rmsnorm(x: np.ndarray, w: np.ndarray, eps: float) -> np.ndarray:
    """x * w / sqrt(mean(x^2) + eps), row-wise."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x * w / np.sqrt(ms + eps)


def rope(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary embedding, half-split pairing: element i is paired with i + dh/2 and rotated by
    the angle pos * base^(-2i/dh).  x is [rows, heads, dh], pos is [rows]."""
    dh = x.shape[-1]
    half = dh // 2
    inv_freq = base ** (-2.0 * np.arange(half, dtype=np.float64) / dh)
    ang = pos.astype(np.float64)[:, None] * inv_freq[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def softmax_rows(s: np.ndarray) -> np.ndarray:
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


# --------------------------------------------------------------------------------------
# Eq. 2, Eq. 3, position ids
# --------------------------------------------------------------------------------------


def extended_input(x: Sequence[int], cands: Sequence[int], k: int, mask_id: int) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 2: I = {x_1..x_l, M^k, c_1, M^k, ..., c_k, M^k}.  Returns (tokens, is_mask)."""
    assert len(cands) == k
    toks: List[int] = list(x)
    is_mask: List[bool] = [False] * len(toks)
    toks += [mask_id] * k
    is_mask += [True] * k
    for c in cands:
        toks.append(int(c))
        is_mask.append(False)
        toks += [mask_id] * k
        is_mask += [True] * k
    return np.asarray(toks, dtype=np.int64), np.asarray(is_mask, dtype=bool)


def mask_group_ids(is_mask: np.ndarray) -> np.ndarray:
    """Index of the maximal run of consecutive mask tokens each mask belongs to (-1 for
    non-mask tokens)."""
    g = np.full(len(is_mask), -1, dtype=np.int64)
    run = -1
    for i, m in enumerate(is_mask):
        if m:
            if i == 0 or not is_mask[i - 1]:
                run += 1
            g[i] = run
    return g


def sar_attention_mask(is_mask: np.ndarray, k: Optional[int] = None, reading: str = "group") -> np.ndarray:
    """Eq. 3.  A[i, j] = 1 iff query i may attend key j.

    clause 1: j <= i and key j is not a mask token;
    clause 2: j <= i and both are mask tokens of the same group (reading="group", the
              prose), or both are mask tokens and i - j < k (reading="literal", as printed).
    """
    n = len(is_mask)
    grp = mask_group_ids(is_mask)
    A = np.zeros((n, n), dtype=np.int64)
    for i in range(n):
        for j in range(i + 1):
            if not is_mask[j]:
                A[i, j] = 1
            elif is_mask[i]:
                if reading == "group":
                    A[i, j] = 1 if grp[i] == grp[j] else 0
                elif reading == "literal":
                    assert k is not None
                    A[i, j] = 1 if (i - j) < k else 0
                else:
                    raise ValueError(reading)
    return A


def position_ids(A: np.ndarray) -> np.ndarray:
    """P-bar_i = sum_j A-bar_ij - 1 (text after Eq. 3)."""
    return A.sum(axis=1) - 1


# --------------------------------------------------------------------------------------
# forward passes
# --------------------------------------------------------------------------------------


def _attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, vis: np.ndarray, scale: float) -> np.ndarray:
    """q [R, H, dh]; k, v [S, Hkv, dh] with Hkv dividing H (query head h reads key/value head
    h // (H / Hkv): grouped-query attention of the larger family members); vis [R, S] in {0,1}.
    Returns [R, H*dh]."""
    R, H, dh = q.shape
    group = H // k.shape[1]
    out = np.empty((R, H, dh), dtype=np.float64)
    for h in range(H):
        s = (q[:, h, :] @ k[:, h // group, :].T) * scale
        s = np.where(vis > 0, s, -np.inf)
        out[:, h, :] = softmax_rows(s) @ v[:, h // group, :]
    return out.reshape(R, H * dh)


def _layer_forward(m: OracleModel, w: Dict[str, np.ndarray], x: np.ndarray, pos: np.ndarray,
                   k_prev: Optional[np.ndarray], v_prev: Optional[np.ndarray], vis: np.ndarray,
                   trace: Optional[Dict[str, np.ndarray]] = None
                   ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """One pre-norm decoder layer over the rows x.  k_prev / v_prev ([S0, H, dh] or None) are
    keys / values that precede these rows; vis is [rows, S0 + rows].  Returns the new x and
    the K / V of these rows ([rows, H, dh])."""
    R = x.shape[0]
    H, Hkv, dh = m.n_heads, m.kv_heads, m.head_dim
    n1 = m.rnd(rmsnorm(x, w["attn_norm"], m.rms_eps))
    q = (n1 @ w["wq"].T).reshape(R, H, dh)
    k = (n1 @ w["wk"].T).reshape(R, Hkv, dh)
    v = (n1 @ w["wv"].T).reshape(R, Hkv, dh)
    q = m.rnd(rope(q, pos, m.rope_base))
    k = m.rnd_kv(rope(k, pos, m.rope_base))
    v = m.rnd_kv(v)
    k_all = k if k_prev is None else np.concatenate([k_prev, k], axis=0)
    v_all = v if v_prev is None else np.concatenate([v_prev, v], axis=0)
    o = _attention(q, k_all, v_all, vis, 1.0 / np.sqrt(dh))
    x = x + m.rnd(o) @ w["wo"].T
    n2 = m.rnd(rmsnorm(x, w["ffn_norm"], m.rms_eps))
    hmid = silu(n2 @ w["w_gate"].T) * (n2 @ w["w_up"].T)
    x = x + m.rnd(hmid) @ w["w_down"].T
    if trace is not None:  # intermediates of this layer, for kernel-level parity tests
        trace.update(xn1=n1, q=q, k=k, v=v, attn_out=m.rnd(o), xn2=n2, h=m.rnd(hmid), x=x)
    return x, k, v


def _logits(m: OracleModel, x: np.ndarray) -> np.ndarray:
    hd = m.head()
    return m.rnd(rmsnorm(x, hd["final_norm"], m.rms_eps)) @ hd["lm_head"].T


def forward_dense(m: OracleModel, tokens: np.ndarray, A: np.ndarray, pos: np.ndarray) -> np.ndarray:
    """P = M(I, A-bar, P-bar) (Algorithm 1, the model invocation): logits of every row of the
    whole sequence, no cache."""
    x = m.head()["embed"][np.asarray(tokens, dtype=np.int64)]
    for l in range(m.n_layers):
        x, _, _ = _layer_forward(m, m.layer(l), x, np.asarray(pos), None, None, A)
    return _logits(m, x)


def causal_forward(m: OracleModel, tokens: Sequence[int]) -> np.ndarray:
    """Plain causal forward with positions 0..n-1 (the textbook autoregressive model)."""
    n = len(tokens)
    A = np.tril(np.ones((n, n), dtype=np.int64))
    return forward_dense(m, np.asarray(tokens), A, np.arange(n))


def ar_greedy(m: OracleModel, prompt: Sequence[int], n_new: int) -> List[int]:
    """Plain greedy autoregressive decoding, full re-forward each token."""
    seq = [int(t) for t in prompt]
    for _ in range(n_new):
        logits = causal_forward(m, seq)
        seq.append(int(np.argmax(logits[-1])))
    return seq


# --------------------------------------------------------------------------------------
# KV cache form
# --------------------------------------------------------------------------------------


class OracleKV:
    """K/V of the committed prefix x_1..x_{l-1}, per layer, as [ctx, H, dh] float64."""

    def __init__(self, m: OracleModel):
        self.k = [np.zeros((0, m.kv_heads, m.head_dim)) for _ in range(m.n_layers)]
        self.v = [np.zeros((0, m.kv_heads, m.head_dim)) for _ in range(m.n_layers)]

    @property
    def length(self) -> int:
        return self.k[0].shape[0]

    def append(self, staged_k: List[np.ndarray], staged_v: List[np.ndarray], rows: Sequence[int]) -> None:
        rows = list(rows)
        for l in range(len(self.k)):
            self.k[l] = np.concatenate([self.k[l], staged_k[l][rows]], axis=0)
            self.v[l] = np.concatenate([self.v[l], staged_v[l][rows]], axis=0)

    def truncate(self, n: int) -> None:
        """Roll the cache back by n positions."""
        if n > 0:
            for l in range(len(self.k)):
                self.k[l] = self.k[l][:-n]
                self.v[l] = self.v[l][:-n]


def block_forward_cached(m: OracleModel, kv: OracleKV, block_tokens: np.ndarray, block_is_mask: np.ndarray,
                         k: Optional[int] = None, reading: str = "group",
                         trace: Optional[List[Dict[str, np.ndarray]]] = None):
    """The model invocation restricted to the rows that are not cached yet.

    The cached keys are non-mask tokens that precede every block row, so by Eq. 3 (clause 1)
    all of them are visible to every row; inside the block Eq. 3 applies unchanged.  Position
    ids are row sums of the full mask minus one.  Returns (logits [rows, V], staged K list,
    staged V list, pos)."""
    ctx = kv.length
    A_blk = sar_attention_mask(block_is_mask, k, reading)
    R = len(block_tokens)
    vis = np.concatenate([np.ones((R, ctx), dtype=np.int64), A_blk], axis=1)
    pos = position_ids(vis)
    x = m.head()["embed"][np.asarray(block_tokens, dtype=np.int64)]
    ks, vs = [], []
    for l in range(m.n_layers):
        tr = {} if trace is not None else None
        x, kk, vv = _layer_forward(m, m.layer(l), x, pos, kv.k[l], kv.v[l], vis, tr)
        if trace is not None:
            trace.append(tr)
        ks.append(kk)
        vs.append(vv)
    return _logits(m, x), ks, vs, pos


def prefill(m: OracleModel, kv: OracleKV, tokens: Sequence[int]) -> np.ndarray:
    """Push committed tokens through the model (all non-mask: the mask is plain causal) and
    keep their K/V.  Returns their logits."""
    toks = np.asarray(tokens, dtype=np.int64)
    logits, ks, vs, _ = block_forward_cached(m, kv, toks, np.zeros(len(toks), dtype=bool))
    kv.append(ks, vs, range(len(toks)))
    return logits


# --------------------------------------------------------------------------------------
# Algorithm 1 (greedy)
# --------------------------------------------------------------------------------------


@dataclass
class StepResult:
    accepted: int            # i*: number of accepted candidates, 0..k
    emitted: List[int]       # accepted candidates followed by the one extra token
    new_cands: List[int]     # L_c for the next step
    argmax: np.ndarray       # argmax of every row the verification may look at (block rows)
    logits: np.ndarray       # logits of those rows


def verify_greedy(P_blk: np.ndarray, k: int, cands: Sequence[int], candidates_valid: bool = True) -> StepResult:
    """Verification and candidate refresh of Algorithm 1 in the greedy setting.

    ``P_blk`` holds the logits of the block rows, i.e. rows l .. l+k(k+2) of the paper's P
    (1-based), so that the paper's P[l + i(k+1)] is P_blk[i(k+1)] and P[idx:idx+k] with
    idx = l+1+i*(k+1) is P_blk[i*(k+1)+1 : i*(k+1)+1+k]."""
    am = np.argmax(P_blk, axis=-1)
    idx = 1
    q_row = 0
    emitted: List[int] = []
    acc = 0
    for i in range(1, k + 1):
        ok = candidates_valid and int(cands[i - 1]) == int(am[q_row])
        if ok:
            emitted.append(int(cands[i - 1]))
            idx += k + 1
            q_row = i * (k + 1)
            acc += 1
        else:
            break
    emitted.append(int(am[q_row]))
    new_cands = [int(t) for t in am[idx: idx + k]]
    return StepResult(acc, emitted, new_cands, am, P_blk)


def space_step_dense(m: OracleModel, seq: Sequence[int], cands: Sequence[int], k: int,
                     candidates_valid: bool = True, reading: str = "group") -> StepResult:
    """One iteration of Algorithm 1 by its definition: full extended input, full mask."""
    l = len(seq)
    toks, is_mask = extended_input(seq, cands, k, m.mask_id)
    A = sar_attention_mask(is_mask, k, reading)
    P = forward_dense(m, toks, A, position_ids(A))
    return verify_greedy(P[l - 1:], k, cands, candidates_valid)


def space_step_cached(m: OracleModel, kv: OracleKV, last_token: int, cands: Sequence[int], k: int,
                      candidates_valid: bool = True, reading: str = "group", commit: bool = True):
    """One iteration of Algorithm 1 with K/V of x_1..x_{l-1} cached.  Commits K/V of x_l and
    of the accepted candidates (all other block rows are dropped).  Returns (StepResult,
    staged K, staged V, pos)."""
    toks, is_mask = extended_input([last_token], cands, k, m.mask_id)
    P, ks, vs, pos = block_forward_cached(m, kv, toks, is_mask, k, reading)
    res = verify_greedy(P, k, cands, candidates_valid)
    if commit:
        kv.append(ks, vs, [g * (k + 1) for g in range(res.accepted + 1)])
    return res, ks, vs, pos


def space_generate(m: OracleModel, prompt: Sequence[int], k: int, n_new: int, form: str = "cached",
                   reading: str = "group", eos_id: Optional[int] = None):
    """Algorithm 1, greedy, stopping once n_new tokens are out (overshoot truncated) or, with
    ``eos_id``, once that token has been generated: then the output ends in front of it (the
    O[:eos_index] of Algorithm 1).  Returns (sequence, list of accepted counts per model invocation)."""
    seq = [int(t) for t in prompt]
    target = len(seq) + n_new
    cands = [0] * k
    valid = False  # P_c = +inf on the first iteration
    accepted_hist: List[int] = []
    kv = None
    if form == "cached":
        kv = OracleKV(m)
        if len(seq) > 1:
            prefill(m, kv, seq[:-1])
    while len(seq) < target:
        if form == "cached":
            res, _, _, _ = space_step_cached(m, kv, seq[-1], cands, k, valid, reading)
        else:
            res = space_step_dense(m, seq, cands, k, valid, reading)
        n_before = len(seq)
        seq.extend(res.emitted)
        accepted_hist.append(res.accepted)
        if eos_id is not None and eos_id in seq[n_before:]:
            return seq[: n_before + seq[n_before:].index(eos_id)][:target], accepted_hist
        cands = res.new_cands
        valid = True
    return seq[:target], accepted_hist
