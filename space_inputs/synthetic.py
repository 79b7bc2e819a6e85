"""Seeded synthetic model weights, prompts and KV fills.

The paper evaluates fine-tuned LLaMA-family checkpoints on public suites (Experimental
Settings, "Training" and "Inference"); neither is available here, so every input is a
seeded random stand-in with the same shapes: LLaMA-shaped decoders with N(0, 0.02)
matrices, unit norm weights, uniform-random prompts.  Canonical weights are the bf16
roundings (round-to-nearest-even) of the fp32 draws, stored as uint16 bit patterns so
that both consumers widen them exactly.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Dict, List

import numpy as np


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    n_kv_heads: int = 0  # 0: one key/value head per query head; else a divisor of n_heads (grouped-query)

    @property
    def kv_heads(self) -> int:
        return self.n_kv_heads if self.n_kv_heads > 0 else self.n_heads

    @property
    def mask_id(self) -> int:
        """The mask token is one extra embedding row past the vocabulary (Experimental
        Settings: it is added as a new special token), so the LM head can never emit it."""
        return self.vocab

    def with_layers(self, n_layers: int) -> "ModelShape":
        return ModelShape(self.name + f"-{n_layers}L", n_layers, self.d_model, self.n_heads,
                          self.head_dim, self.ffn, self.vocab, self.rms_eps, self.rope_base, self.n_kv_heads)


SHAPES: Dict[str, ModelShape] = {
    # small decoder the oracle finishes in seconds
    "tiny": ModelShape("tiny", 2, 256, 4, 64, 688, 1000),
    # head_dim 128 at small width: exercises the 7B attention tile shape cheaply
    "small128": ModelShape("small128", 3, 512, 4, 128, 1376, 2000),
    "7b": ModelShape("7b", 32, 4096, 32, 128, 11008, 32000),
    "13b": ModelShape("13b", 40, 5120, 40, 128, 13824, 32000),
    # grouped-query attention: 8 query heads share 2 key/value heads; the 70B member of the family
    "gqa-small": ModelShape("gqa-small", 3, 512, 8, 64, 1376, 2000, n_kv_heads=2),
    "gqa128": ModelShape("gqa128", 2, 1024, 8, 128, 1376, 2000, n_kv_heads=4),
    "70b": ModelShape("70b", 80, 8192, 64, 128, 28672, 32000, n_kv_heads=8),
}

_TENSOR_IDS = {
    "embed": 1, "lm_head": 2, "final_norm": 3, "attn_norm": 4, "wq": 5, "wk": 6, "wv": 7,
    "wo": 8, "ffn_norm": 9, "w_gate": 10, "w_up": 11, "w_down": 12, "prompt": 13,
    "kv_k": 14, "kv_v": 15, "x": 16, "ctx_len": 17, "accept": 18,
}
_GLOBAL_LAYER = 1 << 20  # layer slot used by tensors that belong to no layer


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 storage (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _gen(seed: int, layer: int, name: str) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, layer, _TENSOR_IDS[name]])))


def _normal_bits(seed: int, layer: int, name: str, shape, std: float) -> np.ndarray:
    g = _gen(seed, layer, name)
    x = g.standard_normal(size=shape, dtype=np.float32)
    x *= np.float32(std)
    return f32_to_bf16_bits(x)


def _ones_bits(n: int) -> np.ndarray:
    return f32_to_bf16_bits(np.ones(n, dtype=np.float32))


def layer_weights(shape: ModelShape, seed: int, layer: int, threads: int = 1) -> Dict[str, np.ndarray]:
    """bf16 bit patterns of one decoder layer; matrices are [out_features, in_features]."""
    d, f, hd = shape.d_model, shape.ffn, shape.n_heads * shape.head_dim
    hkv = shape.kv_heads * shape.head_dim
    specs = {
        "wq": (hd, d), "wk": (hkv, d), "wv": (hkv, d), "wo": (d, hd),
        "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f),
    }
    if threads > 1:
        with ThreadPoolExecutor(threads) as ex:
            futs = {n: ex.submit(_normal_bits, seed, layer, n, s, 0.02) for n, s in specs.items()}
            out = {n: fu.result() for n, fu in futs.items()}
    else:
        out = {n: _normal_bits(seed, layer, n, s, 0.02) for n, s in specs.items()}
    out["attn_norm"] = _ones_bits(d)
    out["ffn_norm"] = _ones_bits(d)
    return out


def head_weights(shape: ModelShape, seed: int) -> Dict[str, np.ndarray]:
    """Embedding table ([vocab + 1, d], last row = mask token), final norm, LM head."""
    return {
        "embed": _normal_bits(seed, _GLOBAL_LAYER, "embed", (shape.vocab + 1, shape.d_model), 0.02),
        "final_norm": _ones_bits(shape.d_model),
        "lm_head": _normal_bits(seed, _GLOBAL_LAYER, "lm_head", (shape.vocab, shape.d_model), 0.02),
    }


def all_weights(shape: ModelShape, seed: int, threads: int = 1) -> Dict[str, object]:
    w: Dict[str, object] = dict(head_weights(shape, seed))
    layers: List[Dict[str, np.ndarray]] = []
    if threads > 1:
        with ThreadPoolExecutor(threads) as ex:
            layers = list(ex.map(lambda l: layer_weights(shape, seed, l), range(shape.n_layers)))
    else:
        layers = [layer_weights(shape, seed, l) for l in range(shape.n_layers)]
    w["layers"] = layers
    return w


def prompt_tokens(shape: ModelShape, seed: int, n: int, batch: int = 1) -> np.ndarray:
    g = _gen(seed, _GLOBAL_LAYER, "prompt")
    return g.integers(0, shape.vocab, size=(batch, n), dtype=np.int64).astype(np.int32)


def normal_bf16(seed: int, layer: int, name: str, shape, std: float = 1.0) -> np.ndarray:
    """bf16 bit patterns of an N(0, std) tensor (KV fills and activations of the
    single-layer micro-benchmark)."""
    return _normal_bits(seed, layer, name, shape, std)


def ragged_context_lengths(seed: int, batch: int, lo: int = 256, hi: int = 4096) -> np.ndarray:
    g = _gen(seed, _GLOBAL_LAYER, "ctx_len")
    return g.integers(lo, hi + 1, size=batch, dtype=np.int64).astype(np.int32)


def geometric_accept_lengths(seed: int, batch: int, k: int, p_fail: float = 0.4, step: int = 0) -> np.ndarray:
    """Accepted-candidate counts: successes before the first failure, capped at k."""
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence(
        [seed, _GLOBAL_LAYER, _TENSOR_IDS["accept"], step])))
    return np.minimum(g.geometric(p_fail, size=batch) - 1, k).astype(np.int32)
