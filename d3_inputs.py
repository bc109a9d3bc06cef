"""Seeded synthetic inputs for the D^3 decode path: model shapes, weights, prompts.

This module is the only code shared by the CPU oracle's tests and the HIP path's
tests/benchmark.  It holds none of the method's arithmetic: it only draws random
numbers and lays them out.  Both sides receive the *same* buffers.

Recipe (stands in for the paper's Llama-2 7B/13B/70B checkpoints and its
GSM8K / BBH few-shot prompts, Section 4.1, which are not available here):

* every linear layer and the embedding table: i.i.d. N(0, 0.02), drawn as
  float32 from numpy's Philox counter-based generator keyed by
  (seed, tensor id), so a depth-truncated model shares its first blocks with
  the full one;
* bf16 models: the float32 draw is rounded once to bf16 (round to nearest
  even) and handed out as uint16 bit patterns;
* RMSNorm gains: 1.0 (float32);
* prompts: token ids uniform in [0, vocab), all sequences of a batch have the
  same length, no EOS, generation runs for a fixed number of tokens.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List

import numpy as np

WEIGHT_STD = 0.02


@dataclass(frozen=True)
class ModelShape:
    """Llama-style decoder shape; field names follow the usual notation
    (L blocks, width d, H query heads, H_kv key/value heads, head dim hd,
    FFN width F, vocabulary V)."""
    name: str
    L: int
    d: int
    H: int
    H_kv: int
    hd: int
    F: int
    V: int
    dtype: str = "bf16"          # "f32" or "bf16": storage type of the linear weights
    eps: float = 1e-6
    rope_base: float = 10000.0

    def truncated(self, L: int) -> "ModelShape":
        return replace(self, L=L, name=f"{self.name}-L{L}")

    @property
    def params_per_block(self) -> int:
        qkv = (self.H + 2 * self.H_kv) * self.hd * self.d
        return qkv + self.H * self.hd * self.d + 3 * self.F * self.d


# Shapes of the benchmark configurations.
TINY = ModelShape("tiny", L=4, d=256, H=4, H_kv=4, hd=64, F=688, V=1024, dtype="f32")
LLAMA_7B = ModelShape("llama-7b", L=32, d=4096, H=32, H_kv=32, hd=128, F=11008, V=32000)
LLAMA_13B = ModelShape("llama-13b", L=40, d=5120, H=40, H_kv=40, hd=128, F=13824, V=32000)
LLAMA_70B = ModelShape("llama-70b", L=80, d=8192, H=64, H_kv=8, hd=128, F=28672, V=32000)
SHAPES = {s.name: s for s in (TINY, LLAMA_7B, LLAMA_13B, LLAMA_70B)}

# tensor ids inside one block (Philox key = [seed, 16*(layer+1) + id])
_BLOCK_TENSORS = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact upcast of bf16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal(seed: int, tensor_id: int, shape, dtype: str) -> np.ndarray:
    g = np.random.Generator(np.random.Philox(key=[seed, tensor_id]))
    n = int(np.prod(shape))
    a = g.standard_normal(n, dtype=np.float32)
    a *= np.float32(WEIGHT_STD)
    a = a.reshape(shape)
    return a if dtype == "f32" else f32_to_bf16_bits(a)


def make_weights(shape: ModelShape, seed: int = 0) -> Dict[str, object]:
    """All weights of the model as numpy arrays (row-major [out, in]).

    Linear weights and the embedding are float32 (dtype "f32") or uint16 bf16 bit
    patterns (dtype "bf16"); gains are float32 ones.  Keys: tok_emb [V,d],
    lm_head [V,d], final_norm [d], layers: list of dicts with attn_norm [d],
    wq [H*hd,d], wk/wv [H_kv*hd,d], wo [d,H*hd], mlp_norm [d], w_gate/w_up [F,d],
    w_down [d,F].
    """
    s = shape
    dims = {
        "wq": (s.H * s.hd, s.d), "wk": (s.H_kv * s.hd, s.d), "wv": (s.H_kv * s.hd, s.d),
        "wo": (s.d, s.H * s.hd), "w_gate": (s.F, s.d), "w_up": (s.F, s.d), "w_down": (s.d, s.F),
    }
    layers: List[Dict[str, np.ndarray]] = []
    for l in range(s.L):
        lw = {"attn_norm": np.ones(s.d, np.float32), "mlp_norm": np.ones(s.d, np.float32)}
        for t, name in enumerate(_BLOCK_TENSORS):
            lw[name] = _normal(seed, 16 * (l + 1) + t, dims[name], s.dtype)
        layers.append(lw)
    return {
        "tok_emb": _normal(seed, 1, (s.V, s.d), s.dtype),
        "lm_head": _normal(seed, 2, (s.V, s.d), s.dtype),
        "final_norm": np.ones(s.d, np.float32),
        "layers": layers,
    }


def weights_as_f64(shape: ModelShape, w: Dict[str, object]) -> Dict[str, object]:
    """The same values as float64 arrays (exact upcast), for NumPy-side checkers."""
    def up(a):
        a = np.asarray(a)
        if a.dtype == np.uint16:
            a = bf16_bits_to_f32(a)
        return a.astype(np.float64)
    out = {k: up(v) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: up(v) for k, v in lw.items()} for lw in w["layers"]]
    return out


def make_prompt(B: int, P: int, vocab: int, seed: int = 1) -> np.ndarray:
    """[B, P] int32 token ids, uniform in [0, vocab)."""
    g = np.random.Generator(np.random.Philox(key=[seed, 0]))
    return g.integers(0, vocab, size=(B, P), dtype=np.int64).astype(np.int32)


def start_layer_from_fraction(L: int, frac: float) -> int:
    """Grid-search 'start' fractions (Table 4) to a 0-based block id."""
    return int(np.floor(frac * L + 1e-9))
