"""Seeded synthetic inputs shared by the CPU oracle and the GPU tests / bench.

This module holds only shapes and random-number recipes.  It contains none of
the method's arithmetic (no normalisation, rotation, attention, planning), so
both the oracle and the HIP path may draw their inputs from it without sharing
any code that matters for parity.

Recipe (stands in for the paper's workloads; Sec. 5.1 "Datasets" of the paper
itself uses synthetic prompts because only token length matters, and its
trained checkpoints are replaced by random weights of the same shapes):

* every weight matrix ~ N(0, 0.02), generated per tensor from
  ``default_rng([seed, layer, tensor_id])`` so single tensors can be produced
  without materialising a whole model;
* norm gains are 1 by default (``gain_jitter`` perturbs them for tests that
  must notice a dropped gain);
* for ``dtype == "bf16"`` every weight is made exactly representable in
  bfloat16 by clearing the low 16 bits of its fp32 pattern, so the fp32 array
  the oracle consumes and the bf16 tensor the GPU consumes hold identical
  values;
* token ids are uniform on [0, vocab).

Matrices are returned in the paper's orientation (Sec. 3: Q = X W_Q), i.e.
``[in_features, out_features]``.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Iterable, Optional

import numpy as np


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_q: int
    n_kv: int
    head_dim: int
    ffn: int
    vocab: int
    dtype: str = "bf16"          # "f32" | "bf16": arithmetic / KV storage type
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def with_(self, **kw) -> "ModelShape":
        return replace(self, **kw)


# Model shapes of the benchmark configurations.
TINY = ModelShape("tiny-f32", 2, 256, 4, 4, 64, 688, 32000, "f32")
LLAMA2_7B = ModelShape("llama2-7b-shape", 32, 4096, 32, 32, 128, 11008, 32000, "bf16")
LLAMA3_8B = ModelShape("llama3-8b-shape", 32, 4096, 32, 8, 128, 14336, 128256, "bf16",
                       rope_theta=500000.0)
LLAMA2_70B = ModelShape("llama2-70b-shape", 80, 8192, 64, 8, 128, 28672, 32000, "bf16")
LONGALPACA_13B = ModelShape("longalpaca-13b-shape", 40, 5120, 40, 40, 128, 13824, 32000, "bf16")

SHAPES = {s.name: s for s in (TINY, LLAMA2_7B, LLAMA3_8B, LLAMA2_70B, LONGALPACA_13B)}

# tensor ids used for per-tensor seeding
_TENSOR_IDS = {
    "embed": 1, "final_norm": 2, "lm_head": 3,
    "attn_norm": 10, "wq": 11, "wk": 12, "wv": 13, "wo": 14,
    "ffn_norm": 15, "w_gate": 16, "w_up": 17, "w_down": 18,
}
LAYER_TENSORS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


def tensor_dims(shape: ModelShape, name: str):
    d, hq, hkv, ff = shape.d_model, shape.n_q * shape.head_dim, shape.n_kv * shape.head_dim, shape.ffn
    return {
        "embed": (shape.vocab, d), "final_norm": (d,), "lm_head": (d, shape.vocab),
        "attn_norm": (d,), "ffn_norm": (d,),
        "wq": (d, hq), "wk": (d, hkv), "wv": (d, hkv), "wo": (hq, d),
        "w_gate": (d, ff), "w_up": (d, ff), "w_down": (ff, d),
    }[name]


def _clear_low_half(a: np.ndarray) -> np.ndarray:
    """Make fp32 values bf16-representable by zeroing the low 16 mantissa bits."""
    u = a.view(np.uint32)
    u &= np.uint32(0xFFFF0000)
    return a


def make_tensor(shape: ModelShape, name: str, layer: int, seed: int,
                std: float = 0.02, gain_jitter: float = 0.0) -> np.ndarray:
    """One weight tensor as float32, in [in, out] orientation (gains: [d])."""
    rng = np.random.default_rng([seed, layer + 1 if layer >= 0 else 0, _TENSOR_IDS[name]])
    dims = tensor_dims(shape, name)
    if name.endswith("norm"):
        g = np.ones(dims, dtype=np.float32)
        if gain_jitter:
            g += (gain_jitter * rng.standard_normal(dims, dtype=np.float32))
        return g  # gains stay fp32 on both sides
    a = rng.standard_normal(dims, dtype=np.float32)
    a *= np.float32(std)
    if shape.dtype == "bf16":
        _clear_low_half(a)
    return a


def make_weights(shape: ModelShape, seed: int = 0, layers: Optional[Iterable[int]] = None,
                 std: float = 0.02, gain_jitter: float = 0.0,
                 with_head: bool = False) -> Dict[str, object]:
    """All tensors the prefill path reads: {"embed", "layers": [ {...}, ... ]}."""
    layer_ids = list(range(shape.n_layers)) if layers is None else list(layers)
    w: Dict[str, object] = {
        "embed": make_tensor(shape, "embed", -1, seed, std),
        "layers": [
            {n: make_tensor(shape, n, l, seed, std, gain_jitter) for n in LAYER_TENSORS}
            for l in layer_ids
        ],
    }
    if with_head:
        w["final_norm"] = make_tensor(shape, "final_norm", -1, seed, std, gain_jitter)
        w["lm_head"] = make_tensor(shape, "lm_head", -1, seed, std)
    return w


def make_tokens(n_tokens: int, vocab: int, seed: int = 1) -> np.ndarray:
    rng = np.random.default_rng([seed, 0xC0FFEE])
    return rng.integers(0, vocab, size=n_tokens, dtype=np.int32)


def make_costs(n: int, seed: int, lo: int = 1, hi: int = 1000):
    """Random integer per-chunk (compute_ns, load_ns) vectors for planner tests."""
    rng = np.random.default_rng([seed, 0xBEEF])
    c = rng.integers(lo, hi + 1, size=n, dtype=np.uint64)
    l = rng.integers(lo, hi + 1, size=n, dtype=np.uint64)
    return c, l
