"""Random-init model weights, produced tensor by tensor from (seed, name).

All matrices are N(0, 0.02^2); RMSNorm gains are 1 (or 1 + N(0, 0.1^2) when
`norm_gain="random"`, used by tests that must notice a dropped gain).  For the
bf16 workloads every tensor is rounded to bfloat16 once, here; `f32(name)`
returns those rounded values widened to fp32 and `bits(name)` the uint16 bit
patterns, so both consumers see identical numbers.
"""
from __future__ import annotations

import numpy as np

from .rng import tensor_normal, to_bf16_bits, bf16_bits_to_f32

_LAYER_MATS = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown")


class ModelWeights:
    def __init__(self, seed: int, shapes: dict, dtype: str, std: float = 0.02,
                 norm_gain: str = "ones", cache: bool = False):
        assert dtype in ("fp32", "bf16")
        self.seed, self.shapes, self.dtype, self.std = seed, shapes, dtype, std
        self.norm_gain = norm_gain
        self._cache = {} if cache else None

    def names(self):
        return list(self.shapes.keys())

    def _raw(self, name: str) -> np.ndarray:
        shape = self.shapes[name]
        if name.endswith("norm"):
            if self.norm_gain == "ones":
                return np.ones(shape, dtype=np.float32)
            return (1.0 + tensor_normal(self.seed, name, shape, 0.1)).astype(np.float32)
        return tensor_normal(self.seed, name, shape, self.std)

    def bits(self, name: str) -> np.ndarray:
        """uint16 bfloat16 bit patterns (bf16 workloads only)."""
        assert self.dtype == "bf16"
        if self._cache is not None:
            return to_bf16_bits(self.f32(name))          # already bf16-representable: exact
        return to_bf16_bits(self._raw(name))

    def f32(self, name: str) -> np.ndarray:
        if self._cache is not None and name in self._cache:
            return self._cache[name]
        x = self._raw(name)
        if self.dtype == "bf16":
            x = bf16_bits_to_f32(to_bf16_bits(x))
        if self._cache is not None:
            self._cache[name] = x
        return x


def _layer_shapes(prefix: str, n_layers: int, H: int, F: int) -> dict:
    s = {}
    for l in range(n_layers):
        p = f"{prefix}layers.{l}."
        s[p + "in_norm"] = (H,)
        s[p + "post_norm"] = (H,)
        for m in ("wq", "wk", "wv", "wo"):
            s[p + m] = (H, H)
        s[p + "wgate"] = (F, H)
        s[p + "wup"] = (F, H)
        s[p + "wdown"] = (H, F)
    return s


def target_weights(cfg: dict, seed: int = 0, **kw) -> ModelWeights:
    H, F, V = cfg["hidden"], cfg["ffn"], cfg["vocab"]
    s = {"embed": (V, H), "lm_head": (V, H), "final_norm": (H,)}
    s.update(_layer_shapes("", cfg["n_layers"], H, F))
    return ModelWeights(seed, s, cfg["dtype"], **kw)


def eagle_weights(cfg: dict, seed: int = 0, **kw) -> ModelWeights:
    H, F = cfg["hidden"], cfg["ffn"]
    s = {"draft.fc": (H, 2 * H)}
    s.update(_layer_shapes("draft.", cfg["K"], H, F))
    return ModelWeights(seed, s, cfg["dtype"], **kw)


def medusa_weights(cfg: dict, seed: int = 0, **kw) -> ModelWeights:
    H = cfg["hidden"]
    s = {}
    for j in range(cfg["medusa_heads"]):
        for k in range(cfg["K"]):
            s[f"medusa.{j}.{k}"] = (H, H)
    return ModelWeights(seed, s, cfg["dtype"], **kw)
