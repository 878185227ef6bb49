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
                 norm_gain: str = "ones", cache: bool = False, overrides: dict | None = None):
        """overrides: name -> function returning that tensor's values (fp32, before any rounding)
        instead of the random stream; used by the structured weight sets below."""
        assert dtype in ("fp32", "bf16")
        self.seed, self.shapes, self.dtype, self.std = seed, shapes, dtype, std
        self.norm_gain = norm_gain
        self.overrides = overrides or {}
        self._cache = {} if cache else None

    def names(self):
        return list(self.shapes.keys())

    def _raw(self, name: str) -> np.ndarray:
        shape = self.shapes[name]
        if name in self.overrides:
            a = np.asarray(self.overrides[name](), dtype=np.float32)
            assert a.shape == tuple(shape), (name, a.shape, shape)
            return a
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


def predictable_pair(cfg: dict, seed: int = 0, sigma: float = 0.0, gain: float = 4.0, **kw):
    """A (target, EAGLE draft) weight pair whose greedy continuation is known by construction, so
    that acceptance lengths in generation tests are not almost always zero as with random weights.

    Target: every attention-output and FFN-down matrix is zero, so the residual stream stays the
    token embedding; LM-head row t is `gain / std` times embedding row t-1 (cyclically), which makes
    the greedy successor of token t the token t+1 (mod vocab) as long as embedding rows are far from
    parallel.  Draft: same zeroed output matrices, fc = [I + sigma * N | 0] on [embedding ; feature]
    with N ~ N(0, 1/hidden): sigma = 0 drafts the target's successor exactly, larger sigma perturbs
    the draft's ranking so that the right token moves to lower ranks or out of the top-k.  All
    other tensors are the usual random ones (they are computed but do not reach the output)."""
    H, V = cfg["hidden"], cfg["vocab"]
    std = 0.02
    zeros_hh = lambda: np.zeros((H, H), np.float32)
    zeros_hf = lambda: np.zeros((H, cfg["ffn"]), np.float32)
    tov, dov = {}, {}
    for l in range(cfg["n_layers"]):
        tov[f"layers.{l}.wo"] = zeros_hh
        tov[f"layers.{l}.wdown"] = zeros_hf
    for k in range(cfg["K"]):
        dov[f"draft.layers.{k}.wo"] = zeros_hh
        dov[f"draft.layers.{k}.wdown"] = zeros_hf
    embed = lambda: tensor_normal(seed, "embed", (V, H), std)
    tov["lm_head"] = lambda: np.roll(embed(), 1, axis=0) * np.float32(gain / std)

    def fc():
        a = np.zeros((H, 2 * H), np.float32)
        a[:, :H] = np.eye(H, dtype=np.float32)
        if sigma:
            a[:, :H] += np.float32(sigma / np.sqrt(H)) * tensor_normal(seed, "draft.fc.noise", (H, H), 1.0)
        return a
    dov["draft.fc"] = fc
    Wt = target_weights(cfg, seed, overrides=tov, **kw)
    Wd = eagle_weights(cfg, seed, overrides=dov, **kw)
    return Wt, Wd
