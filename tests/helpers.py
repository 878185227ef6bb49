"""Shared test helpers: tiny configurations and weight providers."""
import numpy as np

from koala_synth import target_weights, eagle_weights, medusa_weights
from koala_synth.trees import make_tree

NANO = dict(name="nano", dtype="fp32", hidden=32, n_heads=2, head_dim=16, ffn=48, vocab=50,
            n_layers=2, rms_eps=1e-6, rope_base=10000.0, draft="eagle", K=2, medusa_heads=3)


def nano_weights(seed=0, std=0.3, norm_gain="random"):
    """Weights large enough (std 0.3) that attention and FFN branches matter."""
    Wt = target_weights(NANO, seed, std=std, norm_gain=norm_gain, cache=True)
    Wd = eagle_weights(NANO, seed, std=std, norm_gain=norm_gain, cache=True)
    Wm = medusa_weights(NANO, seed, std=std, cache=True)
    return Wt, Wd, Wm


def nano_tree():
    return make_tree([3, 2, 2], [1, 3, 4, 3])
