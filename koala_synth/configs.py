"""The synthetic workloads (shapes, tree templates, context lengths, seeds).

`cfg1`..`cfg5` follow the five benchmark configurations; the `*_small`
entries keep the structure (head_dim 128, bf16, same tree template) at a width
and depth the CPU oracle finishes in seconds, for element-by-element parity.
"""
from __future__ import annotations

import copy

from .trees import make_tree

SEED_WEIGHTS = 0
SEED_INPUTS = 1
SEED_LENGTHS = 2

_TREE_CFG1 = dict(topk=[2, 2], widths=[1, 2, 4])
_TREE_CFG2 = dict(topk=[4, 2, 2, 1, 1], widths=[1, 4, 8, 6, 4, 3])
_TREE_CFG3 = dict(topk=[10, 5, 3, 2], widths=[1, 10, 20, 18, 15])
_TREE_CFG4 = dict(topk=[4, 2, 2, 2, 1, 1], widths=[1, 4, 8, 12, 12, 12, 11])

CONFIGS = {
    "cfg1": dict(
        name="cfg1", dtype="fp32", hidden=256, n_heads=4, head_dim=64, ffn=688, vocab=1000,
        n_layers=4, rms_eps=1e-6, rope_base=10000.0, draft="eagle", K=2, medusa_heads=0,
        tree=_TREE_CFG1, ctx=64, batch=1, kv="prefill", capacity=128),
    "cfg2": dict(
        name="cfg2", dtype="bf16", hidden=4096, n_heads=32, head_dim=128, ffn=11008, vocab=32000,
        n_layers=32, rms_eps=1e-6, rope_base=10000.0, draft="eagle", K=1, medusa_heads=0,
        tree=_TREE_CFG2, ctx=1024, batch=1, kv="normal", capacity=1152),
    "cfg3": dict(
        name="cfg3", dtype="bf16", hidden=4096, n_heads=32, head_dim=128, ffn=11008, vocab=32000,
        n_layers=32, rms_eps=1e-6, rope_base=10000.0, draft="medusa", K=1, medusa_heads=4,
        tree=_TREE_CFG3, ctx=2048, batch=1, kv="normal", capacity=2176),
    "cfg4": dict(
        name="cfg4", dtype="bf16", hidden=5120, n_heads=40, head_dim=128, ffn=13824, vocab=32000,
        n_layers=40, rms_eps=1e-6, rope_base=10000.0, draft="eagle", K=3, medusa_heads=0,
        tree=_TREE_CFG4, ctx=4096, batch=1, kv="normal", capacity=4224),
    "cfg5": dict(
        name="cfg5", dtype="bf16", hidden=6656, n_heads=52, head_dim=128, ffn=17920, vocab=32000,
        n_layers=60, rms_eps=1e-6, rope_base=10000.0, draft="eagle", K=2, medusa_heads=0,
        tree=_TREE_CFG4, ctx=(512, 8192), batch=8, kv="normal", capacity=8320),
}


def _small(base, **over):
    c = copy.deepcopy(CONFIGS[base])
    c.update(over)
    return c


# Reduced-width relatives used by parity tests (same kernels, several tiles, ragged tails).
CONFIGS["cfg2_small"] = _small("cfg2", name="cfg2_small", hidden=512, n_heads=4, ffn=1408,
                               vocab=4000, n_layers=3, ctx=200, capacity=320)
CONFIGS["cfg3_small"] = _small("cfg3", name="cfg3_small", hidden=512, n_heads=4, ffn=1408,
                               vocab=4000, n_layers=3, ctx=300, capacity=448)
CONFIGS["cfg4_small"] = _small("cfg4", name="cfg4_small", hidden=640, n_heads=5, ffn=1664,
                               vocab=4000, n_layers=2, ctx=333, capacity=512)
CONFIGS["cfg5_small"] = _small("cfg5", name="cfg5_small", hidden=512, n_heads=4, ffn=1408,
                               vocab=4000, n_layers=2, ctx=(40, 300), batch=3, capacity=384)


def get_config(name: str, **over) -> dict:
    c = copy.deepcopy(CONFIGS[name])
    c.update(over)
    c["tree_template"] = make_tree(c["tree"]["topk"], c["tree"]["widths"])
    return c
