"""Seeded synthetic inputs for the draft-then-verify path.

This package only *produces data*: weight tensors, KV-cache contents, hidden
states, token ids and static candidate-tree templates.  It holds none of the
method's arithmetic (no normalisation, attention, masks, top-k or acceptance),
so both the CPU oracle and the HIP path may consume what it produces without
sharing any code that computes results.
"""
from .rng import tensor_normal, tensor_uniform_int, tensor_uniform01, to_bf16_bits, bf16_bits_to_f32  # noqa: F401
from .trees import make_tree, chain_tree, TreeTemplate  # noqa: F401
from .configs import CONFIGS, get_config  # noqa: F401
from .weights import ModelWeights, target_weights, eagle_weights, medusa_weights, predictable_pair  # noqa: F401
