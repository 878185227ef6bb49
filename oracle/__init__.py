"""CPU oracle for one draft-then-verify iteration of multi-layer-draft-head
speculative decoding (paper sections 2.1, 2.2 and 3.1) and, in `oracle.train`,
for one adversarial training step of a draft head (section 3.2, Algorithm 1).

TEST INFRASTRUCTURE ONLY.  Plain NumPy, written for checking by eye against the
paper, not for speed.  Only the tests, the smoke check and the `cpu_baseline`
leg of the benchmark may import this package; the product path (the HIP
library and its Python binding) never does, and this package imports nothing
from the product.

Parity status: every function here is pinned by CPU tests against something
other than itself (sequential decoding per Eq. 1, brute-force ancestor closure,
brute-force longest match, full sorts, closed forms; the training step's
backward formulas against finite differences of its losses).  The paper prints no
worked numeric example for this path and its Tables 1-2 need trained weights
and a benchmark that are not available, so those table cells are
"parity unpinned" and out of scope.
"""
from .llama import (rmsnorm, silu, softmax, rope_rotate, attention_row, decoder_layer_rows,  # noqa: F401
                    KVCache)
from .tree import tree_depths, ancestor_mask, children_lists, expanded_nodes  # noqa: F401
from .spec import (target_rows, decode_one, prefill, verify_tree, accept_greedy, commit_path,  # noqa: F401
                   topk_desc, eagle_rows, eagle_expand, medusa_expand, iteration_eagle,
                   greedy_reference, generate_speculative, mean_tokens_per_iteration, n_alpha)
from .sampling import (softmax_t, inverse_cdf, draw_without_replacement, accept_sample,  # noqa: F401
                       eagle_expand_sample, generate_sampled, medusa_expand_sample)
from . import train  # noqa: F401,E402
