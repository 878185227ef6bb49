"""Pins for the oracle's generation loop and its statistics (sections 2.2 and 4.1).

The loop is checked against things it does not compute itself: plain greedy decoding (the
method is lossless whatever the draft proposes), a weight set whose continuation is known in
closed form, drafts recomputed from scratch, and hand-counted statistics."""
import numpy as np
import pytest

import oracle
from koala_synth import get_config, make_tree, chain_tree
from koala_synth.weights import target_weights, eagle_weights, medusa_weights, predictable_pair
from helpers import NANO


def _nano(**kw):
    cfg = dict(NANO)
    cfg.update(kw)
    return cfg


TREE = make_tree([2, 2, 1], [1, 2, 3, 2])


@pytest.mark.parametrize("draft", ["eagle", "medusa"])
def test_generation_is_lossless_with_random_heads(draft):
    cfg = _nano(draft=draft)
    Wt = target_weights(cfg, 3, norm_gain="random", cache=True)
    Wd = (eagle_weights(cfg, 3, norm_gain="random", cache=True) if draft == "eagle"
          else medusa_weights(cfg, 3, cache=True))
    prompt = np.array([7, 1, 30, 12, 5])
    want = oracle.greedy_reference(cfg, Wt, prompt, 14)
    got = oracle.generate_speculative(cfg, Wt, Wd, prompt, 14, TREE.parent, TREE.rank, TREE.topk_per_depth)
    assert got["tokens"] == want
    assert sum(a + 1 for a in got["accept_lens"]) + 1 >= 14
    assert got["C"] == len(prompt) + sum(a + 1 for a in got["accept_lens"])


def test_predictable_pair_continues_cyclically_and_accepts_everything():
    """sigma = 0: the target's successor of token t is t+1 (mod V) and the draft proposes exactly
    that at rank 0, so every iteration accepts a full root path."""
    cfg = get_config("cfg1")
    tree = cfg["tree_template"]
    Wt, Wd = predictable_pair(cfg, 0, sigma=0.0, cache=True)
    prompt = np.array([990, 3, 997, 998])
    n = 13
    got = oracle.generate_speculative(cfg, Wt, Wd, prompt, n, tree.parent, tree.rank, tree.topk_per_depth)
    assert got["tokens"] == [(999 + i) % 1000 for i in range(n)]
    assert got["tokens"] == oracle.greedy_reference(cfg, Wt, prompt, n)
    assert all(a == tree.depth for a in got["accept_lens"])
    assert oracle.mean_tokens_per_iteration(got["accept_lens"]) == tree.depth + 1


def test_noisy_draft_accepts_partially_and_stays_lossless():
    cfg = get_config("cfg1")
    tree = cfg["tree_template"]
    Wt, Wd = predictable_pair(cfg, 0, sigma=5.0, cache=True)
    prompt = np.arange(5, 13)
    got = oracle.generate_speculative(cfg, Wt, Wd, prompt, 30, tree.parent, tree.rank, tree.topk_per_depth)
    assert got["tokens"] == [(13 + i) % 1000 for i in range(30)]
    assert len(set(got["accept_lens"])) == tree.depth + 1        # 0, 1 and 2 all occur


def test_incremental_drafts_equal_drafts_from_scratch():
    """Every tree the loop drafts (catch-up rows of the accepted path only, draft cache kept from
    earlier iterations) equals the tree drafted from an empty draft cache with all committed
    positions as catch-up rows and features from a fresh target prefill."""
    cfg = _nano()
    Wt = target_weights(cfg, 5, norm_gain="random", cache=True)
    Wd = eagle_weights(cfg, 5, norm_gain="random", cache=True)
    prompt = np.array([4, 44, 17])
    got = oracle.generate_speculative(cfg, Wt, Wd, prompt, 8, TREE.parent, TREE.rank, TREE.topk_per_depth)
    toks = list(prompt) + got["tokens"]
    C = len(prompt)
    for it, (a, tree_tokens) in enumerate(zip(got["accept_lens"], got["trees"])):
        ctx = toks[:C]
        tc = oracle.KVCache(cfg["n_layers"], cfg["n_heads"], 64, cfg["head_dim"])
        feats, _ = oracle.prefill(cfg, Wt, tc, ctx)
        dc = oracle.KVCache(cfg["K"], cfg["n_heads"], 64, cfg["head_dim"])
        ref = oracle.eagle_expand(cfg, Wt, Wd, dc, C, feats, np.asarray(ctx[1:] + [toks[C]]), TREE.parent,
                                  TREE.rank, TREE.topk_per_depth)
        np.testing.assert_array_equal(tree_tokens, ref["tokens"], err_msg=f"iteration {it}")
        C += a + 1


def test_statistics_by_hand():
    a = [2, 2, 0, 1, 3, 0]
    assert oracle.mean_tokens_per_iteration(a) == pytest.approx((3 + 3 + 1 + 2 + 4 + 1) / 6)
    # a>=0: 6, a>=1: 4, a>=2: 3, a>=3: 1, a>=4: 0
    al = oracle.n_alpha(a, 5)
    assert al[:4] == pytest.approx([4 / 6, 3 / 4, 1 / 3, 0.0])
    assert np.isnan(al[4])


def test_chain_template_statistics_follow_the_draft_quality():
    """Chain drafting (one candidate per depth): a perfect draft has alpha_n = 1 for every n."""
    cfg = get_config("cfg1")
    ch = chain_tree(3)
    Wt, Wd = predictable_pair(cfg, 0, sigma=0.0, cache=True)
    got = oracle.generate_speculative(cfg, Wt, Wd, np.array([1, 2, 3]), 12, ch.parent, ch.rank, ch.topk_per_depth)
    assert oracle.n_alpha(got["accept_lens"], 3) == [1.0, 1.0, 1.0]
