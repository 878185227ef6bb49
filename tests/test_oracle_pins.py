"""Pins for the CPU oracle: each part is checked against something other than itself.

The paper prints no worked numeric example for the draft-then-verify path, so
the pins are definitions (sequential decoding, Eq. 1), a library
implementation of the Llama architecture, closed forms, brute force on small
inputs, and the losslessness property of section 2.2.
"""
import itertools

import numpy as np
import pytest

import oracle
from oracle import (KVCache, accept_greedy, ancestor_mask, attention_row, commit_path, decode_one,
                    eagle_expand, eagle_rows, greedy_reference, iteration_eagle, medusa_expand,
                    prefill, rmsnorm, rope_rotate, silu, softmax, topk_desc, tree_depths,
                    verify_tree)
from koala_synth import get_config, target_weights, eagle_weights, tensor_uniform_int
from koala_synth.trees import make_tree, chain_tree

from helpers import NANO, nano_weights, nano_tree


# ----------------------------------------------------------------------------- closed forms
def test_rmsnorm_closed_forms():
    x = np.full((3, 8), 2.0)
    g = np.arange(1.0, 9.0)
    np.testing.assert_allclose(rmsnorm(x, g, 1e-6), np.tile(g * 2.0 / np.sqrt(4.0 + 1e-6), (3, 1)), rtol=1e-14)
    rng = np.random.default_rng(0)
    y = rng.standard_normal((4, 16))
    out = rmsnorm(y, np.ones(16), 0.0)
    np.testing.assert_allclose(np.mean(out * out, -1), 1.0, rtol=1e-12)          # unit mean square
    np.testing.assert_allclose(rmsnorm(7.0 * y, np.ones(16), 0.0), out, rtol=1e-12)  # scale invariant
    # eps is added to the mean square, inside the root
    np.testing.assert_allclose(rmsnorm(np.zeros((1, 4)) + 1e-3, np.ones(4), 1.0), 1e-3 / np.sqrt(1e-6 + 1.0))


def test_silu_softmax_closed_forms():
    x = np.linspace(-5, 5, 11)
    np.testing.assert_allclose(silu(x) - silu(-x), x, atol=1e-14)
    assert silu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(silu(np.array([1.0])), 1.0 / (1.0 + np.exp(-1.0)))
    s = np.array([[1.0, 2.0, 3.0], [1000.0, 1000.0, 1000.0]])
    p = softmax(s)
    np.testing.assert_allclose(p.sum(-1), 1.0)
    np.testing.assert_allclose(p[1], 1.0 / 3.0)
    np.testing.assert_allclose(p[0, 2] / p[0, 0], np.exp(2.0))


def test_rope_rotation_properties():
    rng = np.random.default_rng(1)
    q = rng.standard_normal((2, 16))
    k = rng.standard_normal((2, 16))
    np.testing.assert_array_equal(rope_rotate(q, 0, 10000.0), q)                    # position 0: identity
    np.testing.assert_allclose(np.linalg.norm(rope_rotate(q, 37, 10000.0), axis=-1),
                               np.linalg.norm(q, axis=-1), rtol=1e-12)
    # scores depend on the position difference only
    a = np.sum(rope_rotate(q, 5, 1e4) * rope_rotate(k, 2, 1e4), -1)
    b = np.sum(rope_rotate(q, 105, 1e4) * rope_rotate(k, 102, 1e4), -1)
    np.testing.assert_allclose(a, b, rtol=1e-9)
    # head_dim 2: one pair rotated by angle = pos (frequency base^0 = 1), counter-clockwise
    v = rope_rotate(np.array([[1.0, 0.0]]), 0.5, 10000.0)
    np.testing.assert_allclose(v, [[np.cos(0.5), np.sin(0.5)]], rtol=1e-12)
    # head_dim 4: pairs are (0,2) and (1,3); second frequency is base^(-2/4)
    w = rope_rotate(np.array([[0.0, 1.0, 0.0, 0.0]]), 3.0, 100.0)
    np.testing.assert_allclose(w, [[0.0, np.cos(0.3), 0.0, np.sin(0.3)]], atol=1e-12)
    # equivalent complex-multiplication form
    z = (q[:, :8] + 1j * q[:, 8:]) * np.exp(1j * 11 * 10000.0 ** (-2.0 * np.arange(8) / 16))
    np.testing.assert_allclose(rope_rotate(q, 11, 10000.0), np.concatenate([z.real, z.imag], -1), rtol=1e-12)


def test_attention_row_special_cases():
    rng = np.random.default_rng(2)
    nh, dh, cap = 2, 4, 6
    kc = rng.standard_normal((nh, cap, dh))
    vc = rng.standard_normal((nh, cap, dh))
    q = rng.standard_normal((nh, dh))
    # zero query -> all scores equal -> plain average of the visible values
    np.testing.assert_allclose(attention_row(np.zeros((nh, dh)), kc, vc, [0, 2, 5]),
                               vc[:, [0, 2, 5], :].mean(1), rtol=1e-12)
    # one visible slot -> that value
    np.testing.assert_allclose(attention_row(q, kc, vc, [3]), vc[:, 3, :], rtol=1e-12)
    # explicit loops
    slots = [0, 1, 4]
    ref = np.zeros((nh, dh))
    for h in range(nh):
        s = [sum(q[h, d] * kc[h, j, d] for d in range(dh)) / 2.0 for j in slots]   # sqrt(4) = 2
        e = [np.exp(v - max(s)) for v in s]
        for j, w in zip(slots, e):
            ref[h] += w / sum(e) * vc[h, j]
    np.testing.assert_allclose(attention_row(q, kc, vc, slots), ref, rtol=1e-12)


# ----------------------------------------------------------------------------- library pin
def test_target_matches_library_llama():
    """The oracle's sequential decoding equals the `transformers` Llama
    implementation (the architecture of the paper's Vicuna targets) with the
    same weights, on a causal sequence."""
    torch = pytest.importorskip("torch")
    tf = pytest.importorskip("transformers")
    Wt, _, _ = nano_weights()
    c = tf.LlamaConfig(hidden_size=NANO["hidden"], intermediate_size=NANO["ffn"],
                       num_hidden_layers=NANO["n_layers"], num_attention_heads=NANO["n_heads"],
                       num_key_value_heads=NANO["n_heads"], vocab_size=NANO["vocab"],
                       rms_norm_eps=NANO["rms_eps"], rope_theta=NANO["rope_base"],
                       max_position_embeddings=64, attention_bias=False, mlp_bias=False,
                       tie_word_embeddings=False, head_dim=NANO["head_dim"])
    m = tf.LlamaForCausalLM(c).double().eval()
    name_map = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj",
                "wo": "self_attn.o_proj", "wgate": "mlp.gate_proj", "wup": "mlp.up_proj",
                "wdown": "mlp.down_proj", "in_norm": "input_layernorm",
                "post_norm": "post_attention_layernorm"}
    sd = {"model.embed_tokens.weight": Wt.f32("embed"), "lm_head.weight": Wt.f32("lm_head"),
          "model.norm.weight": Wt.f32("final_norm")}
    for l in range(NANO["n_layers"]):
        for k, v in name_map.items():
            sd[f"model.layers.{l}.{v}.weight"] = Wt.f32(f"layers.{l}.{k}")
    missing = m.load_state_dict({k: torch.tensor(v, dtype=torch.float64) for k, v in sd.items()}, strict=False)
    assert not [k for k in missing.missing_keys if "rotary" not in k]
    toks = tensor_uniform_int(5, "lib_tokens", (12,), 0, NANO["vocab"])
    with torch.no_grad():
        out = m(torch.tensor(toks[None].astype(np.int64)), output_hidden_states=True)
    cache = KVCache(NANO["n_layers"], NANO["n_heads"], 16, NANO["head_dim"])
    feats, logits = prefill(NANO, Wt, cache, toks)
    # the library builds its rotary tables in fp32, hence 1e-6-level differences on O(1) values
    np.testing.assert_allclose(logits, out.logits[0].numpy(), rtol=0, atol=3e-5)
    np.testing.assert_allclose(feats, out.hidden_states[-1][0].numpy(), rtol=0, atol=3e-5)
    assert np.abs(logits).max() > 1.0


# ----------------------------------------------------------------------------- tree structure
def _brute_mask(parent):
    T = len(parent)
    m = np.zeros((T, T), bool)
    for i in range(T):
        for j in range(T):
            k = i
            while k != -1:
                if k == j:
                    m[i, j] = True
                k = parent[k]
    return m


def _random_parent(rng, T):
    return np.array([-1] + [int(rng.integers(0, i)) for i in range(1, T)], np.int32)


def test_mask_is_ancestor_closure():
    rng = np.random.default_rng(3)
    trees = [get_config(n)["tree_template"].parent for n in ("cfg1", "cfg2", "cfg3", "cfg4")]
    trees += [_random_parent(rng, T) for T in (1, 2, 5, 17, 64)]
    trees.append(chain_tree(6).parent)
    for parent in trees:
        m = ancestor_mask(parent)
        np.testing.assert_array_equal(m, _brute_mask(parent))
        d = tree_depths(parent)
        np.testing.assert_array_equal(m.sum(1), d + 1)          # a node sees depth+1 nodes
        assert d[0] == 0 and all(d[i] == d[parent[i]] + 1 for i in range(1, len(parent)))


def test_templates_match_benchmark_node_counts():
    for name, T, D in (("cfg1", 7, 2), ("cfg2", 26, 5), ("cfg3", 64, 4), ("cfg4", 60, 6), ("cfg5", 60, 6)):
        t = get_config(name)["tree_template"]
        assert t.n_nodes == T and t.depth == D and int(tree_depths(t.parent).max()) == D
        assert all(t.parent[i] < i for i in range(1, T))
        # siblings have distinct ranks below that depth's k
        seen = set()
        for i in range(1, T):
            key = (int(t.parent[i]), int(t.rank[i]))
            assert key not in seen
            seen.add(key)
            assert t.rank[i] < t.topk_per_depth[tree_depths(t.parent)[i] - 1]


# ----------------------------------------------------------------------------- top-k / argmax
def test_topk_and_argmax_against_full_sort():
    rng = np.random.default_rng(4)
    for _ in range(20):
        x = rng.integers(0, 6, size=40).astype(np.float64)       # many ties
        order = sorted(range(40), key=lambda i: (-x[i], i))
        for k in (1, 2, 5, 10):
            np.testing.assert_array_equal(topk_desc(x, k), order[:k])
        assert int(np.argmax(x)) == order[0]


# ----------------------------------------------------------------------------- verification
def _nano_state(n_ctx=9, seed=0):
    Wt, Wd, Wm = nano_weights(seed)
    toks = tensor_uniform_int(seed + 10, "ctx", (n_ctx + 1,), 0, NANO["vocab"])
    cache = KVCache(NANO["n_layers"], NANO["n_heads"], 48, NANO["head_dim"])
    feats, logits = prefill(NANO, Wt, cache, toks[:n_ctx])
    return Wt, Wd, Wm, toks, cache, feats, logits


def test_verify_equals_sequential_decoding_on_every_path():
    """Eq. 3 must give, for every tree node, the distribution Eq. 1 gives after
    feeding the context and the node's root-to-node path one token at a time."""
    Wt, _, _, toks, cache, _, _ = _nano_state()
    C = 9
    tree = nano_tree()
    T = tree.n_nodes
    tt = tensor_uniform_int(7, "tree_tokens", (T,), 0, NANO["vocab"])
    base = cache.copy()
    feat, logits, greedy = verify_tree(NANO, Wt, cache, C, tt, tree.parent)
    for i in range(T):
        path = []
        k = i
        while k != -1:
            path.append(k)
            k = tree.parent[k]
        path.reverse()
        c2 = base.copy()
        for j, node in enumerate(path):
            f, l = decode_one(NANO, Wt, c2, C + j, int(tt[node]))
        np.testing.assert_allclose(logits[i], l, rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(feat[i], f, rtol=1e-9, atol=1e-11)
        assert greedy[i] == int(np.argmax(l))


def test_single_node_tree_is_a_decode_step():
    Wt, _, _, toks, cache, _, _ = _nano_state()
    c2 = cache.copy()
    feat, logits, _ = verify_tree(NANO, Wt, cache, 9, [int(toks[9])], np.array([-1]))
    f, l = decode_one(NANO, Wt, c2, 9, int(toks[9]))
    np.testing.assert_array_equal(logits[0], l)
    np.testing.assert_array_equal(feat[0], f)


def test_verify_fp32_close_to_fp64():
    cfg = get_config("cfg1")
    Wt = target_weights(cfg, 0, cache=True)
    toks = tensor_uniform_int(1, "ctx", (12,), 0, cfg["vocab"])
    out = []
    for dt in (np.float64, np.float32):
        cache = KVCache(cfg["n_layers"], cfg["n_heads"], 32, cfg["head_dim"], dt)
        prefill(cfg, Wt, cache, toks[:8], dt)
        out.append(verify_tree(cfg, Wt, cache, 8, toks[:7], cfg["tree_template"].parent, dt)[1])
    err = np.abs(out[0] - out[1]).max(-1) / np.abs(out[0]).max(-1)
    assert err.max() < 1e-4


# ----------------------------------------------------------------------------- acceptance
def _brute_accept(tt, g, parent):
    """Deepest node whose whole root path matches; the walk's answer must be that node."""
    best = (0, [0])
    for i in range(len(parent)):
        path = []
        k = i
        while k != -1:
            path.append(k)
            k = parent[k]
        path.reverse()
        if all(tt[c] == g[p] for p, c in zip(path[:-1], path[1:])):
            if len(path) - 1 > best[0]:
                best = (len(path) - 1, path)
    return best


def test_accept_equals_brute_force_longest_match():
    rng = np.random.default_rng(5)
    for name in ("cfg1", "cfg2", "cfg3", "cfg4"):
        t = get_config(name)["tree_template"]
        T = t.n_nodes
        depth = tree_depths(t.parent)
        for trial in range(30):
            # small alphabet so that matches of every length occur; siblings kept distinct
            tt = np.zeros(T, np.int64)
            g = rng.integers(0, 4, T)
            for u in range(T):
                kids = [c for c in range(T) if t.parent[c] == u]
                vals = rng.permutation(max(4, len(kids)))[: len(kids)]
                for c, v in zip(kids, vals):
                    tt[c] = v
            a, path, nxt = accept_greedy(tt, g, t.parent)
            ba, bpath = _brute_accept(tt, g, t.parent)
            assert (a, path) == (ba, bpath)
            assert nxt == g[path[-1]] and a == depth[path[-1]]


def test_accept_planted_paths_of_every_length():
    t = get_config("cfg2")["tree_template"]
    T, D = t.n_nodes, t.depth
    depth = tree_depths(t.parent)
    leaf = [i for i in range(T) if depth[i] == D][-1]
    chain = []
    k = leaf
    while k != -1:
        chain.append(k)
        k = t.parent[k]
    chain.reverse()
    for a_want in range(D + 1):
        tt = 100 + np.arange(T)                   # all distinct
        g = np.full(T, 7)                          # matches nothing
        for p, c in list(zip(chain[:-1], chain[1:]))[:a_want]:
            g[p] = tt[c]
        a, path, nxt = accept_greedy(tt, g, t.parent)
        assert a == a_want and path == chain[: a_want + 1] and nxt == g[chain[a_want]]


def test_accept_chain_counts_leading_matches():
    """On a chain the rule is the one of section 2.2: keep drafted tokens up to
    the first mismatch, then append the target's token."""
    t = chain_tree(5)
    tt = np.array([9, 1, 2, 3, 4, 5])
    g = np.array([1, 2, 3, 0, 5, 6])              # x1..x3 match, x4 does not
    a, path, nxt = accept_greedy(tt, g, t.parent)
    assert (a, path, nxt) == (3, [0, 1, 2, 3], 0)
    a, path, nxt = accept_greedy(tt, np.array([1, 2, 3, 4, 5, 6]), t.parent)
    assert (a, nxt) == (5, 6)                      # all accepted: bonus token from q_{t+1}
    a, path, nxt = accept_greedy(tt, np.array([8, 2, 3, 4, 5, 6]), t.parent)
    assert (a, path, nxt) == (0, [0], 8)


def test_accept_duplicate_siblings_lowest_index_wins():
    parent = np.array([-1, 0, 0, 1, 2])
    tt = np.array([0, 5, 5, 6, 7])
    g = np.array([5, 9, 7, 0, 0])
    a, path, _ = accept_greedy(tt, g, parent)
    assert path == [0, 1] and a == 1


# ----------------------------------------------------------------------------- commit
def test_commit_then_decode_equals_sequential():
    Wt, _, _, toks, cache, _, _ = _nano_state()
    C = 9
    tree = nano_tree()
    tt = tensor_uniform_int(8, "tree_tokens", (tree.n_nodes,), 0, NANO["vocab"])
    path = [0, 2, 6]                                       # a valid root->node path of nano_tree
    assert tree.parent[2] == 0 and tree.parent[6] == 2
    base = cache.copy()
    verify_tree(NANO, Wt, cache, C, tt, tree.parent)
    C2 = commit_path(cache, C, path)
    assert C2 == C + 3
    f1, l1 = decode_one(NANO, Wt, cache, C2, 11)
    seq = base.copy()
    for j, node in enumerate(path):
        decode_one(NANO, Wt, seq, C + j, int(tt[node]))
    f2, l2 = decode_one(NANO, Wt, seq, C + 3, 11)
    np.testing.assert_allclose(l1, l2, rtol=1e-9, atol=1e-11)
    for l in range(NANO["n_layers"]):
        np.testing.assert_allclose(cache.k[l][:, :C2], seq.k[l][:, :C2], rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(cache.v[l][:, :C2], seq.v[l][:, :C2], rtol=1e-9, atol=1e-12)


# ----------------------------------------------------------------------------- draft heads
def _draft_prefill(Wt, Wd, feats, toks, n):
    """Draft cache rows 0..n-1 one row at a time: row i = (feat_i, x_{i+1}) at position i."""
    dc = KVCache(NANO["K"], NANO["n_heads"], 48, NANO["head_dim"])
    outs = []
    for i in range(n):
        outs.append(eagle_rows(NANO, Wt, Wd, dc, [int(toks[i + 1])], feats[i:i + 1], [i], [i], [range(i + 1)])[0])
    return dc, outs


def test_eagle_tree_expansion_equals_chain_drafting_per_path():
    Wt, Wd, _, toks, cache, feats, _ = _nano_state()
    C = 9
    tree = nano_tree()
    # draft cache already holds rows 0..C-3; the m = 2 newest rows are caught up by eagle_expand
    dc, _ = _draft_prefill(Wt, Wd, feats, toks, C - 2)
    out = eagle_expand(NANO, Wt, Wd, dc, C, feats[C - 2:C], toks[C - 1:C + 1], tree.parent, tree.rank,
                       tree.topk_per_depth)
    tt = out["tokens"]
    assert tt[0] == toks[C]
    lm = Wt.f32("lm_head").astype(np.float64)
    depth = tree_depths(tree.parent)
    for leaf in range(tree.n_nodes):
        path = []
        k = leaf
        while k != -1:
            path.append(k)
            k = tree.parent[k]
        path.reverse()
        # chain drafting: feed (token, previous predicted feature) one row at a time
        dc2, outs = _draft_prefill(Wt, Wd, feats, toks, C)        # rows 0..C-1 sequentially
        f = outs[C - 1]
        for d, node in enumerate(path):
            if d > 0:
                f = eagle_rows(NANO, Wt, Wd, dc2, [int(tt[node])], f[None], [C - 1 + d], [C - 1 + d],
                               [range(C + d)])[0]
            if node in out["f_hat"]:
                np.testing.assert_allclose(out["f_hat"][node], f, rtol=1e-9, atol=1e-11)
            kids = [c for c in range(tree.n_nodes) if tree.parent[c] == node]
            if kids:
                order = sorted(range(NANO["vocab"]), key=lambda v: (-(lm @ f)[v], v))
                for c in kids:
                    assert tt[c] == order[tree.rank[c]]
                    np.testing.assert_allclose(out["scores"][c], (lm @ f)[tt[c]], rtol=1e-9)


def test_medusa_tokens_depend_on_depth_and_rank_only():
    Wt, _, Wm, toks, cache, feats, _ = _nano_state()
    tree = make_tree([3, 2, 2], [1, 3, 5, 6])
    out = medusa_expand(NANO, Wt, Wm, feats[-1], int(toks[9]), tree.parent, tree.rank, tree.topk_per_depth)
    depth = tree_depths(tree.parent)
    lm = Wt.f32("lm_head").astype(np.float64)
    assert out["tokens"][0] == toks[9]
    for j in range(3):
        x = feats[-1].astype(np.float64)
        for k in range(NANO["K"]):
            y = Wm.f32(f"medusa.{j}.{k}").astype(np.float64) @ x
            x = x + y / (1.0 + np.exp(-y))
        order = sorted(range(NANO["vocab"]), key=lambda v: (-(lm @ x)[v], v))
        for i in range(1, tree.n_nodes):
            if depth[i] == j + 1:
                assert out["tokens"][i] == order[tree.rank[i]]
    # K = 0 blocks would make every head identical to the target's own LM head on the feature
    cfg0 = dict(NANO, K=0)
    out0 = medusa_expand(cfg0, Wt, Wm, feats[-1], 0, tree.parent, tree.rank, tree.topk_per_depth)
    np.testing.assert_allclose(out0["logits"][0], lm @ feats[-1], rtol=1e-12)


# ----------------------------------------------------------------------------- losslessness
@pytest.mark.parametrize("mode", ["draft", "adversarial", "planted"])
def test_iterations_emit_plain_greedy_decoding(mode):
    """Whatever the draft proposes, the emitted tokens are those of greedy
    autoregressive decoding (section 2.2: results align with the target)."""
    cfg = get_config("cfg1")
    Wt = target_weights(cfg, 0, cache=True)
    Wd = eagle_weights(cfg, 0, cache=True)
    tree = cfg["tree_template"]
    n = 12
    prompt = tensor_uniform_int(1, "ctx", (cfg["ctx"],), 0, cfg["vocab"])[:n]
    want = greedy_reference(cfg, Wt, prompt, 10)
    tc = KVCache(cfg["n_layers"], cfg["n_heads"], 64, cfg["head_dim"])
    dc = KVCache(cfg["K"], cfg["n_heads"], 64, cfg["head_dim"])
    feats, logits = prefill(cfg, Wt, tc, prompt)
    root = int(np.argmax(logits[-1]))
    assert root == want[0]
    C = n
    feat_in, tok_in = feats, np.concatenate([prompt[1:], [root]]).astype(np.int32)
    got = [root]
    rng = np.random.default_rng(0)
    accepted = []
    while len(got) < 10:
        def override(tt, got=got):
            if mode == "draft":
                return tt
            if mode == "adversarial":
                tt[1:] = rng.integers(0, cfg["vocab"], len(tt) - 1)
                return tt
            # planted: put the true continuation on the left-most path as far as it is known
            cur, j = 0, len(got)
            while j < len(want):
                kids = [c for c in range(len(tt)) if tree.parent[c] == cur]
                if not kids:
                    break
                tt[kids[0]] = want[j]
                for c in kids[1:]:
                    tt[c] = (want[j] + 1 + c) % cfg["vocab"]
                cur, j = kids[0], j + 1
            return tt
        it = iteration_eagle(cfg, Wt, Wd, tc, dc, C, feat_in, tok_in, tree.parent, tree.rank,
                             tree.topk_per_depth, override_tokens=override)
        got += it["emitted"]
        accepted.append(it["accept_len"])
        C, feat_in, tok_in = it["C"], it["feat_in"], it["tok_in"]
        assert C == n + len(got) - 1
    assert got[:10] == want[:10]
    if mode == "planted":
        assert max(accepted) == tree.depth         # full-depth acceptance was exercised


# ----------------------------------------------------------------------------- cache storage hook
def test_cache_store_hook_touches_new_keys_and_values_only():
    """KVCache.store models the cache's storage format.  Pins: no hook and the identity hook give the same
    bits; the hook a -> a/2 (exact in binary) gives exactly what halving W_k and W_v gives without a hook
    (keys and values are linear in those matrices and the rotation is linear), which fails if the hook also
    reached the queries, missed the keys or the values, was applied twice, or touched context rows."""
    Wt, _, _, toks, cache, _, _ = _nano_state()
    C = 9
    tree = nano_tree()
    tt = tensor_uniform_int(7, "tree_tokens", (tree.n_nodes,), 0, NANO["vocab"])
    plain, ident, halved_store, halved_w = cache.copy(), cache.copy(), cache.copy(), cache.copy()
    ident.store = lambda a: a
    halved_store.store = lambda a: 0.5 * a
    ref = verify_tree(NANO, Wt, plain, C, tt, tree.parent)
    got = verify_tree(NANO, Wt, ident, C, tt, tree.parent)
    for r, g in zip(ref[:2], got[:2]):
        np.testing.assert_array_equal(r, g)
    for l in range(NANO["n_layers"]):
        np.testing.assert_array_equal(plain.k[l], ident.k[l])
        np.testing.assert_array_equal(plain.v[l], ident.v[l])

    class HalvedKV:
        """The same weights with every W_k and W_v multiplied by 1/2."""
        def f32(self, name):
            w = Wt.f32(name)
            return 0.5 * w if name.endswith(".wk") or name.endswith(".wv") else w
    a = verify_tree(NANO, Wt, halved_store, C, tt, tree.parent)
    b = verify_tree(NANO, HalvedKV(), halved_w, C, tt, tree.parent)
    assert np.abs(a[1] - ref[1]).max() > 1e-6              # the hook changed the result at all
    np.testing.assert_allclose(a[0], b[0], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(a[1], b[1], rtol=1e-12, atol=1e-14)
    for l in range(NANO["n_layers"]):
        np.testing.assert_allclose(halved_store.k[l], halved_w.k[l], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(halved_store.v[l], halved_w.v[l], rtol=1e-12, atol=1e-14)
        np.testing.assert_array_equal(halved_store.k[l][:, :C], cache.k[l][:, :C])   # context rows as given
        np.testing.assert_array_equal(halved_store.v[l][:, :C], cache.v[l][:, :C])
    # layer 0 sees the same input in both runs, so its stored tree rows are exactly half the exact ones
    np.testing.assert_array_equal(halved_store.k[0][:, C:C + tree.n_nodes], 0.5 * plain.k[0][:, C:C + tree.n_nodes])
    np.testing.assert_array_equal(halved_store.v[0][:, C:C + tree.n_nodes], 0.5 * plain.v[0][:, C:C + tree.n_nodes])
