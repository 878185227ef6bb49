"""Pins for the oracle's non-greedy drafting and acceptance (sections 2.2 and 4.4).

What fixes the rule from outside: the emitted tokens must be distributed exactly as samples of
the target (checked by Monte Carlo on small vocabularies, for a chain and for trees with several
children), the closed-form special cases d = q (always accept), disjoint supports (always
reject, replacement from q), a one-hot draft (accept with probability q(x)), and the textbook
frequencies of draws without replacement."""
import numpy as np
import pytest

import oracle
from koala_synth import make_tree, chain_tree


def _rand_dist(rng, V, sharp=1.0):
    return oracle.softmax_t(rng.normal(size=V) * sharp)


def _simulate(tree, q_of, d_of, n_trials, rng, V):
    """Draft by sampling children from d_of(prefix tokens), accept with q_of(prefix tokens).
    Returns the emitted token sequences."""
    T = tree.n_nodes
    ch = [sorted(k, key=lambda c: tree.rank[c]) for k in oracle.children_lists(tree.parent)]
    outs = []
    for _ in range(n_trials):
        tokens = np.zeros(T, np.int64)
        prefix = {0: ()}
        q_rows, d_rows = {}, {}
        for u in range(T):                                   # BFS order: parents first
            q_rows[u] = q_of(prefix[u])
            if ch[u]:
                d_rows[u] = d_of(prefix[u])
                draws = oracle.draw_without_replacement(d_rows[u], rng.random(len(ch[u])))
                for c, x in zip(ch[u], draws):
                    tokens[c] = x
                    prefix[c] = prefix[u] + (x,)
        a, path, nxt = oracle.accept_sample(tokens, tree.parent, tree.rank, q_rows, d_rows, rng.random(T),
                                            rng.random(T))
        outs.append(tuple(int(tokens[p]) for p in path[1:]) + (nxt,))
    return outs


def _tables(V, seed):
    rng = np.random.default_rng(seed)
    q0, d0 = _rand_dist(rng, V, 1.5), _rand_dist(rng, V, 1.5)
    q1 = {x: _rand_dist(rng, V, 1.5) for x in range(V)}
    d1 = {x: _rand_dist(rng, V, 1.5) for x in range(V)}
    q_of = lambda pre: q0 if len(pre) == 0 else q1[pre[-1]] if len(pre) == 1 else q0
    d_of = lambda pre: d0 if len(pre) == 0 else d1[pre[-1]]
    return q0, q1, q_of, d_of


@pytest.mark.parametrize("tree", [chain_tree(2), make_tree([2, 2], [1, 2, 3]), make_tree([3], [1, 3])],
                         ids=["chain2", "tree_2_2", "star3"])
def test_emitted_tokens_are_distributed_as_the_target(tree):
    V, n = 5, 40000
    q0, q1, q_of, d_of = _tables(V, 11)
    rng = np.random.default_rng(5)
    outs = _simulate(tree, q_of, d_of, n, rng, V)
    first = np.bincount([o[0] for o in outs], minlength=V) / n
    sd = np.sqrt(q0 * (1 - q0) / n)
    assert np.all(np.abs(first - q0) < 4.5 * sd), (first, q0)
    # joint of the first two tokens: q0(x1) * q1[x1](x2)  (every trial emits at least one token;
    # those that emit two or more are a biased subset, so condition on nothing: extend by sampling)
    pair = np.zeros((V, V))
    for o in outs:
        x1 = o[0]
        x2 = o[1] if len(o) > 1 else oracle.inverse_cdf(q1[x1], rng.random())
        pair[x1, x2] += 1
    pair /= n
    want = np.array([[q0[a] * q1[a][b] for b in range(V)] for a in range(V)])
    sd2 = np.sqrt(want * (1 - want) / n)
    assert np.all(np.abs(pair - want) < 4.5 * sd2 + 1e-9)


def test_identical_distributions_accept_everything():
    tree = chain_tree(3)
    rng = np.random.default_rng(1)
    p = _rand_dist(rng, 7)
    for _ in range(200):
        toks = np.array([0] + [oracle.inverse_cdf(p, rng.random()) for _ in range(3)])
        a, path, nxt = oracle.accept_sample(toks, tree.parent, tree.rank, {i: p for i in range(4)},
                                            {i: p for i in range(4)}, rng.random(4), rng.random(4))
        assert a == 3 and path == [0, 1, 2, 3]


def test_disjoint_supports_reject_and_resample_from_the_target():
    tree = make_tree([2], [1, 2])
    q = np.array([0.5, 0.5, 0, 0, 0, 0.0])
    d = np.array([0, 0, 0.25, 0.25, 0.25, 0.25])
    rng = np.random.default_rng(2)
    cnt = np.zeros(6)
    for _ in range(4000):
        draws = oracle.draw_without_replacement(d, rng.random(2))
        toks = np.array([0] + draws)
        a, path, nxt = oracle.accept_sample(toks, tree.parent, tree.rank, {0: q, 1: q, 2: q}, {0: d}, rng.random(3),
                                            rng.random(3))
        assert a == 0 and path == [0]
        cnt[nxt] += 1
    assert cnt[2:].sum() == 0 and abs(cnt[0] / 4000 - 0.5) < 0.04


def test_one_hot_draft_is_kept_with_the_target_probability():
    """d = point mass at x: keep x with probability q(x), otherwise draw from q without x."""
    tree = chain_tree(1)
    q = np.array([0.1, 0.6, 0.3])
    d = np.array([0.0, 1.0, 0.0])
    toks = np.array([0, 1])
    qs = {0: q, 1: q}
    a, _, _ = oracle.accept_sample(toks, tree.parent, tree.rank, qs, {0: d}, [0, 0.59], [0, 0])
    assert a == 1
    a, _, nxt = oracle.accept_sample(toks, tree.parent, tree.rank, qs, {0: d}, [0, 0.61], [0.2, 0])
    assert a == 0 and nxt == 0          # residual = (0.25, 0, 0.75): u = 0.2 -> token 0
    a, _, nxt = oracle.accept_sample(toks, tree.parent, tree.rank, qs, {0: d}, [0, 0.61], [0.3, 0])
    assert a == 0 and nxt == 2


def test_section_2_2_worked_example_by_hand():
    """q = (.5,.3,.2), d = (.2,.2,.6), drafted token 2: keep with probability .2/.6 = 1/3;
    on rejection the replacement comes from norm(max(0, q-d)) = (.75, .25, 0)."""
    tree = chain_tree(1)
    q, d = np.array([0.5, 0.3, 0.2]), np.array([0.2, 0.2, 0.6])
    toks = np.array([0, 2])
    a, _, _ = oracle.accept_sample(toks, tree.parent, tree.rank, {0: q, 1: q}, {0: d}, [0, 0.33], [0, 0])
    assert a == 1
    a, _, nxt = oracle.accept_sample(toks, tree.parent, tree.rank, {0: q, 1: q}, {0: d}, [0, 0.34], [0.74, 0])
    assert (a, nxt) == (0, 0)
    a, _, nxt = oracle.accept_sample(toks, tree.parent, tree.rank, {0: q, 1: q}, {0: d}, [0, 0.34], [0.76, 0])
    assert (a, nxt) == (0, 1)


def test_draws_without_replacement_have_textbook_frequencies():
    rng = np.random.default_rng(3)
    d = np.array([0.5, 0.3, 0.15, 0.05])
    n = 40000
    first = np.zeros(4)
    pair = np.zeros((4, 4))
    for _ in range(n):
        i, j = oracle.draw_without_replacement(d, rng.random(2))
        assert i != j
        first[i] += 1
        pair[i, j] += 1
    assert np.all(np.abs(first / n - d) < 4.5 * np.sqrt(d * (1 - d) / n))
    want = np.array([[0 if i == j else d[i] * d[j] / (1 - d[i]) for j in range(4)] for i in range(4)])
    assert np.all(np.abs(pair / n - want) < 4.5 * np.sqrt(want * (1 - want) / n) + 1e-9)


def test_inverse_cdf_against_brute_force():
    rng = np.random.default_rng(4)
    for _ in range(300):
        p = rng.random(9) * (rng.random(9) > 0.3)
        if p.sum() == 0:
            continue
        u = rng.random()
        run, want = 0.0, None
        for i, v in enumerate(p):
            run += v
            if run > u * p.sum():
                want = i
                break
        assert oracle.inverse_cdf(p, u) == want
        assert p[want] > 0
    assert oracle.inverse_cdf([0.25, 0.25, 0.5], 0.0) == 0
    assert oracle.inverse_cdf([0.25, 0.25, 0.5], 0.4999) == 1
    assert oracle.inverse_cdf([0.25, 0.25, 0.5], 0.5) == 2
    assert oracle.inverse_cdf([0.0, 0.0, 0.0], 0.3) == 0            # drawn empty
    assert oracle.draw_without_replacement([0.0, 1.0, 0.0], [0.5, 0.5]) == [1, 0]


def test_sampled_draft_reduces_to_top1_at_low_temperature():
    """temperature -> 0 puts all mass on the argmax, so a chain drafted by sampling equals the
    greedy draft's rank-0 chain."""
    from helpers import NANO
    from koala_synth.weights import target_weights, eagle_weights
    cfg = dict(NANO)
    Wt = target_weights(cfg, 2, norm_gain="random", cache=True)
    Wd = eagle_weights(cfg, 2, norm_gain="random", cache=True)
    ch = chain_tree(3)
    tc = oracle.KVCache(cfg["n_layers"], cfg["n_heads"], 32, cfg["head_dim"])
    prompt = [3, 9, 27, 31]
    feats, logits = oracle.prefill(cfg, Wt, tc, prompt)
    root = int(np.argmax(logits[-1]))
    tok_in = np.array(prompt[1:] + [root])
    d1 = oracle.KVCache(cfg["K"], cfg["n_heads"], 32, cfg["head_dim"])
    d2 = oracle.KVCache(cfg["K"], cfg["n_heads"], 32, cfg["head_dim"])
    g = oracle.eagle_expand(cfg, Wt, Wd, d1, 4, feats, tok_in, ch.parent, ch.rank, ch.topk_per_depth)
    s = oracle.eagle_expand_sample(cfg, Wt, Wd, d2, 4, feats, tok_in, ch.parent, ch.rank,
                                   np.random.default_rng(0).random(4), temperature=1e-7)
    np.testing.assert_array_equal(g["tokens"], s["tokens"])
    for u in (0, 1, 2):
        np.testing.assert_allclose(g["logits"][u], s["logits"][u], rtol=1e-12)


def test_sampled_generation_reduces_to_greedy_generation_at_low_temperature():
    """temperature -> 0: every distribution is one-hot, a drafted token is kept iff it is the target's
    argmax and the replacement is the argmax, so the loop emits plain greedy decoding."""
    from helpers import NANO
    from koala_synth.weights import target_weights, eagle_weights
    from koala_synth import make_tree
    cfg = dict(NANO)
    Wt = target_weights(cfg, 4, norm_gain="random", cache=True)
    Wd = eagle_weights(cfg, 4, norm_gain="random", cache=True)
    tree = make_tree([2, 2], [1, 2, 3])
    prompt = np.array([8, 3, 41, 7])
    rng = np.random.default_rng(9)
    uniforms = [(rng.random(tree.n_nodes), rng.random(tree.n_nodes), rng.random(tree.n_nodes)) for _ in range(16)]
    got = oracle.generate_sampled(cfg, Wt, Wd, prompt, 9, tree.parent, tree.rank, uniforms, temperature=1e-7)
    assert got["tokens"] == oracle.greedy_reference(cfg, Wt, prompt, 9)


def test_sampled_generation_with_a_perfect_draft_accepts_everything_it_can():
    """Draft distribution == target distribution along the chain (the predictable pair at sigma = 0 has
    identical one-hot-like distributions at low temperature): all chain drafts are accepted."""
    from koala_synth import get_config, predictable_pair
    cfg = get_config("cfg1")
    ch = chain_tree(3)
    Wt, Wd = predictable_pair(cfg, 0, sigma=0.0, cache=True)
    rng = np.random.default_rng(10)
    uniforms = [(rng.random(4), rng.random(4), rng.random(4)) for _ in range(8)]
    got = oracle.generate_sampled(cfg, Wt, Wd, np.array([5, 6, 7]), 12, ch.parent, ch.rank, uniforms, temperature=0.02)
    assert got["tokens"] == [(8 + i) % 1000 for i in range(12)]
    assert all(a == 3 for a in got["accept_lens"])


def test_medusa_sampled_draft_special_cases():
    """Chain template at vanishing temperature == the top-1 Medusa draft; two parents of one depth
    draw from the same distribution: equal uniforms give equal children, and the stored logits of a
    parent are those of the head of the next depth."""
    from helpers import NANO
    from koala_synth.weights import target_weights, medusa_weights
    cfg = dict(NANO, draft="medusa")
    Wt = target_weights(cfg, 6, norm_gain="random", cache=True)
    Wm = medusa_weights(cfg, 6, cache=True)
    rng = np.random.default_rng(12)
    feat = rng.normal(size=cfg["hidden"])
    ch = chain_tree(3)
    g = oracle.medusa_expand(cfg, Wt, Wm, feat, 7, ch.parent, ch.rank, ch.topk_per_depth)
    s = oracle.medusa_expand_sample(cfg, Wt, Wm, feat, 7, ch.parent, ch.rank, 3, rng.random(4), temperature=1e-7)
    np.testing.assert_array_equal(g["tokens"], s["tokens"])
    tree = make_tree([2, 2], [1, 2, 4])
    u = rng.random(tree.n_nodes)
    kids = oracle.children_lists(tree.parent)
    a, b = [x for x in range(tree.n_nodes) if tree.parent[x] == 0]           # the two depth-1 parents
    for ca, cb in zip(sorted(kids[a], key=lambda c: tree.rank[c]), sorted(kids[b], key=lambda c: tree.rank[c])):
        u[cb] = u[ca]
    s = oracle.medusa_expand_sample(cfg, Wt, Wm, feat, 7, tree.parent, tree.rank, 2, u, temperature=1.0)
    assert [s["tokens"][c] for c in sorted(kids[a])] == [s["tokens"][c] for c in sorted(kids[b])]
    np.testing.assert_array_equal(s["logits"][a], s["logits"][b])
    np.testing.assert_allclose(s["logits"][0], g["logits"][0])
    np.testing.assert_allclose(s["logits"][a], g["logits"][1])
    assert len(set(int(s["tokens"][c]) for c in kids[a])) == len(kids[a])     # without replacement


def test_inverse_cdf_definition_and_degenerate_cases():
    """Inverse CDF over ascending id against a plain loop; a distribution with no positive weight has no
    index whose running sum exceeds u * 0, and the reading for that case is the lowest id (the same
    preference as in every tie rule of this build: lower id first).  It arises when more children are
    drawn without replacement than the distribution has positive entries."""
    rng = np.random.default_rng(5)
    for _ in range(200):
        V = int(rng.integers(1, 12))
        p = rng.random(V) * (rng.random(V) < 0.7)
        u = rng.random()
        if p.sum() == 0:
            assert oracle.inverse_cdf(p, u) == 0
            continue
        run, want = 0.0, None
        for i in range(V):
            run += p[i]
            if run > u * p.sum():
                want = i
                break
        if want is not None:
            assert oracle.inverse_cdf(p, u) == want
    assert oracle.inverse_cdf(np.zeros(7), 0.3) == 0
    assert oracle.inverse_cdf(np.array([0.0, 0.0, 1.0, 0.0]), 0.999999) == 2
    # a one-hot distribution drawn three times: the one positive id, then the degenerate reading twice
    assert oracle.draw_without_replacement([0.0, 0.0, 0.0, 1.0, 0.0], [0.5, 0.5, 0.9]) == [3, 0, 0]


def test_medusa_sampled_generation_pins():
    """Non-greedy loop with Medusa-style heads.  At vanishing temperature it emits plain greedy decoding of the
    target (the method is lossless whatever the heads propose).  At temperature 1 the bookkeeping must hold:
    the committed length is the prompt plus every emitted token but the last, and every emitted token has
    positive probability under the target when the run is replayed by plain decoding."""
    from helpers import NANO
    from koala_synth.weights import target_weights, medusa_weights
    cfg = dict(NANO, draft="medusa")
    Wt = target_weights(cfg, 6, norm_gain="random", cache=True)
    Wm = medusa_weights(cfg, 6, cache=True)
    tree = make_tree([2, 2, 1], [1, 2, 3, 2])
    prompt = np.array([8, 3, 41, 7])
    rng = np.random.default_rng(19)
    uniforms = [(rng.random(tree.n_nodes), rng.random(tree.n_nodes), rng.random(tree.n_nodes)) for _ in range(24)]
    cold = oracle.generate_sampled(cfg, Wt, Wm, prompt, 11, tree.parent, tree.rank, uniforms, temperature=1e-7)
    assert cold["tokens"] == oracle.greedy_reference(cfg, Wt, prompt, 11)
    warm = oracle.generate_sampled(cfg, Wt, Wm, prompt, 11, tree.parent, tree.rank, uniforms, temperature=1.0)
    assert warm["C"] == len(prompt) + sum(a + 1 for a in warm["accept_lens"])
    assert len(warm["tokens"]) == 11 and warm["tokens"] != cold["tokens"]
    # replaying the emitted tokens through plain decoding: each had positive probability under the target
    cache = oracle.KVCache(cfg["n_layers"], cfg["n_heads"], 64, cfg["head_dim"])
    _, logits = oracle.prefill(cfg, Wt, cache, prompt)
    last, C = logits[-1], len(prompt)
    for t in warm["tokens"][:-1]:
        assert oracle.softmax_t(last, 1.0)[t] > 0
        _, last = oracle.decode_one(cfg, Wt, cache, C, t)
        C += 1
