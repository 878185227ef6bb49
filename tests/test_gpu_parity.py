"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the
same seeded inputs.  Integer results are compared exactly (greedy ids and drafted tokens
except where the oracle's own margin is below the tolerance); logits and features within
1e-4 (fp32) / 2e-2 (bf16) of the row maximum."""
import numpy as np
import pytest

import oracle
from koala_synth import tensor_uniform_int

from gpu_harness import Case, rel_err_rows, compare_logits_and_greedy, compare_draft_tokens

pytestmark = pytest.mark.gpu


def _prefilled_cfg1(n_ctx=64, **kw):
    case = Case("cfg1", max_m=64, **kw)
    prompt = tensor_uniform_int(1, "ctx", (case.cfg["ctx"],), 0, case.V)[:n_ctx]
    feats, logits = case.prefill_oracle(prompt)
    root = int(np.argmax(logits[-1]))
    return case, prompt, feats, root


# --------------------------------------------------------------------------- cfg 1 (fp32)
def test_cfg1_verify_matches_oracle():
    case, prompt, feats, root = _prefilled_cfg1()
    case.upload_kv()
    tt = case.random_tree_tokens()
    tt[0, 0] = root
    feat, logits, greedy = case.gpu_verify(tt)
    rfeat, rlogits, rgreedy = case.oracle_verify(tt)
    skipped, err = compare_logits_and_greedy(case, logits, greedy, rlogits, rgreedy)
    assert skipped == 0
    assert rel_err_rows(feat, rfeat).max() < case.tol
    # the tree rows' keys/values were written to slots C..C+T-1 of every layer
    k, v = case.download_kv()
    C = case.ctx_lens[0]
    for l in range(case.cfg["n_layers"]):
        rk = case.tc[0].k[l][:, C:C + case.T]
        rv = case.tc[0].v[l][:, C:C + case.T]
        assert np.abs(k[l, 0][:, C:C + case.T] - rk).max() < 1e-4 * np.abs(rk).max()
        assert np.abs(v[l, 0][:, C:C + case.T] - rv).max() < 1e-4 * np.abs(rv).max()
        # context rows untouched
        np.testing.assert_array_equal(k[l, 0][:, :C], case.tc[0].k[l][:, :C].astype(np.float32))


def test_cfg1_draft_expand_matches_oracle():
    case, prompt, feats, root = _prefilled_cfg1()
    case.upload_kv()
    n = len(prompt)
    feat_in = feats[None].astype(np.float32)                                   # [1, n, H]
    tok_in = np.concatenate([prompt[1:], [root]]).astype(np.int32)[None]        # [1, n]
    tokens, scores = case.gpu_draft(feat_in, tok_in)
    ref = case.oracle_draft(feat_in.astype(np.float64), tok_in)
    n_cmp, n_skip = compare_draft_tokens(case, tokens, scores, ref)
    assert n_cmp == case.T - 1 and n_skip == 0
    # draft cache rows 0..C-1 now hold the catch-up rows
    k, v = case.download_kv("draft")
    for l in range(case.cfg["K"]):
        rk = case.dc[0].k[l][:, :n]
        assert np.abs(k[l, 0][:, :n] - rk).max() < 1e-4 * np.abs(rk).max()


def test_cfg1_catchup_in_two_calls_equals_one():
    """Draft cache built by m=40 then m=24 catch-up rows gives the same tree as m=64 at once."""
    case, prompt, feats, root = _prefilled_cfg1()
    case.upload_kv()
    feat_in = feats[None].astype(np.float32)
    tok_in = np.concatenate([prompt[1:], [root]]).astype(np.int32)[None]
    t_all, s_all = case.gpu_draft(feat_in, tok_in)
    # second device state: pretend the context was 40 long, catch up, then extend to 64
    case2, _, _, _ = _prefilled_cfg1()
    case2.upload_kv()
    case2.kv["ctx_len"].fill_(40)
    case2.gpu_draft(feat_in[:, :40], tok_in[:, :40])
    case2.kv["ctx_len"].fill_(64)
    t_two, s_two = case2.gpu_draft(feat_in[:, 40:], tok_in[:, 40:])
    np.testing.assert_array_equal(t_all, t_two)
    np.testing.assert_allclose(s_all, s_two, rtol=1e-4, atol=1e-5)


def test_cfg1_iterations_are_lossless_and_match_oracle():
    """Full loop on the device: draft -> verify -> accept+commit, fed back; the emitted tokens
    are those of plain greedy decoding (section 2.2) and every step equals the oracle's."""
    case, prompt, feats, root = _prefilled_cfg1(n_ctx=40)
    case.upload_kv()
    cfg, tree = case.cfg, case.tree
    want = oracle.greedy_reference(cfg, case.Wt, prompt, 12)
    assert want[0] == root
    feat_in = feats.astype(np.float32)
    tok_in = np.concatenate([prompt[1:], [root]]).astype(np.int32)
    ofeat, otok = feats, tok_in.copy()
    C = len(prompt)
    got = [root]
    plant_rng = np.random.default_rng(0)
    it_no = 0
    while len(got) < 12:
        tokens, scores = case.gpu_draft(feat_in[None], tok_in[None])
        ref = oracle.eagle_expand(cfg, case.Wt, case.Wd, case.dc[0], C, ofeat, otok, tree.parent, tree.rank,
                                  tree.topk_per_depth)
        np.testing.assert_array_equal(tokens[0], ref["tokens"])
        tt = tokens.copy()
        if it_no % 2 == 1:                      # plant the true continuation on a random root path
            cur, j = 0, len(got)
            while j < len(want):
                kids = [c for c in range(case.T) if tree.parent[c] == cur]
                if not kids:
                    break
                pick = kids[int(plant_rng.integers(0, len(kids)))]
                for c in kids:
                    tt[0, c] = want[j] if c == pick else (want[j] + 1 + c) % case.V
                cur, j = pick, j + 1
        feat, logits, greedy = case.gpu_verify(tt)
        rfeat, rlogits, rgreedy = case.oracle_verify(tt)
        skipped, _ = compare_logits_and_greedy(case, logits, greedy, rlogits, rgreedy)
        assert skipped == 0
        a, path, nxt = case.gpu_accept(tt, greedy, commit=True)
        ra, rpath, rnxt = oracle.accept_greedy(tt[0], rgreedy[0], tree.parent)
        assert a[0] == ra and nxt[0] == rnxt
        assert list(path[0][:ra + 1]) == rpath and all(path[0][ra + 1:] == -1)
        C2 = oracle.commit_path(case.tc[0], C, rpath)
        assert int(case.kv["ctx_len"][0].item()) == C2
        emitted = [int(tt[0, p]) for p in rpath[1:]] + [rnxt]
        got += emitted
        feat_in = feat[0][rpath].astype(np.float32)
        tok_in = np.asarray(emitted, np.int32)
        ofeat, otok = rfeat[0][rpath], tok_in.copy()
        C = C2
        case.ctx_lens = [C]
        it_no += 1
    assert got[:12] == want[:12]
    # committed device rows equal the oracle's committed rows
    k, v = case.download_kv()
    for l in range(cfg["n_layers"]):
        rk = case.tc[0].k[l][:, :C]
        assert np.abs(k[l, 0][:, :C] - rk).max() < 1e-4 * np.abs(rk).max()


def test_chain_template_prefill_equals_oracle_prefill():
    """A chain is a tree: verifying a 32-token chain on an empty cache and committing all of it
    reproduces sequential decoding (Eq. 1) of those tokens."""
    case = Case("cfg1", tree=dict(topk=[1] * 31, widths=[1] * 32), capacity=96)
    case.ctx_lens = [0]
    case.upload_kv()
    toks = tensor_uniform_int(1, "ctx", (64,), 0, case.V)[:32]
    feat, logits, greedy = case.gpu_verify(toks[None])
    oc = oracle.KVCache(case.cfg["n_layers"], case.cfg["n_heads"], 96, case.cfg["head_dim"])
    rfeat, rlogits = oracle.prefill(case.cfg, case.Wt, oc, toks)
    assert rel_err_rows(logits[0], rlogits).max() < case.tol
    # plant "greedy == next token" so that the whole chain is accepted and committed
    g = np.concatenate([toks[1:], [5]]).astype(np.int32)[None]
    a, path, nxt = case.gpu_accept(toks[None], g, commit=True)
    assert a[0] == 31 and nxt[0] == 5 and list(path[0]) == list(range(32))
    assert int(case.kv["ctx_len"][0].item()) == 32


# --------------------------------------------------------------------------- acceptance (integers: exact)
@pytest.mark.parametrize("cfgname", ["cfg2_small", "cfg3_small", "cfg5_small"])
def test_accept_prefix_is_exact(cfgname):
    case = Case(cfgname, n_layers=1, K=1)
    case.fill_kv_normal()
    case.upload_kv()
    rng = np.random.default_rng(7)
    t = case.tree
    kids = [[c for c in range(case.T) if t.parent[c] == u] for u in range(case.T)]
    for trial in range(12):
        tt = np.zeros((case.B, case.T), np.int32)
        g = rng.integers(0, 4, (case.B, case.T)).astype(np.int32)
        for b in range(case.B):
            for u in range(case.T):
                vals = rng.permutation(max(4, len(kids[u])))[: len(kids[u])]
                for c, v in zip(kids[u], vals):
                    tt[b, c] = v
        if trial == 0:                           # full-depth planted path in sequence 0
            node = case.T - 1                        # the last node is at the deepest level
            while t.parent[node] != -1:
                g[0, t.parent[node]] = tt[0, node]
                node = int(t.parent[node])
        a, path, nxt = case.gpu_accept(tt, g, commit=False)
        for b in range(case.B):
            ra, rpath, rnxt = oracle.accept_greedy(tt[b], g[b], t.parent)
            assert a[b] == ra and nxt[b] == rnxt
            assert list(path[b][:ra + 1]) == rpath and all(path[b][ra + 1:] == -1)
        if trial == 0:
            assert a[0] == case.D


def test_commit_moves_rows_bit_exactly():
    case = Case("cfg5_small", n_layers=2, K=1)
    case.fill_kv_normal()
    t = case.tree
    # put recognisable values into the tree slots of every layer
    for b in range(case.B):
        C = case.ctx_lens[b]
        for l in range(2):
            for i in range(case.T):
                case.tc[b].k[l][:, C + i] = 100 * (l + 1) + i
                case.tc[b].v[l][:, C + i] = -(100 * (l + 1) + i)
    case.upload_kv()
    before_k, before_v = case.download_kv()
    tt = np.tile(1000 + np.arange(case.T, dtype=np.int32), (case.B, 1))
    g = np.full((case.B, case.T), 3, np.int32)
    # sequence b accepts a path of length b+2 ending at the last node of that depth
    depth = oracle.tree_depths(t.parent)
    want_paths = []
    for b in range(case.B):
        node = [i for i in range(case.T) if depth[i] == b + 2][-1]
        path = []
        while node != -1:
            path.append(node)
            node = int(t.parent[node])
        path.reverse()
        for p, c in zip(path[:-1], path[1:]):
            g[b, p] = tt[b, c]
        want_paths.append(path)
    a, path, nxt = case.gpu_accept(tt, g, commit=True)
    k, v = case.download_kv()
    for b in range(case.B):
        C = case.ctx_lens[b]
        assert a[b] == b + 2 and list(path[b][:b + 3]) == want_paths[b]
        assert int(case.kv["ctx_len"][b].item()) == C + b + 3
        for l in range(2):
            for j, node in enumerate(want_paths[b]):
                np.testing.assert_array_equal(k[l, b][:, C + j], before_k[l, b][:, C + node])
                np.testing.assert_array_equal(v[l, b][:, C + j], before_v[l, b][:, C + node])
            np.testing.assert_array_equal(k[l, b][:, :C], before_k[l, b][:, :C])


# --------------------------------------------------------------------------- bf16, reduced width
@pytest.mark.parametrize("cfgname,K", [("cfg2_small", 1), ("cfg2_small", 2), ("cfg4_small", 3),
                                        ("cfg5_small", 2), ("cfg3_small", 1)])
def test_bf16_verify_matches_oracle(cfgname, K):
    case = Case(cfgname, K=K)
    case.fill_kv_normal()
    case.upload_kv()
    tt = case.random_tree_tokens()
    feat, logits, greedy = case.gpu_verify(tt)
    rfeat, rlogits, rgreedy = case.oracle_verify(tt)
    skipped, err = compare_logits_and_greedy(case, logits, greedy, rlogits, rgreedy)
    assert skipped <= max(1, case.B * case.T // 10)
    assert rel_err_rows(feat, rfeat).max() < case.tol
    # verification without materialised logits gives the same greedy ids
    case.upload_kv()
    _, _, greedy2 = case.gpu_verify(tt, want_logits=False)
    np.testing.assert_array_equal(greedy, greedy2)


@pytest.mark.parametrize("cfgname,K", [("cfg2_small", 1), ("cfg2_small", 2), ("cfg4_small", 3),
                                        ("cfg5_small", 2), ("cfg3_small", 1), ("cfg3_small", 2)])
def test_bf16_draft_expand_matches_oracle(cfgname, K):
    case = Case(cfgname, K=K)
    case.fill_kv_normal()
    case.upload_kv()
    feat_in, tok_in = case.normal_draft_inputs()
    tokens, scores = case.gpu_draft(feat_in, tok_in)
    ref = case.oracle_draft(feat_in.astype(np.float64), tok_in)
    n_cmp, n_skip = compare_draft_tokens(case, tokens, scores, ref)
    assert n_skip <= max(1, n_cmp // 10), f"{n_skip} of {n_cmp} drafted tokens skipped by the margin rule"
    for b in range(case.B):
        assert len(set(tokens[b, 1:1 + case.tree.topk_per_depth[0]])) == case.tree.topk_per_depth[0]


# --------------------------------------------------------------------------- bf16, long contexts
@pytest.mark.parametrize("cfgname,ctx", [("cfg2_small", 4096), ("cfg4_small", 2500), ("cfg3_small", 1777)])
def test_bf16_verify_long_context_matches_oracle(cfgname, ctx):
    """Contexts long enough that every attention wave runs several 32-key steps (the running maximum and
    sum of the softmax are rescaled between steps), with a ragged last step."""
    case = Case(cfgname, n_layers=2, ctx=ctx, capacity=ctx + 128)
    case.fill_kv_normal()
    case.upload_kv()
    tt = case.random_tree_tokens()
    feat, logits, greedy = case.gpu_verify(tt)
    rfeat, rlogits, rgreedy = case.oracle_verify(tt)
    skipped, err = compare_logits_and_greedy(case, logits, greedy, rlogits, rgreedy)
    assert skipped <= max(1, case.B * case.T // 10)
    assert rel_err_rows(feat, rfeat).max() < case.tol


def test_bf16_long_context_softmax_with_a_dominant_late_key():
    """The last 40 context rows get keys 8 x larger than the rest (a power of two: still exact in the
    cache's storage type), so that the row maxima of the scores sit at the end of the context: every
    earlier step's running maximum is replaced there and its partial sums are scaled down."""
    case = Case("cfg2_small", n_layers=1, ctx=3000, capacity=3128)
    case.fill_kv_normal()
    C = case.ctx_lens[0]
    for c in case.tc:
        c.k[0][:, C - 40:C] *= 8.0
    case.upload_kv()
    tt = case.random_tree_tokens()
    feat, logits, greedy = case.gpu_verify(tt)
    rfeat, rlogits, rgreedy = case.oracle_verify(tt)
    compare_logits_and_greedy(case, logits, greedy, rlogits, rgreedy)
    assert rel_err_rows(feat, rfeat).max() < case.tol


# --------------------------------------------------------------------------- bf16, heads of 64 dimensions
@pytest.mark.parametrize("cfgname,ctx", [("cfg2_small", 200), ("cfg4_small", 1100)])
def test_bf16_head_dim_64_matches_oracle(cfgname, ctx):
    """The benchmark shapes all have heads of 128 dimensions; the library also takes 64 (its attention kernel,
    the rotary pairs and the query fragments of the QKV projection are laid out per head size).  Same widths
    with twice the heads: verification (26 and 60 rows, one and several key steps per wave) and drafting."""
    from koala_synth import get_config
    hidden = get_config(cfgname)["hidden"]
    case = Case(cfgname, n_layers=2, ctx=ctx, capacity=ctx + 128, head_dim=64, n_heads=hidden // 64)
    assert case.cfg["head_dim"] == 64 and case.cfg["n_heads"] * 64 == hidden
    case.fill_kv_normal()
    case.upload_kv()
    tt = case.random_tree_tokens()
    feat, logits, greedy = case.gpu_verify(tt)
    rfeat, rlogits, rgreedy = case.oracle_verify(tt)
    skipped, err = compare_logits_and_greedy(case, logits, greedy, rlogits, rgreedy)
    assert skipped <= max(1, case.B * case.T // 10)
    assert rel_err_rows(feat, rfeat).max() < case.tol
    case.upload_kv()
    feat_in, tok_in = case.normal_draft_inputs()
    tokens, scores = case.gpu_draft(feat_in, tok_in)
    ref = case.oracle_draft(feat_in.astype(np.float64), tok_in)
    n_cmp, n_skip = compare_draft_tokens(case, tokens, scores, ref)
    assert n_skip <= max(1, n_cmp // 10), f"{n_skip} of {n_cmp} drafted tokens skipped by the margin rule"


# --------------------------------------------------------------------------- bf16, many rows
@pytest.mark.parametrize("batch", [2, 4, 5])
def test_bf16_batched_verify_many_rows_matches_oracle(batch):
    """Batches whose row count needs the GEMM's passes of eight activation tiles: 2 x 60 rows = 8 tiles (one
    pass of eight), 4 x 60 = 16 tiles (two passes of eight), 5 x 60 = 20 tiles (two of eight and one of four).
    Ragged contexts; every logit of every row is compared."""
    case = Case("cfg5_small", batch=batch, n_layers=2)
    case.fill_kv_normal()
    case.upload_kv()
    tt = case.random_tree_tokens()
    feat, logits, greedy = case.gpu_verify(tt)
    rfeat, rlogits, rgreedy = case.oracle_verify(tt)
    skipped, err = compare_logits_and_greedy(case, logits, greedy, rlogits, rgreedy)
    assert skipped <= max(1, case.B * case.T // 10)
    assert rel_err_rows(feat, rfeat).max() < case.tol
