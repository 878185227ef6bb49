"""GPU parity of non-greedy drafting and acceptance (section 2.2; temperature 1 in section 4.4)
against the oracle, with the same uniform random numbers on both sides.

A drawn or accepted token is an integer decided by floating point (a running sum or a ratio
crossing a uniform).  The oracle decides in fp64, the device with fp32 exponentials and fp64
sums, so a trial is compared only if the oracle's own decisions do not change when every uniform
is moved by +-delta (delta an order of magnitude above the arithmetic difference, 1e-7 relative
for the fp32 exponentials; it cannot be much larger, because with 32000 tokens neighbouring
boundaries of the running sum are only ~3e-5 apart); all other trials must agree exactly.  The fraction of compared trials is asserted to be high."""
import numpy as np
import pytest

import oracle
from koala_synth import tensor_normal, tensor_uniform01, tensor_uniform_int, chain_tree

from gpu_harness import Case, rel_err_rows

pytestmark = pytest.mark.gpu


def _robust(fn, us, delta):
    """fn(list of uniform arrays) -> hashable decision; None if it changes under +-delta."""
    base = fn(us)
    for sgn in (-1.0, 1.0):
        moved = [np.clip(u.astype(np.float64) + sgn * delta, 0.0, 1.0 - 1e-12) for u in us]
        if fn(moved) != base:
            return None
    return base


def _compare_sampled_tree(tree, ref, got_tokens, u_draw, temperature, delta):
    """Node by node: the children of a node whose own token (and all of its ancestors') agreed are
    compared with the oracle's draws from the oracle's distribution at that node, provided those
    draws do not change when the uniforms move by +-delta; a child that is not compared or differs
    within that margin taints its subtree.  Returns (nodes compared, nodes in the tree - 1)."""
    T = tree.n_nodes
    ch = [sorted(k, key=lambda c: tree.rank[c]) for k in oracle.children_lists(tree.parent)]
    ok = {0}
    compared = 0
    for u in range(T):                                     # BFS numbering: parents first
        if u not in ok or not ch[u]:
            continue
        p = oracle.softmax_t(ref["logits"][u], temperature)
        us = np.array([u_draw[c] for c in ch[u]], np.float64)
        base = oracle.draw_without_replacement(p, us)
        lo = oracle.draw_without_replacement(p, np.clip(us - delta, 0, 1))
        hi = oracle.draw_without_replacement(p, np.clip(us + delta, 0, 1 - 1e-12))
        assert base == [int(ref["tokens"][c]) for c in ch[u]]
        for j, c in enumerate(ch[u]):
            robust = lo[:j + 1] == base[:j + 1] == hi[:j + 1]
            if robust:
                assert int(got_tokens[c]) == base[j], (u, c)
                compared += 1
                ok.add(c)
            elif int(got_tokens[c]) == base[j] and lo[:j] == base[:j] == hi[:j]:
                ok.add(c)
            else:
                break                                      # later siblings were drawn from a different remainder
    return compared, T - 1


def _accept_case(case, seed, n_trials, temperature, scale, delta=3e-6):
    """Synthetic logits straight into the acceptance kernel (no model): every sequence of the batch
    is one trial."""
    B, T, V, tree = case.B, case.T, case.V, case.tree
    compared = 0
    for trial in range(n_trials):
        tl = tensor_normal(seed, f"tl{trial}", (B, T, V), scale)
        dl = tl + tensor_normal(seed, f"dl{trial}", (B, T, V), 0.7 * scale)
        ua = tensor_uniform01(seed, f"ua{trial}", (B, T))
        ur = tensor_uniform01(seed, f"ur{trial}", (B, T))
        u_draw = tensor_uniform01(seed, f"ud{trial}", (B, T))
        # tokens: children drawn from the draft distribution of their parent, as the draft step does
        toks = np.zeros((B, T), np.int32)
        ch = [sorted(k, key=lambda c: tree.rank[c]) for k in oracle.children_lists(tree.parent)]
        for b in range(B):
            for u in range(T):
                if ch[u]:
                    draws = oracle.draw_without_replacement(oracle.softmax_t(dl[b, u], temperature),
                                                            [u_draw[b, c] for c in ch[u]])
                    for c, x in zip(ch[u], draws):
                        toks[b, c] = x
        a, path, nxt = case.gpu_accept_sample(toks, tl, dl, ua, ur, temperature)
        for b in range(B):
            q = {i: oracle.softmax_t(tl[b, i], temperature) for i in range(T)}
            d = {i: oracle.softmax_t(dl[b, i], temperature) for i in range(T)}
            fn = lambda us: tuple(map(str, oracle.accept_sample(toks[b], tree.parent, tree.rank, q, d, us[0], us[1])))
            want = _robust(fn, [ua[b], ur[b]], delta)
            if want is None:
                continue
            compared += 1
            ra, rpath, rnxt = oracle.accept_sample(toks[b], tree.parent, tree.rank, q, d, ua[b], ur[b])
            assert a[b] == ra and nxt[b] == rnxt, (trial, b)
            assert list(path[b][:ra + 1]) == rpath and all(path[b][ra + 1:] == -1)
    return compared


def test_accept_sample_kernel_full_vocab_tree():
    """7B-sized vocabulary (32000), a 60-node tree of depth 6, batch 3, temperature 1."""
    case = Case("cfg5_small", batch=3, vocab=32000, n_layers=1)
    n = 6
    compared = _accept_case(case, 21, n, 1.0, 2.5)
    assert compared >= 0.8 * n * case.B


def test_accept_sample_kernel_chain_and_temperature():
    case = Case("cfg1", tree=dict(topk=[1, 1, 1, 1], widths=[1, 1, 1, 1, 1]))
    assert list(case.tree.parent) == list(chain_tree(4).parent)
    for temperature in (1.0, 0.6):
        compared = _accept_case(case, 22, 24, temperature, 2.0)
        assert compared >= 18


def test_accepted_lengths_cover_the_range():
    """The synthetic trials are not degenerate: all accepted lengths 0..depth occur (oracle side)."""
    tree = chain_tree(4)
    seen = set()
    for trial in range(24):
        tl = tensor_normal(22, f"tl{trial}", (1, 5, 1000), 2.0)
        dl = tl + tensor_normal(22, f"dl{trial}", (1, 5, 1000), 1.4)
        ua, ur = tensor_uniform01(22, f"ua{trial}", (1, 5)), tensor_uniform01(22, f"ur{trial}", (1, 5))
        ud = tensor_uniform01(22, f"ud{trial}", (1, 5))
        toks = np.zeros(5, np.int32)
        for u in range(4):
            toks[u + 1] = oracle.draw_without_replacement(oracle.softmax_t(dl[0, u]), [ud[0, u + 1]])[0]
        q = {i: oracle.softmax_t(tl[0, i]) for i in range(5)}
        d = {i: oracle.softmax_t(dl[0, i]) for i in range(5)}
        seen.add(oracle.accept_sample(toks, tree.parent, tree.rank, q, d, ua[0], ur[0])[0])
    assert len(seen) >= 4


@pytest.mark.parametrize("temperature", [1.0, 0.5])
def test_cfg1_sampled_draft_and_acceptance_match_oracle(temperature):
    """Whole non-greedy iteration on the fp32 model: sampled draft -> verify -> stochastic accept."""
    case = Case("cfg1", max_m=64)
    cfg, tree, T = case.cfg, case.tree, case.T
    prompt = tensor_uniform_int(1, "ctx", (64,), 0, case.V)[:20]
    feats, logits = case.prefill_oracle(prompt)
    case.upload_kv()
    C = len(prompt)
    root = int(np.argmax(logits[-1]))
    tok_in = np.concatenate([prompt[1:], [root]]).astype(np.int32)
    compared_draws = total_draws = compared_acc = 0
    n_trials = 12
    for trial in range(n_trials):
        ud = tensor_uniform01(31, f"ud{trial}", (1, T))
        ua = tensor_uniform01(31, f"ua{trial}", (1, T))
        ur = tensor_uniform01(31, f"ur{trial}", (1, T))
        tokens, dl_dev = case.gpu_draft_sample(feats, tok_in, ud, temperature)

        def draft(us):
            dc = oracle.KVCache(cfg["K"], cfg["n_heads"], case.cap, cfg["head_dim"])
            return oracle.eagle_expand_sample(cfg, case.Wt, case.Wd, dc, C, feats, tok_in, tree.parent, tree.rank,
                                              us[0], temperature)
        ref = draft([ud[0]])
        n_cmp, n_all = _compare_sampled_tree(tree, ref, tokens[0], ud[0], temperature, 1e-5)
        compared_draws += n_cmp
        total_draws += n_all
        if not np.array_equal(tokens[0], ref["tokens"]):
            continue                                        # a draw within the margin: the trees differ from there on
        dl = dl_dev.cpu().numpy()
        for u, row in ref["logits"].items():
            if any(tree.parent[c] == u for c in range(T)):
                assert rel_err_rows(dl[0, u][None], row[None]).max() < case.tol
        # verification of the drafted tree, then the stochastic walk on the device's own logits buffers
        feat, tlog, greedy = case.gpu_verify(tokens)
        tc = case.tc[0].copy()
        rfeat, rlog, _ = oracle.verify_tree(cfg, case.Wt, tc, C, tokens[0], tree.parent)
        assert rel_err_rows(tlog[0], rlog).max() < case.tol
        a, path, nxt = case.gpu_accept_sample(tokens, tlog, dl_dev, ua, ur, temperature)
        q = {i: oracle.softmax_t(rlog[i], temperature) for i in range(T)}
        d = {u: oracle.softmax_t(row, temperature) for u, row in ref["logits"].items()}
        fn = lambda us: tuple(map(str, oracle.accept_sample(tokens[0], tree.parent, tree.rank, q, d, us[0], us[1])))
        wa = _robust(fn, [ua[0], ur[0]], 2e-5)
        if wa is None:
            continue
        compared_acc += 1
        ra, rpath, rnxt = oracle.accept_sample(tokens[0], tree.parent, tree.rank, q, d, ua[0], ur[0])
        assert a[0] == ra and nxt[0] == rnxt and list(path[0][:ra + 1]) == rpath
    assert compared_draws >= 0.8 * total_draws and compared_acc >= 0.5 * n_trials


def test_bf16_sampled_draft_matches_oracle():
    """bf16 path.  The random head's logits are nearly flat over 4000 tokens, so at temperature 1
    neighbouring draw boundaries lie closer together than the bf16 path's arithmetic difference;
    a low temperature concentrates the mass on few tokens and makes most draws decidable."""
    TEMP = 0.05
    case = Case("cfg2_small", ctx=24, max_m=24, kv_storage_rounding=True)
    cfg, tree, T = case.cfg, case.tree, case.T
    prompt = tensor_uniform_int(1, "ctx", (64,), 0, case.V)[:24]
    feats, logits = case.prefill_oracle(prompt)
    case.upload_kv()
    C = len(prompt)
    root = int(np.argmax(logits[-1]))
    tok_in = np.concatenate([prompt[1:], [root]]).astype(np.int32)
    compared = total = 0
    for trial in range(6):
        ud = tensor_uniform01(32, f"ud{trial}", (1, T))
        tokens, dl_dev = case.gpu_draft_sample(feats, tok_in, ud, TEMP)

        def draft(us):
            dc = oracle.KVCache(cfg["K"], cfg["n_heads"], case.cap, cfg["head_dim"], store=case.tc[0].store)
            return oracle.eagle_expand_sample(cfg, case.Wt, case.Wd, dc, C, feats, tok_in, tree.parent, tree.rank,
                                              us[0], TEMP)
        n_cmp, n_all = _compare_sampled_tree(tree, draft([ud[0]]), tokens[0], ud[0], TEMP, 5e-5)
        compared += n_cmp
        total += n_all
    print(f"bf16 sampled draft: {compared} of {total} draws decidable and compared")
    assert compared >= 0.8 * total


@pytest.mark.parametrize("K", [1, 2])
def test_medusa_sampled_draft_matches_oracle(K):
    """Medusa-style heads (bf16 path, 64-node tree): every parent draws its children from the
    distribution of the next depth's head; also the stored logits equal that head's."""
    TEMP = 0.05
    case = Case("cfg3_small", K=K)
    cfg, tree, T = case.cfg, case.tree, case.T
    feat = tensor_normal(1, "medusa_feat", (1, 1, case.H))
    tok = np.array([[11]], np.int32)
    compared = total = 0
    for trial in range(3):
        ud = tensor_uniform01(33, f"ud{trial}", (1, T))
        tokens, dl_dev = case.gpu_draft_sample(feat, tok, ud, TEMP)
        ref = oracle.medusa_expand_sample(cfg, case.Wt, case.Wd, feat[0, 0].astype(np.float64), 11, tree.parent,
                                          tree.rank, tree.depth, ud[0], TEMP)
        n_cmp, n_all = _compare_sampled_tree(tree, ref, tokens[0], ud[0], TEMP, 5e-5)
        compared += n_cmp
        total += n_all
        dl = dl_dev.cpu().numpy()
        for u, row in ref["logits"].items():
            assert rel_err_rows(dl[0, u][None], row[None]).max() < case.tol
    print(f"Medusa sampled draft K={K}: {compared} of {total} draws decidable and compared")
    assert compared >= 0.8 * total


def test_sampling_argument_errors():
    import paper_2408_08146_amd as K
    case2 = Case("cfg1")
    with pytest.raises(K.KoalaError):    # temperature must be positive
        case2.gpu_draft_sample(np.zeros((1, 1, case2.H), np.float32), np.zeros((1, 1), np.int32),
                               np.zeros((1, case2.T), np.float32), temperature=0.0)


def test_first_emitted_token_follows_the_target_distribution():
    """Distribution-level check on the device (section 2.2: the method samples from the target's
    distribution): over 2048 independent trials of sampled draft -> verify -> stochastic acceptance
    from the same state, the first token an iteration emits (the accepted depth-1 child, or the
    replacement) is distributed as softmax(target logits at the root / temperature), which the
    oracle computes by plain decoding.  Temperature 0.1 concentrates the mass of the random model
    enough that single tokens have measurable frequencies, while the draft's and the target's
    distributions still overlap, so that accepted and replaced tokens both contribute."""
    TEMP, B, CALLS = 0.1, 16, 128
    case = Case("cfg1", batch=B, max_m=16)
    cfg, tree, T = case.cfg, case.tree, case.T
    prompt = tensor_uniform_int(1, "ctx", (64,), 0, case.V)[:12]
    feats, logits = oracle.prefill(cfg, case.Wt, case.tc[0], prompt)
    for b in range(1, B):
        case.tc[b] = case.tc[0].copy()
    case.ctx_lens = [len(prompt)] * B
    case.upload_kv()
    C = len(prompt)
    root = int(np.argmax(logits[-1]))
    tok_in = np.tile(np.concatenate([prompt[1:], [root]]).astype(np.int32), (B, 1))
    feat_in = np.tile(feats.astype(np.float32), (B, 1, 1))
    _, root_logits = oracle.decode_one(cfg, case.Wt, case.tc[0].copy(), C, root)
    q0 = oracle.softmax_t(root_logits, TEMP)
    counts = np.zeros(case.V)
    accepted = 0
    for call in range(CALLS):
        ud = tensor_uniform01(41, f"ud{call}", (B, T))
        ua = tensor_uniform01(41, f"ua{call}", (B, T))
        ur = tensor_uniform01(41, f"ur{call}", (B, T))
        tokens, dl_dev = case.gpu_draft_sample(feat_in, tok_in, ud, TEMP)
        assert (tokens[:, 0] == root).all()
        torch = case.torch
        tl_dev = torch.empty(B, T, case.V, dtype=torch.float32, device=case.device)
        feat = torch.empty(B, T, case.H, dtype=torch.float32, device=case.device)
        greedy = torch.empty(B, T, dtype=torch.int32, device=case.device)
        case.gpu.tree_verify(B, case.t(tokens), feat, tl_dev, greedy)
        a, path, nxt = case.gpu_accept_sample(tokens, tl_dev, dl_dev, ua, ur, TEMP)
        for b in range(B):
            if a[b] >= 1:
                counts[tokens[b, path[b, 1]]] += 1
                accepted += 1
            else:
                counts[nxt[b]] += 1
    n = B * CALLS
    assert 0.1 * n < accepted < 0.9 * n, accepted        # both branches are exercised
    top = np.argsort(-q0)[:8]
    assert q0[top].sum() > 0.4, q0[top]
    freq = counts / n
    sd = np.sqrt(q0 * (1 - q0) / n)
    assert np.all(np.abs(freq[top] - q0[top]) < 4.5 * sd[top]), (freq[top], q0[top])
    rest_q, rest_f = 1 - q0[top].sum(), 1 - freq[top].sum()
    assert abs(rest_f - rest_q) < 4.5 * np.sqrt(rest_q * (1 - rest_q) / n)
