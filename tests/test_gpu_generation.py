"""GPU parity of the generation loop (koala_generate) against the oracle's loop: the tokens are
those of plain greedy decoding (the method is lossless, section 2.2), and the accepted length of
every iteration, hence tokens per iteration and n-alpha (section 4.1), equals the oracle's.

Weight sets: the usual random ones (the draft is almost never right), and `predictable_pair`,
whose greedy continuation is t -> t+1 by construction and whose draft quality is set by sigma, so
that every accepted length occurs.  Token margins of the predictable sets are far above the
tolerance, so ids are compared exactly."""
import numpy as np
import pytest

import oracle
from koala_synth import chain_tree, predictable_pair, tensor_uniform_int

from gpu_harness import Case

pytestmark = pytest.mark.gpu


def _hist(accept_lens, n=64):
    h = [0] * n
    for a in accept_lens:
        h[a] += 1
    return h


def _run(case, prompt, n_new, use_draft=True):
    """Oracle prefill -> upload -> device generation.  Returns (device tokens, stats, root)."""
    feats, logits = case.prefill_oracle(prompt)
    case.upload_kv()
    root = int(np.argmax(logits[-1]))
    if case.eagle and use_draft:
        feat_in, tok_in = feats, np.concatenate([prompt[1:], [root]])
    else:
        feat_in, tok_in = feats[-1:], np.array([root])
    toks, stats = case.gpu_generate(feat_in, tok_in, n_new - 1, use_draft=use_draft)
    return [root] + [int(t) for t in toks], stats


@pytest.mark.parametrize("sigma", [0.0, 5.0])
def test_cfg1_generation_matches_oracle_loop(sigma):
    case = Case("cfg1", max_m=16, weights=lambda cfg: predictable_pair(cfg, 0, sigma=sigma, cache=True))
    tree = case.tree
    prompt = np.arange(5, 13)
    n = 30
    ref = oracle.generate_speculative(case.cfg, case.Wt, case.Wd, prompt, n, tree.parent, tree.rank,
                                      tree.topk_per_depth)
    got, stats = _run(case, prompt, n)
    assert got == ref["tokens"] == [(13 + i) % 1000 for i in range(n)]
    # the device stops once n-1 new tokens exist; the oracle once n (root included): same iterations
    assert stats["iterations"] == len(ref["accept_lens"])
    assert stats["accept_hist"] == _hist(ref["accept_lens"])
    assert stats["tokens"] == sum(a + 1 for a in ref["accept_lens"])
    assert int(case.kv["ctx_len"][0].item()) == ref["C"]
    if sigma:
        assert len(set(ref["accept_lens"])) == tree.depth + 1


def test_cfg1_generation_with_random_heads_is_lossless():
    case = Case("cfg1", max_m=40)
    tree = case.tree
    prompt = tensor_uniform_int(1, "ctx", (64,), 0, case.V)[:24]
    n = 10
    want = oracle.greedy_reference(case.cfg, case.Wt, prompt, n)
    ref = oracle.generate_speculative(case.cfg, case.Wt, case.Wd, prompt, n, tree.parent, tree.rank,
                                      tree.topk_per_depth)
    got, stats = _run(case, prompt, n)
    assert got == want == ref["tokens"]
    assert stats["accept_hist"] == _hist(ref["accept_lens"])


def test_plain_decoding_mode_equals_greedy_reference():
    case = Case("cfg1", tree=dict(topk=[], widths=[1]),
                weights=lambda cfg: predictable_pair(cfg, 0, sigma=0.0, cache=True))
    prompt = np.array([100, 7, 512])
    n = 9
    want = oracle.greedy_reference(case.cfg, case.Wt, prompt, n)
    got, stats = _run(case, prompt, n, use_draft=False)
    assert got == want
    assert stats["iterations"] == n - 1 and stats["accept_hist"][0] == n - 1


def test_chain_template_n_alpha_matches_oracle():
    ch = chain_tree(4)
    case = Case("cfg1", max_m=16, tree=dict(topk=[1, 1, 1, 1], widths=[1, 1, 1, 1, 1]),
                weights=lambda cfg: predictable_pair(cfg, 0, sigma=4.5, cache=True))
    assert list(case.tree.parent) == list(ch.parent)
    prompt = np.arange(40, 46)
    n = 40
    ref = oracle.generate_speculative(case.cfg, case.Wt, case.Wd, prompt, n, ch.parent, ch.rank, ch.topk_per_depth)
    got, stats = _run(case, prompt, n)
    assert got == ref["tokens"]
    h = stats["accept_hist"]
    ge = [sum(h[a:]) for a in range(6)]
    alpha = [ge[k] / ge[k - 1] if ge[k - 1] else float("nan") for k in range(1, 5)]
    want = oracle.n_alpha(ref["accept_lens"], 4)
    np.testing.assert_allclose(alpha, want, equal_nan=True)
    assert 0.0 < want[0] < 1.0


def test_bf16_generation_matches_oracle_loop():
    """bf16 path (MFMA kernels) inside the loop, tree of 26 nodes and depth 5."""
    case = Case("cfg2_small", ctx=16, max_m=16, weights=lambda cfg: predictable_pair(cfg, 0, sigma=6.0, cache=True))
    tree = case.tree
    prompt = np.arange(200, 216)
    n = 24
    ref = oracle.generate_speculative(case.cfg, case.Wt, case.Wd, prompt, n, tree.parent, tree.rank,
                                      tree.topk_per_depth)
    got, stats = _run(case, prompt, n)
    assert got == ref["tokens"] == [(216 + i) % case.V for i in range(n)]
    assert stats["accept_hist"] == _hist(ref["accept_lens"])


def test_generate_argument_errors():
    import paper_2408_08146_amd as K
    case = Case("cfg1", max_m=2)        # depth 2 tree needs max_m >= 3 for the loop
    feats, logits = case.prefill_oracle(np.array([1, 2]))
    case.upload_kv()
    with pytest.raises(K.KoalaError):
        case.gpu_generate(feats, np.array([2, 3]), 4)
    with pytest.raises(K.KoalaError):   # plain decoding needs a single-node tree
        case.gpu_generate(feats[-1:], np.array([3]), 4, use_draft=False)
    case2 = Case("cfg1", max_m=8)
    feats, logits = case2.prefill_oracle(np.array([1, 2]))
    case2.upload_kv()
    with pytest.raises(K.KoalaError):   # capacity 128
        case2.gpu_generate(feats, np.array([2, 3]), 200)
    case2.ctx_lens = [5]                # host's idea of the context length is wrong
    with pytest.raises(K.KoalaError):
        case2.gpu_generate(feats, np.array([2, 3]), 4)


@pytest.mark.parametrize("temperature", [1.0, 0.3])
def test_nongreedy_generation_matches_oracle_loop(temperature):
    """koala_generate_sample against the oracle's non-greedy loop with the same uniforms.  The oracle's
    whole run is repeated with every uniform moved by +-2e-5; only if nothing changes (it does not
    for these seeds: the predictable weights give concentrated distributions) is the device run
    compared, and then exactly."""
    from koala_synth import tensor_uniform01
    case = Case("cfg1", max_m=16, weights=lambda cfg: predictable_pair(cfg, 0, sigma=5.0, cache=True))
    tree, T = case.tree, case.T
    Tp = (T + 3) // 4 * 4
    prompt = np.arange(5, 13)
    n, iters = 24, 40
    U = tensor_uniform01(52, "gen_uniforms", (iters, 3, Tp))

    def run(delta):
        us = [tuple(np.clip(U[i, j, :T].astype(np.float64) + delta, 0.0, 1.0 - 1e-12) for j in range(3))
              for i in range(iters)]
        r = oracle.generate_sampled(case.cfg, case.Wt, case.Wd, prompt, n, tree.parent, tree.rank, us, temperature)
        return r["tokens"], r["accept_lens"], r["C"]
    ref = run(0.0)
    assert ref == run(-2e-5) == run(2e-5), "pick another seed: the oracle's own decisions are within the margin"
    assert len(set(ref[1])) >= 3                      # several accepted lengths occur
    feats, logits = case.prefill_oracle(prompt)
    case.upload_kv()
    root = oracle.inverse_cdf(oracle.softmax_t(logits[-1], temperature), U[0, 2, 0])
    assert root == ref[0][0]
    torch = case.torch
    out = torch.full((n - 1,), -1, dtype=torch.int32, device=case.device)
    stats = case.gpu.generate_sample(case.t(feats.astype(np.float32)),
                                     case.t(np.concatenate([prompt[1:], [root]]).astype(np.int32)), len(prompt),
                                     len(prompt), n - 1, case.t(U), temperature, out)
    got = [root] + [int(t) for t in out.cpu().numpy()]
    assert got == ref[0]
    assert stats["accept_hist"] == _hist(ref[1]) and stats["iterations"] == len(ref[1])
    assert int(case.kv["ctx_len"][0].item()) == ref[2]


@pytest.mark.parametrize("temperature", [0.1, 0.05])
def test_nongreedy_generation_with_medusa_heads_matches_oracle_loop(temperature):
    """koala_generate_sample with Medusa-style heads (section 4.4 evaluates both kinds) against the oracle's
    loop with the same uniforms, compared exactly where the oracle's own run does not change when every
    uniform moves by +-2e-5.  The random model's distributions over 1000 tokens are nearly flat at
    temperature 1 (draw boundaries then lie closer together than that margin), so the temperatures are low;
    accepted lengths 0, 1 and 2 all occur."""
    from koala_synth import tensor_uniform01
    case = None
    for seed in (61, 62, 63, 64):
        case = case or Case("cfg1", draft="medusa", medusa_heads=2, K=1)
        tree, T = case.tree, case.T
        Tp = (T + 3) // 4 * 4
        prompt = np.arange(5, 13)
        n, iters = 16, 40
        U = tensor_uniform01(seed, "gen_uniforms_medusa", (iters, 3, Tp))

        def run(delta):
            us = [tuple(np.clip(U[i, j, :T].astype(np.float64) + delta, 0.0, 1.0 - 1e-12) for j in range(3))
                  for i in range(iters)]
            r = oracle.generate_sampled(case.cfg, case.Wt, case.Wd, prompt, n, tree.parent, tree.rank, us, temperature)
            return r["tokens"], r["accept_lens"], r["C"]
        ref = run(0.0)
        if ref == run(-2e-5) == run(2e-5):
            break
    else:
        pytest.fail("no seed whose oracle run is outside the margin")
    case.tc[0] = oracle.KVCache(case.cfg["n_layers"], case.cfg["n_heads"], case.cap, case.cfg["head_dim"])
    feats, logits = case.prefill_oracle(prompt)
    case.upload_kv()
    root = oracle.inverse_cdf(oracle.softmax_t(logits[-1], temperature), U[0, 2, 0])
    assert root == ref[0][0]
    torch = case.torch
    out = torch.full((n - 1,), -1, dtype=torch.int32, device=case.device)
    stats = case.gpu.generate_sample(case.t(feats[-1:].astype(np.float32)), case.t(np.array([root], np.int32)), 1,
                                     len(prompt), n - 1, case.t(U), temperature, out)
    got = [root] + [int(t) for t in out.cpu().numpy()]
    assert got == ref[0]
    assert stats["accept_hist"] == _hist(ref[1]) and stats["iterations"] == len(ref[1])
    assert int(case.kv["ctx_len"][0].item()) == ref[2]


def test_nongreedy_generation_runs_out_of_uniforms_cleanly():
    import paper_2408_08146_amd as K
    from koala_synth import tensor_uniform01
    case = Case("cfg1", max_m=16)
    prompt = np.arange(5, 13)
    feats, logits = case.prefill_oracle(prompt)
    case.upload_kv()
    torch = case.torch
    out = torch.full((30,), -1, dtype=torch.int32, device=case.device)
    U = case.t(tensor_uniform01(53, "few", (2, 3, 8)))       # two iterations cannot yield 30 tokens
    with pytest.raises(K.KoalaError):
        case.gpu.generate_sample(case.t(feats.astype(np.float32)),
                                 case.t(np.concatenate([prompt[1:], [3]]).astype(np.int32)), len(prompt), len(prompt),
                                 30, U, 1.0, out)
