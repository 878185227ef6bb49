"""Edge cases on the device: degenerate trees, largest tree / most catch-up rows, host-side
rejection of bad arguments at bind and call time (no kernel is launched for a rejected call)."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
import paper_2408_08146_amd as K
from paper_2408_08146_amd.binding import KoalaError
from koala_synth import tensor_uniform_int

from gpu_harness import Case, rel_err_rows, compare_logits_and_greedy, compare_draft_tokens

pytestmark = pytest.mark.gpu


def test_single_node_tree_is_plain_decoding_bf16():
    """A 1-node tree is one autoregressive step (Eq. 1): verify it, accept (a = 0), commit, repeat;
    the device must follow the oracle's sequential decoding."""
    case = Case("cfg2_small", tree=dict(topk=[], widths=[1]))
    case.fill_kv_normal()
    case.upload_kv()
    tok = 17
    C0 = case.ctx_lens[0]
    for step in range(3):
        feat, logits, greedy = case.gpu_verify(np.array([[tok]], np.int32))
        f, l = oracle.decode_one(case.cfg, case.Wt, case.tc[0], C0 + step, tok)
        assert rel_err_rows(logits[0], l[None]).max() < case.tol
        a, path, nxt = case.gpu_accept(np.array([[tok]], np.int32), greedy, commit=True)
        assert a[0] == 0 and path[0][0] == 0 and nxt[0] == greedy[0, 0]
        assert int(case.kv["ctx_len"][0].item()) == C0 + step + 1
        tok = int(np.argmax(l))
        assert tok == greedy[0, 0]


@pytest.mark.parametrize("topk,widths", [([3, 2, 1], [1, 3, 6, 6]), ([4, 2, 1], [1, 4, 6, 6]),
                                         ([4, 2, 2, 1], [1, 4, 8, 10, 9]), ([4, 2, 2, 1], [1, 4, 8, 10, 10]),
                                         ([4, 2, 2, 2], [1, 4, 8, 13, 14]), ([4, 2, 2, 2], [1, 4, 8, 16, 20])])
def test_tree_sizes_around_the_row_tile_boundaries_bf16(topk, widths):
    """Trees of 16, 17, 32, 33, 40 and 49 nodes: a full row tile, one row into the second, two full tiles, one
    row into the second group of tiles, and groups with a part-filled and an empty tile."""
    case = Case("cfg2_small", n_layers=2, tree=dict(topk=topk, widths=widths))
    assert case.T == sum(widths)
    case.fill_kv_normal()
    case.upload_kv()
    tt = case.random_tree_tokens()
    feat, logits, greedy = case.gpu_verify(tt)
    rfeat, rlogits, rgreedy = case.oracle_verify(tt)
    skipped, err = compare_logits_and_greedy(case, logits, greedy, rlogits, rgreedy)
    assert skipped <= max(1, case.T // 10)
    assert rel_err_rows(feat, rfeat).max() < case.tol


def test_largest_tree_and_most_catchup_rows_bf16():
    """64 tree nodes (Medusa template) verified, and an EAGLE catch-up of m = 64 rows."""
    case = Case("cfg3_small")
    assert case.T == 64
    case.fill_kv_normal()
    case.upload_kv()
    tt = case.random_tree_tokens()
    feat, logits, greedy = case.gpu_verify(tt)
    rfeat, rlogits, rgreedy = case.oracle_verify(tt)
    compare_logits_and_greedy(case, logits, greedy, rlogits, rgreedy)

    case = Case("cfg2_small", max_m=64)
    case.fill_kv_normal(m=64)
    case.upload_kv()
    feat_in, tok_in = case.normal_draft_inputs(m=64)
    tokens, scores = case.gpu_draft(feat_in, tok_in)
    ref = case.oracle_draft(feat_in.astype(np.float64), tok_in)
    n_cmp, n_skip = compare_draft_tokens(case, tokens, scores, ref)
    assert n_skip <= max(1, n_cmp // 10)


def test_bind_and_call_argument_errors():
    case = Case("cfg2_small", n_layers=1)
    ctx, lib = case.gpu, case.gpu.lib
    kv, ws = case.kv, case.ws
    w = case.gpu._keep[0]
    # workspace too small
    with pytest.raises(KoalaError) as e:
        ctx.bind(w, kv, ws[: ws.numel() // 2])
    assert e.value.status == -6
    ctx.bind(w, kv, ws)                                    # still usable after a rejected bind
    # misaligned workspace
    with pytest.raises(KoalaError) as e:
        ctx.bind(w, kv, torch.empty(ws.numel() + 64, dtype=torch.uint8, device="cuda")[16:])
    assert e.value.status == -3
    # capacity smaller than the tree
    small = dict(kv)
    small["capacity"] = case.T
    with pytest.raises(KoalaError) as e:
        ctx.bind(w, small, ws)
    assert e.value.status == -4
    # a missing weight pointer
    bad = dict(w)
    bad["lm_head"] = None
    with pytest.raises(KoalaError) as e:
        ctx.bind(bad, kv, ws)
    assert e.value.status == -1
    ctx.bind(w, kv, ws)
    B, T = case.B, case.T
    tt = torch.zeros(B, T, dtype=torch.int32, device="cuda")
    feat = torch.full((B, T, case.H), 7.0, dtype=torch.float32, device="cuda")
    greedy = torch.full((B, T), -3, dtype=torch.int32, device="cuda")
    # batch out of range, NULL outputs, misaligned output: rejected, outputs untouched
    for bad_batch in (0, B + 1):
        with pytest.raises(KoalaError) as e:
            ctx.tree_verify(bad_batch, tt, feat, None, greedy)
        assert e.value.status == -2
    with pytest.raises(KoalaError) as e:
        ctx.tree_verify(B, tt, None, None, greedy)
    assert e.value.status == -1
    with pytest.raises(KoalaError) as e:
        ctx.tree_verify(B, tt, feat.view(-1)[1:1 + B * T * case.H - 4].view(-1), None, greedy)
    assert e.value.status == -3
    with pytest.raises(KoalaError) as e:                   # m above max_m
        f = torch.zeros(B, 2, case.H, dtype=torch.float32, device="cuda")
        t2 = torch.zeros(B, 2, dtype=torch.int32, device="cuda")
        ctx.draft_expand(B, f, t2, 2, tt, None)
    assert e.value.status == -2
    torch.cuda.synchronize()
    assert float(feat.min()) == 7.0 and int(greedy.max()) == -3


def test_results_are_run_to_run_identical():
    """Split-K partials are summed in a fixed order and no float atomics are used: two runs on the
    same inputs give bit-identical logits and features."""
    case = Case("cfg4_small", K=3)
    case.fill_kv_normal()
    tt = case.random_tree_tokens()
    outs = []
    for _ in range(2):
        case.upload_kv()
        outs.append(case.gpu_verify(tt))
    np.testing.assert_array_equal(outs[0][1], outs[1][1])
    np.testing.assert_array_equal(outs[0][0], outs[1][0])


@pytest.mark.parametrize("name,batch", [("cfg4_small", 1), ("cfg5_small", 5)])
def test_results_do_not_depend_on_what_the_workspace_held(name, batch):
    """Partial results cross workgroups inside kernels (key splits of the attention, split-K sums): a consumer that
    read one before its producer had written it would pick up whatever the workspace held.  Twelve verifications,
    the workspace refilled with 0x7f bytes (3.4e38) and bound again before each: every run must reproduce the first
    bit for bit."""
    case = Case(name, batch=batch, n_layers=2)
    case.fill_kv_normal()
    tt = case.random_tree_tokens()
    case.upload_kv()
    first = case.gpu_verify(tt)
    assert np.isfinite(first[1]).all()
    for _ in range(12):
        case.ws.fill_(0x7f)
        case.gpu.bind(*case.gpu._keep)
        case.upload_kv()
        again = case.gpu_verify(tt)
        np.testing.assert_array_equal(first[1], again[1])
        np.testing.assert_array_equal(first[0], again[0])


def test_weights_to_half_is_exact_and_rejects_bad_arguments():
    """koala_weights_to_half re-encodes bfloat16 values as fp16 in place: bit for bit what a conversion through
    fp32 with round-to-nearest-even gives, and the same number wherever fp16 can hold it (magnitudes 2^-14 ..
    65504 here; down to 2^-24 the eight significant bits still fit the subnormal grid), for both signs, zeros and
    the exponent range a weight can have.  Bad sizes, alignments and pointers are refused before any launch."""
    from paper_2408_08146_amd.binding import weights_to_half_status, STATUS_BY_NAME
    rng = np.random.default_rng(5)
    n = 1 << 16
    vals = np.exp2(rng.uniform(-30.0, 17.0, n)).astype(np.float32) * rng.choice([-1.0, 1.0], n).astype(np.float32)
    vals[:64] = [0.0, -0.0, 65504.0, -65504.0, 2.0 ** -14, 2.0 ** -24, 2.0 ** -25, 1.0] * 8
    bits = (vals.view(np.uint32) >> 16).astype(np.uint16)          # any bf16 bit pattern will do: truncate
    as_f32 = (bits.astype(np.uint32) << 16).view(np.float32)       # the bf16 values
    with np.errstate(over="ignore"):
        ref = as_f32.astype(np.float16)                            # numpy: round to nearest even, inf beyond 65504
    t = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    out = K.weights_to_f16(t)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    np.testing.assert_array_equal(got.view(np.uint16), ref.view(np.uint16))
    exact = (np.abs(as_f32) >= 2.0 ** -14) & (np.abs(as_f32) <= 65504.0)
    assert exact.sum() > n // 2
    np.testing.assert_array_equal(got.astype(np.float32)[exact], as_f32[exact])
    buf = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    assert weights_to_half_status(0, 64) == STATUS_BY_NAME["KOALA_E_NULL"]
    assert weights_to_half_status(buf.data_ptr(), 12) == STATUS_BY_NAME["KOALA_E_SHAPE"]
    assert weights_to_half_status(buf.data_ptr() + 2, 8) == STATUS_BY_NAME["KOALA_E_ALIGN"]
    torch.cuda.synchronize()
    assert float(buf.float().abs().max().item()) == 0.0


def test_activations_beyond_the_fp16_range_saturate_instead_of_overflowing():
    """GEMM inputs are fp16: a hidden state beyond +-65504 (here embedding rows of +-3e5) is clamped to the largest
    fp16 value where it is written as a GEMM input, so every projection, the features and the logits stay finite
    (they differ from the exact result, which is the documented limit of the format)."""
    from koala_synth import target_weights, eagle_weights

    def weights(cfg):
        shape = (cfg["vocab"], cfg["hidden"])
        sign = np.where(np.arange(shape[0] * shape[1]).reshape(shape) % 3 == 0, -1.0, 1.0).astype(np.float32)
        return (target_weights(cfg, 0, cache=True, overrides={"embed": lambda: 3.0e5 * sign}),
                eagle_weights(cfg, 0, cache=True))

    case = Case("cfg2_small", n_layers=2, weights=weights)
    case.fill_kv_normal()
    case.upload_kv()
    feat, logits, greedy = case.gpu_verify(case.random_tree_tokens())
    assert np.isfinite(feat).all() and np.isfinite(logits).all()
    assert np.abs(logits).max() > 0.0
