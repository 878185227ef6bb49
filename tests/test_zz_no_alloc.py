"""koala_accept_sample_static, the entry point that allocates nothing (its scratch is a fixed array inside
the library), against koala_accept_sample on the same inputs: accepted length, path and next token must be
equal bit for bit, on two calls in a row, the second with a smaller input (fewer sequences, smaller
vocabulary, another context), and with the KV commit switched on."""
import numpy as np
import pytest

from koala_synth import tensor_normal, tensor_uniform01

from gpu_harness import Case

pytestmark = pytest.mark.gpu


def _both(case, seed, temperature, commit):
    torch = case.torch
    B, T, V, D = case.B, case.T, case.V, case.D
    tt = case.random_tree_tokens(f"static_tt{seed}")
    # target logits = draft logits + noise: acceptance ratios are neither all near 0 nor all 1
    dl_h = tensor_normal(seed, "static_dl", (B, T, V)).astype(np.float32) * 2.0
    tl = case.t(dl_h + 0.7 * tensor_normal(seed, "static_tl", (B, T, V)).astype(np.float32))
    dl = case.t(dl_h)
    # children carry tokens the draft distribution favours, so that acceptances happen
    dlh = dl.cpu().numpy()
    for b in range(B):
        for i in range(1, T):
            p = int(case.tree.parent[i])
            order = np.argsort(-dlh[b, p])
            tt[b, i] = order[int(case.tree.rank[i])]
    ua = case.t(tensor_uniform01(seed, "static_ua", (B, T)))
    ur = case.t(tensor_uniform01(seed, "static_ur", (B, T)))
    ttd = case.t(np.asarray(tt, np.int32).reshape(B, T))
    outs = []
    for fn in (case.gpu.accept_sample, case.gpu.accept_sample_static):
        case.upload_kv()
        a = torch.full((B,), -7, dtype=torch.int32, device=case.device)
        path = torch.full((B, D + 1), -7, dtype=torch.int32, device=case.device)
        nxt = torch.full((B,), -7, dtype=torch.int32, device=case.device)
        fn(B, ttd, tl, dl, ua, ur, temperature, a, path, nxt, commit)
        torch.cuda.synchronize()
        k, v = case.download_kv()
        outs.append((a.cpu().numpy(), path.cpu().numpy(), nxt.cpu().numpy(), case.kv["ctx_len"].cpu().numpy(), k, v))
    for x, y in zip(*outs):
        np.testing.assert_array_equal(x, y)
    return outs[0][0]


def test_static_scratch_entry_point_equals_workspace_entry_point():
    import paper_2408_08146_amd as K
    big = Case("cfg2_small", n_layers=1, K=1, batch=3)
    big.fill_kv_normal()
    small = Case("cfg1", batch=1)
    a1 = _both(big, 51, 1.0, commit=True)          # 3 sequences x 4000 tokens
    a2 = _both(small, 52, 0.7, commit=True)        # then 1 sequence x 1000 tokens: part of the array keeps old contents
    a3 = _both(big, 53, 1.0, commit=False)
    assert max(a1.max(), a3.max()) >= 1             # acceptances occurred
    # beyond the fixed array: rejected before anything is launched
    huge = Case("cfg2_small", n_layers=1, K=1, batch=70)
    torch = huge.torch
    z = torch.zeros(70, huge.T, huge.V, device=huge.device)
    i32 = lambda *s: torch.zeros(*s, dtype=torch.int32, device=huge.device)
    u = torch.zeros(70, huge.T, device=huge.device)
    with pytest.raises(K.KoalaError) as e:
        huge.gpu.accept_sample_static(70, i32(70, huge.T), z, z, u, u, 1.0, i32(70), i32(70, huge.D + 1), i32(70), False)
    assert e.value.status == -4
