"""The three iteration calls only enqueue kernels on the caller's stream and keep the context length
on the device, so an iteration can be captured into a HIP graph.  Replays (with other work and
synchronisations between them) must reproduce the eager results bit for bit."""
import numpy as np
import pytest

from koala_synth import tensor_normal

from gpu_harness import Case

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfgname", ["cfg1", "cfg2_small"])
def test_captured_iteration_replays_like_eager(cfgname):
    import torch
    case = Case(cfgname, ctx=48 if cfgname == "cfg1" else None)
    case.fill_kv_normal()
    case.upload_kv()
    B, T, D, H, dev = case.B, case.T, case.D, case.H, case.device
    feat_in = case.t(tensor_normal(1, "graph_feat", (B, 1, H)))
    tok_in = case.t(np.full((B, 1), 5, np.int32))
    tokens = torch.zeros(B, T, dtype=torch.int32, device=dev)
    scores = torch.zeros(B, T, dtype=torch.float32, device=dev)
    feat = torch.zeros(B, T, H, dtype=torch.float32, device=dev)
    greedy = torch.zeros(B, T, dtype=torch.int32, device=dev)
    a = torch.zeros(B, dtype=torch.int32, device=dev)
    path = torch.zeros(B, D + 1, dtype=torch.int32, device=dev)
    nxt = torch.zeros(B, dtype=torch.int32, device=dev)
    ctx0 = case.kv["ctx_len"].clone()
    outs = (tokens, scores, feat, greedy, a, path, nxt)

    def step():
        case.kv["ctx_len"].copy_(ctx0)
        case.gpu.draft_expand(B, feat_in, tok_in, 1, tokens, scores)
        case.gpu.tree_verify(B, tokens, feat, None, greedy)
        case.gpu.accept_prefix(B, tokens, greedy, a, path, nxt, True)

    step()
    torch.cuda.synchronize()
    want = [o.clone() for o in outs]
    want_len = case.kv["ctx_len"].clone()
    want_k = case.kv["target_k"].clone()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream's side
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for replay in range(3):
        for o in outs:
            o.fill_(-1)
        junk = torch.randn(1 << 20, device=dev)  # the program's own eager work between replays
        assert torch.isfinite(junk.sum()).item()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(outs, want):
            assert torch.equal(got, ref), replay
        assert torch.equal(case.kv["ctx_len"], want_len)
        assert torch.equal(case.kv["target_k"], want_k)
