#!/usr/bin/env python3
"""Benchmark of one draft-then-verify iteration (draft_expand + tree_verify + accept_prefix) on one MI355X.

A step is one full iteration on the 7B-shape EAGLE-style workload: 32-layer bf16 target, K draft
layers, 26-node depth-5 tree, 1024-token KV context, batch 1, synthetic N(0, 0.02) weights and
N(0, 1) KV / features (all resident in HBM before timing starts).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

# what "dtype" in the JSON line stands for
DTYPE_NOTE = ("GEMMs multiply fp16 x fp16 into fp32 on the matrix pipe: the workload's bf16 weights re-encoded exactly as "
              "fp16, activations rounded to fp16; attention multiplies bf16 (cache) x bf16 hi+lo; KV cache, embeddings "
              "and norm gains are stored in bf16; parity bar: the bf16 one, 2e-2 of a row's largest logit")

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
# kernel arguments in device memory: shaves about a microsecond off every launch (set before HIP starts)
os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes(cfg, T, ctx_lens, D, K, levels, medusa_heads):
    """Bytes that must move per call (bf16 = 2 bytes): weights once per pass, KV context read,
    tree KV written; activations of T*H size are ignored (<1%)."""
    H, F, V, L = cfg["hidden"], cfg["ffn"], cfg["vocab"], cfg["n_layers"]
    b, B, sumC = 2, len(ctx_lens), sum(ctx_lens)
    P_l = 4 * H * H + 3 * H * F
    verify = b * (L * P_l + V * H) + b * L * 2 * H * sumC + b * L * 2 * H * T * B + b * T * B * H
    if cfg["draft"] == "medusa":
        draft = b * (medusa_heads * K * H * H + V * H)
    else:
        passes = 1 + sum(1 for n in levels[1:D] if n > 0)      # catch-up/root pass + expanded levels
        draft = passes * b * (2 * H * H + K * P_l + V * H) + b * K * 2 * H * sumC * passes
    return verify, draft


def device_weights(cfg, torch, K, dev):
    """Random-init weights generated on the device (seeded), in the library's layout."""
    import paper_2408_08146_amd as KO
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    H, F, V = cfg["hidden"], cfg["ffn"], cfg["vocab"]

    def mat(n, k):
        return (torch.randn(n, k, generator=g, device=dev, dtype=torch.float32) * 0.02).to(torch.bfloat16)

    def layer():
        wqkv = KO.device_matrix(mat(3 * H, H))
        wo = KO.device_matrix(mat(H, H))
        gu = mat(2 * F, H)                                       # rows already in the library's order (gate/up
                                                                 # interleaved, rotary pairs adjacent): random anyway
        wgu = KO.device_matrix(gu)
        wd = KO.device_matrix(mat(H, F))
        one = torch.ones(H, dtype=torch.bfloat16, device=dev)
        return (one, wqkv, wo, one.clone(), wgu, wd)

    w = dict(embed=mat(V, H), lm_head=KO.device_matrix(mat(V, H)),
             final_norm=torch.ones(H, dtype=torch.bfloat16, device=dev),
             layers=[layer() for _ in range(cfg["n_layers"])])
    if cfg["draft"] == "medusa":
        w["fc"] = None
        w["draft"] = [KO.device_matrix(mat(H, H)) for _ in range(cfg["medusa_heads"] * K)]
    else:
        w["fc"] = KO.device_matrix(mat(H, 2 * H))
        w["draft"] = [t for _ in range(K) for t in layer()]
    return w


def predictable_device_weights(cfg, torch, K, dev, sigma, gain=4.0):
    """Device-side build of the weight pair koala_synth.predictable_pair describes (greedy successor of
    token t is t+1; the draft's ranking of it is perturbed by sigma), in the library's layout."""
    import paper_2408_08146_amd as KO
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    H, F, V = cfg["hidden"], cfg["ffn"], cfg["vocab"]
    bf = torch.bfloat16

    def mat(n, k):
        return (torch.randn(n, k, generator=g, device=dev, dtype=torch.float32) * 0.02).to(bf)

    def layer():
        one = torch.ones(H, dtype=bf, device=dev)
        return (one, KO.device_matrix(mat(3 * H, H)), KO.device_matrix(torch.zeros(H, H, dtype=bf, device=dev)),
                one.clone(), KO.device_matrix(mat(2 * F, H)), KO.device_matrix(torch.zeros(H, F, dtype=bf, device=dev)))

    embed = mat(V, H)
    lm = (torch.roll(embed.float(), 1, dims=0) * (gain / 0.02)).to(bf)
    w = dict(embed=embed, lm_head=KO.device_matrix(lm), final_norm=torch.ones(H, dtype=bf, device=dev),
             layers=[layer() for _ in range(cfg["n_layers"])])
    fc = torch.zeros(H, 2 * H, dtype=torch.float32, device=dev)
    fc[:, :H] = torch.eye(H, device=dev)
    if sigma:
        fc[:, :H] += sigma / H ** 0.5 * torch.randn(H, H, generator=g, device=dev, dtype=torch.float32)
    w["fc"] = KO.device_matrix(fc.to(bf))
    w["draft"] = [t for _ in range(K) for t in layer()]
    return w


def generation_bench(args):
    """Generation loop (sections 2.2, 4.1): tokens per second of speculative decoding against plain
    autoregressive decoding with the same target on the same device, mean tokens per iteration and the
    accepted-length histogram, for a synthetic weight pair of adjustable draft quality."""
    import torch
    import paper_2408_08146_amd as KO
    from koala_synth import get_config, make_tree
    dev = "cuda:0"
    cfg = get_config(args.config)
    assert cfg["dtype"] == "bf16" and cfg["draft"] == "eagle"
    if cfg["batch"] != 1 or isinstance(cfg["ctx"], tuple):      # the loop runs one sequence: take the shape only
        cfg["batch"], cfg["ctx"] = 1, 1024
    if args.layers:
        cfg["n_layers"] = args.layers
    K = args.K if args.K > 0 else (1 if args.config == "cfg2" else cfg["K"])
    tree = cfg["tree_template"]
    T, D, H, V = tree.n_nodes, tree.depth, cfg["hidden"], cfg["vocab"]
    C, N = int(cfg["ctx"]), args.generate
    cap = C + N + D + T + 64
    shape = dict(hidden=H, n_heads=cfg["n_heads"], head_dim=cfg["head_dim"], ffn=cfg["ffn"], vocab=V,
                 n_layers=cfg["n_layers"], rms_eps=cfg["rms_eps"], rope_base=cfg["rope_base"], dtype=KO.KOALA_BF16)
    w = (predictable_device_weights(cfg, torch, K, dev, args.sigma) if args.sigma >= 0
         else device_weights(cfg, torch, K, dev))
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    kv = KO.alloc_kv(cfg, 1, cap, dev, K)
    for name in ("target_k", "target_v", "draft_k", "draft_v"):
        for l in range(kv[name].shape[0]):
            view = kv[name][l, 0, :, :C]
            view.copy_(torch.randn(view.shape, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16))
    spec = KO.KoalaContext(shape, dict(kind=KO.KOALA_DRAFT_EAGLE, K=K, medusa_heads=0, max_m=D + 1), tree, 1)
    plain = KO.KoalaContext(shape, dict(kind=KO.KOALA_DRAFT_EAGLE, K=K, medusa_heads=0, max_m=1),
                            make_tree([], [1]), 1)
    ws = torch.empty(max(spec.workspace_bytes(), plain.workspace_bytes()), dtype=torch.uint8, device=dev)
    feat_in = torch.randn(1, H, generator=g, device=dev, dtype=torch.float32)
    tok_in = torch.tensor([123], dtype=torch.int32, device=dev)
    out = torch.zeros(N, dtype=torch.int32, device=dev)
    res = {}
    Tp = (T + 3) // 4 * 4
    uniforms = torch.rand(N + 1, 3, Tp, generator=g, device=dev, dtype=torch.float32)
    for name, c, use_draft in (("plain", plain, False), ("speculative", spec, True)):
        c.bind(w, kv, ws)
        best = None
        for rep in range(args.warmup_gen + args.repeat_gen):
            kv["ctx_len"].fill_(C)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            if use_draft and args.sample:
                st = c.generate_sample(feat_in, tok_in, 1, C, N, uniforms, 1.0, out)
            else:
                st = c.generate(feat_in, tok_in, 1, C, N, out, use_draft=use_draft)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            if rep >= args.warmup_gen and (best is None or dt < best[0]):
                best = (dt, st)
        dt, st = best
        res[name] = dict(seconds=dt, iterations=st["iterations"], tokens=st["tokens"],
                         tokens_per_s=st["tokens"] / dt, ms_per_iteration=dt / st["iterations"] * 1e3,
                         mean_tokens_per_iteration=st["tokens"] / st["iterations"],
                         accept_hist=st["accept_hist"][:D + 1], first_tokens=out[:4].tolist())
    spec.close()
    plain.close()
    ratio = res["speculative"]["tokens_per_s"] / res["plain"]["tokens_per_s"]
    print(json.dumps({
        "metric": "speedup_over_autoregressive_decoding", "value": ratio, "unit": "x", "n_gpus": 1,
        "higher_is_better": True, "vs_baseline": None, "dtype": "f16", "dtype_note": DTYPE_NOTE, "data": "synthetic",
        "config": {"workload": f"{args.config}: generation of {N} tokens after a {C}-token context, EAGLE-style K={K}, "
                               f"T={T} depth {D}, {cfg['n_layers']} target layers, batch 1",
                   "weights": (f"predictable pair, sigma={args.sigma}" if args.sigma >= 0 else "random"),
                   "best_of": args.repeat_gen,
                   "acceptance": "stochastic, temperature 1" if args.sample else "greedy"},
        "speculative": res["speculative"], "plain": res["plain"]}))


def training_bench(args):
    """One adversarial training step (section 3.2, Algorithm 1) at the 7B head's sizes: discriminator step,
    draft-head loss/gradient at the logits, and a Medusa-style head's forward + update; fp32, synthetic data."""
    import torch
    import paper_2408_08146_amd as KO
    dev = "cuda:0"
    H, V, DH, n_fc, Kb, N = 4096, 32000, 1024, 2, 2, args.train
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    rnd = lambda *s: torch.randn(*s, generator=g, device=dev, dtype=torch.float32)
    D = KO.Discriminator(rnd(V, H) * 0.02, [rnd(DH, V) * 0.02, rnd(1, DH) * 0.02], [rnd(DH) * 0.02, rnd(1) * 0.02],
                         fc_hidden=DH)
    head = KO.MedusaHeadTrainer([rnd(H, H) * 0.02 for _ in range(Kb)], rnd(V, H) * 0.02)
    h, q = rnd(N, H), rnd(N, V) * 2.0
    d = torch.zeros(N, V, device=dev)
    grad = torch.zeros(N, V, device=dev)
    loss = torch.zeros(3, device=dev)

    def step():
        head.forward(h, d)
        D.gen_grad(h, q, d, 0.5, loss[:2], grad)
        head.step(h, grad, 1e-3)
        D.step(h, q, d, 1e-3, loss[2:])
    for _ in range(2):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    flops = 2.0 * N * (V * H * 4 + DH * V * 5 + Kb * H * H * 3 + V * H * 2)   # dense products of one g-step + d-step
    print(json.dumps({"metric": "adversarial_training_steps_per_s", "value": 1e3 / ms, "unit": "steps/s", "n_gpus": 1,
                      "steps": args.steps, "ms_per_step": ms, "higher_is_better": True, "dtype": "f32",
                      "data": "synthetic", "vs_baseline": None,
                      "config": {"workload": f"one g-step + one d-step, {N} positions, hidden {H}, vocab {V}, "
                                             f"discriminator Linear + {n_fc} FC (width {DH}), Medusa-style head K={Kb}"},
                      "approx_tflops": flops / (ms * 1e-3) / 1e12, "losses_adv_distill_disc": loss.tolist()}))


def cpu_baseline(cfg, tree, K, levels):
    """Time the unmodified fp32 oracle on a bounded sample: tree_verify over 2 of the target layers
    plus final norm / LM head / argmax, and one EAGLE draft pass (fc + K layers + LM head + top-k) for
    the root row; scale linearly to 32 layers and the iteration's draft passes."""
    import numpy as np
    import oracle
    from koala_synth import get_config, target_weights, eagle_weights, tensor_normal, tensor_uniform_int
    import copy
    Ls = 2
    c = copy.deepcopy(cfg)
    c["n_layers"], c["K"] = Ls, K
    Wt = target_weights(c, 0, cache=True)
    Wd = eagle_weights(c, 0, cache=True)
    for n in Wt.names() + Wd.names():                            # generate outside the timed part
        (Wt if n in Wt.shapes else Wd).f32(n)
    T, C = tree.n_nodes, cfg["ctx"]
    dt = np.float32
    tc = oracle.KVCache(Ls, c["n_heads"], C + T + 8, c["head_dim"], dt)
    dc = oracle.KVCache(K, c["n_heads"], C + T + 8, c["head_dim"], dt)
    for l in range(Ls):
        tc.k[l][:, :C] = tensor_normal(1, f"bk{l}", (c["n_heads"], C, c["head_dim"]))
        tc.v[l][:, :C] = tensor_normal(1, f"bv{l}", (c["n_heads"], C, c["head_dim"]))
    for l in range(K):
        dc.k[l][:, :C - 1] = tensor_normal(1, f"dk{l}", (c["n_heads"], C - 1, c["head_dim"]))
        dc.v[l][:, :C - 1] = tensor_normal(1, f"dv{l}", (c["n_heads"], C - 1, c["head_dim"]))
    tt = tensor_uniform_int(1, "tt", (T,), 0, c["vocab"])
    feat = tensor_normal(1, "feat", (1, c["hidden"]))
    # repeat the sample until about 12 s of oracle work has been timed; keep the mean of each part
    t_full = t_head = t_pass = 0.0
    reps = 0
    t_start = time.perf_counter()
    while reps < 3 or time.perf_counter() - t_start < 12.0:
        t0 = time.perf_counter()
        oracle.verify_tree(c, Wt, tc, C, tt, tree.parent, dt)                 # Ls layers + head
        t1 = time.perf_counter()
        oracle.verify_tree(c, Wt, tc, C, tt, tree.parent, dt, n_layers=0)     # head only
        t2 = time.perf_counter()
        # single-node tree: only the root pass of the draft runs (fc + K layers), then LM head + top-k
        oracle.eagle_expand(c, Wt, Wd, dc, C, feat, tt[:1], np.array([-1], np.int32), np.array([0], np.int32),
                            np.array([], np.int32), dt)
        _ = oracle.topk_desc(Wt.f32("lm_head") @ feat[0], 4)
        t3 = time.perf_counter()
        t_full += t1 - t0
        t_head += t2 - t1
        t_pass += t3 - t2
        reps += 1
    t_full, t_head, t_pass = t_full / reps, t_head / reps, t_pass / reps
    passes = 1 + sum(1 for n in levels[1:tree.depth] if n > 0)
    t_layer = (t_full - t_head) / Ls
    est = cfg["n_layers"] * t_layer + t_head + passes * t_pass
    one_thread = None
    try:
        import threadpoolctl
        threads = max([p["num_threads"] for p in threadpoolctl.threadpool_info()] + [1])
        with threadpoolctl.threadpool_limits(limits=1):          # the same sample once on a single core
            t0 = time.perf_counter()
            oracle.verify_tree(c, Wt, tc, C, tt, tree.parent, dt)
            t1 = time.perf_counter()
            oracle.verify_tree(c, Wt, tc, C, tt, tree.parent, dt, n_layers=0)
            t2 = time.perf_counter()
            oracle.eagle_expand(c, Wt, Wd, dc, C, feat, tt[:1], np.array([-1], np.int32), np.array([0], np.int32),
                                np.array([], np.int32), dt)
            _ = oracle.topk_desc(Wt.f32("lm_head") @ feat[0], 4)
            t3 = time.perf_counter()
        est1 = cfg["n_layers"] * ((t1 - t0) - (t2 - t1)) / Ls + (t2 - t1) + passes * (t3 - t2)
        one_thread = dict(value=1.0 / est1, unit="iterations/s", cores=1, seconds_per_iteration_est=est1,
                          sample="the same sample, one repetition, BLAS limited to one thread")
    except Exception:
        threads = os.cpu_count()
    return dict(value=1.0 / est, unit="iterations/s", cores=int(threads), kind="oracle",
                sample=(f"fp32 NumPy oracle, mean of {reps} repetitions (~12 s of CPU work): tree_verify on {Ls} of "
                        f"{cfg['n_layers']} target layers + LM head ({t_full:.2f}s, head {t_head:.2f}s) and one "
                        f"EAGLE draft pass ({t_pass:.2f}s), scaled "
                        f"linearly to {cfg['n_layers']} layers and {passes} draft passes; "
                        f"host has {os.cpu_count()} logical CPUs"),
                seconds_per_iteration_est=est, single_thread=one_thread)


def gpu_state():
    """Clock levels, power and performance level of the first AMD GPU as sysfs reports them (plain file reads:
    no child process is started once the GPU is in use); None where the files are not there."""
    import glob
    out = {}
    for dev in sorted(glob.glob("/sys/class/drm/card*/device")):
        if not os.path.exists(os.path.join(dev, "pp_dpm_sclk")):
            continue

        def rd(name):
            try:
                return open(os.path.join(dev, name)).read().strip()
            except OSError:
                return None
        for key in ("pp_dpm_sclk", "pp_dpm_mclk", "pp_dpm_fclk", "power_dpm_force_performance_level"):
            v = rd(key)
            if v is not None:
                active = [ln.strip() for ln in v.splitlines() if ln.strip().endswith("*")]
                out[key] = active[0] if active else v.splitlines()[-1] if key.startswith("pp_dpm") else v
        for hw in glob.glob(os.path.join(dev, "hwmon", "hwmon*")):
            for key in ("power1_average", "power1_input", "power1_cap"):
                try:
                    out[key + "_W"] = int(open(os.path.join(hw, key)).read()) / 1e6
                except (OSError, ValueError):
                    pass
        break
    return out or None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--K", type=int, default=0, help="draft layers per head (0: 1 for cfg2, else the config's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layers", type=int, default=0, help="override target layer count (debug only)")
    ap.add_argument("--graph", type=int, default=0, help="1: replay the iteration as a captured HIP graph")
    ap.add_argument("--calib-copy", type=int, default=0,
                    help="MiB: first run one plain device copy of this size (reference for counter scaling)")
    ap.add_argument("--generate", type=int, default=0,
                    help="N > 0: instead of the iteration benchmark, generate N tokens with and without the draft "
                         "head and report the speed-up ratio and tokens per iteration")
    ap.add_argument("--sigma", type=float, default=-1.0,
                    help="--generate: draft-quality knob of the predictable weight pair (0 = perfect draft); "
                         "negative = random weights (the draft is almost never right)")
    ap.add_argument("--sample", type=int, default=0,
                    help="1: time the non-greedy iteration (sampled draft, stochastic acceptance) instead of the greedy one")
    ap.add_argument("--train", type=int, default=0,
                    help="N > 0: time one adversarial training step (g-step + d-step) on N positions instead")
    ap.add_argument("--warmup-gen", type=int, default=1)
    ap.add_argument("--repeat-gen", type=int, default=3)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    if args.generate > 0:
        return generation_bench(args)
    if args.train > 0:
        return training_bench(args)

    import torch
    import paper_2408_08146_amd as KO
    from koala_synth import get_config
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    KO.load_library()
    dev = "cuda:0"
    cfg = get_config(args.config)
    assert cfg["dtype"] == "bf16"
    if args.layers:
        cfg["n_layers"] = args.layers
    eagle = cfg["draft"] == "eagle"
    K = args.K if args.K > 0 else (1 if args.config == "cfg2" else cfg["K"])
    B = cfg["batch"]
    tree = cfg["tree_template"]
    T, D, H, V = tree.n_nodes, tree.depth, cfg["hidden"], cfg["vocab"]
    cap = cfg["capacity"]
    if isinstance(cfg["ctx"], tuple):                            # ragged batch: lengths from seed 2
        from koala_synth import tensor_uniform_int
        from koala_synth.configs import SEED_LENGTHS
        ctx_lens = [int(v) for v in tensor_uniform_int(SEED_LENGTHS, "ctx_lens", (B,), cfg["ctx"][0], cfg["ctx"][1] + 1)]
    else:
        ctx_lens = [int(cfg["ctx"])] * B
    C = max(ctx_lens)

    shape = dict(hidden=H, n_heads=cfg["n_heads"], head_dim=cfg["head_dim"], ffn=cfg["ffn"], vocab=V,
                 n_layers=cfg["n_layers"], rms_eps=cfg["rms_eps"], rope_base=cfg["rope_base"], dtype=KO.KOALA_BF16)
    ctx = KO.KoalaContext(shape, dict(kind=KO.KOALA_DRAFT_EAGLE if eagle else KO.KOALA_DRAFT_MEDUSA, K=K,
                                      medusa_heads=cfg["medusa_heads"], max_m=1), tree, B)
    w = device_weights(cfg, torch, K, dev)
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    kv = KO.alloc_kv(cfg, B, cap, dev, K if eagle else 0)
    for name in ("target_k", "target_v", "draft_k", "draft_v"):
        if kv[name] is None:
            continue
        for l in range(kv[name].shape[0]):                       # layer by layer: bounded temporaries
            for b in range(B):
                view = kv[name][l, b, :, :ctx_lens[b]]
                view.copy_(torch.randn(view.shape, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16))
    ws = torch.empty(ctx.workspace_bytes(), dtype=torch.uint8, device=dev)
    ctx.bind(w, kv, ws)

    feat_in = torch.randn(B, 1, H, generator=g, device=dev, dtype=torch.float32)
    tok_in = torch.randint(0, V, (B, 1), generator=g, device=dev, dtype=torch.int32)
    tree_tokens = torch.zeros(B, T, dtype=torch.int32, device=dev)
    scores = torch.zeros(B, T, dtype=torch.float32, device=dev)
    feat_out = torch.zeros(B, T, H, dtype=torch.float32, device=dev)
    greedy = torch.zeros(B, T, dtype=torch.int32, device=dev)
    a_len = torch.zeros(B, dtype=torch.int32, device=dev)
    path = torch.zeros(B, D + 1, dtype=torch.int32, device=dev)
    nxt = torch.zeros(B, dtype=torch.int32, device=dev)
    ctx0 = torch.tensor(ctx_lens, dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream()

    if args.sample:                                              # non-greedy iteration (section 2.2 rule, temperature 1)
        assert eagle, "--sample needs an EAGLE-style draft head"
        u_draw = torch.rand(B, T, generator=g, device=dev, dtype=torch.float32)
        u_acc = torch.rand(B, T, generator=g, device=dev, dtype=torch.float32)
        u_res = torch.rand(B, T, generator=g, device=dev, dtype=torch.float32)
        draft_logits = torch.zeros(B, T, V, dtype=torch.float32, device=dev)
        target_logits = torch.zeros(B, T, V, dtype=torch.float32, device=dev)

    def step(events=None):
        kv["ctx_len"].copy_(ctx0)                                # same workload every step
        if events: events[0].record(stream)
        if args.sample:
            ctx.draft_expand_sample(B, feat_in, tok_in, 1, u_draw, 1.0, tree_tokens, draft_logits)
        else:
            ctx.draft_expand(B, feat_in, tok_in, 1, tree_tokens, scores)
        if events: events[1].record(stream)
        ctx.tree_verify(B, tree_tokens, feat_out, target_logits if args.sample else None, greedy)
        if events: events[2].record(stream)
        if args.sample:
            ctx.accept_sample(B, tree_tokens, target_logits, draft_logits, u_acc, u_res, 1.0, a_len, path, nxt, True)
        else:
            ctx.accept_prefix(B, tree_tokens, greedy, a_len, path, nxt, True)
        if events: events[3].record(stream)
        # feed the result back (device side): the root's feature and the target's next token
        feat_in.copy_(feat_out[:, :1])
        tok_in.copy_(nxt.view(B, 1))

    if args.calib_copy:
        src = torch.ones(args.calib_copy << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                                           # reads and writes calib_copy MiB exactly once
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    run = step
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        run = graph.replay
        for _ in range(3):
            run()
        torch.cuda.synchronize()
    acc_sum = 0
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # per-call breakdown, spread of the iteration time and accepted lengths (separate pass, events on the
    # launch stream around every call)
    n_b = min(args.steps, 200)
    parts = [0.0, 0.0, 0.0]
    iter_ms = []
    for _ in range(n_b):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        step(ev)
        torch.cuda.synchronize()
        for i in range(3):
            parts[i] += ev[i].elapsed_time(ev[i + 1]) / n_b
        iter_ms.append(ev[0].elapsed_time(ev[3]))
        acc_sum += float(a_len.float().mean().item())
    mean_tokens = 1.0 + acc_sum / n_b
    iter_ms.sort()
    pct = lambda q: iter_ms[min(len(iter_ms) - 1, int(q * len(iter_ms)))]

    # what this device delivers for a plain streaming read of 2 GiB (same load instructions as the GEMM)
    probe = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
    probe.fill_(1)
    torch.cuda.synchronize()
    stream_read_gbs = KO.measure_stream_read(probe, repeats=5)
    del probe
    state = gpu_state()                                          # right after sustained work

    # dominant kernel: the weight-streaming GEMM; HIP events around each of its launches
    ctx.profile_begin(8192)
    n_p = min(args.steps, 5)
    for _ in range(n_p):
        step()
    torch.cuda.synchronize()
    gemm_ms, gemm_launches, gemm_bytes = ctx.profile_end()

    levels = [sum(1 for i in range(T) if len(tree.paths[i]) == d and any(tree.parent[j] == i for j in range(T)))
              for d in range(D + 1)]
    vb, db = algorithmic_bytes(cfg, T, ctx_lens, D, K, levels, cfg["medusa_heads"])
    achieved = gemm_bytes / (gemm_ms * 1e-3) / 1e9 if gemm_ms > 0 else 0.0
    traffic = None                                               # HBM bytes per launch from the rocprofv3 PMC runs
    tfile = os.path.join(ROOT, "profiles", f"traffic_weight_gemm_{args.config}.txt")
    if os.path.exists(tfile) and K == 1 and not args.layers:
        for line in open(tfile):
            if line.startswith("traffic_bytes_per_launch="):
                traffic = float(line.split("=")[1])
    out = {
        "metric": "draft_verify_iterations_per_s", "value": 1e3 / ms_per_step, "unit": "iterations/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16", "dtype_note": DTYPE_NOTE, "data": "synthetic",
        "config": {"workload": f"{args.config}: hidden {H}, {'EAGLE' if eagle else 'Medusa'}-style K={K}, T={T} depth "
                               f"{D}, ctx {ctx_lens if B > 1 else C}, {cfg['n_layers']} target layers, batch {B}",
                   "K": K, "tree_nodes": T, "ctx": C, "batch": B,
                   "launch": "hip_graph" if args.graph else "stream",
                   "acceptance": "stochastic, temperature 1" if args.sample else "greedy"},
        "tokens_per_s": 1e3 / ms_per_step * mean_tokens * B, "mean_tokens_per_iteration": mean_tokens,
        "ms_draft_expand": parts[0], "ms_tree_verify": parts[1], "ms_accept_prefix": parts[2],
        "iteration_ms_p10_p50_p90": [pct(0.1), pct(0.5), pct(0.9)], "iterations_in_spread": n_b,
        "measured_stream_read_GBs": stream_read_gbs,
        "verify_frac_of_measured_stream_read": vb / (parts[1] * 1e-3) / 1e9 / stream_read_gbs,
        "verify_bytes": vb, "draft_bytes": db,
        "verify_hbm_frac": vb / (parts[1] * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "iteration_hbm_frac": (vb + db) / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "gpu_state": state,
        "roofline": {"bound": "hbm", "kernel": "k_gemm_rows (weight-streaming GEMM; k_gemm_packed for the LM head)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "launches_timed": gemm_launches, "avg_launch_us": gemm_ms * 1e3 / max(1, gemm_launches),
                     "avg_launch_bytes": gemm_bytes / max(1, gemm_launches)},
    }
    # context only: tokens/s this iteration rate would give at the average tokens per iteration the paper reports
    # for a trained head of this kind on Vicuna 7B (Table 1: EAGLE 3.91 at K=1, 4.20 at K=2, 4.36 at K=3)
    paper_l = {("cfg2", 1): 3.91, ("cfg2", 2): 4.20, ("cfg2", 3): 4.36}.get((args.config, K))
    if paper_l and eagle and not args.sample:
        out["projection_context_only"] = {"tokens_per_iteration_from_paper_table_1": paper_l,
                                          "tokens_per_s": 1e3 / ms_per_step * paper_l}
    if not args.no_cpu_baseline and eagle and B == 1:
        out["cpu_baseline"] = cpu_baseline(cfg, tree, K, levels)
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
