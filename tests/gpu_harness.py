"""Builds one workload twice - as oracle state (NumPy) and as device state bound to
the HIP library - from the same seeded inputs, and holds the comparison rules."""
from __future__ import annotations

import numpy as np

import oracle
from koala_synth import (get_config, target_weights, eagle_weights, medusa_weights, tensor_normal,
                         tensor_uniform_int, to_bf16_bits, bf16_bits_to_f32)
from koala_synth.configs import SEED_WEIGHTS, SEED_INPUTS, SEED_LENGTHS

TOL = {"fp32": 1e-4, "bf16": 2e-2}


def rel_err_rows(got, ref):
    """Per row: max |got - ref| / max |ref|."""
    got = np.asarray(got, np.float64).reshape(-1, got.shape[-1])
    ref = np.asarray(ref, np.float64).reshape(-1, ref.shape[-1])
    return np.abs(got - ref).max(-1) / np.maximum(np.abs(ref).max(-1), 1e-30)


def top_margin(ref_row, k=1):
    """Smallest gap between consecutive entries among the k+1 largest, relative to max |ref|."""
    s = np.sort(np.asarray(ref_row, np.float64))[::-1][: k + 1]
    return float(np.min(s[:-1] - s[1:]) / max(np.abs(ref_row).max(), 1e-30))


def _round(cfg, x):
    return bf16_bits_to_f32(to_bf16_bits(x)) if cfg["dtype"] == "bf16" else x.astype(np.float32)


class Case:
    def __init__(self, name, device="cuda", n_layers=None, norm_gain="random", batch=None, ctx=None,
                 K=None, max_m=None, make_gpu=True, kv_storage_rounding=False, weights=None, **over):
        import torch
        cfg = get_config(name, **over)
        if n_layers is not None:
            cfg["n_layers"] = n_layers
        if K is not None:
            cfg["K"] = K
        if batch is not None:
            cfg["batch"] = batch
        if ctx is not None:
            cfg["ctx"] = ctx
        self.cfg, self.tree = cfg, cfg["tree_template"]
        self.B, self.T, self.D = cfg["batch"], self.tree.n_nodes, self.tree.depth
        self.H, self.V = cfg["hidden"], cfg["vocab"]
        self.tol = TOL[cfg["dtype"]]
        self.eagle = cfg["draft"] == "eagle"
        if weights is not None:          # weights: function cfg -> (target, draft) weight providers
            self.Wt, self.Wd = weights(cfg)
        else:
            self.Wt = target_weights(cfg, SEED_WEIGHTS, norm_gain=norm_gain, cache=True)
            self.Wd = (eagle_weights if self.eagle else medusa_weights)(
                cfg, SEED_WEIGHTS, **({"norm_gain": norm_gain} if self.eagle else {}), cache=True)
        if isinstance(cfg["ctx"], list):          # explicit length per sequence
            assert len(cfg["ctx"]) == self.B
            self.ctx_lens = [int(v) for v in cfg["ctx"]]
        elif isinstance(cfg["ctx"], tuple):
            lo, hi = cfg["ctx"]
            self.ctx_lens = [int(v) for v in tensor_uniform_int(SEED_LENGTHS, "ctx_lens", (self.B,), lo, hi + 1)]
        else:
            self.ctx_lens = [int(cfg["ctx"])] * self.B
        self.cap = cfg["capacity"]
        assert self.cap >= max(self.ctx_lens) + self.T
        self.max_m = max_m or 1
        self.device = device
        L, nh, dh = cfg["n_layers"], cfg["n_heads"], cfg["head_dim"]
        # kv_storage_rounding: the oracle rounds every key/value row it writes to the cache's bf16
        # storage format (the device cache is bf16); off = rows stay exact
        store = None
        if kv_storage_rounding and cfg["dtype"] == "bf16":
            store = lambda a: bf16_bits_to_f32(to_bf16_bits(np.asarray(a, np.float32))).astype(np.float64)
        self.tc = [oracle.KVCache(L, nh, self.cap, dh, store=store) for _ in range(self.B)]
        self.dc = ([oracle.KVCache(cfg["K"], nh, self.cap, dh, store=store) for _ in range(self.B)]
                   if self.eagle else None)
        self.gpu = None
        if make_gpu:
            self._make_gpu(torch)

    # ---------------------------------------------------------------- device side
    def _make_gpu(self, torch):
        import paper_2408_08146_amd as K
        cfg = self.cfg
        shape = dict(hidden=cfg["hidden"], n_heads=cfg["n_heads"], head_dim=cfg["head_dim"], ffn=cfg["ffn"],
                     vocab=cfg["vocab"], n_layers=cfg["n_layers"], rms_eps=cfg["rms_eps"],
                     rope_base=cfg["rope_base"], dtype=K.KOALA_BF16 if cfg["dtype"] == "bf16" else K.KOALA_FP32)
        draft = dict(kind=K.KOALA_DRAFT_EAGLE if self.eagle else K.KOALA_DRAFT_MEDUSA, K=cfg["K"],
                     medusa_heads=cfg["medusa_heads"], max_m=self.max_m)
        self.gpu = K.KoalaContext(shape, draft, self.tree, self.B)
        w = K.pack_target_weights(self.Wt, cfg, self.device)
        w.update((K.pack_eagle_weights if self.eagle else K.pack_medusa_weights)(self.Wd, cfg, self.device))
        self.kv = K.alloc_kv(cfg, self.B, self.cap, self.device, cfg["K"] if self.eagle else 0)
        # every byte 0x7f (3.4e38 as fp32 or bf16): a kernel that reads workspace memory nobody has written gets a
        # value that wrecks the comparison instead of a zero that happens to be harmless
        self.ws = torch.full((self.gpu.workspace_bytes(),), 0x7f, dtype=torch.uint8, device=self.device)
        self.gpu.bind(w, self.kv, self.ws)
        self.torch = torch

    def upload_kv(self):
        """Copy the oracle caches (all slots) and context lengths to the device."""
        torch = self.torch
        td = torch.bfloat16 if self.cfg["dtype"] == "bf16" else torch.float32

        def put(dst, caches, which):
            for b, c in enumerate(caches):
                arr = np.stack(getattr(c, which)).astype(np.float32)          # [L, nh, cap, dh]
                dst[:, b].copy_(torch.from_numpy(arr).to(self.device).to(td))
        put(self.kv["target_k"], self.tc, "k")
        put(self.kv["target_v"], self.tc, "v")
        if self.eagle:
            put(self.kv["draft_k"], self.dc, "k")
            put(self.kv["draft_v"], self.dc, "v")
        self.kv["ctx_len"].copy_(torch.tensor(self.ctx_lens, dtype=torch.int32))

    def download_kv(self, which="target"):
        k = self.kv[f"{which}_k"].float().cpu().numpy()
        v = self.kv[f"{which}_v"].float().cpu().numpy()
        return k, v                                                            # [L, B, nh, cap, dh]

    # ---------------------------------------------------------------- inputs
    def fill_kv_normal(self, m=1):
        """KV caches ~ N(0,1) (keys taken as already rotated), rounded to the model dtype:
        target rows 0..C-1, draft rows 0..C-m-1."""
        cfg = self.cfg
        for b in range(self.B):
            C = self.ctx_lens[b]
            for which, caches, rows in (("target", self.tc, C), ("draft", self.dc, C - m)):
                if caches is None:
                    continue
                c = caches[b]
                for l in range(len(c.k)):
                    shp = (cfg["n_heads"], rows, cfg["head_dim"])
                    c.k[l][:, :rows] = _round(cfg, tensor_normal(SEED_INPUTS, f"kv.{which}.k.{b}.{l}", shp))
                    c.v[l][:, :rows] = _round(cfg, tensor_normal(SEED_INPUTS, f"kv.{which}.v.{b}.{l}", shp))

    def normal_draft_inputs(self, m=1):
        feat = tensor_normal(SEED_INPUTS, "feat_in", (self.B, m, self.H)).astype(np.float32)
        tok = tensor_uniform_int(SEED_INPUTS, "tok_in", (self.B, m), 0, self.V)
        return feat, tok

    def random_tree_tokens(self, tag="tree_tokens"):
        return tensor_uniform_int(SEED_INPUTS, tag, (self.B, self.T), 0, self.V)

    def prefill_oracle(self, prompt_tokens):
        """Real prefill with the oracle (single sequence): fills the target cache, returns feats, logits."""
        assert self.B == 1
        feats, logits = oracle.prefill(self.cfg, self.Wt, self.tc[0], prompt_tokens)
        self.ctx_lens = [len(prompt_tokens)]
        return feats, logits

    # ---------------------------------------------------------------- device calls
    def t(self, arr, dtype=None):
        torch = self.torch
        x = torch.from_numpy(np.ascontiguousarray(arr)).to(self.device)
        return x if dtype is None else x.to(dtype)

    def gpu_verify(self, tree_tokens, want_logits=True):
        torch = self.torch
        B, T = self.B, self.T
        tt = self.t(np.asarray(tree_tokens, np.int32).reshape(B, T))
        feat = torch.empty(B, T, self.H, dtype=torch.float32, device=self.device)
        logits = torch.empty(B, T, self.V, dtype=torch.float32, device=self.device) if want_logits else None
        greedy = torch.empty(B, T, dtype=torch.int32, device=self.device)
        self.gpu.tree_verify(B, tt, feat, logits, greedy)
        torch.cuda.synchronize()
        return feat.cpu().numpy(), (logits.cpu().numpy() if want_logits else None), greedy.cpu().numpy()

    def gpu_generate(self, feat_in, tok_in, max_new, use_draft=True):
        """koala_generate on sequence 0.  Returns (tokens[max_new], stats dict)."""
        torch = self.torch
        feat_in = np.asarray(feat_in, np.float32).reshape(-1, self.H)
        tok_in = np.asarray(tok_in, np.int32).reshape(-1)
        m = len(tok_in)
        out = torch.full((max_new,), -1, dtype=torch.int32, device=self.device)
        stats = self.gpu.generate(self.t(feat_in), self.t(tok_in), m, self.ctx_lens[0], max_new, out,
                                  use_draft=use_draft)
        torch.cuda.synchronize()
        return out.cpu().numpy(), stats

    def gpu_draft_sample(self, feat_in, tok_in, u_draw, temperature=1.0):
        """koala_draft_expand_sample.  Returns (tokens[B,T], draft_logits[B,T,V])."""
        torch = self.torch
        B, T = self.B, self.T
        feat_in = np.asarray(feat_in, np.float32).reshape(B, -1, self.H)
        tok_in = np.asarray(tok_in, np.int32).reshape(B, -1)
        m = tok_in.shape[1]
        tokens = torch.full((B, T), -1, dtype=torch.int32, device=self.device)
        dl = torch.zeros(B, T, self.V, dtype=torch.float32, device=self.device)
        self.gpu.draft_expand_sample(B, self.t(feat_in), self.t(tok_in), m,
                                     self.t(np.asarray(u_draw, np.float32).reshape(B, T)), temperature, tokens, dl)
        torch.cuda.synchronize()
        return tokens.cpu().numpy(), dl

    def gpu_accept_sample(self, tree_tokens, target_logits, draft_logits, u_accept, u_resample, temperature=1.0,
                          commit=False):
        """koala_accept_sample; logits may be numpy arrays or device tensors [B,T,V]."""
        torch = self.torch
        B, T, D = self.B, self.T, self.D
        as_dev = lambda x: x if isinstance(x, torch.Tensor) else self.t(np.asarray(x, np.float32).reshape(B, T, self.V))
        a = torch.full((B,), -7, dtype=torch.int32, device=self.device)
        path = torch.full((B, D + 1), -7, dtype=torch.int32, device=self.device)
        nxt = torch.full((B,), -7, dtype=torch.int32, device=self.device)
        self.gpu.accept_sample(B, self.t(np.asarray(tree_tokens, np.int32).reshape(B, T)), as_dev(target_logits),
                               as_dev(draft_logits), self.t(np.asarray(u_accept, np.float32).reshape(B, T)),
                               self.t(np.asarray(u_resample, np.float32).reshape(B, T)), temperature, a, path, nxt,
                               commit)
        torch.cuda.synchronize()
        return a.cpu().numpy(), path.cpu().numpy(), nxt.cpu().numpy()

    def gpu_draft(self, feat_in, tok_in):
        torch = self.torch
        B, T = self.B, self.T
        m = tok_in.shape[1]
        f = self.t(np.asarray(feat_in, np.float32).reshape(B, m, self.H))
        tk = self.t(np.asarray(tok_in, np.int32).reshape(B, m))
        tt = torch.full((B, T), -1, dtype=torch.int32, device=self.device)
        sc = torch.zeros(B, T, dtype=torch.float32, device=self.device)
        self.gpu.draft_expand(B, f, tk, m, tt, sc)
        torch.cuda.synchronize()
        return tt.cpu().numpy(), sc.cpu().numpy()

    def gpu_accept(self, tree_tokens, greedy, commit):
        torch = self.torch
        B, T, D = self.B, self.T, self.D
        tt = self.t(np.asarray(tree_tokens, np.int32).reshape(B, T))
        g = self.t(np.asarray(greedy, np.int32).reshape(B, T))
        a = torch.full((B,), -7, dtype=torch.int32, device=self.device)
        path = torch.full((B, D + 1), -7, dtype=torch.int32, device=self.device)
        nxt = torch.full((B,), -7, dtype=torch.int32, device=self.device)
        self.gpu.accept_prefix(B, tt, g, a, path, nxt, commit)
        torch.cuda.synchronize()
        return a.cpu().numpy(), path.cpu().numpy(), nxt.cpu().numpy()

    # ---------------------------------------------------------------- oracle calls
    def oracle_verify(self, tree_tokens):
        outs = [oracle.verify_tree(self.cfg, self.Wt, self.tc[b], self.ctx_lens[b],
                                   np.asarray(tree_tokens).reshape(self.B, self.T)[b], self.tree.parent)
                for b in range(self.B)]
        return (np.stack([o[0] for o in outs]), np.stack([o[1] for o in outs]), np.stack([o[2] for o in outs]))

    def oracle_draft(self, feat_in, tok_in):
        t = self.tree
        outs = []
        for b in range(self.B):
            if self.eagle:
                outs.append(oracle.eagle_expand(self.cfg, self.Wt, self.Wd, self.dc[b], self.ctx_lens[b],
                                                feat_in[b], tok_in[b], t.parent, t.rank, t.topk_per_depth))
            else:
                outs.append(oracle.medusa_expand(self.cfg, self.Wt, self.Wd, feat_in[b][-1], int(tok_in[b][-1]),
                                                 t.parent, t.rank, t.topk_per_depth))
        return outs


def compare_logits_and_greedy(case, got_logits, got_greedy, ref_logits, ref_greedy):
    """Logit rows within tolerance; greedy ids equal except where the oracle's top-2 margin is
    below the tolerance.  Returns the number of rows skipped by the margin rule."""
    err = rel_err_rows(got_logits, ref_logits)
    assert err.max() < case.tol, f"logit error {err.max():.3e} exceeds {case.tol}"
    skipped = 0
    G = np.asarray(got_greedy).reshape(-1)
    R = np.asarray(ref_greedy).reshape(-1)
    RL = np.asarray(ref_logits).reshape(len(R), -1)
    for i in range(len(R)):
        if G[i] != R[i]:
            assert top_margin(RL[i]) < case.tol, f"row {i}: greedy {G[i]} != {R[i]} with a clear margin"
            skipped += 1
    return skipped, float(err.max())


def compare_draft_tokens(case, got_tokens, got_scores, ref_outs):
    """Tree tokens equal the oracle's; a node may differ only if, under its parent, the oracle's
    top-(k+1) logits are closer than the tolerance - its subtree is then not compared."""
    t = case.tree
    depth = oracle.tree_depths(t.parent)
    n_cmp = n_skip = 0
    for b, ref in enumerate(ref_outs):
        tainted = set()
        for i in range(case.T):
            p = int(t.parent[i])
            if p in tainted:
                tainted.add(i)
                continue
            if i == 0:
                assert got_tokens[b, 0] == ref["tokens"][0]
                continue
            n_cmp += 1
            if got_tokens[b, i] != ref["tokens"][i]:
                d = int(depth[i])
                row = ref["logits"][p] if case.eagle else ref["logits"][d - 1]
                assert top_margin(row, int(t.topk_per_depth[d - 1])) < case.tol, \
                    f"seq {b} node {i}: token {got_tokens[b, i]} != {ref['tokens'][i]} with clear margins"
                tainted.add(i)
                n_skip += 1
                continue
            scale = np.abs(ref["logits"][p] if case.eagle else ref["logits"][depth[i] - 1]).max()
            assert abs(got_scores[b, i] - ref["scores"][i]) <= case.tol * scale
    return n_cmp, n_skip
