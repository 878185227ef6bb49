"""ctypes binding of the C ABI declared in include/koala.h (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os

KOALA_FP32, KOALA_BF16 = 0, 1
KOALA_DRAFT_EAGLE, KOALA_DRAFT_MEDUSA = 0, 1

EXPORTS = ("koala_create", "koala_workspace_bytes", "koala_bind", "koala_draft_expand",
           "koala_tree_verify", "koala_accept_prefix", "koala_generate", "koala_draft_expand_sample",
           "koala_accept_sample", "koala_accept_sample_static", "koala_generate_sample", "koala_weights_to_half",
           "koala_measure_stream_read", "koala_profile_begin",
           "koala_profile_end", "koala_train_workspace_bytes", "koala_train_disc_step", "koala_train_gen_grad",
           "koala_train_medusa_workspace_bytes", "koala_train_medusa_head_forward", "koala_train_medusa_head_step",
           "koala_last_error", "koala_destroy")

_STATUS = {0: "KOALA_OK", -1: "KOALA_E_NULL", -2: "KOALA_E_SHAPE", -3: "KOALA_E_ALIGN",
           -4: "KOALA_E_CAPACITY", -5: "KOALA_E_UNSUPPORTED", -6: "KOALA_E_WORKSPACE",
           -7: "KOALA_E_DEVICE"}


STATUS_BY_NAME = {name: code for code, name in _STATUS.items()}


class KoalaError(RuntimeError):
    def __init__(self, status, msg=""):
        self.status = status
        super().__init__(f"{_STATUS.get(status, status)}: {msg}")


class _Shape(C.Structure):
    _fields_ = [("hidden", C.c_int), ("n_heads", C.c_int), ("head_dim", C.c_int), ("ffn", C.c_int),
                ("vocab", C.c_int), ("n_layers", C.c_int), ("rms_eps", C.c_float),
                ("rope_base", C.c_float), ("dtype", C.c_int)]


class _DraftShape(C.Structure):
    _fields_ = [("kind", C.c_int), ("K", C.c_int), ("medusa_heads", C.c_int), ("max_m", C.c_int)]


class _Tree(C.Structure):
    _fields_ = [("n_nodes", C.c_int), ("depth", C.c_int), ("parent", C.POINTER(C.c_int32)),
                ("rank", C.POINTER(C.c_int32)), ("topk_per_depth", C.POINTER(C.c_int32))]


class _Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("layer_w", C.POINTER(C.c_void_p)), ("fc", C.c_void_p),
                ("draft_w", C.POINTER(C.c_void_p))]


class _GenStats(C.Structure):
    _fields_ = [("iterations", C.c_int32), ("tokens", C.c_int32), ("accept_hist", C.c_int32 * 64)]


class _DiscShape(C.Structure):
    _fields_ = [("hidden", C.c_int), ("vocab", C.c_int), ("fc_hidden", C.c_int), ("n_fc", C.c_int)]


class _DiscParams(C.Structure):
    _fields_ = [("w_lin", C.c_void_p), ("w_fc", C.c_void_p * 3), ("b_fc", C.c_void_p * 3)]


class _KV(C.Structure):
    _fields_ = [("target_k", C.c_void_p), ("target_v", C.c_void_p), ("draft_k", C.c_void_p),
                ("draft_v", C.c_void_p), ("capacity", C.c_int), ("ctx_len", C.c_void_p)]


def library_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libkoala.so")


_LIB = None


def load_library():
    """Load libkoala.so; there is no fallback - a missing library is an error."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise KoalaError(-7, f"{path} not found: build it with `python -m paper_2408_08146_amd.build` "
                             "(or __graft_entry__.build())")
    # PyTorch first: it ships its own HIP runtime, and the pointers and streams handed to the library come
    # from it.  Loading the library before torch would bring a second runtime into the process.
    import torch  # noqa: F401
    lib = C.CDLL(path)
    vp, ip = C.c_void_p, C.c_int
    lib.koala_create.argtypes = [C.POINTER(_Shape), C.POINTER(_DraftShape), C.POINTER(_Tree), ip, C.POINTER(vp)]
    lib.koala_workspace_bytes.argtypes = [vp, C.POINTER(C.c_size_t)]
    lib.koala_bind.argtypes = [vp, C.POINTER(_Weights), C.POINTER(_KV), vp, C.c_size_t]
    lib.koala_draft_expand.argtypes = [vp, vp, ip, vp, vp, ip, vp, vp]
    lib.koala_tree_verify.argtypes = [vp, vp, ip, vp, vp, vp, vp]
    lib.koala_accept_prefix.argtypes = [vp, vp, ip, vp, vp, vp, vp, vp, ip]
    lib.koala_generate.argtypes = [vp, vp, vp, vp, ip, ip, ip, ip, vp, C.POINTER(_GenStats)]
    lib.koala_draft_expand_sample.argtypes = [vp, vp, ip, vp, vp, ip, vp, C.c_float, vp, vp]
    lib.koala_accept_sample.argtypes = [vp, vp, ip, vp, vp, vp, vp, vp, C.c_float, vp, vp, vp, ip]
    lib.koala_accept_sample_static.argtypes = lib.koala_accept_sample.argtypes
    lib.koala_generate_sample.argtypes = [vp, vp, vp, vp, ip, ip, ip, vp, ip, C.c_float, vp, C.POINTER(_GenStats)]
    lib.koala_weights_to_half.argtypes = [vp, vp, C.c_size_t]
    lib.koala_measure_stream_read.argtypes = [vp, vp, C.c_size_t, vp, ip, C.POINTER(C.c_double)]
    lib.koala_profile_begin.argtypes = [vp, ip]
    lib.koala_profile_end.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(ip), C.POINTER(C.c_double)]
    fl = C.c_float
    lib.koala_train_workspace_bytes.argtypes = [C.POINTER(_DiscShape), ip, C.POINTER(C.c_size_t)]
    lib.koala_train_disc_step.argtypes = [C.POINTER(_DiscShape), C.POINTER(_DiscParams), vp, ip, vp, vp, vp, fl, vp,
                                          C.c_size_t, vp]
    lib.koala_train_gen_grad.argtypes = [C.POINTER(_DiscShape), C.POINTER(_DiscParams), vp, ip, vp, vp, vp, fl, vp,
                                         C.c_size_t, vp, vp]
    lib.koala_train_medusa_workspace_bytes.argtypes = [ip, ip, ip, C.POINTER(C.c_size_t)]
    lib.koala_train_medusa_head_forward.argtypes = [vp, ip, ip, ip, ip, C.POINTER(vp), vp, vp, vp, C.c_size_t, vp]
    lib.koala_train_medusa_head_step.argtypes = [vp, ip, ip, ip, ip, C.POINTER(vp), vp, vp, vp, fl, vp, C.c_size_t]
    lib.koala_last_error.argtypes = [vp]
    lib.koala_last_error.restype = C.c_char_p
    lib.koala_destroy.argtypes = [vp]
    lib.koala_destroy.restype = None
    for n in EXPORTS[:20]:
        getattr(lib, n).restype = C.c_int
    _LIB = lib
    return lib


def weights_to_f16(packed, stream=None):
    """A fragment-major bfloat16 weight matrix (flat device tensor) rewritten in place as fp16 by the library
    (koala_weights_to_half); returns the same memory viewed as float16.  Call once per matrix."""
    import torch
    lib = load_library()
    assert packed.dtype == torch.bfloat16 and packed.is_cuda and packed.is_contiguous()
    rc = lib.koala_weights_to_half(_stream(stream), C.c_void_p(packed.data_ptr()), packed.numel())
    if rc != 0:
        raise KoalaError(rc, "koala_weights_to_half failed")
    return packed.view(torch.float16)


def weights_to_half_status(ptr, n_elements, stream=None):
    """The raw status of koala_weights_to_half for a device address and an element count (tests of its argument
    checks use this; everyone else wants weights_to_f16)."""
    return load_library().koala_weights_to_half(_stream(stream), C.c_void_p(ptr), n_elements)


def measure_stream_read(buffer, repeats=5, stream=None):
    """GB/s at which the device streams the whole tensor `buffer` through a plain read kernel."""
    import torch
    lib = load_library()
    out = C.c_double()
    sink = torch.zeros(64, dtype=torch.int32, device=buffer.device)
    rc = lib.koala_measure_stream_read(_stream(stream), C.c_void_p(buffer.data_ptr()),
                                       buffer.numel() * buffer.element_size(), C.c_void_p(sink.data_ptr()), repeats,
                                       C.byref(out))
    if rc != 0:
        raise KoalaError(rc, "koala_measure_stream_read failed")
    return out.value


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is not None:
        return C.c_void_p(stream.cuda_stream)
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class KoalaContext:
    """One model shape + draft head + tree template bound to device memory.

    shape: dict(hidden, n_heads, head_dim, ffn, vocab, n_layers, rms_eps, rope_base, dtype)
    draft: dict(kind, K, medusa_heads, max_m); tree: object with parent, rank,
    topk_per_depth (int32 numpy arrays) and depth.
    """

    def __init__(self, shape: dict, draft: dict, tree, max_batch: int = 1):
        import numpy as np
        self.lib = load_library()
        self._h = C.c_void_p()
        self.shape, self.draft, self.tree, self.max_batch = dict(shape), dict(draft), tree, max_batch
        sh = _Shape(shape["hidden"], shape["n_heads"], shape["head_dim"], shape["ffn"], shape["vocab"],
                    shape["n_layers"], shape["rms_eps"], shape["rope_base"], shape["dtype"])
        dr = _DraftShape(draft["kind"], draft["K"], draft.get("medusa_heads", 0), draft.get("max_m", 1))
        par = np.ascontiguousarray(tree.parent, dtype=np.int32)
        rnk = np.ascontiguousarray(tree.rank, dtype=np.int32)
        tk = np.ascontiguousarray(tree.topk_per_depth, dtype=np.int32)
        i32p = C.POINTER(C.c_int32)
        tr = _Tree(len(par), int(tree.depth), par.ctypes.data_as(i32p), rnk.ctypes.data_as(i32p),
                   tk.ctypes.data_as(i32p))
        st = self.lib.koala_create(C.byref(sh), C.byref(dr), C.byref(tr), max_batch, C.byref(self._h))
        if st != 0:
            raise KoalaError(st, "koala_create rejected the configuration")
        self.n_nodes, self.depth = len(par), int(tree.depth)
        self._keep = None

    def _check(self, st):
        if st != 0:
            raise KoalaError(st, self.lib.koala_last_error(self._h).decode())

    def workspace_bytes(self) -> int:
        n = C.c_size_t()
        self._check(self.lib.koala_workspace_bytes(self._h, C.byref(n)))
        return n.value

    def bind(self, weights: dict, kv: dict, workspace):
        """weights: embed, lm_head, final_norm, layers (list of 6-tuples), fc (or None),
        draft (list of tensors).  kv: target_k, target_v, draft_k, draft_v, capacity, ctx_len."""
        lw = [t for layer in weights["layers"] for t in layer]
        dw = list(weights["draft"])
        lw_arr = (C.c_void_p * len(lw))(*[t.data_ptr() for t in lw])
        dw_arr = (C.c_void_p * max(1, len(dw)))(*[t.data_ptr() for t in dw])
        w = _Weights(_ptr(weights["embed"]), _ptr(weights["lm_head"]), _ptr(weights["final_norm"]),
                     C.cast(lw_arr, C.POINTER(C.c_void_p)), _ptr(weights.get("fc")),
                     C.cast(dw_arr, C.POINTER(C.c_void_p)))
        k = _KV(_ptr(kv["target_k"]), _ptr(kv["target_v"]), _ptr(kv.get("draft_k")), _ptr(kv.get("draft_v")),
                int(kv["capacity"]), _ptr(kv["ctx_len"]))
        self._check(self.lib.koala_bind(self._h, C.byref(w), C.byref(k), _ptr(workspace),
                                        workspace.numel() * workspace.element_size()))
        self._keep = (weights, kv, workspace)       # the library borrows these

    def draft_expand(self, batch, feat_in, tok_in, m, tree_tokens, tree_scores=None, stream=None):
        self._check(self.lib.koala_draft_expand(self._h, _stream(stream), batch, _ptr(feat_in), _ptr(tok_in), m,
                                                _ptr(tree_tokens), _ptr(tree_scores)))

    def tree_verify(self, batch, tree_tokens, feat_out, logits_out, greedy_out, stream=None):
        self._check(self.lib.koala_tree_verify(self._h, _stream(stream), batch, _ptr(tree_tokens), _ptr(feat_out),
                                               _ptr(logits_out), _ptr(greedy_out)))

    def accept_prefix(self, batch, tree_tokens, greedy, accept_len, accept_path, next_token, commit,
                      stream=None):
        self._check(self.lib.koala_accept_prefix(self._h, _stream(stream), batch, _ptr(tree_tokens), _ptr(greedy),
                                                 _ptr(accept_len), _ptr(accept_path), _ptr(next_token),
                                                 1 if commit else 0))

    def generate(self, feat_in, tok_in, m, ctx_len0, max_new, out_tokens, use_draft=True, stream=None):
        """Returns dict(iterations, tokens, accept_hist[list])."""
        st = _GenStats()
        self._check(self.lib.koala_generate(self._h, _stream(stream), _ptr(feat_in), _ptr(tok_in), m, ctx_len0,
                                            max_new, 1 if use_draft else 0, _ptr(out_tokens), C.byref(st)))
        return dict(iterations=st.iterations, tokens=st.tokens, accept_hist=list(st.accept_hist))

    def generate_sample(self, feat_in, tok_in, m, ctx_len0, max_new, uniforms, temperature, out_tokens, stream=None):
        """uniforms: device fp32 [max_iters, 3, n_nodes rounded up to 4].  Returns the statistics dict."""
        st = _GenStats()
        self._check(self.lib.koala_generate_sample(self._h, _stream(stream), _ptr(feat_in), _ptr(tok_in), m, ctx_len0,
                                                   max_new, _ptr(uniforms), int(uniforms.shape[0]), float(temperature),
                                                   _ptr(out_tokens), C.byref(st)))
        return dict(iterations=st.iterations, tokens=st.tokens, accept_hist=list(st.accept_hist))

    def draft_expand_sample(self, batch, feat_in, tok_in, m, u_draw, temperature, tree_tokens, draft_logits,
                            stream=None):
        self._check(self.lib.koala_draft_expand_sample(self._h, _stream(stream), batch, _ptr(feat_in), _ptr(tok_in), m,
                                                       _ptr(u_draw), float(temperature), _ptr(tree_tokens),
                                                       _ptr(draft_logits)))

    def accept_sample(self, batch, tree_tokens, target_logits, draft_logits, u_accept, u_resample, temperature,
                      accept_len, accept_path, next_token, commit, stream=None):
        self._check(self.lib.koala_accept_sample(self._h, _stream(stream), batch, _ptr(tree_tokens),
                                                 _ptr(target_logits), _ptr(draft_logits), _ptr(u_accept),
                                                 _ptr(u_resample), float(temperature), _ptr(accept_len),
                                                 _ptr(accept_path), _ptr(next_token), 1 if commit else 0))

    def accept_sample_static(self, batch, tree_tokens, target_logits, draft_logits, u_accept, u_resample,
                             temperature, accept_len, accept_path, next_token, commit, stream=None):
        self._check(self.lib.koala_accept_sample_static(self._h, _stream(stream), batch, _ptr(tree_tokens),
                                                        _ptr(target_logits), _ptr(draft_logits), _ptr(u_accept),
                                                        _ptr(u_resample), float(temperature), _ptr(accept_len),
                                                        _ptr(accept_path), _ptr(next_token), 1 if commit else 0))

    def profile_begin(self, max_launches=4096):
        self._check(self.lib.koala_profile_begin(self._h, max_launches))

    def profile_end(self):
        """Returns (summed GEMM kernel ms, timed launches, weight bytes streamed by them)."""
        ms, n, b = C.c_double(), C.c_int(), C.c_double()
        self._check(self.lib.koala_profile_end(self._h, C.byref(ms), C.byref(n), C.byref(b)))
        return ms.value, n.value, b.value

    def close(self):
        if self._h:
            self.lib.koala_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Discriminator:
    """Discriminator of the adversarial training step (section 3.2) bound to fp32 device tensors:
    w_lin [vocab, hidden], w_fc / b_fc lists of the fully connected layers' weights and biases."""

    def __init__(self, w_lin, w_fc, b_fc, fc_hidden=0):
        self.lib = load_library()
        self.w_lin, self.w_fc, self.b_fc = w_lin, list(w_fc), list(b_fc)
        V, H = w_lin.shape
        self.shape = _DiscShape(H, V, int(fc_hidden), len(self.w_fc))
        p = _DiscParams()
        p.w_lin = w_lin.data_ptr()
        for k in range(len(self.w_fc)):
            p.w_fc[k] = self.w_fc[k].data_ptr()
            p.b_fc[k] = self.b_fc[k].data_ptr()
        self.params = p
        self._ws = None

    def _workspace(self, n):
        import torch
        need = C.c_size_t()
        rc = self.lib.koala_train_workspace_bytes(C.byref(self.shape), n, C.byref(need))
        if rc != 0:
            raise KoalaError(rc, "koala_train_workspace_bytes")
        if self._ws is None or self._ws.numel() < need.value:
            self._ws = torch.empty(need.value, dtype=torch.uint8, device=self.w_lin.device)
        return self._ws

    def step(self, h, q_logits, d_logits, lr, loss_out, stream=None):
        ws = self._workspace(h.shape[0])
        rc = self.lib.koala_train_disc_step(C.byref(self.shape), C.byref(self.params), _stream(stream), h.shape[0],
                                            _ptr(h), _ptr(q_logits), _ptr(d_logits), float(lr), _ptr(ws), ws.numel(),
                                            _ptr(loss_out))
        if rc != 0:
            raise KoalaError(rc, "koala_train_disc_step")

    def gen_grad(self, h, q_logits, d_logits, lam, loss_out, grad_d, stream=None):
        ws = self._workspace(h.shape[0])
        rc = self.lib.koala_train_gen_grad(C.byref(self.shape), C.byref(self.params), _stream(stream), h.shape[0],
                                           _ptr(h), _ptr(q_logits), _ptr(d_logits), float(lam), _ptr(ws), ws.numel(),
                                           _ptr(loss_out), _ptr(grad_d))
        if rc != 0:
            raise KoalaError(rc, "koala_train_gen_grad")


class MedusaHeadTrainer:
    """One Medusa-style head in training: blocks = list of K fp32 device tensors [hidden, hidden] (updated in
    place), w_lm [vocab, hidden] fixed."""

    def __init__(self, blocks, w_lm):
        self.lib = load_library()
        self.blocks, self.w_lm = list(blocks), w_lm
        self.K = len(self.blocks)
        self.V, self.H = w_lm.shape
        self._arr = (C.c_void_p * self.K)(*[b.data_ptr() for b in self.blocks])
        self._ws = None

    def _workspace(self, n):
        import torch
        need = C.c_size_t()
        rc = self.lib.koala_train_medusa_workspace_bytes(n, self.H, self.K, C.byref(need))
        if rc != 0:
            raise KoalaError(rc, "koala_train_medusa_workspace_bytes")
        if self._ws is None or self._ws.numel() < need.value:
            self._ws = torch.empty(need.value, dtype=torch.uint8, device=self.w_lm.device)
        return self._ws

    def forward(self, h, d_logits, stream=None):
        ws = self._workspace(h.shape[0])
        rc = self.lib.koala_train_medusa_head_forward(_stream(stream), h.shape[0], self.H, self.V, self.K,
                                                      C.cast(self._arr, C.POINTER(C.c_void_p)), _ptr(self.w_lm),
                                                      _ptr(h), _ptr(ws), ws.numel(), _ptr(d_logits))
        if rc != 0:
            raise KoalaError(rc, "koala_train_medusa_head_forward")

    def step(self, h, grad_d, lr, stream=None):
        ws = self._workspace(h.shape[0])
        rc = self.lib.koala_train_medusa_head_step(_stream(stream), h.shape[0], self.H, self.V, self.K,
                                                   C.cast(self._arr, C.POINTER(C.c_void_p)), _ptr(self.w_lm), _ptr(h),
                                                   _ptr(grad_d), float(lr), _ptr(ws), ws.numel())
        if rc != 0:
            raise KoalaError(rc, "koala_train_medusa_head_step")
