"""Host-side checks of the C ABI that need no GPU: the built library exports every symbol the
header declares, and koala_create validates shapes and trees before anything touches a device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2408_08146_amd as K
from paper_2408_08146_amd.binding import KoalaContext, KoalaError
from koala_synth import get_config
from koala_synth.trees import make_tree

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _built():
    if not os.path.exists(K.library_path()):
        from paper_2408_08146_amd.build import build_library
        build_library(verbose=False)


def test_library_exports_every_declared_symbol():
    _built()
    header = open(os.path.join(ROOT, "include", "koala.h")).read()
    declared = set(re.findall(r"\b(koala_[a-z_]+)\s*\(", header))
    assert declared == set(K.EXPORTS)
    lib = C.CDLL(K.library_path())
    for name in declared:
        assert getattr(lib, name) is not None


SHAPE = dict(hidden=256, n_heads=4, head_dim=64, ffn=688, vocab=1000, n_layers=4, rms_eps=1e-6,
             rope_base=1e4, dtype=K.KOALA_FP32)
DRAFT = dict(kind=K.KOALA_DRAFT_EAGLE, K=2, medusa_heads=0, max_m=8)


def _status(shape=SHAPE, draft=DRAFT, tree=None, max_batch=1):
    _built()
    tree = tree or get_config("cfg1")["tree_template"]
    try:
        KoalaContext(shape, draft, tree, max_batch).close()
        return 0
    except KoalaError as e:
        return e.status


class _T:
    def __init__(self, parent, rank, topk, depth):
        self.parent, self.rank, self.topk_per_depth, self.depth = (np.asarray(parent, np.int32),
                                                                   np.asarray(rank, np.int32),
                                                                   np.asarray(topk, np.int32), depth)


def test_create_accepts_all_benchmark_trees():
    for name in ("cfg1", "cfg2", "cfg3", "cfg4"):
        assert _status(tree=get_config(name)["tree_template"],
                       draft=dict(DRAFT, medusa_heads=4)) == 0
    assert _status(tree=make_tree([], [1])) == 0                     # single-node tree: plain decoding


def test_create_rejects_bad_shapes():
    assert _status(shape=dict(SHAPE, hidden=250)) == -2               # hidden != n_heads * head_dim
    assert _status(shape=dict(SHAPE, n_heads=8, head_dim=32)) == -5   # head_dim not supported
    assert _status(shape=dict(SHAPE, dtype=7)) == -5
    assert _status(shape=dict(SHAPE, dtype=K.KOALA_BF16, ffn=688)) == -5   # bf16 needs ffn % 64 == 0
    assert _status(draft=dict(DRAFT, K=0)) == -2
    assert _status(draft=dict(DRAFT, max_m=65)) == -2
    assert _status(draft=dict(DRAFT, kind=3)) == -5
    assert _status(max_batch=0) == -2


def test_create_rejects_malformed_trees():
    assert _status(tree=_T([0, 0], [0, 0], [1], 1)) == -2            # root's parent must be -1
    assert _status(tree=_T([-1, 1], [0, 0], [1], 1)) == -2           # parent[i] < i
    assert _status(tree=_T([-1, 0, 0], [0, 0], [2], 1)) == -2        # siblings share a rank
    assert _status(tree=_T([-1, 0, 0], [0, 2], [2], 1)) == -2        # rank >= k of its depth
    assert _status(tree=_T([-1, 0, 1], [0, 0, 0], [1], 1)) == -2     # deeper than declared
    assert _status(tree=_T([-1, 0, 1, 0], [0, 0, 0, 1], [2, 1], 2)) == -2   # not ordered by depth
    t65 = make_tree([1] * 64, [1] * 65)
    assert _status(tree=t65) == -2                                   # more than 64 nodes
    assert _status(draft=dict(kind=K.KOALA_DRAFT_MEDUSA, K=1, medusa_heads=1, max_m=1)) == -2  # heads < depth


def test_unbound_context_refuses_compute_calls():
    _built()
    ctx = KoalaContext(SHAPE, DRAFT, get_config("cfg1")["tree_template"], 1)
    assert ctx.workspace_bytes() > 0
    with pytest.raises(KoalaError) as e:
        ctx.lib.koala_tree_verify.restype = C.c_int
        st = ctx.lib.koala_tree_verify(ctx._h, None, 1, None, None, None, None)
        ctx._check(st)
    assert e.value.status == -6
    ctx.close()


def test_every_compute_entry_point_refuses_an_unbound_or_missing_context():
    """No compute call may touch the device before a successful bind: each returns
    KOALA_E_WORKSPACE (-6) for an unbound context and KOALA_E_NULL (-1) for a null one, on the host."""
    _built()
    ctx = KoalaContext(SHAPE, DRAFT, get_config("cfg1")["tree_template"], 1)
    lib = ctx.lib
    stats = (C.c_int32 * 66)()
    f1 = C.c_float(1.0)
    calls = {
        "koala_draft_expand": lambda h: lib.koala_draft_expand(h, None, 1, None, None, 1, None, None),
        "koala_tree_verify": lambda h: lib.koala_tree_verify(h, None, 1, None, None, None, None),
        "koala_accept_prefix": lambda h: lib.koala_accept_prefix(h, None, 1, None, None, None, None, None, 0),
        "koala_draft_expand_sample": lambda h: lib.koala_draft_expand_sample(h, None, 1, None, None, 1, None, f1, None,
                                                                             None),
        "koala_accept_sample": lambda h: lib.koala_accept_sample(h, None, 1, None, None, None, None, None, f1, None,
                                                                 None, None, 0),
        "koala_generate": lambda h: lib.koala_generate(h, None, None, None, 1, 1, 1, 1, None,
                                                       C.cast(stats, C.POINTER(K.binding._GenStats))),
        "koala_generate_sample": lambda h: lib.koala_generate_sample(h, None, None, None, 1, 1, 1, None, 1, f1, None,
                                                                     C.cast(stats, C.POINTER(K.binding._GenStats))),
    }
    for name, call in calls.items():
        got = call(ctx._h)
        assert got in (-6, -1), (name, got)          # unbound (-6), or a null argument found first (-1)
        assert call(None) == -1, name
    # with every pointer present the unbound context itself is what is refused
    dummy = C.c_void_p(256)
    assert lib.koala_tree_verify(ctx._h, None, 1, dummy, dummy, None, dummy) == -6
    assert lib.koala_accept_prefix(ctx._h, None, 1, dummy, dummy, dummy, dummy, dummy, 0) == -6
    ctx.close()
