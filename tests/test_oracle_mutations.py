"""The pins are only worth something if plausible mistakes fail them.  Each
case plants one mistake in the oracle (on the CPU) and checks that the named pin
test then fails."""
import numpy as np
import pytest

import oracle.llama as ol
import oracle.spec as osp
import oracle.tree as otr
import test_oracle_pins as pins


def _wrong_rope(x, pos, base):                       # rotation in the opposite direction
    return ol_rope(x, -pos, base)


def _rope_interleaved(x, pos, base):                 # pairs (2i, 2i+1) instead of (i, i+dh/2)
    dh = x.shape[-1]
    ang = float(pos) * base ** (-2.0 * np.arange(dh // 2) / dh)
    c, s = np.cos(ang), np.sin(ang)
    out = np.empty_like(x)
    out[..., 0::2] = x[..., 0::2] * c - x[..., 1::2] * s
    out[..., 1::2] = x[..., 1::2] * c + x[..., 0::2] * s
    return out


ol_rope = ol.rope_rotate
ol_rms = ol.rmsnorm
ol_att = ol.attention_row
ol_silu = ol.silu

MUTATIONS = [
    ("rope direction", ol, "rope_rotate", _wrong_rope, "test_target_matches_library_llama"),
    ("rope pairing", ol, "rope_rotate", _rope_interleaved, "test_target_matches_library_llama"),
    ("norm gain dropped", ol, "rmsnorm", lambda x, g, eps: ol_rms(x, np.ones_like(g), eps),
     "test_target_matches_library_llama"),
    ("eps outside root", ol, "rmsnorm",
     lambda x, g, eps: x / (np.sqrt(np.mean(x * x, -1, keepdims=True)) + eps) * g,
     "test_rmsnorm_closed_forms_via_module"),
    ("score scale dropped", ol, "attention_row",
     lambda q, kc, vc, slots: ol_att(q * np.sqrt(float(q.shape[-1])), kc, vc, slots),
     "test_target_matches_library_llama"),
    ("gelu-ish activation", ol, "silu", lambda x: x / (1.0 + np.exp(-1.702 * x)),
     "test_target_matches_library_llama"),
    ("mask transposed", osp, "ancestor_mask", lambda p: otr.ancestor_mask(p).T,
     "test_verify_equals_sequential_decoding_on_every_path"),
    ("depth off by one", osp, "tree_depths", lambda p: otr.tree_depths(p) + (np.arange(len(p)) > 0),
     "test_verify_equals_sequential_decoding_on_every_path"),
    ("top-k ascending", osp, "topk_desc", lambda x, k: np.argsort(x, kind="stable")[:k].astype(np.int32),
     "test_eagle_tree_expansion_equals_chain_drafting_per_path"),
]


def test_rmsnorm_closed_forms_via_module():
    x = np.zeros((1, 4)) + 1e-3
    np.testing.assert_allclose(ol.rmsnorm(x, np.ones(4), 1.0), 1e-3 / np.sqrt(1e-6 + 1.0))


@pytest.mark.parametrize("label,mod,attr,repl,victim", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(monkeypatch, label, mod, attr, repl, victim):
    monkeypatch.setattr(mod, attr, repl)
    if mod is ol:                                   # functions imported by name elsewhere
        for m in (osp, pins):
            if hasattr(m, attr):
                monkeypatch.setattr(m, attr, repl)
    fn = globals().get(victim) or getattr(pins, victim)
    with pytest.raises(AssertionError):
        fn()
