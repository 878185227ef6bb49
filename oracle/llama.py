"""Llama-style decoder layer, one row at a time (oracle; test infrastructure only).

The target model M_q of the paper (section 4.1: Vicuna 7B/13B/33B) and the
decoder layers of the EAGLE-style draft head (section 3.1) are Llama decoder
layers: RMSNorm, rotary multi-head attention without biases, SwiGLU FFN, both
with residual connections.  Everything is written per row with explicit lists
of visible cache slots, so no mask arithmetic can hide a mistake.
"""
from __future__ import annotations

import numpy as np


def rmsnorm(x, g, eps):
    """x / sqrt(mean(x^2) + eps) * g over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def silu(x):
    return x / (1.0 + np.exp(-x))


def softmax(s):
    e = np.exp(s - np.max(s, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def rope_rotate(x, pos, base):
    """Rotary embedding with half-split pairing: element i is paired with
    i + dh/2 and the pair is rotated by the angle pos * base^(-2i/dh).
    x: [..., dh]; pos: scalar position id."""
    dh = x.shape[-1]
    half = dh // 2
    i = np.arange(half, dtype=np.float64)
    ang = float(pos) * base ** (-2.0 * i / dh)
    c, s = np.cos(ang).astype(x.dtype), np.sin(ang).astype(x.dtype)
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


class KVCache:
    """Per-layer key/value rows of one sequence: k[l], v[l] are [n_heads, capacity, head_dim]."""

    def __init__(self, n_layers, n_heads, capacity, head_dim, dtype=np.float64, store=None):
        """store: optional function applied to every key/value row as it is written, modelling the
        storage format of the cache (e.g. rounding to bfloat16); None keeps rows exact."""
        self.k = [np.zeros((n_heads, capacity, head_dim), dtype) for _ in range(n_layers)]
        self.v = [np.zeros((n_heads, capacity, head_dim), dtype) for _ in range(n_layers)]
        self.capacity = capacity
        self.store = store

    def copy(self):
        c = KVCache.__new__(KVCache)
        c.k = [a.copy() for a in self.k]
        c.v = [a.copy() for a in self.v]
        c.capacity = self.capacity
        c.store = self.store
        return c


def attention_row(q, kc, vc, slots):
    """Softmax attention of one query row over the cache rows listed in `slots`.
    q: [nh, dh]; kc, vc: [nh, cap, dh]; returns [nh, dh]."""
    nh, dh = q.shape
    k = kc[:, slots, :]                       # [nh, S, dh]
    v = vc[:, slots, :]
    s = np.einsum("hsd,hd->hs", k, q) / np.sqrt(float(dh))
    p = softmax(s)
    return np.einsum("hs,hsd->hd", p, v)


def decoder_layer_rows(x, pos, slots, visible, lw, kc, vc, n_heads, head_dim, eps, base, store=None):
    """One decoder layer over T new rows.

    x[T,H] residual stream in; pos[T] rotary position ids; slots[T] cache slot
    each row's key/value is written to; visible[i] = list of cache slots row i
    attends to (it must contain slots[i]); lw = dict of this layer's tensors
    (in_norm, wq, wk, wv, wo, post_norm, wgate, wup, wdown; matrices [out,in]).
    All new keys/values are written (through `store`, if given: the cache's storage format)
    before any row attends.  Returns x_out[T,H].
    """
    if store is None:
        store = lambda a: a
    T, H = x.shape
    a = rmsnorm(x, lw["in_norm"], eps)
    q = (a @ lw["wq"].T).reshape(T, n_heads, head_dim)
    k = (a @ lw["wk"].T).reshape(T, n_heads, head_dim)
    v = (a @ lw["wv"].T).reshape(T, n_heads, head_dim)
    for i in range(T):
        q[i] = rope_rotate(q[i], pos[i], base)
        kc[:, slots[i], :] = store(rope_rotate(k[i], pos[i], base))
        vc[:, slots[i], :] = store(v[i])
    o = np.empty((T, H), x.dtype)
    for i in range(T):
        o[i] = attention_row(q[i], kc, vc, list(visible[i])).reshape(H)
    x = x + o @ lw["wo"].T
    m = rmsnorm(x, lw["post_norm"], eps)
    x = x + (silu(m @ lw["wgate"].T) * (m @ lw["wup"].T)) @ lw["wdown"].T
    return x
