"""Put named weight tensors into the device layout the library expects
(pure data movement: concatenation, row interleaving, dtype views; the one change of number format, the Linear
weights of the bfloat16 path to fp16, is a library call)."""
from __future__ import annotations

import numpy as np


def _dev(provider, name, device, dtype):
    import torch
    if dtype == "bf16":
        return torch.from_numpy(provider.bits(name).view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(provider.f32(name))).to(device)


def fragment_major(w):
    """Reorder a row-major [N, K] matrix into the fragment-major storage the bf16 kernels stream
    (see include/koala.h): N is padded with zero rows to a multiple of 64, K must be a multiple
    of 64; tiles of 64 rows x 64 k, each tile 8 fragments (row/16, k/32) of 64 lanes x 8 values,
    lane = row%16 + 16*((k%32)/8).  Returns a flat tensor of Npad*K elements."""
    import torch
    N, K = w.shape
    assert K % 64 == 0
    Np = (N + 63) // 64 * 64
    if Np != N:
        w = torch.cat([w, torch.zeros(Np - N, K, dtype=w.dtype, device=w.device)], dim=0)
    v = w.reshape(Np // 64, 4, 16, K // 64, 2, 4, 8)          # rb, t, li, kt, s, lg, e
    return v.permute(0, 3, 1, 4, 5, 2, 6).contiguous().reshape(-1)


def device_matrix(w):
    """A row-major bfloat16 [N, K] Linear weight on the device in the form koala_bind takes: fragment-major,
    then handed once to the library, which rewrites it as fp16 (koala_weights_to_half)."""
    from .binding import weights_to_f16
    return weights_to_f16(fragment_major(w))


def _mat(w, dtype):
    return device_matrix(w) if dtype == "bf16" else w.contiguous()


def rotary_pair_interleave(w, head_dim):
    """Reorder the rows of W_q or W_k [n_heads * head_dim, K] inside every head so that the two members of a
    rotary pair are neighbours: new row 2i holds dimension i, new row 2i + 1 dimension i + head_dim / 2."""
    n, k = w.shape
    half = head_dim // 2
    return w.reshape(n // head_dim, 2, half, k).transpose(1, 2).reshape(n, k)


def _layer(provider, prefix, l, device, dtype, head_dim):
    import torch
    g = lambda n: _dev(provider, f"{prefix}layers.{l}.{n}", device, dtype)
    if dtype == "bf16":
        wqkv = torch.cat([rotary_pair_interleave(g("wq"), head_dim), rotary_pair_interleave(g("wk"), head_dim),
                          g("wv")], dim=0)
    else:
        wqkv = torch.cat([g("wq"), g("wk"), g("wv")], dim=0)
    gate, up = g("wgate"), g("wup")
    wgu = torch.stack([gate, up], dim=1).reshape(2 * gate.shape[0], gate.shape[1])
    return (g("in_norm"), _mat(wqkv, dtype), _mat(g("wo"), dtype), g("post_norm"), _mat(wgu, dtype),
            _mat(g("wdown"), dtype))


def pack_target_weights(provider, cfg, device="cuda"):
    dt = cfg["dtype"]
    return dict(embed=_dev(provider, "embed", device, dt), lm_head=_mat(_dev(provider, "lm_head", device, dt), dt),
                final_norm=_dev(provider, "final_norm", device, dt),
                layers=[_layer(provider, "", l, device, dt, cfg["head_dim"]) for l in range(cfg["n_layers"])])


def pack_eagle_weights(provider, cfg, device="cuda"):
    dt = cfg["dtype"]
    layers = [_layer(provider, "draft.", k, device, dt, cfg["head_dim"]) for k in range(cfg["K"])]
    return dict(fc=_mat(_dev(provider, "draft.fc", device, dt), dt), draft=[t for layer in layers for t in layer])


def pack_medusa_weights(provider, cfg, device="cuda"):
    dt = cfg["dtype"]
    return dict(fc=None, draft=[_mat(_dev(provider, f"medusa.{j}.{k}", device, dt), dt)
                                for j in range(cfg["medusa_heads"]) for k in range(cfg["K"])])


def alloc_kv(cfg, max_batch, capacity, device="cuda", draft_layers=0):
    """Zeroed KV caches [layer][batch][n_heads][capacity][head_dim] and ctx_len int32[max_batch]."""
    import torch
    td = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    shp = (cfg["n_layers"], max_batch, cfg["n_heads"], capacity, cfg["head_dim"])
    kv = dict(target_k=torch.zeros(shp, dtype=td, device=device),
              target_v=torch.zeros(shp, dtype=td, device=device),
              draft_k=None, draft_v=None, capacity=capacity,
              ctx_len=torch.zeros(max_batch, dtype=torch.int32, device=device))
    if draft_layers:
        dshp = (draft_layers,) + shp[1:]
        kv["draft_k"] = torch.zeros(dshp, dtype=td, device=device)
        kv["draft_v"] = torch.zeros(dshp, dtype=td, device=device)
    return kv
