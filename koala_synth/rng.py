"""Counter-based, per-tensor seeded random tensors.

Every tensor is identified by (seed, name).  Its flattened storage is cut into
fixed chunks of CHUNK elements; chunk c is drawn from a Philox stream keyed by
(seed, crc32(name), c).  The result therefore does not depend on how many
threads fill it, on the order in which tensors are asked for, or on which other
tensors exist - a layer of a 7B-shaped model can be produced on its own.
"""
from __future__ import annotations

import os
import zlib
from concurrent.futures import ThreadPoolExecutor

import numpy as np

CHUNK = 1 << 20


def _key(seed: int, name: str, chunk: int):
    h = zlib.crc32(name.encode("utf-8")) & 0xFFFFFFFF
    return np.array([(int(seed) << 32) | h, int(chunk)], dtype=np.uint64)


def _n_threads() -> int:
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit() and int(env) > 0:
        return min(int(env), 32)
    return max(1, min(os.cpu_count() or 1, 16))


def _fill(out_flat: np.ndarray, seed: int, name: str, draw):
    n = out_flat.size
    n_chunks = (n + CHUNK - 1) // CHUNK

    def work(c):
        lo = c * CHUNK
        hi = min(n, lo + CHUNK)
        g = np.random.Generator(np.random.Philox(key=_key(seed, name, c)))
        out_flat[lo:hi] = draw(g, hi - lo)

    if n_chunks <= 2:
        for c in range(n_chunks):
            work(c)
    else:
        with ThreadPoolExecutor(max_workers=_n_threads()) as ex:
            list(ex.map(work, range(n_chunks)))


def tensor_normal(seed: int, name: str, shape, std: float = 1.0) -> np.ndarray:
    """fp32 tensor of N(0, std^2) values for (seed, name)."""
    out = np.empty(int(np.prod(shape)), dtype=np.float32)
    s = np.float32(std)
    _fill(out, seed, name, lambda g, k: g.standard_normal(k, dtype=np.float32) * s)
    return out.reshape(shape)


def tensor_uniform_int(seed: int, name: str, shape, lo: int, hi: int) -> np.ndarray:
    """int32 tensor uniform in [lo, hi)."""
    out = np.empty(int(np.prod(shape)), dtype=np.int32)
    _fill(out, seed, name, lambda g, k: g.integers(lo, hi, size=k, dtype=np.int32))
    return out.reshape(shape)


def tensor_uniform01(seed: int, name: str, shape) -> np.ndarray:
    """fp32 tensor uniform in [0, 1) (the random numbers of sampling tests; fp32 so that both
    consumers read the very same values)."""
    out = np.empty(int(np.prod(shape)), dtype=np.float32)
    _fill(out, seed, name, lambda g, k: g.random(k, dtype=np.float32))
    return out.reshape(shape)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to fp32."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)
