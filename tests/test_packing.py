"""The fragment-major weight layout produced by the packer equals the index formula in koala.h."""
import numpy as np
import torch

from paper_2408_08146_amd import fragment_major


def test_fragment_major_matches_header_formula():
    N, K = 100, 192                                   # N is padded to 128
    w = torch.arange(N * K, dtype=torch.float32).reshape(N, K)
    packed = fragment_major(w).numpy()
    Np = 128
    assert packed.shape == (Np * K,)
    ref = np.zeros(Np * K, np.float32)
    for n in range(N):
        for k in range(K):
            idx = (((((n // 64) * (K // 64) + k // 64) * 4 + (n % 64) // 16) * 2 + (k % 64) // 32) * 64
                   + (n % 16) + 16 * ((k % 32) // 8)) * 8 + k % 8
            ref[idx] = n * K + k
    np.testing.assert_array_equal(packed, ref)
