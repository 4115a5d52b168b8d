"""The torch-permute reference of the step-tiled K and V caches (tests/layout_ref.py) against the byte formulas
that include/amph.h states (CPU only: pure data movement).  The library's own converters are checked against
the same reference on the GPU (tests/test_gpu_kernels.py)."""
import pytest
import torch

import layout_ref as D


@pytest.mark.parametrize("dt,E", [(torch.bfloat16, 2), (torch.float32, 4)])
@pytest.mark.parametrize("dh", [64, 128])
def test_tiled_cache_helpers_follow_the_header_formulas(dt, E, dh):
    P = 16 // E                       # elements per 16 bytes; a key step is 4P rows
    R = 3 * 4 * P
    rows = (torch.arange(R * dh) % 251).float().reshape(R, dh).to(dt)      # exactly representable in bf16
    kt, vt = D.keys_to_tiled(rows).reshape(-1), D.values_to_tiled(rows).reshape(-1)
    for r in range(R):
        for c in range(dh):
            s, kk = r // (4 * P), r % (4 * P)
            t, i, ds = (kk % P) // 4, (kk // P) * 4 + kk % 4, c * E // 64
            off_k = ((s * (P // 4) + t) * (dh * E // 64) + ds) * 1024 + i * 64 + (c * E) % 64
            off_v = (s * (dh // 16) + c // 16) * 1024 + (c % 16) * 64 + (r % (4 * P)) * E
            assert kt[off_k // E] == rows[r, c] and vt[off_v // E] == rows[r, c]
    assert torch.equal(D.tiled_to_keys(D.keys_to_tiled(rows)), rows)
    assert torch.equal(D.tiled_to_values(D.values_to_tiled(rows)), rows)


def test_tiled_cache_helpers_keep_leading_dimensions():
    x = torch.randn(2, 3, 64, 128)
    assert torch.equal(D.keys_to_tiled(x)[1, 2], D.keys_to_tiled(x[1, 2]))
    assert torch.equal(D.values_to_tiled(x)[0, 1], D.values_to_tiled(x[0, 1]))
