"""The step-tiled K and V cache layouts of include/amph.h written as torch permutes (test-side reference only:
pure data movement).  tests/test_layouts_cpu.py checks them against the header's byte formulas; the GPU tests check
amph_pack_kv / amph_unpack_kv against them."""
from __future__ import annotations

import torch


def _step(t: torch.Tensor):
    """(rows per key step, elements per 64 bytes): 32 for bf16, 16 for float32 (both numbers coincide)."""
    return 64 // t.element_size()


def keys_to_tiled(k_rows: torch.Tensor) -> torch.Tensor:
    """[..., rows, head_dim] -> the step-tiled key-cache layout of amph_verify_attn (same shape, permuted
    storage).  rows must be a multiple of the key step."""
    P = _step(k_rows)                     # rows per step == elements per 64-byte piece
    nt = P // 16                          # fragments of 16 rows per step
    *lead, R, dh = k_rows.shape
    assert R % P == 0 and dh % P == 0
    # row = s*P + grp*(4*nt) + t*4 + lo  (slot i = grp*4 + lo);  dim = ds*P + w
    x = k_rows.reshape(*lead, R // P, 4, nt, 4, dh // P, P)
    n = len(lead)
    x = x.permute(*range(n), n, n + 2, n + 4, n + 1, n + 3, n + 5)      # [s, t, ds, grp, lo, w]
    return x.contiguous().reshape(*lead, R, dh)


def tiled_to_keys(k_tiled: torch.Tensor) -> torch.Tensor:
    P = _step(k_tiled)
    nt = P // 16
    *lead, R, dh = k_tiled.shape
    x = k_tiled.reshape(*lead, R // P, nt, dh // P, 4, 4, P)
    n = len(lead)
    x = x.permute(*range(n), n, n + 3, n + 1, n + 4, n + 2, n + 5)      # [s, grp, t, lo, ds, w]
    return x.contiguous().reshape(*lead, R, dh)


def values_to_tiled(v_rows: torch.Tensor) -> torch.Tensor:
    """[..., rows, head_dim] -> the step-tiled value-cache layout of amph_verify_attn."""
    P = _step(v_rows)
    *lead, R, dh = v_rows.shape
    assert R % P == 0 and dh % 16 == 0
    x = v_rows.reshape(*lead, R // P, P, dh // 16, 16)                  # [s, kk, db, r]
    n = len(lead)
    x = x.permute(*range(n), n, n + 2, n + 3, n + 1)                    # [s, db, r, kk]
    return x.contiguous().reshape(*lead, R, dh)


def tiled_to_values(v_tiled: torch.Tensor) -> torch.Tensor:
    P = _step(v_tiled)
    *lead, R, dh = v_tiled.shape
    x = v_tiled.reshape(*lead, R // P, dh // 16, 16, P)
    n = len(lead)
    x = x.permute(*range(n), n, n + 3, n + 1, n + 2)                    # [s, kk, db, r]
    return x.contiguous().reshape(*lead, R, dh)
