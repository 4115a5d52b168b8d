"""Host->device marshalling of synthetic tensors (data movement and layout only, no arithmetic)."""
from __future__ import annotations

from typing import Dict

import numpy as np
import torch

from .binding import (AMPH_BF16, AMPH_F32, AMPH_PACK_DOWN, AMPH_PACK_GATEUP, AMPH_PACK_LMHEAD, AMPH_PACK_QKV,
                      AMPH_PACK_WO, amph_layer_tiled)


def dtype_code(name: str) -> int:
    return AMPH_BF16 if name == "bf16" else AMPH_F32


def torch_dtype(name: str):
    return torch.bfloat16 if name == "bf16" else torch.float32


def to_device(t, device="cuda:0") -> torch.Tensor:
    """synth_inputs.Tensor -> device tensor holding exactly the same values (bf16 patterns or float32)."""
    if t.dtype == "bf16":
        return torch.from_numpy(t.dev.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(t.dev)).to(device)


def layer_to_device(lw: Dict[str, object], device="cuda:0") -> Dict[str, torch.Tensor]:
    return {k: to_device(v, device) for k, v in lw.items()}


def draft_to_device(dw: Dict[str, object], device="cuda:0") -> Dict[str, object]:
    out = {}
    for k, v in dw.items():
        if k == "sal":
            out[k] = [layer_to_device(l, device) for l in v]
        elif k == "fc":
            out[k] = [to_device(x, device) for x in v]
        else:
            out[k] = to_device(v, device)
    return out


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


def pack_layer(ctx, lw: Dict[str, torch.Tensor]):
    """Tiled copies of one target layer's matrices (amph_pack_weights).  Returns (amph_layer_tiled, tensors):
    the caller keeps `tensors` alive as long as the struct is used."""
    dev = lw["wq"].device

    def buf(role):
        return torch.empty(ctx.amph_tiled_bytes(role), dtype=torch.uint8, device=dev)

    t = {"qkv": buf(AMPH_PACK_QKV), "wo": buf(AMPH_PACK_WO), "gate_up": buf(AMPH_PACK_GATEUP), "down": buf(AMPH_PACK_DOWN)}
    ctx.amph_pack_weights(AMPH_PACK_QKV, lw["wq"], lw["wk"], lw["wv"], t["qkv"])
    ctx.amph_pack_weights(AMPH_PACK_WO, lw["wo"], None, None, t["wo"])
    ctx.amph_pack_weights(AMPH_PACK_GATEUP, lw["w_gate"], lw["w_up"], None, t["gate_up"])
    ctx.amph_pack_weights(AMPH_PACK_DOWN, lw["w_down"], None, None, t["down"])
    s = amph_layer_tiled(*[t[k].data_ptr() for k in ("qkv", "wo", "gate_up", "down")])
    return s, t


def pack_lm_head(ctx, lm_head: torch.Tensor) -> torch.Tensor:
    out = torch.empty(ctx.amph_tiled_bytes(AMPH_PACK_LMHEAD), dtype=torch.uint8, device=lm_head.device)
    ctx.amph_pack_weights(AMPH_PACK_LMHEAD, lm_head, None, None, out)
    return out
