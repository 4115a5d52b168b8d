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


def _kv_check(ctx, t: torch.Tensor) -> int:
    """Number of [max_kv, head_dim] caches in t (all leading dimensions); shape and type must be the context's."""
    assert t.is_contiguous() and t.shape[-2] == ctx.cfg.max_kv and t.shape[-1] == ctx.cfg.head_dim, tuple(t.shape)
    assert t.dtype == (torch.bfloat16 if ctx.cfg.dtype == AMPH_BF16 else torch.float32)
    return t.numel() // (t.shape[-2] * t.shape[-1])


def pack_kv(ctx, k_rows: torch.Tensor, v_rows: torch.Tensor):
    """Row-major caches [..., max_kv, head_dim] -> their step-tiled storage (amph_pack_kv); same shapes."""
    k_t, v_t = torch.empty_like(k_rows), torch.empty_like(v_rows)
    n = _kv_check(ctx, k_rows)
    assert _kv_check(ctx, v_rows) == n
    ctx.amph_pack_kv(k_rows, v_rows, k_t, v_t, n)
    return k_t, v_t


def unpack_kv(ctx, k_tiled: torch.Tensor, v_tiled: torch.Tensor):
    """Step-tiled caches -> row-major [..., max_kv, head_dim] (amph_unpack_kv)."""
    k_r, v_r = torch.empty_like(k_tiled), torch.empty_like(v_tiled)
    n = _kv_check(ctx, k_tiled)
    assert _kv_check(ctx, v_tiled) == n
    ctx.amph_unpack_kv(k_tiled, v_tiled, k_r, v_r, n)
    return k_r, v_r


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
