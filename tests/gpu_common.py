"""Helpers shared by the GPU parity tests: build a context for a synthetic configuration, move the
seeded inputs to the device, and compare against the oracle with the stated tolerances."""
from __future__ import annotations

import sys

import numpy as np
import torch

import synth_inputs as si
from paper_2406_13170_amd import binding as B
from paper_2406_13170_amd import device as D

DEV = "cuda:0"

# Tolerances (row-normwise: max_i |g_i - o_i| <= tol * max_i |o_i| per output row).
# bf16 storage with float32 accumulation against the float64 oracle: 2e-2; all-float32: 1e-4.
TOL = {"bf16": 2e-2, "f32": 1e-4}


def say(msg: str):
    print(msg, flush=True)
    sys.stdout.flush()


def make_ctx(cfg: si.Config, T: int | None = None, batch: int | None = None, max_kv: int | None = None, **variant) -> B.Context:
    """variant: n_stages, aeb_layers, lm_rank (the structural switches of amph_config)."""
    return B.Context(d_model=cfg.d_model, n_heads=cfg.n_heads, head_dim=cfg.head_dim, d_ffn=cfg.d_ffn, vocab=cfg.vocab,
                     K=cfg.K, topk=cfg.topk, max_tree=T or cfg.T, max_kv=max_kv or cfg.max_kv, batch=batch or cfg.batch,
                     dtype=D.dtype_code(cfg.dtype), rms_eps=cfg.rms_eps, rope_theta=cfg.rope_theta, device=DEV, **variant)


def rowwise_ok(got: np.ndarray, ref: np.ndarray, tol: float):
    """Returns (ok, worst ratio) of max|g - o| / max|o| over rows (last axis = row)."""
    got = np.asarray(got, dtype=np.float64).reshape(-1, got.shape[-1])
    ref = np.asarray(ref, dtype=np.float64).reshape(-1, ref.shape[-1])
    err = np.abs(got - ref).max(axis=1)
    scale = np.abs(ref).max(axis=1)
    ratio = err / np.maximum(scale, 1e-30)
    return bool(np.all(np.isfinite(got)) and np.all(ratio <= tol)), float(ratio.max())


def assert_rows_close(got, ref, tol, what=""):
    ok, worst = rowwise_ok(got, ref, tol)
    assert ok, f"{what}: worst row error {worst:.3e} > {tol:.1e}"
    return worst


def topk_consistent(g_idx: np.ndarray, o_logits: np.ndarray, k: int, tol_abs: float):
    """The GPU's rank-r index must be one the oracle could have chosen up to near-ties: its oracle
    logit lies within tol_abs of the oracle's rank-r value; and indices must be distinct."""
    order = np.lexsort((np.arange(o_logits.shape[0]), -o_logits))
    bad = []
    for r in range(k):
        if abs(o_logits[g_idx[r]] - o_logits[order[r]]) > tol_abs:
            bad.append(r)
    return (len(set(int(i) for i in g_idx)) == k) and not bad, bad


def f32_to_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def i32_to_dev(a) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def cfg_tensor_to_dev(t: si.Tensor) -> torch.Tensor:
    return D.to_device(t, DEV)


def act_to_dev(cfg: si.Config, a32: np.ndarray) -> torch.Tensor:
    """float32 values (exactly representable in cfg.dtype) -> device tensor of the storage type."""
    t = torch.from_numpy(np.ascontiguousarray(a32, dtype=np.float32)).to(DEV)
    return t.to(D.torch_dtype(cfg.dtype))


def np_of(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy() if t.is_floating_point() else t.detach().cpu().numpy()


def f32_layers(layers):
    return [{k: v.f32 for k, v in lw.items()} for lw in layers]


def draft_f32(dw):
    return dict(embed=dw["embed"].f32, fc=[x.f32 for x in dw["fc"]], sal=f32_layers(dw["sal"]), mlp=dw["mlp"].f32,
                pe=dw["pe"].f32, aeb_wq=dw["aeb_wq"].f32, aeb_wk=dw["aeb_wk"].f32, aeb_wv=dw["aeb_wv"].f32,
                aeb_wo=dw["aeb_wo"].f32, lm_head=dw["lm_head"].f32)
