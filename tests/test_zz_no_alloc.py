"""amph_verify_attn_static (the entry point for callers that cannot allocate: its key-split partials live in a
static device array of the library) against amph_verify_attn on the same inputs: same kernels, same arithmetic, so
the outputs must be bit-identical; both are also held to the oracle's tolerance.  Two calls in a row share the
array, the second with a smaller input."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import amphista_oracle as orc
from paper_2406_13170_amd import binding as B
from paper_2406_13170_amd import device as D

from gpu_common import DEV, TOL, assert_rows_close, cfg_tensor_to_dev, i32_to_dev, make_ctx, np_of, say

pytestmark = pytest.mark.gpu


def one_case(cfg, T, caps, L, B_, seed, heads):
    K = len(caps)
    cfgx = si.with_(cfg, batch=B_, K=K, topk=min(16, max(caps)))
    max_kv = (L + T + 31) // 32 * 32 + 32
    ctx = make_ctx(cfgx, T=T, batch=B_, max_kv=max_kv)
    paths = si.tree_paths(T, caps)
    tree = B.Tree(paths, K)
    otree = orc.tree_from_paths(paths, K)
    n_h, d_h = cfg.n_heads, cfg.head_dim
    q = si.normal(cfgx, seed, "na.q", (B_, T, n_h, d_h), 1.0)
    k = si.normal(cfgx, seed, "na.k", (B_, n_h, L + T, d_h), 1.0)
    v = si.normal(cfgx, seed, "na.v", (B_, n_h, L + T, d_h), 1.0)
    tdt = D.torch_dtype(cfg.dtype)
    k_rows = torch.full((B_, n_h, max_kv, d_h), float("nan"), dtype=tdt, device=DEV)
    v_rows = torch.full((B_, n_h, max_kv, d_h), float("nan"), dtype=tdt, device=DEV)
    k_rows[:, :, :L + T], v_rows[:, :, :L + T] = cfg_tensor_to_dev(k), cfg_tensor_to_dev(v)
    kc, vc = D.pack_kv(ctx, k_rows, v_rows)
    kv_len = i32_to_dev(np.full(B_, L))
    q_d = cfg_tensor_to_dev(q)
    out_ws = torch.full((B_, T, n_h, d_h), float("nan"), dtype=tdt, device=DEV)
    out_st = torch.full((B_, T, n_h, d_h), float("nan"), dtype=tdt, device=DEV)
    ctx.amph_verify_attn(tree, q_d, kc, vc, kv_len, out_ws)
    ctx.amph_verify_attn_static(tree, q_d, kc, vc, kv_len, out_st)
    torch.cuda.synchronize()
    assert ctx.device_status() == 0
    assert torch.equal(out_ws.view(torch.int16 if cfg.dtype == "bf16" else torch.int32),
                       out_st.view(torch.int16 if cfg.dtype == "bf16" else torch.int32)), "static-scratch call differs"
    got = np_of(out_st)
    worst = 0.0
    for b in range(B_):
        for h in heads:
            ref = orc.tree_attention(q.f32[b][:, h:h + 1], k.f32[b][h:h + 1], v.f32[b][h:h + 1], L, otree.mask)
            worst = max(worst, assert_rows_close(got[b][:, h], ref[:, 0], TOL[cfg.dtype], f"static verify_attn b={b} h={h}"))
    return worst


def test_static_scratch_entry_point_two_calls_second_smaller():
    say("amph_verify_attn_static: 7B shape (key splits: 4.1 MiB of partials in the static array)")
    w = one_case(si.V7B, 64, (10,) * 4, 1024, 1, seed=31, heads=[0, 13, 31])
    say(f"  worst row error {w:.2e}")
    say("amph_verify_attn_static: smaller input right after it (Mini, T = 22, L = 37, batch 2)")
    w = one_case(si.MINI, 22, (10,) * 4, 37, 2, seed=32, heads=range(si.MINI.n_heads))
    say(f"  worst row error {w:.2e}")


def test_static_scratch_entry_point_rejects_oversized_shapes():
    say("amph_verify_attn_static: a shape whose partials exceed the array is refused before anything is launched")
    # 8 heads, 128 queries, a long cache, the LDS-ring kernel forced: 32 key splits x 8 heads x 128 x 130 floats = 17 MB
    ctx = B.Context(d_model=1024, n_heads=8, head_dim=128, d_ffn=1024, vocab=1024, K=4, topk=10, max_tree=128, max_kv=8192,
                    batch=1, dtype=B.AMPH_BF16, device=DEV)
    ctx.amph_verify_kernel(1)
    tree = B.Tree(si.tree_paths(128, (10,) * 4), 4)
    t = torch.zeros(64, dtype=torch.bfloat16, device=DEV)
    out = torch.zeros(64, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(B.AmphError) as e:
        ctx.amph_verify_attn_static(tree, t, t, t, t, out)
    assert e.value.status == B.AMPH_ESHAPE and "static scratch" in str(e.value)
