"""Full-depth parity at Vicuna-7B shapes: all 32 target layers over the 64 tree tokens, device against
oracle (about two minutes; set AMPH_SKIP_FULL_DEPTH=1 to leave it out).  Layers are generated, given to the
oracle and uploaded one at a time, so that only one layer's float32 copy is alive on the host.

Activation rounding alone (bf16 at the five points of a layer where the device stores bf16) moves a 32-layer
stack by more than 2e-2: its noise grows like the square root of the depth (tests/test_bf16_noise_cpu.py), and
two runs that round at slightly different values decorrelate within a few layers, so no reference can follow the
device through 32 layers more closely than that noise.  The stated 2e-2 is therefore held where it can be:
  * EVERY layer on its own, teacher-forced: the device gets the oracle's input to that layer (rounded to bf16,
    as both sides then see it) and its output rows and tree K/V rows must match the oracle's at 2e-2;
  * the whole chain against the exact oracle is bounded by 1.5 x the drift that the oracle shows when its own
    values are rounded at those five points on the same inputs (tests/bf16_noise_model.py), and that drift is
    printed next to 2e-2."""
import os

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import amphista_oracle as orc
from paper_2406_13170_amd import binding as B
from paper_2406_13170_amd import device as D

import bf16_noise_model as nm
from gpu_common import DEV, TOL, assert_rows_close, cfg_tensor_to_dev, i32_to_dev, make_ctx, np_of, say

pytestmark = pytest.mark.gpu


@pytest.mark.skipif(os.environ.get("AMPH_SKIP_FULL_DEPTH") == "1", reason="AMPH_SKIP_FULL_DEPTH=1")
def test_target_forward_vicuna7b_all_32_layers():
    cfg = si.V7B
    seed, T, L, n_layers = 0, cfg.T, cfg.kv_len, cfg.n_layers
    n_h, d_h, d, V = cfg.n_heads, cfg.head_dim, cfg.d_model, cfg.vocab
    max_kv = cfg.max_kv
    ctx = make_ctx(cfg)
    paths = si.tree_paths(T, cfg.tree_caps)
    tree, otree = B.Tree(paths, cfg.K), orc.tree_from_paths(paths, cfg.K)
    tdt = D.torch_dtype(cfg.dtype)
    embed = si.normal(cfg, seed, "target.embed", (V, d), si.W_STD)
    lm_head = si.normal(cfg, seed, "target.lm_head", (V, d), si.W_STD)
    final_norm = si.ones(cfg, (d,))
    tok = si.tokens(cfg, seed, "tree.tok", (1, T))
    pos = (L + otree.depth).astype(np.int32)[None, :]
    k_caches = torch.zeros((n_layers, 1, n_h, max_kv, d_h), dtype=tdt, device=DEV)
    v_caches = torch.zeros((n_layers, 1, n_h, max_kv, d_h), dtype=tdt, device=DEV)
    structs, tiled, keep = [], [], []
    forced = []                                      # per layer: (input rows on the device, oracle's normed output, its K/V rows)
    xe = embed.f32[tok[0]].astype(np.float64)        # exact oracle
    xr = xe.copy()                                   # rounding model
    for li in range(n_layers):
        lw = si.decoder_layer(cfg, seed, f"target.layer{li}")
        kc = si.normal(cfg, seed, f"tkv{li}.k", (1, n_h, L, d_h), 1.0)
        vc = si.normal(cfg, seed, f"tkv{li}.v", (1, n_h, L, d_h), 1.0)
        lw64 = {k: v.f32 for k, v in lw.items()}
        # teacher forcing: this layer alone on the oracle's input to it, rounded to the type the device's table holds
        xb = nm.bf16(xe)
        o_tf, k_tf, v_tf, _, _ = orc.decoder_layer_rows(xb, lw64, kc.f32[0], vc.f32[0], list(pos[0]), otree.mask, n_h, cfg.rms_eps,
                                                        cfg.rope_theta)
        forced.append((torch.from_numpy(xb.astype(np.float32)).to(DEV).to(tdt), orc.rmsnorm(o_tf, final_norm.f32, cfg.rms_eps), k_tf, v_tf))
        # exact: the oracle's own layer on top of its own previous output; model: the same with rounding
        xe = orc.decoder_layer_rows(xe, lw64, kc.f32[0], vc.f32[0], list(pos[0]), otree.mask, n_h, cfg.rms_eps, cfg.rope_theta)[0]
        xr = nm.layer(xr, lw64, kc.f32[0], vc.f32[0], list(pos[0]), otree.mask, n_h, cfg.rms_eps, cfg.rope_theta, nm.bf16)[0]
        # device: upload, tile, drop the row-major matrices
        ld = D.layer_to_device(lw, DEV)
        ts, tt = D.pack_layer(ctx, ld)
        torch.cuda.synchronize()
        structs.append(B.amph_layer_w(rms1=ld["rms1"].data_ptr(), rms2=ld["rms2"].data_ptr()))
        tiled.append(ts)
        keep.append((tt, ld["rms1"], ld["rms2"]))
        kr = torch.zeros((1, n_h, max_kv, d_h), dtype=tdt, device=DEV)
        vr = torch.zeros((1, n_h, max_kv, d_h), dtype=tdt, device=DEV)
        kr[:, :, :L], vr[:, :, :L] = cfg_tensor_to_dev(kc), cfg_tensor_to_dev(vc)
        k_caches[li], v_caches[li] = D.pack_kv(ctx, kr, vr)
        del lw, lw64, ld, kc, vc, kr, vr
        if li % 8 == 7:
            say(f"  layer {li + 1}/{n_layers} through the oracle, the rounding model and onto the device")
    hidden_e, logits_e = nm.head(xe, final_norm.f32, lm_head.f32, cfg.rms_eps, nm.exact)
    hidden_m, logits_m = nm.head(xr, final_norm.f32, lm_head.f32, cfg.rms_eps, nm.bf16)
    embed_d, fn_d, lm_d = cfg_tensor_to_dev(embed), cfg_tensor_to_dev(final_norm), cfg_tensor_to_dev(lm_head)
    lm_t = D.pack_lm_head(ctx, lm_d)
    hidden = torch.zeros((1, T, d), dtype=torch.float32, device=DEV)
    logits = torch.zeros((1, T, V), dtype=torch.float32, device=DEV)
    tgt = torch.zeros((1, T), dtype=torch.int32, device=DEV)
    ctx.amph_target_forward(tree, structs, embed_d, fn_d, None, i32_to_dev(tok), i32_to_dev(pos), k_caches, v_caches,
                            i32_to_dev([L]), hidden, logits, tgt, tiled_structs=tiled, lm_head_tiled=lm_t)
    torch.cuda.synchronize()
    assert ctx.device_status() == 0
    g_hidden, g_logits, g_tgt = np_of(hidden)[0], np_of(logits)[0], np_of(tgt)[0]
    assert np.all(np.isfinite(g_logits))
    tol = TOL[cfg.dtype]
    # ---- the whole chain against the exact oracle: bounded by the rounding model's own drift on these inputs
    d_h_, d_l_ = nm.worst_row(hidden_m, hidden_e), nm.worst_row(logits_m, logits_e)
    e_h, e_l = nm.worst_row(g_hidden, hidden_e), nm.worst_row(g_logits, logits_e)
    say(f"  32 layers, worst row error against the exact oracle: hidden {e_h:.3e}, logits {e_l:.3e}; the oracle with its own "
        f"values rounded at the device's five rounding points is {d_h_:.3e} / {d_l_:.3e} from the exact one: activation rounding "
        f"alone {'exceeds' if max(d_h_, d_l_) > tol else 'stays below'} {tol:.0e} at this depth")
    assert e_h <= 1.5 * d_h_ and e_l <= 1.5 * d_l_, "further from the exact oracle than 1.5 x the rounding model's drift"
    # ---- every layer on its own at the stated tolerance (teacher-forced: the layer's input is the oracle's)
    rows = i32_to_dev(np.arange(T)[None])
    per_node = lambda a: np.transpose(a, (1, 0, 2)).reshape(a.shape[1], -1)
    per_head = lambda a: a.reshape(-1, a.shape[-1])
    worst_out = worst_node = worst_head = 0.0
    for li, (x_dev, want, k_tf, v_tf) in enumerate(forced):
        tf_tgt = torch.zeros((1, T), dtype=torch.int32, device=DEV)
        ctx.amph_target_forward(tree, structs[li:li + 1], x_dev, fn_d, None, rows, i32_to_dev(pos), k_caches[li:li + 1],
                                v_caches[li:li + 1], i32_to_dev([L]), hidden, logits if li == n_layers - 1 else None, tf_tgt,
                                tiled_structs=tiled[li:li + 1], lm_head_tiled=lm_t)
        torch.cuda.synchronize()
        assert ctx.device_status() == 0
        worst_out = max(worst_out, assert_rows_close(np_of(hidden)[0], want, tol, f"layer {li} alone: output rows"))
        k_rows, v_rows = D.unpack_kv(ctx, k_caches[li], v_caches[li])
        kc, vc = np_of(k_rows[0][:, L:L + T]), np_of(v_rows[0][:, L:L + T])
        worst_node = max(worst_node, assert_rows_close(per_node(kc), per_node(k_tf), tol, f"layer {li} alone: tree keys"),
                         assert_rows_close(per_node(vc), per_node(v_tf), tol, f"layer {li} alone: tree values"))
        worst_head = max(worst_head, assert_rows_close(per_head(kc), per_head(k_tf), tol, f"layer {li} alone: tree keys per head"),
                         assert_rows_close(per_head(vc), per_head(v_tf), tol, f"layer {li} alone: tree values per head"))
    say(f"  each of the 32 layers alone (bound {tol:.0e}): worst output row {worst_out:.2e}, tree K/V per node {worst_node:.2e}, "
        f"per (head, node) {worst_head:.2e}")
    # ---- argmax of the chain: exact on the device's own logits, and a near-tie of the exact oracle's within the band
    # the chain's rounding noise allows (with random weights the logits are nearly flat, so few gaps exceed it)
    band_rel = 2 * 1.5 * d_l_
    for i in range(T):
        o = logits_e[i]
        assert g_tgt[i] == orc.row_argmax(g_logits[i]), "argmax of the device's own logits"
        assert o[g_tgt[i]] >= o.max() - band_rel * np.abs(o).max(), f"node {i}: the device's argmax is not a near-tie of the oracle's"
    agree_e = int((g_tgt == np.array([orc.row_argmax(r) for r in logits_e])).sum())
    say(f"  chain argmax: {agree_e}/{T} nodes agree with the exact oracle")
    # ---- argmax at the stated tolerance: the last layer alone (its forced run above left its logits and argmax):
    # equal to the oracle's wherever the oracle's top-1/top-2 gap exceeds twice the tolerance, and such nodes exist
    want_logits = orc.linear(lm_head.f32, forced[-1][1])
    tf_logits, tf_arg = np_of(logits)[0], np_of(tf_tgt)[0]
    w_l = assert_rows_close(tf_logits, want_logits, tol, "last layer alone: logits")
    clear = ok = 0
    for i in range(T):
        o = want_logits[i]
        s_ = np.sort(o)
        band = 2 * tol * np.abs(o).max()
        assert tf_arg[i] == orc.row_argmax(tf_logits[i])
        assert o[tf_arg[i]] >= s_[-1] - band
        if s_[-1] - s_[-2] > band:
            clear += 1
            ok += int(tf_arg[i] == orc.row_argmax(o))
    say(f"  last layer alone: logits {w_l:.2e}; argmax equal on {ok}/{clear} nodes with a clear gap (of {T})")
    assert clear > 0, "no node has a clear top-1/top-2 gap: the argmax comparison would be empty"
    assert ok == clear
