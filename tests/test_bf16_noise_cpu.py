"""How much of the bf16 tolerance is used up by activation rounding alone?  (CPU only.)

The GPU path keeps the residual stream in float32 but hands the matrix cores bf16 activations at five
points of a decoder layer: the two normalised inputs, q/k/v, the attention output and the SwiGLU
product.  This test rounds the oracle's float64 values at exactly those points and compares with the
unrounded oracle.  It pins the fact the bf16 tolerance rests on: this inherent noise is a few 1e-3 per
layer at small widths (it grows with width: 1.4e-2 at d 6656 / FFN 17920 / 96 rows, measured once with the
same code), i.e. the same order as the 2e-2 bound the parity tests use."""
import numpy as np

import synth_inputs as si
from oracle import amphista_oracle as orc


def bf16(a):
    return si.bf16_bits_to_f32(si.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))).astype(np.float64)


def layer(x, lw, kc, vc, positions, visible, n_heads, eps, theta, rnd):
    """One decoder layer over the tree rows (Sec. 2 "Tree Attention"), with `rnd` applied where the GPU stores bf16."""
    R, d = x.shape
    d_h = d // n_heads
    n = rnd(orc.rmsnorm(x, lw["rms1"], eps))
    q = orc.linear(lw["wq"], n).reshape(R, n_heads, d_h)
    k = orc.linear(lw["wk"], n).reshape(R, n_heads, d_h)
    v = orc.linear(lw["wv"], n).reshape(R, n_heads, d_h)
    for r in range(R):
        q[r], k[r] = orc.rope(q[r], positions[r], theta), orc.rope(k[r], positions[r], theta)
    q, k, v = rnd(q), rnd(k), rnd(v)
    k_new, v_new = np.transpose(k, (1, 0, 2)), np.transpose(v, (1, 0, 2))
    attn = np.zeros((R, n_heads, d_h))
    for h in range(n_heads):
        for r in range(R):
            sel = np.nonzero(visible[r])[0]
            attn[r, h] = orc.attend_segments(q[r, h], [(kc[h], vc[h]), (k_new[h][sel], v_new[h][sel])])
    y = x + orc.linear(lw["wo"], rnd(attn).reshape(R, d))
    m = rnd(orc.rmsnorm(y, lw["rms2"], eps))
    act = rnd(orc.silu(orc.linear(lw["w_gate"], m)) * orc.linear(lw["w_up"], m))
    return y + orc.linear(lw["w_down"], act)


def test_bf16_activation_rounding_alone_costs_a_few_1e3_per_layer():
    d, n_h, f, L, T = 1024, 8, 2752, 512, 64
    cfg = si.with_(si.MINI, d_model=d, n_heads=n_h, head_dim=d // n_h, d_ffn=f, vocab=512, n_layers=1, T=T, kv_len=L)
    tw = si.target_weights(cfg, 0, 1)
    otree = orc.tree_from_paths(si.tree_paths(T, (10,) * 4), 4)
    tok = si.tokens(cfg, 0, "tree.tok", (1, T))[0]
    pos = list((L + otree.depth).astype(np.int32))
    kc = si.normal(cfg, 0, "tkv0.k", (1, n_h, L, d // n_h), 1.0).f32[0].astype(np.float64)
    vc = si.normal(cfg, 0, "tkv0.v", (1, n_h, L, d // n_h), 1.0).f32[0].astype(np.float64)
    lw = {k: v.f32.astype(np.float64) for k, v in tw["layers"][0].items()}
    x0 = tw["embed"].f32.astype(np.float64)[tok]
    fn = tw["final_norm"].f32.astype(np.float64)
    exact = orc.rmsnorm(layer(x0, lw, kc, vc, pos, otree.mask, n_h, 1e-6, 10000.0, lambda a: a), fn, 1e-6)
    noisy = orc.rmsnorm(layer(x0, lw, kc, vc, pos, otree.mask, n_h, 1e-6, 10000.0, bf16), fn, 1e-6)
    # the unrounded layer is the oracle's own layer
    ref = orc.decoder_layer_rows(x0, tw["layers"][0] and {k: v.f32 for k, v in tw["layers"][0].items()}, kc, vc, pos,
                                 otree.mask, n_h, 1e-6, 10000.0)[0]
    assert np.allclose(orc.rmsnorm(ref, fn, 1e-6), exact, rtol=0, atol=1e-12)
    err = (np.abs(noisy - exact).max(axis=1) / np.abs(exact).max(axis=1)).max()
    assert 2e-3 < err < 1.2e-2, err
