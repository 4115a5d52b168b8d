"""The oracle's decoder layer with a rounding function applied where the device stores bf16 (test-side model of
the device's activation precision; built from the oracle's own functions, used by CPU and GPU tests only).

The device keeps the residual stream in float32 and hands the matrix cores bf16 activations at five points of a
decoder layer: the two normalised inputs, q/k/v (after RoPE), the attention output and the SwiGLU product; the LM
head reads the bf16 final-normed hidden state.  With rnd = identity every function here is the oracle's."""
from __future__ import annotations

import numpy as np

import synth_inputs as si
from oracle import amphista_oracle as orc


def bf16(a):
    return si.bf16_bits_to_f32(si.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))).astype(np.float64)


def exact(a):
    return a


def layer(x, lw, kc, vc, positions, visible, n_heads, eps, theta, rnd):
    """One decoder layer over the tree rows (Sec. 2 "Tree Attention").  Returns (out, k_new, v_new) with k_new, v_new
    [n_heads, R, d_h] as the cache would hold them."""
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
    return y + orc.linear(lw["w_down"], act), k_new, v_new


def head(x, final_norm, lm_head, eps, rnd):
    """Final RMSNorm and LM head: (hidden, logits); the LM head reads the rounded hidden state."""
    hidden = orc.rmsnorm(x, final_norm, eps)
    return hidden, orc.linear(lm_head, rnd(hidden))


def worst_row(got, ref):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    got, ref = got.reshape(-1, got.shape[-1]), ref.reshape(-1, ref.shape[-1])
    return float((np.abs(got - ref).max(axis=1) / np.abs(ref).max(axis=1)).max())


def target_forward(tw, tree_tok, tree_pos, mask, k_caches, v_caches, n_heads, eps, theta, rnd):
    """The oracle's target pass over the tree tokens with rnd at the device's rounding points.  Same arguments as the
    oracle's target_forward; returns hidden, logits and per layer the tree's new K/V rows."""
    x = np.asarray(tw["embed"], dtype=np.float64)[np.asarray(tree_tok)]
    layers = []
    for li, lw in enumerate(tw["layers"]):
        x, k_new, v_new = layer(x, lw, np.asarray(k_caches[li], dtype=np.float64), np.asarray(v_caches[li], dtype=np.float64),
                                list(tree_pos), mask, n_heads, eps, theta, rnd)
        layers.append(dict(k_new=k_new, v_new=v_new))
    hidden, logits = head(x, tw["final_norm"], tw["lm_head"], eps, rnd)
    return dict(hidden=hidden, logits=logits, layers=layers)
