"""Pins for the oracle's attention pieces: tree-masked attention (Sec. 2 "Tree Attention",
Appendix "Draft Tree"), the adaptation layer's cached single-position attention (Eq. 1) and
the bi-directional self-attention of Eq. 5.  Each check compares the oracle with something
other than itself: brute force over root-to-leaf paths, torch's attention routine, closed
forms, invariants."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import amphista_oracle as orc


def causal_attention_plain(q, k, v):
    """Textbook causal attention of a sequence, written independently of the oracle.
    q, k, v [S, d_h]; row i attends to rows 0..i."""
    S, d_h = q.shape
    out = np.zeros_like(q)
    for i in range(S):
        s = np.array([np.dot(q[i], k[j]) for j in range(i + 1)]) / np.sqrt(d_h)
        w = np.exp(s - s.max())
        w /= w.sum()
        for j in range(i + 1):
            out[i] += w[j] * v[j]
    return out


def random_case(rng, T, n_h, d_h, L):
    q = rng.standard_normal((T, n_h, d_h))
    k = rng.standard_normal((n_h, L + T, d_h))
    v = rng.standard_normal((n_h, L + T, d_h))
    return q, k, v


@pytest.mark.parametrize("T,caps,L", [(16, (4, 2, 2, 2), 5), (22, (10, 10, 10, 10), 3), (9, (2, 3), 0)])
def test_tree_attention_equals_per_path_causal(T, caps, L):
    """Every node's output equals plain causal attention run on [cache ; its root-to-leaf path]."""
    rng = np.random.default_rng(1)
    K = len(caps)
    tree = orc.tree_from_paths(si.tree_paths(T, caps), K)
    n_h, d_h = 2, 8
    q, k, v = random_case(rng, T, n_h, d_h, L)
    got = orc.tree_attention(q, k, v, L, tree.mask)
    seen = np.zeros(T, dtype=bool)
    for path in tree.retrieve:
        nodes = [int(n) for n in path if n >= 0]
        for h in range(n_h):
            # queries for cache rows are irrelevant: use zeros, only path rows are compared
            qs = np.concatenate([np.zeros((L, d_h)), q[nodes, h]], axis=0)
            ks = np.concatenate([k[h, :L], k[h, [L + n for n in nodes]]], axis=0)
            vs = np.concatenate([v[h, :L], v[h, [L + n for n in nodes]]], axis=0)
            ref = causal_attention_plain(qs, ks, vs)[L:]
            np.testing.assert_allclose(got[nodes, h], ref, rtol=1e-12, atol=1e-12)
        seen[nodes] = True
    assert seen.all()


def test_chain_tree_is_causal_attention():
    rng = np.random.default_rng(2)
    K, L, n_h, d_h = 4, 7, 3, 16
    tree = orc.tree_from_paths(si.chain_tree_paths(K), K)
    assert tree.T == K + 1
    assert np.array_equal(tree.mask, np.tril(np.ones((K + 1, K + 1), dtype=bool)))
    q, k, v = random_case(rng, K + 1, n_h, d_h, L)
    got = orc.tree_attention(q, k, v, L, tree.mask)
    for h in range(n_h):
        qs = np.concatenate([np.zeros((L, d_h)), q[:, h]], axis=0)
        ref = causal_attention_plain(qs, k[h], v[h])[L:]
        np.testing.assert_allclose(got[:, h], ref, rtol=1e-12, atol=1e-12)


def test_star_tree_sees_cache_root_and_self_only():
    rng = np.random.default_rng(3)
    n, L, n_h, d_h = 5, 4, 2, 8
    tree = orc.tree_from_paths(si.star_tree_paths(n), 1)
    q, k, v = random_case(rng, n + 1, n_h, d_h, L)
    got = orc.tree_attention(q, k, v, L, tree.mask)
    for i in range(1, n + 1):
        rows = list(range(L)) + [L, L + i]
        for h in range(n_h):
            s = k[h, rows] @ q[i, h] / np.sqrt(d_h)
            w = np.exp(s - s.max()); w /= w.sum()
            np.testing.assert_allclose(got[i, h], w @ v[h, rows], rtol=1e-12)


def test_tree_attention_matches_torch_sdpa():
    """Same result from torch's attention routine given the explicit boolean mask."""
    rng = np.random.default_rng(4)
    T, L, n_h, d_h = 64, 40, 4, 32
    tree = orc.tree_from_paths(si.tree_paths(T, (10,) * 4), 4)
    q, k, v = random_case(rng, T, n_h, d_h, L)
    got = orc.tree_attention(q, k, v, L, tree.mask)
    full = np.concatenate([np.ones((T, L), dtype=bool), tree.mask], axis=1)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).permute(1, 0, 2)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None],
        attn_mask=torch.from_numpy(full)[None, None])
    np.testing.assert_allclose(got, ref[0].permute(1, 0, 2).numpy(), rtol=1e-10, atol=1e-12)


def test_mask_invariants():
    for T, caps in [(16, (4, 2, 2, 2)), (64, (10,) * 4), (96, (10,) * 5)]:
        tree = orc.tree_from_paths(si.tree_paths(T, caps), len(caps))
        assert np.array_equal(tree.mask.sum(axis=1), tree.depth + 1)          # ancestors + self
        assert not np.triu(tree.mask, 1).any()                                 # parents come first
        assert tree.mask[:, 0].all()                                           # everyone sees the root
        for i in range(1, T):
            assert np.array_equal(tree.mask[i] & ~np.eye(T, dtype=bool)[i], tree.mask[tree.parent[i]])


# ---------------------------------------------------------------------------- Eq. 5
def make_aeb(rng, K, d):
    return [rng.standard_normal((d, d)) * 0.2 for _ in range(4)], rng.standard_normal((K, d))


def test_biattention_single_row_closed_form():
    """K = 1: softmax over one key is 1, so attn_o = Wo Wv H_p."""
    rng = np.random.default_rng(5)
    (wq, wk, wv, wo), Hp = make_aeb(rng, 1, 32)
    got = orc.bi_self_attention(Hp, wq, wk, wv, wo, n_heads=4)
    np.testing.assert_allclose(got[0], wo @ (wv @ Hp[0]), rtol=1e-12)


def test_biattention_zero_query_gives_mean_of_values():
    rng = np.random.default_rng(6)
    (wq, wk, wv, wo), Hp = make_aeb(rng, 4, 32)
    got = orc.bi_self_attention(Hp, np.zeros_like(wq), wk, wv, wo, n_heads=4)
    mean_v = (Hp @ wv.T).mean(axis=0)
    for r in range(4):
        np.testing.assert_allclose(got[r], wo @ mean_v, rtol=1e-12)


def test_biattention_is_row_permutation_equivariant_and_not_causal():
    rng = np.random.default_rng(7)
    (wq, wk, wv, wo), Hp = make_aeb(rng, 4, 32)
    got = orc.bi_self_attention(Hp, wq, wk, wv, wo, n_heads=4)
    perm = np.array([2, 0, 3, 1])
    got_p = orc.bi_self_attention(Hp[perm], wq, wk, wv, wo, n_heads=4)
    np.testing.assert_allclose(got_p, got[perm], rtol=1e-11, atol=1e-13)
    # the first row must depend on the last one (a causal mask would forbid that)
    Hp2 = Hp.copy(); Hp2[3] += 1.0
    got2 = orc.bi_self_attention(Hp2, wq, wk, wv, wo, n_heads=4)
    assert np.abs(got2[0] - got[0]).max() > 1e-6


def test_biattention_matches_torch_mha():
    """torch.nn.functional.multi_head_attention_forward with the same four matrices, no mask."""
    rng = np.random.default_rng(8)
    K, d, n_h = 5, 48, 4
    (wq, wk, wv, wo), Hp = make_aeb(rng, K, d)
    got = orc.bi_self_attention(Hp, wq, wk, wv, wo, n_heads=n_h)
    x = torch.from_numpy(Hp)[:, None, :]
    ref, _ = torch.nn.functional.multi_head_attention_forward(
        x, x, x, d, n_h, in_proj_weight=None, in_proj_bias=None, bias_k=None, bias_v=None, add_zero_attn=False,
        dropout_p=0.0, out_proj_weight=torch.from_numpy(wo), out_proj_bias=None, use_separate_proj_weight=True,
        q_proj_weight=torch.from_numpy(wq), k_proj_weight=torch.from_numpy(wk), v_proj_weight=torch.from_numpy(wv),
        need_weights=False)
    np.testing.assert_allclose(got, ref[:, 0].numpy(), rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------------------- building blocks
def test_rope_is_a_plane_rotation():
    """d_h = 2: theta^0 = 1, so the single pair is rotated by exactly `pos` radians."""
    out = orc.rope(np.array([[1.0, 0.0]]), 3, 10000.0)
    np.testing.assert_allclose(out[0], [np.cos(3.0), np.sin(3.0)], rtol=1e-14)
    out = orc.rope(np.array([[0.0, 1.0]]), 3, 10000.0)
    np.testing.assert_allclose(out[0], [-np.sin(3.0), np.cos(3.0)], rtol=1e-14)


def test_rope_pairs_half_split_and_relative():
    rng = np.random.default_rng(9)
    d_h = 16
    q, k = rng.standard_normal(d_h), rng.standard_normal(d_h)
    # norm preserved, dot product depends on m - n only
    assert np.isclose(np.linalg.norm(orc.rope(q, 11, 1e4)), np.linalg.norm(q))
    a = np.dot(orc.rope(q, 9, 1e4), orc.rope(k, 4, 1e4))
    b = np.dot(orc.rope(q, 105, 1e4), orc.rope(k, 100, 1e4))
    assert np.isclose(a, b, rtol=1e-10)
    # component i pairs with i + d_h/2 and uses frequency theta^(-2i/d_h)
    x = np.zeros(d_h); x[3] = 1.0
    y = orc.rope(x, 2, 1e4)
    ang = 2 * 1e4 ** (-2 * 3 / d_h)
    expect = np.zeros(d_h); expect[3] = np.cos(ang); expect[3 + d_h // 2] = np.sin(ang)
    np.testing.assert_allclose(y, expect, atol=1e-15)


def test_rmsnorm_and_silu_match_torch():
    rng = np.random.default_rng(10)
    x, w = rng.standard_normal((3, 40)), rng.standard_normal(40)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (40,), torch.from_numpy(w), eps=1e-6)
    np.testing.assert_allclose(orc.rmsnorm(x, w, 1e-6), ref.numpy(), rtol=1e-12)
    np.testing.assert_allclose(orc.silu(x), torch.nn.functional.silu(torch.from_numpy(x)).numpy(), rtol=1e-12)
    y = orc.rmsnorm(x, np.ones(40), 0.0)
    np.testing.assert_allclose(np.sqrt((y * y).mean(axis=-1)), 1.0, rtol=1e-12)


def test_linear_is_a_plain_matvec():
    rng = np.random.default_rng(11)
    W, x = rng.standard_normal((5, 7)), rng.standard_normal(7)
    ref = [sum(W[i, j] * x[j] for j in range(7)) for i in range(5)]
    np.testing.assert_allclose(orc.linear(W, x), ref, rtol=1e-13)
    X = rng.standard_normal((3, 7))
    np.testing.assert_allclose(orc.linear(W, X), (torch.from_numpy(X) @ torch.from_numpy(W).T).numpy(), rtol=1e-13)


# ---------------------------------------------------------------------------- SAL layer, Eq. 1
def small_layer(rng, d, f):
    g = lambda *s: rng.standard_normal(s) * 0.2
    return dict(rms1=1 + 0.1 * rng.standard_normal(d), rms2=1 + 0.1 * rng.standard_normal(d),
                wq=g(d, d), wk=g(d, d), wv=g(d, d), wo=g(d, d), w_gate=g(f, d), w_up=g(f, d), w_down=g(d, f))


def test_sal_incremental_equals_full_causal_recompute():
    """Feeding positions one at a time through the cache gives the last row of a full causal pass."""
    rng = np.random.default_rng(12)
    d, n_h, f, S = 32, 4, 48, 6
    d_h = d // n_h
    lw = small_layer(rng, d, f)
    xs = rng.standard_normal((S, d))
    full, _, _, _, _ = orc.decoder_layer_rows(xs, lw, np.zeros((n_h, 0, d_h)), np.zeros((n_h, 0, d_h)),
                                              list(range(S)), np.tril(np.ones((S, S), dtype=bool)), n_h, 1e-6, 1e4)
    kc, vc = np.zeros((n_h, 0, d_h)), np.zeros((n_h, 0, d_h))
    for t in range(S):
        out, k_new, v_new = orc.sal_stage(xs[t], lw, kc, vc, n_h, 1e-6, 1e4)
        np.testing.assert_allclose(out, full[t], rtol=1e-10, atol=1e-12)
        kc = np.concatenate([kc, k_new[:, None, :]], axis=1)
        vc = np.concatenate([vc, v_new[:, None, :]], axis=1)


def test_sal_empty_cache_attention_returns_value():
    """With nothing cached the only key is the new one: attention output = its value vector."""
    rng = np.random.default_rng(13)
    d, n_h, f = 32, 4, 48
    lw = small_layer(rng, d, f)
    x = rng.standard_normal(d)
    _, k_new, v_new, q, attn = orc.decoder_layer_rows(x[None], lw, np.zeros((n_h, 0, 8)), np.zeros((n_h, 0, 8)),
                                                      [0], np.ones((1, 1), dtype=bool), n_h, 1e-6, 1e4)
    np.testing.assert_allclose(attn[0], v_new[:, 0, :], rtol=1e-13)
    n = orc.rmsnorm(x, lw["rms1"], 1e-6)
    np.testing.assert_allclose(v_new[:, 0, :].reshape(-1), lw["wv"] @ n, rtol=1e-12)
    np.testing.assert_allclose(k_new[:, 0, :].reshape(-1), lw["wk"] @ n, rtol=1e-12)   # position 0: no rotation
