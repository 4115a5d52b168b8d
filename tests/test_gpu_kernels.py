"""GPU parity of the single kernels behind the C ABI against the CPU oracle, element by element, on
seeded inputs: the weight-streaming GEMV, the matrix-core skinny GEMM, tree-masked verification
attention, candidate-tree construction and greedy acceptance."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import amphista_oracle as orc
from paper_2406_13170_amd import binding as B
from paper_2406_13170_amd import device as D

from gpu_common import (DEV, TOL, act_to_dev, assert_rows_close, cfg_tensor_to_dev, f32_to_dev, i32_to_dev, make_ctx,
                        np_of, say)

pytestmark = pytest.mark.gpu


# ---------------------------------------------------------------------------- GEMV (A1-A5 building block)
@pytest.mark.parametrize("cfg,M,N,Kd", [
    (si.TINY, 1, 256, 512), (si.TINY, 4, 1024, 256), (si.TINY, 1, 256, 688), (si.TINY, 5, 77, 264),
    (si.MINI, 1, 512, 1024), (si.MINI, 4, 2048, 512), (si.MINI, 1, 512, 1376), (si.MINI, 8, 203, 520), (si.MINI, 3, 64, 8),
    (si.V7B, 1, 4096, 4096), (si.V7B, 1, 4096, 11008), (si.V7B, 4, 32000, 4096),
])
def test_gemv_matches_oracle(cfg, M, N, Kd):
    say(f"gemv {cfg.name} M={M} N={N} Kd={Kd}")
    ctx = make_ctx(cfg)
    W = si.normal(cfg, 11, f"gemv.W.{N}.{Kd}", (N, Kd), si.W_STD)
    x = si.as_f32_exact(cfg, 11, f"gemv.x.{M}.{Kd}", (M, Kd), 1.0)
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
    ctx.amph_gemv(f32_to_dev(x), cfg_tensor_to_dev(W), y, M, N, Kd)
    torch.cuda.synchronize()
    ref = orc.linear(W.f32, x)
    assert_rows_close(np_of(y), ref, 1e-4, "gemv")          # exact products, float32 accumulation in both dtypes


# ---------------------------------------------------------------------------- skinny GEMM (A7/A9 building block)
@pytest.mark.parametrize("cfg,M,N,Kd,split", [
    (si.TINY, 16, 256, 256, 1), (si.TINY, 16, 256, 688 // 16 * 16, 2), (si.TINY, 37, 100, 256, 0),
    (si.MINI, 64, 512, 512, 1), (si.MINI, 64, 512, 1376, 4), (si.MINI, 130, 203, 512, 2), (si.MINI, 7, 64, 32, 1),
    (si.MINI, 64, 2048, 512, 8),
    (si.V7B, 64, 4096, 4096, 0), (si.V7B, 64, 4096, 11008, 0), (si.V7B, 64, 1024, 4096, 8),
])
def test_gemm_matches_oracle(cfg, M, N, Kd, split):
    say(f"gemm {cfg.name} M={M} N={N} Kd={Kd} split={split}")
    ctx = make_ctx(cfg)
    W = si.normal(cfg, 12, f"gemm.W.{N}.{Kd}", (N, Kd), si.W_STD)
    x = si.normal(cfg, 12, f"gemm.x.{M}.{Kd}", (M, Kd), 1.0)
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
    ctx.amph_gemm(cfg_tensor_to_dev(x), cfg_tensor_to_dev(W), y, M, N, Kd, split)
    torch.cuda.synchronize()
    ref = orc.linear(W.f32, x.f32)
    assert_rows_close(np_of(y), ref, 1e-4, "gemm")
    # split-K partials are folded in a fixed order: a second run is bit-identical
    y2 = torch.empty_like(y)
    ctx.amph_gemm(cfg_tensor_to_dev(x), cfg_tensor_to_dev(W), y2, M, N, Kd, split)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)


# ---------------------------------------------------------------------------- A8 tree-masked attention
KERNELS = [0, 1]        # amph_verify_kernel: operands through registers / through the LDS ring
KERNEL_IDS = ["regs", "ring"]


def verify_case(cfg, T, caps, L, B_=1, seed=21, heads=None, lens=None, kernel=-1):
    K = len(caps)
    cfgx = si.with_(cfg, batch=B_, K=K, topk=min(16, max(caps)))
    lens = [L] * B_ if lens is None else list(lens)      # committed rows per batch element (L = the largest)
    assert max(lens) == L and len(lens) == B_
    max_kv = (L + T + 31) // 32 * 32 + 32
    ctx = make_ctx(cfgx, T=T, batch=B_, max_kv=max_kv)
    ctx.amph_verify_kernel(kernel)
    paths = si.tree_paths(T, caps)
    tree = B.Tree(paths, K)
    otree = orc.tree_from_paths(paths, K)
    n_h, d_h = cfg.n_heads, cfg.head_dim
    q = si.normal(cfgx, seed, "va.q", (B_, T, n_h, d_h), 1.0)
    k = si.normal(cfgx, seed, "va.k", (B_, n_h, L + T, d_h), 1.0)
    v = si.normal(cfgx, seed, "va.v", (B_, n_h, L + T, d_h), 1.0)
    tdt = D.torch_dtype(cfg.dtype)
    # caches start as NaN everywhere outside the valid rows: nothing beyond L + T may leak in
    k_rows = torch.full((B_, n_h, max_kv, d_h), float("nan"), dtype=tdt, device=DEV)
    v_rows = torch.full((B_, n_h, max_kv, d_h), float("nan"), dtype=tdt, device=DEV)
    for b in range(B_):                                   # element b uses rows [0, lens[b] + T) of its random rows
        k_rows[b, :, :lens[b] + T] = cfg_tensor_to_dev(k)[b, :, :lens[b] + T]
        v_rows[b, :, :lens[b] + T] = cfg_tensor_to_dev(v)[b, :, :lens[b] + T]
    kc, vc = D.pack_kv(ctx, k_rows, v_rows)
    out = torch.full((B_, T, n_h, d_h), float("nan"), dtype=tdt, device=DEV)
    kv_len = i32_to_dev(np.asarray(lens))
    ctx.amph_verify_attn(tree, cfg_tensor_to_dev(q), kc, vc, kv_len, out)
    torch.cuda.synchronize()
    assert ctx.device_status() == 0
    got = np_of(out)
    hs = range(n_h) if heads is None else heads
    worst = 0.0
    for b in range(B_):
        for h in hs:
            n = lens[b] + T
            ref = orc.tree_attention(q.f32[b][:, h:h + 1], k.f32[b][h:h + 1, :n], v.f32[b][h:h + 1, :n], lens[b], otree.mask)
            worst = max(worst, assert_rows_close(got[b][:, h], ref[:, 0], TOL[cfg.dtype], f"verify_attn b={b} h={h}"))
    return worst


@pytest.mark.parametrize("cfg,T,caps,L", [
    (si.TINY, 16, (4, 2, 2, 2), 128),
    (si.TINY, 16, (4, 2, 2, 2), 0),             # empty cache: only root/ancestors/self
    (si.TINY, 22, (10,) * 4, 37),               # ragged: 22 queries in 2 blocks, L not a multiple of the key step
    (si.TINY, 5, (1, 1, 1, 1), 9),              # chain tree = causal attention
    (si.MINI, 64, (10,) * 4, 200),
    (si.MINI, 64, (10,) * 4, 1),
    (si.MINI, 96, (10,) * 5, 333),              # two query groups of three 16-query blocks
    (si.MINI, 35, (10,) * 4, 1000),
    (si.MINI, 128, (10,) * 8, 64),              # the largest tree (eight 16-query blocks), depth 8
    (si.MINI, 1, (4, 4, 4, 4), 96),             # the root alone = one-token decoding
    (si.TINY, 1, (4, 4, 4, 4), 0),              # one query, one key (itself)
])
@pytest.mark.parametrize("kernel", KERNELS, ids=KERNEL_IDS)
def test_verify_attn_matches_oracle(cfg, T, caps, L, kernel):
    say(f"verify_attn {cfg.name} T={T} L={L} kernel={kernel}")
    worst = verify_case(cfg, T, caps, L, kernel=kernel)
    say(f"  worst row error {worst:.2e}")


@pytest.mark.parametrize("kernel", KERNELS, ids=KERNEL_IDS)
def test_verify_attn_batch_independent_lengths_share_a_launch(kernel):
    say(f"verify_attn batch=3, committed lengths 77 / 5 / 40 in one launch, kernel={kernel}")
    verify_case(si.MINI, 64, (10,) * 4, 77, B_=3, lens=[77, 5, 40], kernel=kernel)
    say("verify_attn batch=2, one element with an empty cache")
    verify_case(si.MINI, 35, (10,) * 4, 130, B_=2, lens=[0, 130], kernel=kernel)


@pytest.mark.parametrize("cfg,T,caps,L,B_", [
    (si.MINI, 64, (10,) * 4, 77, 4),            # 4 x 4 heads x 4 query blocks
    (si.MINI, 22, (10,) * 4, 37, 8),            # ragged last query block
    (si.TINY, 64, (10,) * 4, 130, 4),           # float32 (16-key steps, 64-wide heads)
    (si.MINI, 64, (10,) * 4, 0, 4),             # empty cache
])
@pytest.mark.parametrize("kernel", KERNELS, ids=KERNEL_IDS)
def test_verify_attn_many_workgroups(cfg, T, caps, L, B_, kernel):
    """Batches large enough that (batch, head, query block) alone fill a quarter of the chip: the launch
    heuristics then pick few or no key splits."""
    say(f"verify_attn {cfg.name} T={T} L={L} B={B_} kernel={kernel}")
    worst = verify_case(cfg, T, caps, L, B_=B_, kernel=kernel)
    say(f"  worst row error {worst:.2e}")


@pytest.mark.parametrize("kernel", [-1, 1], ids=["auto", "ring"])
def test_verify_attn_vicuna7b_shape(kernel):
    """Full 7B layer shape (32 heads x 128, L = 1024, T = 64) in the launch configuration the bench uses
    (kernel chosen by shape), and with the other kernel; every head checked against the oracle."""
    say(f"verify_attn vicuna7b L=1024 T=64 kernel={kernel}")
    worst = verify_case(si.V7B, 64, (10,) * 4, 1024, kernel=kernel)
    say(f"  worst row error {worst:.2e}")


def test_verify_attn_long_cache_whole_head_per_workgroup():
    """Shape for which the choice by shape takes the LDS ring without key splits (batch x heads above the number of
    compute units) and every workgroup walks a long cache: 9 x 32 heads, L = 2500 (79 key steps, ragged)."""
    say("verify_attn vicuna7b heads, batch 9, L=2500 T=64, kernel by shape")
    worst = verify_case(si.V7B, 64, (10,) * 4, 2500, B_=9, heads=[0, 13, 31], lens=[2500, 17, 1200, 2499, 0, 64, 2048, 999, 2500])
    say(f"  worst row error {worst:.2e}")


@pytest.mark.parametrize("cfg,T,caps,heads", [
    (si.TINY, 22, (10,) * 4, [0, 3]),           # float32, 64-wide heads, two query waves per key group
    (si.TINY, 1, (4, 4, 4, 4), [1]),            # one query
    (si.MINI, 112, (10,) * 7, [2]),             # bf16, 128-wide heads, seven query waves per key group: 1024 threads
    (si.MINI, 96, (10,) * 5, [0]),              # the 33B tree size
])
def test_verify_attn_ring_two_key_groups(cfg, T, caps, heads):
    """Batch x heads above the number of compute units: the LDS ring runs without key splits and with two groups of
    math waves that take alternate key steps and merge through LDS.  The committed lengths give every count of key
    steps from 1 upwards (odd counts leave the second group without a step in the last stage; one step leaves it
    with none at all), full and ragged last steps, and an empty cache."""
    B_ = 33
    kstep = 16 if cfg.dtype == si.F32 else 32
    lens = [0, 1, kstep - 1, kstep, kstep + 1, 2 * kstep, 3 * kstep - T % kstep, 5 * kstep + 3, 8 * kstep, 9 * kstep + 7, 301]
    lens = [max(0, x) for x in lens]
    lens = (lens * 3)[:B_]
    say(f"verify_attn ring, two key groups: {cfg.name} T={T} batch={B_}")
    worst = verify_case(cfg, T, caps, max(lens), B_=B_, heads=heads, lens=lens, kernel=1)
    say(f"  worst row error {worst:.2e}")


def test_verify_kernel_selector_rejects_unknown_values():
    ctx = make_ctx(si.TINY, T=16)
    for bad in (-2, 2, 7):
        with pytest.raises(RuntimeError):
            ctx.amph_verify_kernel(bad)
    ctx.amph_verify_kernel(-1)


def test_verify_attn_flags_cache_overflow():
    cfg = si.TINY
    ctx = make_ctx(cfg, T=16, max_kv=64)
    tree = B.Tree(si.tree_paths(16, (4, 2, 2, 2)), 4)
    tdt = D.torch_dtype(cfg.dtype)
    q = torch.zeros((1, 16, cfg.n_heads, cfg.head_dim), dtype=tdt, device=DEV)
    kc = torch.zeros((1, cfg.n_heads, 64, cfg.head_dim), dtype=tdt, device=DEV)
    vc = torch.zeros((1, cfg.n_heads, cfg.head_dim, 64), dtype=tdt, device=DEV)
    out = torch.full_like(q, 7.0)
    ctx.amph_verify_attn(tree, q, kc, vc, i32_to_dev([60]), out)       # 60 + 16 > 64
    assert ctx.device_status() == B.AMPH_DEV_KV_OVERFLOW
    assert torch.all(out == 7.0)                                        # nothing written
    assert ctx.device_status() == 0                                     # the flag was cleared by the read


# ---------------------------------------------------------------------------- A6 / A10 integer work
@pytest.mark.parametrize("T,caps,B_", [(16, (4, 2, 2, 2), 1), (64, (10,) * 4, 1), (96, (10,) * 5, 4),
                                       (128, (10,) * 8, 2),        # the largest tree and the most heads the library takes
                                       (1, (4, 4, 4, 4), 1),       # the root alone: nothing to accept
                                       (5, (1, 1, 1, 1), 1)])      # a chain
def test_tree_build_and_accept_are_bit_exact(T, caps, B_):
    say(f"tree_build/accept T={T} B={B_}")
    K = len(caps)
    cfg = si.with_(si.MINI, K=K, batch=B_, topk=10 if caps[0] > 4 else 4)
    ctx = make_ctx(cfg, T=T, batch=B_)
    paths = si.tree_paths(T, caps)
    tree = B.Tree(paths, K)
    otree = orc.tree_from_paths(paths, K)
    rng = np.random.default_rng(5)
    for trial in range(8):
        vocab = 13                      # tiny vocabulary so that many drafts hit the target's choice
        topk = np.stack([[rng.permutation(vocab)[:cfg.topk] for _ in range(K)] for _ in range(B_)]).astype(np.int32)
        root = rng.integers(0, vocab, size=B_).astype(np.int32)
        kvl = rng.integers(0, 1000, size=B_).astype(np.int32)
        tok = torch.empty((B_, T), dtype=torch.int32, device=DEV)
        pos = torch.empty((B_, T), dtype=torch.int32, device=DEV)
        ctx.amph_tree_build(tree, i32_to_dev(root), i32_to_dev(topk), i32_to_dev(kvl), tok, pos)
        tgt = rng.integers(0, vocab, size=(B_, T)).astype(np.int32)
        a_len = torch.empty(B_, dtype=torch.int32, device=DEV)
        a_path = torch.empty((B_, K + 1), dtype=torch.int32, device=DEV)
        nxt = torch.empty(B_, dtype=torch.int32, device=DEV)
        best = torch.empty(B_, dtype=torch.int32, device=DEV)
        ctx.amph_accept(tree, tok, i32_to_dev(tgt), None, a_len, a_path, nxt, best)
        torch.cuda.synchronize()
        for b in range(B_):
            o_tok, o_pos = orc.tree_tokens(otree, int(root[b]), topk[b], int(kvl[b]))
            np.testing.assert_array_equal(np_of(tok)[b], o_tok)
            np.testing.assert_array_equal(np_of(pos)[b], o_pos)
            oa, opath, onxt, obest = orc.accept_greedy(otree, o_tok, tgt[b])
            assert int(a_len[b]) == oa and int(best[b]) == obest and int(nxt[b]) == onxt
            np.testing.assert_array_equal(np_of(a_path)[b], opath)


@pytest.mark.parametrize("seed", range(6))
def test_random_irregular_trees_build_accept_and_attention(seed):
    """Irregular topologies end to end: tree tokens and positions, greedy acceptance with planted accepted paths, and
    the tree-masked attention of both kernels, each against the oracle."""
    rng = np.random.default_rng(100 + seed)
    K = int(rng.integers(2, 9))
    topk = int(rng.integers(2, 17))
    T = int(min(rng.integers(2, 129), sum(topk ** j for j in range(1, K + 1)) + 1))
    B_ = int(rng.integers(1, 4))
    say(f"random tree seed={seed}: T={T} K={K} topk={topk} B={B_}")
    cfg = si.with_(si.MINI, K=K, batch=B_, topk=topk)
    paths = si.random_tree_paths(T, K, topk, seed)
    tree = B.Tree(paths, K)
    otree = orc.tree_from_paths(paths, K)
    ctx = make_ctx(cfg, T=T, batch=B_)
    vocab = 11
    for trial in range(4):
        top = np.stack([[rng.permutation(max(vocab, topk))[:topk] for _ in range(K)] for _ in range(B_)]).astype(np.int32)
        root = rng.integers(0, vocab, size=B_).astype(np.int32)
        kvl = rng.integers(0, 500, size=B_).astype(np.int32)
        tok = torch.empty((B_, T), dtype=torch.int32, device=DEV)
        pos = torch.empty((B_, T), dtype=torch.int32, device=DEV)
        ctx.amph_tree_build(tree, i32_to_dev(root), i32_to_dev(top), i32_to_dev(kvl), tok, pos)
        torch.cuda.synchronize()
        tgt = rng.integers(0, vocab, size=(B_, T)).astype(np.int32)
        o_toks = []
        for b in range(B_):
            o_tok, o_pos = orc.tree_tokens(otree, int(root[b]), top[b], int(kvl[b]))
            np.testing.assert_array_equal(np_of(tok)[b], o_tok)
            np.testing.assert_array_equal(np_of(pos)[b], o_pos)
            o_toks.append(o_tok)
            # plant an accepted path down to a random node: the target picks the drafted token at every ancestor
            node = int(rng.integers(0, T))
            while node > 0:
                tgt[b, otree.parent[node]] = o_tok[node]
                node = int(otree.parent[node])
        a_len = torch.empty(B_, dtype=torch.int32, device=DEV)
        a_path = torch.empty((B_, K + 1), dtype=torch.int32, device=DEV)
        nxt = torch.empty(B_, dtype=torch.int32, device=DEV)
        best = torch.empty(B_, dtype=torch.int32, device=DEV)
        ctx.amph_accept(tree, tok, i32_to_dev(tgt), None, a_len, a_path, nxt, best)
        torch.cuda.synchronize()
        for b in range(B_):
            oa, opath, onxt, obest = orc.accept_greedy(otree, o_toks[b], tgt[b])
            assert int(a_len[b]) == oa and int(best[b]) == obest and int(nxt[b]) == onxt
            np.testing.assert_array_equal(np_of(a_path)[b], opath)
    # attention with this tree's mask, both kernels
    L = int(rng.integers(0, 300))
    for kernel in KERNELS:
        verify_case_paths(si.MINI, paths, K, topk, L, B_, kernel)


def verify_case_paths(cfg, paths, K, topk, L, B_, kernel, seed=23):
    T = len(paths) + 1
    cfgx = si.with_(cfg, batch=B_, K=K, topk=topk)
    max_kv = (L + T + 31) // 32 * 32 + 32
    ctx = make_ctx(cfgx, T=T, batch=B_, max_kv=max_kv)
    ctx.amph_verify_kernel(kernel)
    tree = B.Tree(paths, K)
    otree = orc.tree_from_paths(paths, K)
    n_h, d_h = cfg.n_heads, cfg.head_dim
    q = si.normal(cfgx, seed, "vr.q", (B_, T, n_h, d_h), 1.0)
    k = si.normal(cfgx, seed, "vr.k", (B_, n_h, L + T, d_h), 1.0)
    v = si.normal(cfgx, seed, "vr.v", (B_, n_h, L + T, d_h), 1.0)
    tdt = D.torch_dtype(cfg.dtype)
    k_rows = torch.full((B_, n_h, max_kv, d_h), float("nan"), dtype=tdt, device=DEV)
    v_rows = torch.full((B_, n_h, max_kv, d_h), float("nan"), dtype=tdt, device=DEV)
    k_rows[:, :, :L + T] = cfg_tensor_to_dev(k)
    v_rows[:, :, :L + T] = cfg_tensor_to_dev(v)
    out = torch.full((B_, T, n_h, d_h), float("nan"), dtype=tdt, device=DEV)
    kc, vc = D.pack_kv(ctx, k_rows, v_rows)
    ctx.amph_verify_attn(tree, cfg_tensor_to_dev(q), kc, vc, i32_to_dev(np.full(B_, L)), out)
    torch.cuda.synchronize()
    assert ctx.device_status() == 0
    got = np_of(out)
    for b in range(B_):
        for h in range(n_h):
            ref = orc.tree_attention(q.f32[b][:, h:h + 1], k.f32[b][h:h + 1], v.f32[b][h:h + 1], L, otree.mask)
            assert_rows_close(got[b][:, h], ref[:, 0], TOL[cfg.dtype], f"random-tree verify_attn b={b} h={h} kernel={kernel}")


def test_accept_from_logits_takes_argmax_with_lowest_id_on_ties():
    cfg = si.with_(si.TINY, vocab=1024)
    T, K = 16, 4
    ctx = make_ctx(cfg, T=T)
    paths = si.tree_paths(T, (4, 2, 2, 2))
    tree = B.Tree(paths, K)
    otree = orc.tree_from_paths(paths, K)
    rng = np.random.default_rng(6)
    logits = rng.standard_normal((1, T, cfg.vocab)).astype(np.float32)
    logits[0, :, 700] = logits[0].max(axis=1) + 1.0
    logits[0, :, 300] = logits[0, :, 700]                 # exact tie: 300 must win
    logits[0, 3, 5] = logits[0, 3, 300]                   # three-way tie at node 3: 5 wins
    tgt = np.array([orc.row_argmax(r) for r in logits[0]], dtype=np.int32)
    assert tgt[0] == 300 and tgt[3] == 5
    tok = np.zeros(T, dtype=np.int32)
    tok[1:] = rng.integers(0, cfg.vocab, size=T - 1)
    # plant a full accepted path so that the logits-derived argmax decides every hop
    path = [int(n) for n in otree.retrieve[np.argmax((otree.retrieve >= 0).sum(axis=1))] if n >= 0]
    for par, ch in zip(path[:-1], path[1:]):
        tok[ch] = tgt[par]
    a_len = torch.empty(1, dtype=torch.int32, device=DEV)
    a_path = torch.empty((1, K + 1), dtype=torch.int32, device=DEV)
    nxt = torch.empty(1, dtype=torch.int32, device=DEV)
    best = torch.empty(1, dtype=torch.int32, device=DEV)
    ctx.amph_accept(tree, i32_to_dev(tok[None]), None, f32_to_dev(logits), a_len, a_path, nxt, best)
    torch.cuda.synchronize()
    oa, opath, onxt, obest = orc.accept_greedy(otree, tok, tgt)
    assert oa == 4
    assert (int(a_len[0]), int(best[0]), int(nxt[0])) == (oa, obest, onxt)
    np.testing.assert_array_equal(np_of(a_path)[0], opath)


# ---------------------------------------------------------------------------- K/V cache layout converters
@pytest.mark.parametrize("cfg,max_kv,lead", [(si.TINY, 96, (2, 1, 4)), (si.MINI, 160, (3, 2, 4)), (si.V7B, 1088, (1, 1, 32))])
def test_pack_and_unpack_kv_follow_the_header_formulas(cfg, max_kv, lead):
    """amph_pack_kv / amph_unpack_kv against the torch-permute reference of the header's byte formulas
    (tests/layout_ref.py, itself checked against those formulas on the CPU): pure data movement, bit-exact."""
    import layout_ref as R
    say(f"pack_kv / unpack_kv {cfg.name} max_kv={max_kv} caches={lead}")
    ctx = make_ctx(cfg, max_kv=max_kv)
    tdt = D.torch_dtype(cfg.dtype)
    g = torch.Generator(device="cpu").manual_seed(5)
    shape = (*lead, max_kv, cfg.head_dim)
    k_rows = torch.randn(shape, generator=g).to(tdt).to(DEV)
    v_rows = torch.randn(shape, generator=g).to(tdt).to(DEV)
    k_t, v_t = D.pack_kv(ctx, k_rows, v_rows)
    torch.cuda.synchronize()
    assert torch.equal(k_t, R.keys_to_tiled(k_rows)) and torch.equal(v_t, R.values_to_tiled(v_rows))
    k_back, v_back = D.unpack_kv(ctx, k_t, v_t)
    torch.cuda.synchronize()
    assert torch.equal(k_back, k_rows) and torch.equal(v_back, v_rows)
    # keys alone / values alone leave the other destination untouched
    only_k = torch.zeros_like(k_rows)
    ctx.amph_pack_kv(k_rows, None, only_k, None, k_rows.numel() // (max_kv * cfg.head_dim))
    torch.cuda.synchronize()
    assert torch.equal(only_k, k_t)
    with pytest.raises(B.AmphError):
        ctx.amph_pack_kv(k_rows, None, None, v_t, 1)          # a destination without its source
    with pytest.raises(B.AmphError):
        ctx.amph_pack_kv(k_rows, None, k_rows, None, 1)       # in place
