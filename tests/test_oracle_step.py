"""Pins for the rest of the oracle: Eq. 1-4 and 6 closed forms, top-k, the draft tree, greedy
acceptance, losslessness against the target's own autoregressive decoding, and a Hugging Face
Llama decoder stack run with identical weights and the same tree mask."""
import os

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import amphista_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


# ---------------------------------------------------------------------------- Eq. 1-4
def test_fc_concat_order_hidden_then_embedding():
    d = 6
    rng = np.random.default_rng(0)
    h, e = rng.standard_normal(d), rng.standard_normal(d)
    W_h = np.concatenate([np.eye(d), np.zeros((d, d))], axis=1)
    W_e = np.concatenate([np.zeros((d, d)), np.eye(d)], axis=1)
    np.testing.assert_array_equal(orc.fc_concat(W_h, h, e), h)
    np.testing.assert_array_equal(orc.fc_concat(W_e, h, e), e)


@pytest.mark.parametrize("K,first_half", [(4, 2), (5, 2), (2, 1)])
def test_heads_split_between_the_two_stages(K, first_half):
    """Eq. 2: heads 1..floor(K/2) read h^1, the others h^2.  With W = 0, SiLU(0) = 0, so row k is h^s + PE_k."""
    d = 8
    rng = np.random.default_rng(1)
    h1, h2, pe = rng.standard_normal(d), rng.standard_normal(d), rng.standard_normal((K, d))
    Hp = orc.head_inputs(h1, h2, np.zeros((K, d, d)), pe)
    for k in range(K):
        np.testing.assert_allclose(Hp[k], (h1 if k < first_half else h2) + pe[k], rtol=1e-15)


def test_head_mlp_form():
    rng = np.random.default_rng(2)
    d = 8
    W, h = rng.standard_normal((d, d)), rng.standard_normal(d)
    z = W @ h
    np.testing.assert_allclose(orc.head_mlp(W, h), h + z / (1 + np.exp(-z)), rtol=1e-13)


# ---------------------------------------------------------------------------- Eq. 6 / top-k
def test_topk_equals_full_sort_and_breaks_ties_by_lower_id():
    rng = np.random.default_rng(3)
    v = rng.standard_normal(500)
    idx, val = orc.topk_sorted(v, 10)
    ref = torch.topk(torch.from_numpy(v), 10)
    np.testing.assert_array_equal(idx, ref.indices.numpy())
    np.testing.assert_array_equal(val, ref.values.numpy())
    v[[7, 400, 33]] = v.max() + 1.0           # exact three-way tie at the top
    v[[100, 50]] = v.max() - 0.5              # and a two-way tie below it
    idx, val = orc.topk_sorted(v, 6)
    assert list(idx[:5]) == [7, 33, 400, 50, 100]
    assert np.all(np.diff(val) <= 0)


def test_lm_head_is_shared_across_rows():
    rng = np.random.default_rng(4)
    W, A = rng.standard_normal((50, 8)), rng.standard_normal((4, 8))
    logits, idx, val = orc.lm_head_topk(W, A, 3)
    for r in range(4):
        full = W @ A[r]
        np.testing.assert_allclose(logits[r], full, rtol=1e-13)
        assert list(idx[r]) == list(np.argsort(-full, kind="stable")[:3])


# ---------------------------------------------------------------------------- tree
def test_caption_example_two_heads():
    g = {r[0]: [int(x) for x in r[1:]] for r in read_golden("tree_caption_example.txt")}
    tree = orc.tree_from_paths(si.dense_tree_paths(g["widths"]), len(g["widths"]))
    assert tree.T == g["nodes_with_root"][0]
    assert len(tree.leaves) == g["candidate_sequences"][0]
    assert tree.retrieve.shape == (6, 3)
    assert len({tuple(r) for r in tree.retrieve}) == 6


def test_generator_counts_and_invariants():
    for name, T, caps, counts, leaves in read_golden("tree_generator_counts.txt"):
        T, leaves = int(T), int(leaves)
        caps = tuple(int(c) for c in caps.split(","))
        counts = [int(c) for c in counts.split(",")]
        paths = si.tree_paths(T, caps)
        tree = orc.tree_from_paths(paths, len(caps))
        assert tree.T == T
        assert [int((tree.depth == m).sum()) for m in range(1, len(caps) + 1)] == counts
        assert len(tree.leaves) == leaves
        S = set(paths)
        for p in paths:
            assert len(p) <= len(caps)
            assert len(p) == 1 or p[:-1] in S                      # parent present
            assert p[-1] == 0 or p[:-1] + (p[-1] - 1,) in S        # sibling-rank closure
        # node order: by depth, then lexicographic rank path
        assert tree.paths == sorted(tree.paths, key=lambda p: (len(p), p))


def test_tree_tokens_by_direct_indexing():
    rng = np.random.default_rng(5)
    tree = orc.tree_from_paths(si.tree_paths(64, (10,) * 4), 4)
    topk = rng.permutation(4 * 10).reshape(4, 10).astype(np.int32) + 100
    tok, pos = orc.tree_tokens(tree, 7, topk, 1000)
    assert tok[0] == 7 and pos[0] == 1000
    for i in range(1, 64):
        path = tree.paths[i]
        assert tok[i] == topk[len(path) - 1][path[-1]]
        assert pos[i] == 1000 + len(path)


def test_malformed_trees_rejected():
    with pytest.raises(ValueError):
        orc.tree_from_paths([(0,), (1, 0)], 4)          # parent (1,) missing
    with pytest.raises(ValueError):
        orc.tree_from_paths([(0,), (0,)], 4)            # duplicate
    with pytest.raises(ValueError):
        orc.tree_from_paths([(0,), (0, 0), (0, 0, 0)], 2)   # deeper than K


# ---------------------------------------------------------------------------- acceptance
def brute_force_accept(tree, tok, tgt):
    """Walk every root-to-leaf path and count how many draft tokens match the target's argmax."""
    best = (0, 0)
    for path in tree.retrieve:
        nodes = [int(n) for n in path if n >= 0]
        a = 0
        for par, ch in zip(nodes[:-1], nodes[1:]):
            if tok[ch] != tgt[par]:
                break
            a += 1
        if a > best[0]:
            best = (a, nodes[a])
    return best


def test_accept_against_path_walk():
    rng = np.random.default_rng(6)
    tree = orc.tree_from_paths(si.tree_paths(64, (10,) * 4), 4)
    for trial in range(200):
        topk = np.stack([rng.permutation(12)[:10] for _ in range(4)]).astype(np.int32)   # small vocab: many hits
        tok, _ = orc.tree_tokens(tree, 0, topk, 0)
        tgt = rng.integers(0, 12, size=64).astype(np.int32)
        a, path, nxt, best = orc.accept_greedy(tree, tok, tgt)
        ra, rbest = brute_force_accept(tree, tok, tgt)
        assert (a, best) == (ra, rbest)
        assert nxt == tgt[best]
        assert list(path[:a + 1]) == [int(n) for n in tree.retrieve[[best in r for r in tree.retrieve].index(True)][:a + 1]]
        assert (path[a + 1:] == -1).all()


# ---------------------------------------------------------------------------- whole-step invariants on Tiny
def tiny_setup(seed=0, n_layers=2, L=12):
    cfg = si.with_(si.TINY, d_model=64, n_heads=4, head_dim=16, d_ffn=96, vocab=97, kv_len=L, sal_len=L)
    f = lambda t: t.f32
    dw_t = si.draft_weights(cfg, seed)
    tw_t = si.target_weights(cfg, seed, n_layers)
    # larger weights than N(0, 0.02): at this width the logits would otherwise be nearly flat
    scale = 8.0
    conv_layer = lambda lw: {k: (f(v) * (scale if k.startswith("w") else 1.0)) for k, v in lw.items()}
    dw = dict(embed=f(dw_t["embed"]) * scale, fc=[f(x) * scale for x in dw_t["fc"]],
              sal=[conv_layer(l) for l in dw_t["sal"]], mlp=f(dw_t["mlp"]) * scale, pe=f(dw_t["pe"]),
              aeb_wq=f(dw_t["aeb_wq"]) * scale, aeb_wk=f(dw_t["aeb_wk"]) * scale, aeb_wv=f(dw_t["aeb_wv"]) * scale,
              aeb_wo=f(dw_t["aeb_wo"]) * scale, lm_head=f(dw_t["lm_head"]) * scale)
    tw = dict(embed=dw["embed"], layers=[conv_layer(l) for l in tw_t["layers"]],
              final_norm=f(tw_t["final_norm"]), lm_head=f(tw_t["lm_head"]) * scale)
    return cfg, dw, tw


def target_prefill(cfg, tw, tokens):
    """Run the oracle target causally over a prompt; returns per-layer caches and the last argmax."""
    n_h, d_h = cfg.n_heads, cfg.head_dim
    S = len(tokens)
    empty = [np.zeros((n_h, 0, d_h)) for _ in tw["layers"]]
    t = orc.target_forward(tw, np.asarray(tokens), np.arange(S), np.tril(np.ones((S, S), dtype=bool)),
                           empty, empty, n_h, cfg.rms_eps, cfg.rope_theta, keep=True)
    kc = [l["k_new"] for l in t["layers"]]
    vc = [l["v_new"] for l in t["layers"]]
    return kc, vc, t


def greedy_continuation(cfg, tw, prompt, n):
    """The target's own autoregressive greedy decoding: one token at a time, full recompute."""
    toks = list(prompt)
    for _ in range(n):
        _, _, t = target_prefill(cfg, tw, toks)
        toks.append(int(t["tgt"][-1]))
    return toks[len(prompt):]


def test_planted_argmax_is_accepted_to_exactly_the_planted_depth():
    """Plant the target's own argmax along one path depth by depth; a node's logits depend only on
    its ancestors, so planting depth m never changes shallower decisions."""
    cfg, dw, tw = tiny_setup()
    rng = np.random.default_rng(7)
    prompt = rng.integers(0, cfg.vocab, size=cfg.kv_len + 1)
    kc, vc, _ = target_prefill(cfg, tw, prompt[:-1])
    tree = orc.tree_from_paths(si.tree_paths(16, (4, 2, 2, 2)), 4)
    leaf_path = [int(n) for n in tree.retrieve[np.argmax((tree.retrieve >= 0).sum(axis=1))] if n >= 0]
    assert len(leaf_path) == 5
    L = cfg.kv_len
    tok = np.full(16, -1, dtype=np.int32)           # -1 never equals an argmax
    tok[0] = prompt[-1]
    pos = L + tree.depth
    for m in range(1, 5):
        t = orc.target_forward(tw, np.where(tok < 0, 0, tok), pos, tree.mask, kc, vc, cfg.n_heads, cfg.rms_eps, cfg.rope_theta)
        a, path, nxt, best = orc.accept_greedy(tree, tok, t["tgt"])
        assert a == m - 1 and best == leaf_path[m - 1]
        tok[leaf_path[m]] = t["tgt"][leaf_path[m - 1]]
    t = orc.target_forward(tw, np.where(tok < 0, 0, tok), pos, tree.mask, kc, vc, cfg.n_heads, cfg.rms_eps, cfg.rope_theta)
    a, path, nxt, best = orc.accept_greedy(tree, tok, t["tgt"])
    assert a == 4 and list(path) == leaf_path
    # a wrong token at depth 3 cuts the accepted prefix to 2
    tok2 = tok.copy(); tok2[leaf_path[3]] = (tok2[leaf_path[3]] + 1) % cfg.vocab
    t2 = orc.target_forward(tw, np.where(tok2 < 0, 0, tok2), pos, tree.mask, kc, vc, cfg.n_heads, cfg.rms_eps, cfg.rope_theta)
    assert orc.accept_greedy(tree, tok2, t2["tgt"])[0] == 2


def test_step_output_equals_autoregressive_greedy_continuation():
    """Losslessness (Sec. 2 "Speculative Decoding"; Appendix "Case Study"): whatever the draft
    proposes, the a + 1 tokens a step emits are the target's own greedy continuation, and a is the
    length of the longest tree path that agrees with it."""
    cfg, dw, tw = tiny_setup(seed=1)
    rng = np.random.default_rng(8)
    tree = orc.tree_from_paths(si.tree_paths(16, (4, 2, 2, 2)), 4)
    n_h, d_h, L = cfg.n_heads, cfg.head_dim, cfg.kv_len
    hits = 0
    for trial in range(6):
        prompt = rng.integers(0, cfg.vocab, size=L + 1)
        kc, vc, _ = target_prefill(cfg, tw, prompt[:-1])
        ar = greedy_continuation(cfg, tw, prompt, 5)
        # drafts: mix the true continuation into random candidates so that some paths get accepted
        topk = np.stack([rng.permutation(cfg.vocab)[:4] for _ in range(4)]).astype(np.int32)
        for m in range(trial % 5):
            if ar[m] not in topk[m]:
                topk[m][rng.integers(0, 2)] = ar[m]
        tok, pos = orc.tree_tokens(tree, int(prompt[-1]), topk, L)
        t = orc.target_forward(tw, tok, pos, tree.mask, kc, vc, n_h, cfg.rms_eps, cfg.rope_theta)
        a, path, nxt, best = orc.accept_greedy(tree, tok, t["tgt"])
        emitted = [int(tok[n]) for n in path[1:a + 1]] + [nxt]
        assert emitted == ar[:a + 1]
        # a is maximal: no tree path matches a longer prefix of the AR continuation
        longest = 0
        for r in tree.retrieve:
            nodes = [int(n) for n in r if n >= 0][1:]
            m = 0
            while m < len(nodes) and tok[nodes[m]] == ar[m]:
                m += 1
            longest = max(longest, m)
        assert a == longest
        hits += a
    assert hits > 0          # the test exercised at least one accepted draft token


def test_generator_emits_the_autoregressive_greedy_continuation():
    """N steps of the whole loop (draft over the newly committed positions, tree, verification, greedy
    acceptance, commit) emit exactly the target's own greedy tokens, whatever the draft proposes; and the
    committed caches after the loop are the caches of a causal pass over the same tokens."""
    cfg, dw, tw = tiny_setup(seed=2)
    rng = np.random.default_rng(11)
    tree = orc.tree_from_paths(si.tree_paths(16, (4, 2, 2, 2)), 4)
    prompt = [int(t) for t in rng.integers(0, cfg.vocab, size=9)]
    emitted, recs = orc.generate(dw, tw, tree, prompt, 4, cfg.n_heads, 4, cfg.rms_eps, cfg.rope_theta)
    assert len(emitted) == sum(r["accept_len"] + 1 for r in recs) >= 4
    assert emitted == greedy_continuation(cfg, tw, prompt, len(emitted))
    # cache bookkeeping: the length grows by a + 1 per step and the adaptation layers see one row per position
    L = len(prompt) - 1
    for r in recs:
        assert r["kv_len"] == L and len(r["toks"]) == len(r["h_rows"])
        L += r["accept_len"] + 1
    # the first step's draft saw positions 0..P-2 with the tokens that follow them
    assert recs[0]["toks"] == prompt[1:]


def test_draft_catchup_is_the_single_position_draft_repeated():
    cfg, dw, tw = tiny_setup(seed=3)
    rng = np.random.default_rng(5)
    n_h, d_h, d = cfg.n_heads, cfg.head_dim, cfg.d_model
    sal_k = [rng.standard_normal((n_h, 5, d_h)) for _ in range(2)]
    sal_v = [rng.standard_normal((n_h, 5, d_h)) for _ in range(2)]
    hs, toks = rng.standard_normal((3, d)), [3, 9, 27]
    dl, k3, v3 = orc.draft_catchup(dw, hs, toks, sal_k, sal_v, n_h, 4, cfg.rms_eps, cfg.rope_theta)
    # by hand: two single-position drafts to grow the caches, then the third gives the heads
    k, v = [x.copy() for x in sal_k], [x.copy() for x in sal_v]
    for j in range(2):
        dj = orc.draft(dw, hs[j], toks[j], k, v, n_h, 4, cfg.rms_eps, cfg.rope_theta)
        k = [np.concatenate([k[s], dj["k_new"][s][:, None]], axis=1) for s in range(2)]
        v = [np.concatenate([v[s], dj["v_new"][s][:, None]], axis=1) for s in range(2)]
    d3 = orc.draft(dw, hs[2], toks[2], k, v, n_h, 4, cfg.rms_eps, cfg.rope_theta)
    assert np.array_equal(dl["topk_idx"], d3["topk_idx"]) and np.allclose(dl["logits"], d3["logits"], rtol=0, atol=1e-12)
    assert all(k3[s].shape[1] == 8 for s in range(2))
    # the order of the positions matters (each row attends to the earlier ones)
    dr, _, _ = orc.draft_catchup(dw, hs[::-1], toks[::-1], sal_k, sal_v, n_h, 4, cfg.rms_eps, cfg.rope_theta)
    assert not np.allclose(dr["logits"], dl["logits"])


def test_catchup_with_one_adaptation_layer_equals_a_causal_recompute():
    """The variant with a single adaptation layer (Sec. 4.3) through the catch-up over several new positions: the
    incremental result (one position at a time, each appending a cache row) must equal the textbook recompute, i.e.
    the same decoder layer applied to all new rows at once under a causal mask on top of the committed cache; the
    heads then read the last row, every head the first (only) stage's output."""
    cfg, dw, tw = tiny_setup(seed=6)
    one = {**dw, "sal": dw["sal"][:1], "fc": dw["fc"][:1]}
    rng = np.random.default_rng(15)
    n_h, d_h, d, K = cfg.n_heads, cfg.head_dim, cfg.d_model, 4
    sal_k, sal_v = [rng.standard_normal((n_h, 5, d_h))], [rng.standard_normal((n_h, 5, d_h))]
    hs, toks = rng.standard_normal((3, d)), [3, 9, 27]
    dl, k3, v3 = orc.draft_catchup(one, hs, toks, sal_k, sal_v, n_h, 4, cfg.rms_eps, cfg.rope_theta)
    assert len(k3) == 1 and len(v3) == 1 and k3[0].shape[1] == 8 and len(dl["h"]) == 1
    x_rows = np.stack([orc.fc_concat(one["fc"][0], hs[j], one["embed"][toks[j]]) for j in range(3)])
    h_rows, k_new, v_new, _, _ = orc.decoder_layer_rows(x_rows, one["sal"][0], sal_k[0], sal_v[0], [5, 6, 7],
                                                        np.tril(np.ones((3, 3), dtype=bool)), n_h, cfg.rms_eps, cfg.rope_theta)
    assert np.allclose(dl["h"][0], h_rows[2], rtol=0, atol=1e-10)
    assert np.allclose(k3[0][:, 5:], k_new, rtol=0, atol=1e-10) and np.allclose(v3[0][:, 5:], v_new, rtol=0, atol=1e-10)
    for k in range(K):
        assert np.allclose(dl["Hp"][k], orc.head_mlp(one["mlp"][k], h_rows[2]) + one["pe"][k], rtol=0, atol=1e-9)
    # the two-stage model's first stage is the same computation: its first-stage rows agree with the one-stage run
    two_k = [sal_k[0], rng.standard_normal((n_h, 5, d_h))]
    two_v = [sal_v[0], rng.standard_normal((n_h, 5, d_h))]
    d2, k2, _ = orc.draft_catchup(dw, hs, toks, two_k, two_v, n_h, 4, cfg.rms_eps, cfg.rope_theta)
    assert len(k2) == 2 and np.array_equal(k2[0], k3[0]) and np.array_equal(d2["h"][0], dl["h"][0])
    # and the generator runs with one stage (it keeps one adaptation-layer cache per stage of the weights)
    tree = orc.tree_from_paths(si.tree_paths(16, (4, 2, 2, 2)), 4)
    emitted, recs = orc.generate(one, tw, tree, [5, 17, 3, 44], 3, n_h, 4, cfg.rms_eps, cfg.rope_theta)
    want, _ = orc.generate(dw, tw, tree, [5, 17, 3, 44], 6, n_h, 4, cfg.rms_eps, cfg.rope_theta)
    n = min(len(emitted), len(want))
    assert n >= 3 and emitted[:n] == want[:n]          # both emit the target's own greedy continuation


def test_commit_rows_keeps_the_path_in_order():
    old = np.arange(2 * 3 * 4, dtype=float).reshape(2, 3, 4)
    new = 100 + np.arange(2 * 6 * 4, dtype=float).reshape(2, 6, 4)
    out = orc.commit_rows(old, new, [0, 2, 5])
    assert out.shape == (2, 6, 4)
    assert np.array_equal(out[:, :3], old) and np.array_equal(out[:, 3], new[:, 0])
    assert np.array_equal(out[:, 4], new[:, 2]) and np.array_equal(out[:, 5], new[:, 5])


def test_structural_variants_of_the_draft_reduce_to_known_cases():
    """The ablation variants (Sec. 4.3; Appendix) are switches on the same formulas; each is pinned to a case whose
    answer is known without running the variant's own code path."""
    cfg, dw, tw = tiny_setup(seed=4)
    rng = np.random.default_rng(12)
    n_h, d_h, d, K = cfg.n_heads, cfg.head_dim, cfg.d_model, 4
    sal_k = [rng.standard_normal((n_h, 6, d_h)) for _ in range(2)]
    sal_v = [rng.standard_normal((n_h, 6, d_h)) for _ in range(2)]
    h, tok = rng.standard_normal(d), 5
    run = lambda w: orc.draft(w, h, tok, sal_k, sal_v, n_h, 4, cfg.rms_eps, cfg.rope_theta)
    base = run(dw)
    # no position encoding == a zero position encoding
    a = run({**dw, "pe": None}); b = run({**dw, "pe": np.zeros_like(dw["pe"])})
    assert np.array_equal(a["logits"], b["logits"]) and not np.allclose(a["logits"], base["logits"])
    # one adaptation layer: the first stage is the full model's first stage, and every head reads its output
    one = run({**dw, "sal": dw["sal"][:1], "fc": dw["fc"][:1]})
    assert np.array_equal(one["h"][0], base["h"][0]) and len(one["h"]) == 1
    for k in range(K):
        want = orc.head_mlp(dw["mlp"][k], base["h"][0]) + dw["pe"][k]
        assert np.allclose(one["Hp"][k], want, rtol=0, atol=1e-12)
    # second self-attention layer with Wq = Wk = 0 (uniform attention) and Wv = Wo = I: every row becomes the mean
    I, Z = np.eye(d), np.zeros((d, d))
    al = run({**dw, "aeb2_wq": Z, "aeb2_wk": Z, "aeb2_wv": I, "aeb2_wo": I})
    assert np.allclose(al["attn_o"], np.broadcast_to(base["attn_o"].mean(axis=0), (K, d)), rtol=0, atol=1e-12)
    # low-rank head: with r = d and lm_a = I it is the full head; in general it is the head lm_b @ lm_a
    lo = run({**dw, "lm_a": I, "lm_b": dw["lm_head"]})
    assert np.allclose(lo["logits"], base["logits"], rtol=0, atol=1e-10)
    A, Bm = rng.standard_normal((8, d)), rng.standard_normal((cfg.vocab, 8))
    lo = run({**dw, "lm_a": A, "lm_b": Bm}); full = run({**dw, "lm_head": Bm @ A})
    assert np.allclose(lo["logits"], full["logits"], rtol=0, atol=1e-9)


def test_draft_step_shapes_and_cache_rows():
    cfg, dw, tw = tiny_setup(seed=2)
    rng = np.random.default_rng(9)
    n_h, d_h, Ls = cfg.n_heads, cfg.head_dim, 5
    sal_k = [rng.standard_normal((n_h, Ls, d_h)) for _ in range(2)]
    sal_v = [rng.standard_normal((n_h, Ls, d_h)) for _ in range(2)]
    h = rng.standard_normal(cfg.d_model)
    out = orc.draft(dw, h, 3, sal_k, sal_v, n_h, 4, cfg.rms_eps, cfg.rope_theta)
    assert out["logits"].shape == (4, cfg.vocab) and out["topk_idx"].shape == (4, 4)
    # stage 2 consumes stage 1's output and the same token embedding (Eq. 1)
    x2 = orc.fc_concat(dw["fc"][1], out["h"][0], dw["embed"][3])
    np.testing.assert_allclose(out["x"][1], x2, rtol=1e-13)
    # each row's top-k comes from the shared head applied to that row of attn_o (Eq. 6)
    for k in range(4):
        full = dw["lm_head"].astype(np.float64) @ out["attn_o"][k]
        assert list(out["topk_idx"][k]) == list(np.argsort(-full, kind="stable")[:4])


# ---------------------------------------------------------------------------- independent library pin
def test_target_forward_matches_huggingface_llama_with_tree_mask():
    """The whole Llama-style reading (pre-RMSNorm, half-split RoPE, SwiGLU, residuals, final norm, LM
    head, 1/sqrt(d_h) scaling) against transformers' LlamaForCausalLM in float64 with the same weights,
    fed [prompt ; tree tokens] with position ids L + depth and a 4-D mask = causal prompt + tree mask."""
    transformers = pytest.importorskip("transformers")
    from transformers import LlamaConfig, LlamaForCausalLM
    cfg, dw, tw = tiny_setup(seed=3)
    rng = np.random.default_rng(10)
    L, T = cfg.kv_len, 16
    hf_cfg = LlamaConfig(vocab_size=cfg.vocab, hidden_size=cfg.d_model, intermediate_size=cfg.d_ffn,
                         num_hidden_layers=len(tw["layers"]), num_attention_heads=cfg.n_heads,
                         num_key_value_heads=cfg.n_heads, rms_norm_eps=cfg.rms_eps, rope_theta=cfg.rope_theta,
                         max_position_embeddings=512, attention_bias=False, mlp_bias=False,
                         tie_word_embeddings=False, attn_implementation="eager")
    try:
        model = LlamaForCausalLM(hf_cfg).to(torch.float64).eval()
    except Exception as e:  # pragma: no cover
        pytest.skip(f"transformers could not build the model: {e}")
    sd = {"model.embed_tokens.weight": tw["embed"], "model.norm.weight": tw["final_norm"], "lm_head.weight": tw["lm_head"]}
    names = dict(rms1="input_layernorm", rms2="post_attention_layernorm", wq="self_attn.q_proj", wk="self_attn.k_proj",
                 wv="self_attn.v_proj", wo="self_attn.o_proj", w_gate="mlp.gate_proj", w_up="mlp.up_proj", w_down="mlp.down_proj")
    for i, lw in enumerate(tw["layers"]):
        for k, v in lw.items():
            sd[f"model.layers.{i}.{names[k]}.weight"] = v
    missing, unexpected = model.load_state_dict({k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in sd.items()}, strict=False)
    assert not [m for m in missing if "rotary" not in m] and not unexpected
    prompt = rng.integers(0, cfg.vocab, size=L + 1)
    tree = orc.tree_from_paths(si.tree_paths(T, (4, 2, 2, 2)), 4)
    topk = np.stack([rng.permutation(cfg.vocab)[:4] for _ in range(4)]).astype(np.int32)
    tok, pos = orc.tree_tokens(tree, int(prompt[-1]), topk, L)
    kc, vc, pre = target_prefill(cfg, tw, prompt[:-1])
    got = orc.target_forward(tw, tok, pos, tree.mask, kc, vc, cfg.n_heads, cfg.rms_eps, cfg.rope_theta)

    ids = torch.from_numpy(np.concatenate([prompt[:-1], tok]).astype(np.int64))[None]
    position_ids = torch.from_numpy(np.concatenate([np.arange(L), pos]).astype(np.int64))[None]
    allow = np.zeros((L + T, L + T), dtype=bool)
    allow[:L, :L] = np.tril(np.ones((L, L), dtype=bool))
    allow[L:, :L] = True
    allow[L:, L:] = tree.mask
    add = torch.zeros((1, 1, L + T, L + T), dtype=torch.float64)
    add[0, 0][~torch.from_numpy(allow)] = torch.finfo(torch.float64).min
    with torch.no_grad():
        ref = model(input_ids=ids, attention_mask=add, position_ids=position_ids).logits[0].numpy()
    # the library builds its rotary cos/sin tables in float32 whatever the model dtype, so agreement
    # stops near 1e-6; any error of convention (pairing, sign, scaling, residual order) is of order 1
    np.testing.assert_allclose(pre["logits"], ref[:L], rtol=1e-4, atol=2e-5)
    np.testing.assert_allclose(got["logits"], ref[L:], rtol=1e-4, atol=2e-5)
    assert np.abs(ref).max() > 1.0
