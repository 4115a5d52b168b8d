"""GPU parity of the loop around the step: amph_commit, amph_draft over several new positions, and the
whole generator (draft -> tree -> target -> accept -> commit, repeated) against the oracle's generator
and the target's autoregressive greedy decoding."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import amphista_oracle as orc
from paper_2406_13170_amd import binding as B
from paper_2406_13170_amd import device as D

from gpu_common import (DEV, TOL, assert_rows_close, cfg_tensor_to_dev, draft_f32, f32_to_dev, i32_to_dev, make_ctx, np_of,
                        say, topk_consistent)

pytestmark = pytest.mark.gpu


# ---------------------------------------------------------------------------- amph_commit
@pytest.mark.parametrize("cfg,T,caps,L,B_", [(si.TINY, 16, (4, 2, 2, 2), 21, 1), (si.MINI, 64, (10,) * 4, 77, 2)])
def test_commit_moves_the_accepted_rows_and_gathers_the_next_draft_inputs(cfg, T, caps, L, B_):
    say(f"commit {cfg.name} T={T} L={L} B={B_}")
    K = len(caps)
    cfgx = si.with_(cfg, batch=B_, K=K, topk=min(16, max(caps)))
    n_h, d_h, d = cfg.n_heads, cfg.head_dim, cfg.d_model
    n_layers = 2
    max_kv = (L + T + 31) // 32 * 32
    ctx = make_ctx(cfgx, T=T, batch=B_, max_kv=max_kv)
    paths = si.tree_paths(T, caps)
    tree = B.Tree(paths, K)
    otree = orc.tree_from_paths(paths, K)
    tdt = D.torch_dtype(cfg.dtype)
    rows_k = [si.normal(cfgx, 5, f"cm{li}.k", (B_, n_h, L + T, d_h), 1.0) for li in range(n_layers)]
    rows_v = [si.normal(cfgx, 5, f"cm{li}.v", (B_, n_h, L + T, d_h), 1.0) for li in range(n_layers)]
    kr = torch.zeros((n_layers, B_, n_h, max_kv, d_h), dtype=tdt, device=DEV)
    vr = torch.zeros_like(kr)
    for li in range(n_layers):
        kr[li, :, :, :L + T] = cfg_tensor_to_dev(rows_k[li])
        vr[li, :, :, :L + T] = cfg_tensor_to_dev(rows_v[li])
    k_caches, v_caches = D.pack_kv(ctx, kr, vr)
    # one accepted path per batch element: a whole leaf path, and a short one
    full = [[int(n) for n in r if n >= 0] for r in otree.retrieve]
    chosen = [max(full, key=len), min(full, key=len)][:B_]
    a = [len(p) - 1 - (b % 2) for b, p in enumerate(chosen)]               # second element: one node short of its leaf
    path = np.full((B_, K + 1), -1, dtype=np.int32)
    for b, p in enumerate(chosen):
        path[b, :a[b] + 1] = p[:a[b] + 1]
    hidden = si.as_f32_exact(cfgx, 5, "cm.hidden", (B_, T, d), 1.0)
    tree_tok = si.tokens(cfgx, 5, "cm.tok", (B_, T))
    nxt = si.tokens(cfgx, 5, "cm.nxt", (B_,))
    kv_len = i32_to_dev(np.full(B_, L))
    h_new = torch.full((B_, K + 1, d), float("nan"), dtype=torch.float32, device=DEV)
    tok_new = torch.full((B_, K + 1), -5, dtype=torch.int32, device=DEV)
    n_new = torch.full((B_,), -5, dtype=torch.int32, device=DEV)
    ctx.amph_commit(tree, n_layers, k_caches, v_caches, kv_len, i32_to_dev(a), i32_to_dev(path), i32_to_dev(nxt),
                    i32_to_dev(tree_tok), f32_to_dev(hidden), h_new, tok_new, n_new)
    torch.cuda.synchronize()
    assert ctx.device_status() == 0
    assert list(np_of(kv_len)) == [L + x + 1 for x in a] and list(np_of(n_new)) == [x + 1 for x in a]
    kg, vg = D.unpack_kv(ctx, k_caches, v_caches)
    for b in range(B_):
        nodes = [int(n) for n in path[b, :a[b] + 1]]
        for li in range(n_layers):
            for got, rows in ((kg, rows_k), (vg, rows_v)):
                ref = orc.commit_rows(rows[li].f32[b][:, :L], rows[li].f32[b][:, L:], nodes)
                assert np.array_equal(np_of(got[li, b, :, :L + a[b] + 1]).astype(np.float64), ref)     # data movement: exact
        assert np.array_equal(np_of(h_new[b, :a[b] + 1]), hidden[b][nodes])
        assert np.all(np_of(h_new[b, a[b] + 1:]) == 0.0)
        want_tok = [int(tree_tok[b][n]) for n in nodes[1:]] + [int(nxt[b])]
        assert list(np_of(tok_new[b, :a[b] + 1])) == want_tok


# ---------------------------------------------------------------------------- amph_draft over several new positions
# five concatenated [h ; e] rows of this width do not fit in LDS as float32: Eq. 1's product then runs as two launches
# over half the columns each
WIDE_FC = si.with_(si.MINI, name="mini_wide_fc", d_model=3584, n_heads=28, d_ffn=512, vocab=512)
# five rows of this FFN width do not fit in LDS either: W_down's product runs as launches over slices of its columns
WIDE_FFN = si.with_(si.MINI, name="mini_wide_ffn", d_ffn=8192)


@pytest.mark.parametrize("cfg,n_rows,n_live", [(si.TINY, 5, 5), (si.TINY, 5, 2), (si.MINI, 5, 3), (si.MINI, 3, 1),
                                               (WIDE_FC, 5, 4), (WIDE_FFN, 5, 5)])
def test_draft_catches_up_over_new_positions(cfg, n_rows, n_live):
    """h_new carries n_rows positions of which the first n_live count (n_valid on the device)."""
    say(f"draft catch-up {cfg.name} rows={n_rows} live={n_live}")
    seed = 9
    Ls = 37
    n_h, d_h, d, V, K = cfg.n_heads, cfg.head_dim, cfg.d_model, cfg.vocab, cfg.K
    max_kv = (Ls + n_rows + 31) // 32 * 32
    ctx = make_ctx(cfg, max_kv=max_kv)
    dw = si.draft_weights(cfg, seed)
    dwd = D.draft_to_device(dw, DEV)
    dstruct = B.Context.draft_struct(dwd)
    hs = si.as_f32_exact(cfg, seed, "cu.h", (1, n_rows, d), 1.0)
    toks = si.tokens(cfg, seed, "cu.tok", (1, n_rows))
    tdt = D.torch_dtype(cfg.dtype)
    sal_k = [si.normal(cfg, seed, f"sal{s}.k", (1, n_h, Ls, d_h), 1.0) for s in range(2)]
    sal_v = [si.normal(cfg, seed, f"sal{s}.v", (1, n_h, Ls, d_h), 1.0) for s in range(2)]
    sal_kv = torch.full((2, 1, 2, n_h, max_kv, d_h), float("nan"), dtype=tdt, device=DEV)
    for s in range(2):
        sal_kv[s, :, 0, :, :Ls] = cfg_tensor_to_dev(sal_k[s])
        sal_kv[s, :, 1, :, :Ls] = cfg_tensor_to_dev(sal_v[s])
    sal_len = i32_to_dev([Ls])
    topk_idx = torch.full((1, K, cfg.topk), -7, dtype=torch.int32, device=DEV)
    topk_val = torch.full((1, K, cfg.topk), float("nan"), dtype=torch.float32, device=DEV)
    logits = torch.full((1, K, V), float("nan"), dtype=torch.float32, device=DEV)
    ctx.amph_draft(dstruct, f32_to_dev(hs), i32_to_dev(toks), sal_kv, sal_len, topk_idx, topk_val, logits, n_new=n_rows,
                   n_valid=i32_to_dev([n_live]))
    torch.cuda.synchronize()
    assert ctx.device_status() == 0
    assert int(np_of(sal_len)[0]) == Ls + n_live
    o, ok_, ov_ = orc.draft_catchup(draft_f32(dw), hs[0][:n_live], toks[0][:n_live], [k.f32[0] for k in sal_k],
                                    [v.f32[0] for v in sal_v], n_h, cfg.topk, cfg.rms_eps, cfg.rope_theta)
    tol = TOL[cfg.dtype]
    assert_rows_close(np_of(logits)[0], o["logits"], tol, "catch-up logits")
    for k in range(K):
        good, bad = topk_consistent(np_of(topk_idx)[0, k], o["logits"][k], cfg.topk, tol * np.abs(o["logits"][k]).max())
        assert good, f"head {k}: ranks {bad}"
    for s in range(2):
        got_k = np_of(sal_kv[s, 0, 0, :, Ls:Ls + n_live]); got_v = np_of(sal_kv[s, 0, 1, :, Ls:Ls + n_live])
        assert_rows_close(got_k, ok_[s][:, Ls:], tol, f"stage {s} new keys")
        assert_rows_close(got_v, ov_[s][:, Ls:], tol, f"stage {s} new values")
        assert torch.isnan(sal_kv[s, 0, :, :, Ls + n_live:].float()).all(), "rows of ignored positions must stay untouched"


# ---------------------------------------------------------------------------- the generator
def generator_weights():
    """Weights scaled so that decisions have margins and a vocabulary of 8 tokens (top-4 candidates per head) so that
    an untrained draft is accepted by chance.  Returns (cfg, draft weights, target weights) as float arrays."""
    cfg = si.with_(si.TINY, kv_len=5, sal_len=0, vocab=8)
    seed, scale = 8, 6.0
    f = lambda t: (t.f32 * np.float32(scale)).astype(np.float32)
    dw_t, tw_t = si.draft_weights(cfg, seed), si.target_weights(cfg, seed)
    conv = lambda lw: {k: (f(v) if k.startswith("w") else v.f32) for k, v in lw.items()}
    dw = dict(embed=f(dw_t["embed"]), fc=[f(x) for x in dw_t["fc"]], sal=[conv(l) for l in dw_t["sal"]], mlp=f(dw_t["mlp"]),
              pe=dw_t["pe"].f32, aeb_wq=f(dw_t["aeb_wq"]), aeb_wk=f(dw_t["aeb_wk"]), aeb_wv=f(dw_t["aeb_wv"]),
              aeb_wo=f(dw_t["aeb_wo"]), lm_head=f(dw_t["lm_head"]))
    tw = dict(embed=dw["embed"], layers=[conv(l) for l in tw_t["layers"]], final_norm=tw_t["final_norm"].f32,
              lm_head=f(tw_t["lm_head"]))
    return cfg, dw, tw


def generator_state(n_steps_max=8, prompts=None, one_stage=False):
    """The device state after the prompts (one per batch element, 2 .. K + 2 tokens each, lengths may differ): the
    target's caches from the oracle's causal pass over each prompt, empty adaptation-layer caches, the inputs of the
    first draft (each element's prompt positions, n_new = its count).  one_stage: the variant with a single
    adaptation layer."""
    cfg, dw, tw = generator_weights()
    if one_stage:
        dw = {**dw, "sal": dw["sal"][:1], "fc": dw["fc"][:1]}
    n_h, d_h, d, V, K, T = cfg.n_heads, cfg.head_dim, cfg.d_model, cfg.vocab, cfg.K, cfg.T
    paths = si.tree_paths(T, cfg.tree_caps)
    otree = orc.tree_from_paths(paths, K)
    if prompts is None:
        rng = np.random.default_rng(3)
        prompts = [[int(t) for t in rng.integers(0, V, size=K + 2)]]      # K + 1 prompt positions feed the first draft
    Bn = len(prompts)
    Ps = [len(p) - 1 for p in prompts]
    assert all(1 <= P <= K + 1 for P in Ps)
    n_layers = len(tw["layers"])
    max_kv = (max(Ps) + n_steps_max * (K + 1) + T + 31) // 32 * 32
    # ---- device state: weights, the prompt's target caches (from the oracle's causal pass), empty adaptation-layer caches
    ctx = make_ctx(cfg, max_kv=max_kv, batch=Bn, **({"n_stages": 1} if one_stage else {}))
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)
    lay = lambda lw: {k: to(v) for k, v in lw.items()}
    dwd = dict(embed=to(dw["embed"]), fc=[to(x) for x in dw["fc"]], sal=[lay(l) for l in dw["sal"]], mlp=to(dw["mlp"]),
               pe=to(dw["pe"]), aeb_wq=to(dw["aeb_wq"]), aeb_wk=to(dw["aeb_wk"]), aeb_wv=to(dw["aeb_wv"]), aeb_wo=to(dw["aeb_wo"]),
               lm_head=to(dw["lm_head"]))
    dstruct = B.Context.draft_struct(dwd)
    layers_d = [lay(l) for l in tw["layers"]]
    structs = [B.Context.layer_struct(l) for l in layers_d]
    fn_d, lm_d = to(tw["final_norm"]), to(tw["lm_head"])
    tree = B.Tree(paths, K)
    kr = torch.zeros((n_layers, Bn, n_h, max_kv, d_h), dtype=torch.float32, device=DEV)
    vr = torch.zeros_like(kr)
    i32 = lambda *shape: torch.zeros(shape, dtype=torch.int32, device=DEV)
    h_new = torch.zeros((Bn, K + 1, d), dtype=torch.float32, device=DEV)
    tok_new = i32(Bn, K + 1)
    for b, prompt in enumerate(prompts):
        P = Ps[b]
        pre = orc.target_forward(tw, np.asarray(prompt[:-1]), np.arange(P), np.tril(np.ones((P, P), dtype=bool)),
                                 [np.zeros((n_h, 0, d_h))] * n_layers, [np.zeros((n_h, 0, d_h))] * n_layers, n_h, cfg.rms_eps,
                                 cfg.rope_theta, keep=True)
        for li in range(n_layers):
            kr[li, b, :, :P] = to(pre["layers"][li]["k_new"])
            vr[li, b, :, :P] = to(pre["layers"][li]["v_new"])
        h_new[b, :P] = to(pre["hidden"])
        tok_new[b, :P] = i32_to_dev(prompt[1:])
    k_caches, v_caches = D.pack_kv(ctx, kr, vr)
    sal_kv = torch.zeros((2, Bn, 2, n_h, max_kv, d_h), dtype=torch.float32, device=DEV)
    kv_len, sal_len = i32_to_dev(Ps), i32_to_dev([0] * Bn)
    n_new, root = i32_to_dev(Ps), i32_to_dev([p[-1] for p in prompts])
    topk_idx, topk_val = i32(Bn, K, cfg.topk), torch.zeros((Bn, K, cfg.topk), dtype=torch.float32, device=DEV)
    tree_tok, tree_pos, tgt = i32(Bn, T), i32(Bn, T), i32(Bn, T)
    hidden = torch.zeros((Bn, T, d), dtype=torch.float32, device=DEV)
    a_len, a_path, nxt, best = i32(Bn), i32(Bn, K + 1), i32(Bn), i32(Bn)
    return dict(cfg=cfg, dw=dw, tw=tw, otree=otree, prompt=prompts[0], prompts=prompts, P=Ps[0], n_layers=n_layers, ctx=ctx,
                dstruct=dstruct, dwd=dwd,
                structs=structs, fn_d=fn_d, lm_d=lm_d, tree=tree, k_caches=k_caches, v_caches=v_caches, sal_kv=sal_kv,
                kv_len=kv_len, sal_len=sal_len, h_new=h_new, tok_new=tok_new, n_new=n_new, root=root, topk_idx=topk_idx,
                topk_val=topk_val, tree_tok=tree_tok, tree_pos=tree_pos, tgt=tgt, hidden=hidden, a_len=a_len, a_path=a_path,
                nxt=nxt, best=best)


def run_device_generator(st, recs_per_seq, n_steps):
    """n_steps of the device loop for every sequence of the batch at once, each step compared with that sequence's
    oracle generator record.  Returns the tokens each sequence emitted."""
    cfg, n_layers = st["cfg"], st["n_layers"]
    K = cfg.K
    ctx, dstruct, dwd, structs, fn_d, lm_d, tree = st["ctx"], st["dstruct"], st["dwd"], st["structs"], st["fn_d"], st["lm_d"], st["tree"]
    k_caches, v_caches, sal_kv, kv_len, sal_len = st["k_caches"], st["v_caches"], st["sal_kv"], st["kv_len"], st["sal_len"]
    h_new, tok_new, n_new, root = st["h_new"], st["tok_new"], st["n_new"], st["root"]
    topk_idx, topk_val, tree_tok, tree_pos, tgt, hidden = st["topk_idx"], st["topk_val"], st["tree_tok"], st["tree_pos"], st["tgt"], st["hidden"]
    a_len, a_path, nxt, best = st["a_len"], st["a_path"], st["nxt"], st["best"]
    Bn = len(recs_per_seq)
    got = [[] for _ in range(Bn)]
    for step in range(n_steps):
        ctx.amph_draft(dstruct, h_new, tok_new, sal_kv, sal_len, topk_idx, topk_val, None, n_new=K + 1, n_valid=n_new)
        ctx.amph_tree_build(tree, root, topk_idx, kv_len, tree_tok, tree_pos)
        ctx.amph_target_forward(tree, structs, dwd["embed"], fn_d, lm_d, tree_tok, tree_pos, k_caches, v_caches, kv_len, hidden,
                                None, tgt)
        ctx.amph_accept(tree, tree_tok, tgt, None, a_len, a_path, nxt, best)
        tt, al, ap, nx = np_of(tree_tok), np_of(a_len), np_of(a_path), np_of(nxt)            # before the commit
        ctx.amph_commit(tree, n_layers, k_caches, v_caches, kv_len, a_len, a_path, nxt, tree_tok, hidden, h_new, tok_new, n_new)
        root.copy_(nxt)
        torch.cuda.synchronize()
        assert ctx.device_status() == 0
        for b in range(Bn):
            r = recs_per_seq[b][step]
            assert np.array_equal(tt[b], r["tree_tok"]), f"step {step} sequence {b}: tree tokens differ from the oracle's"
            a = int(al[b])
            assert a == r["accept_len"] and int(nx[b]) == r["next_tok"] and list(ap[b, :a + 1]) == r["nodes"], f"step {step} sequence {b}"
            # the target's caches are committed; the adaptation layers have seen the positions before this step
            assert int(np_of(kv_len)[b]) == r["kv_len"] + a + 1 and int(np_of(sal_len)[b]) == r["kv_len"]
            got[b] += [int(tt[b][n]) for n in r["nodes"][1:]] + [int(nx[b])]
        say(f"  step {step}: accepted {[int(x) for x in al]}")
    return got


def test_generator_matches_oracle_and_autoregressive_greedy():
    """Eight steps of the whole loop on the device, float32 configuration.  The draft module is untrained,
    so the vocabulary is cut to 8 tokens (top-4 candidates per head) to make acceptances happen by chance:
    with this seed the oracle's generator accepts 1, 0, 0, 1, 1, 1, 2, 1 draft tokens, and every decision
    of the target and every top-4 boundary of the draft has a margin above 2e-2 (float32 error: ~1e-5).
    Every step's tree, accepted path and next token must equal the oracle generator's, and the emitted
    tokens are the target's own greedy continuation."""
    say("generator tiny (vocabulary 8), 8 steps")
    n_steps = 8
    st = generator_state(n_steps)
    cfg, dw, tw, otree, prompt, P, n_layers = st["cfg"], st["dw"], st["tw"], st["otree"], st["prompt"], st["P"], st["n_layers"]
    n_h, d_h, K, T = cfg.n_heads, cfg.head_dim, cfg.K, cfg.T
    ctx, dstruct, dwd, structs, fn_d, lm_d, tree = st["ctx"], st["dstruct"], st["dwd"], st["structs"], st["fn_d"], st["lm_d"], st["tree"]
    k_caches, v_caches, sal_kv, kv_len, sal_len = st["k_caches"], st["v_caches"], st["sal_kv"], st["kv_len"], st["sal_len"]
    h_new, tok_new, n_new, root = st["h_new"], st["tok_new"], st["n_new"], st["root"]
    topk_idx, topk_val, tree_tok, tree_pos, tgt, hidden = st["topk_idx"], st["topk_val"], st["tree_tok"], st["tree_pos"], st["tgt"], st["hidden"]
    a_len, a_path, nxt, best = st["a_len"], st["a_path"], st["nxt"], st["best"]
    emitted, recs = orc.generate(dw, tw, otree, prompt, n_steps, n_h, cfg.topk, cfg.rms_eps, cfg.rope_theta)
    ar = list(prompt)
    for _ in range(len(emitted)):                                          # autoregressive greedy, full recompute
        S = len(ar)
        t = orc.target_forward(tw, np.asarray(ar), np.arange(S), np.tril(np.ones((S, S), dtype=bool)),
                               [np.zeros((n_h, 0, d_h))] * len(tw["layers"]), [np.zeros((n_h, 0, d_h))] * len(tw["layers"]),
                               n_h, cfg.rms_eps, cfg.rope_theta)
        ar.append(int(t["tgt"][-1]))
    assert emitted == ar[len(prompt):]

    got_emitted = run_device_generator(st, [recs], n_steps)[0]
    assert got_emitted == emitted == ar[len(prompt):]
    assert [r["accept_len"] for r in recs] == [1, 0, 0, 1, 1, 1, 2, 1]


def test_generator_batch_of_three_with_unequal_prompts():
    """The loop at batch 3: prompts of 6, 3 and 4 tokens (5, 2 and 3 positions feed the first draft), so every
    per-sequence length on the device differs, and the catch-up call carries 3 x (K + 1) = 15 adaptation-layer rows
    (two launches of the 8-row kernels).  Every step of every sequence must equal that sequence's own oracle
    generator, which emits the target's greedy continuation of its prompt."""
    say("generator tiny (vocabulary 8), batch 3, unequal prompts, 4 steps")
    n_steps = 4
    prompts = [[5, 1, 7, 2, 6, 3], [4, 4, 0], [2, 7, 1, 5]]
    st = generator_state(n_steps, prompts=prompts)
    cfg, dw, tw, otree = st["cfg"], st["dw"], st["tw"], st["otree"]
    n_h = cfg.n_heads
    recs, emitted = [], []
    for p in prompts:
        e, r = orc.generate(dw, tw, otree, p, n_steps, n_h, cfg.topk, cfg.rms_eps, cfg.rope_theta)
        emitted.append(e); recs.append(r)
    got = run_device_generator(st, recs, n_steps)
    assert got == emitted
    assert any(r["accept_len"] > 0 for rs in recs for r in rs), "the seeded case must exercise an acceptance"


def test_generator_with_one_adaptation_layer():
    """The single-adaptation-layer variant (Sec. 4.3) through commit and catch-up: batch 2, 4 steps, against the oracle's
    generator run on the same one-stage weights."""
    say("generator tiny (vocabulary 8), one adaptation layer, batch 2, 4 steps")
    n_steps = 4
    prompts = [[5, 1, 7, 2, 6, 3], [2, 7, 1, 5]]
    st = generator_state(n_steps, prompts=prompts, one_stage=True)
    cfg, dw, tw, otree = st["cfg"], st["dw"], st["tw"], st["otree"]
    assert len(dw["sal"]) == 1
    recs, emitted = [], []
    for p in prompts:
        e, r = orc.generate(dw, tw, otree, p, n_steps, cfg.n_heads, cfg.topk, cfg.rms_eps, cfg.rope_theta)
        emitted.append(e); recs.append(r)
    got = run_device_generator(st, recs, n_steps)
    assert got == emitted
    assert torch.count_nonzero(st["sal_kv"][1]) == 0, "the second stage's cache must never be touched"
