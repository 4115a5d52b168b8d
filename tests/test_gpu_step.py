"""GPU parity of the composite calls (amph_draft, amph_target_forward) and of a whole
speculate-and-verify step against the CPU oracle, on seeded inputs."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import amphista_oracle as orc
from paper_2406_13170_amd import binding as B
from paper_2406_13170_amd import device as D

import bf16_noise_model as nm
from gpu_common import (DEV, TOL, assert_rows_close, cfg_tensor_to_dev, draft_f32, f32_layers, f32_to_dev, i32_to_dev,
                        make_ctx, np_of, say, topk_consistent)

pytestmark = pytest.mark.gpu


# ---------------------------------------------------------------------------- amph_draft (A1-A5)
def apply_variant(cfg, dw, seed, variant):
    """The ablation variants as changes of the weight dictionary (synth_inputs tensors) + amph_config switches."""
    dw = dict(dw)
    sw = {}
    d, V = cfg.d_model, cfg.vocab
    if variant.get("one_stage"):
        dw["sal"], dw["fc"] = dw["sal"][:1], dw["fc"][:1]
        sw["n_stages"] = 1
    if variant.get("no_pe"):
        dw["pe"] = None
    if variant.get("alpha"):
        for k in ("wq", "wk", "wv", "wo"):
            dw["aeb2_" + k] = si.normal(cfg, seed, "draft.aeb2." + k, (d, d), si.W_STD)
        sw["aeb_layers"] = 2
    if variant.get("lm_rank"):
        r = variant["lm_rank"]
        dw["lm_a"] = si.normal(cfg, seed, "draft.lm_a", (r, d), si.W_STD)
        dw["lm_b"] = si.normal(cfg, seed, "draft.lm_b", (V, r), si.W_STD)
        dw["lm_head"] = None
        sw["lm_rank"] = r
    return dw, sw


def variant_to_device(dw):
    out = {}
    for k, v in dw.items():
        if v is None:
            out[k] = None
        elif k == "sal":
            out[k] = [D.layer_to_device(l, DEV) for l in v]
        elif k == "fc":
            out[k] = [D.to_device(x, DEV) for x in v]
        else:
            out[k] = D.to_device(v, DEV)
    return out


def variant_f32(dw):
    f = lambda t: None if t is None else t.f32
    return {k: ([{kk: vv.f32 for kk, vv in l.items()} for l in v] if k == "sal" else [x.f32 for x in v] if k == "fc" else f(v))
            for k, v in dw.items()}


def run_draft(cfg: si.Config, seed=0, Bsz=1, sal_len=None, variant=None):
    cfg = si.with_(cfg, batch=Bsz)
    Ls = cfg.sal_len if sal_len is None else sal_len
    n_h, d_h, d, V, K = cfg.n_heads, cfg.head_dim, cfg.d_model, cfg.vocab, cfg.K
    max_kv = (max(Ls + 1, cfg.T) + 31) // 32 * 32
    dw = si.draft_weights(cfg, seed)
    sw = {}
    if variant:
        dw, sw = apply_variant(cfg, dw, seed, variant)
    ctx = make_ctx(cfg, batch=Bsz, max_kv=max_kv, **sw)
    dwd = variant_to_device(dw) if variant else D.draft_to_device(dw, DEV)
    dstruct = B.Context.draft_struct(dwd)
    h = si.as_f32_exact(cfg, seed, "draft.h_t", (Bsz, d), 1.0)
    tok = si.tokens(cfg, seed, "draft.tok", (Bsz,))
    tdt = D.torch_dtype(cfg.dtype)
    # committed SAL rows ~ N(0,1); the rest of the cache is NaN so that a stray read shows up
    sal_k = [si.normal(cfg, seed, f"sal{s}.k", (Bsz, n_h, Ls, d_h), 1.0) for s in range(2)]
    sal_v = [si.normal(cfg, seed, f"sal{s}.v", (Bsz, n_h, Ls, d_h), 1.0) for s in range(2)]
    sal_kv = torch.full((2, Bsz, 2, n_h, max_kv, d_h), float("nan"), dtype=tdt, device=DEV)
    for s in range(2):
        sal_kv[s, :, 0, :, :Ls] = cfg_tensor_to_dev(sal_k[s])
        sal_kv[s, :, 1, :, :Ls] = cfg_tensor_to_dev(sal_v[s])
    sal_len_d = i32_to_dev(np.full(Bsz, Ls))
    topk_idx = torch.full((Bsz, K, cfg.topk), -7, dtype=torch.int32, device=DEV)
    topk_val = torch.full((Bsz, K, cfg.topk), float("nan"), dtype=torch.float32, device=DEV)
    logits = torch.full((Bsz, K, V), float("nan"), dtype=torch.float32, device=DEV)
    ctx.amph_draft(dstruct, f32_to_dev(h), i32_to_dev(tok), sal_kv, sal_len_d, topk_idx, topk_val, logits)
    torch.cuda.synchronize()
    assert ctx.device_status() == 0
    dwo = variant_f32(dw) if variant else draft_f32(dw)
    outs = []
    for b in range(Bsz):
        o = orc.draft(dwo, h[b], int(tok[b]), [sal_k[s].f32[b] for s in range(2)], [sal_v[s].f32[b] for s in range(2)],
                      n_h, cfg.topk, cfg.rms_eps, cfg.rope_theta)
        outs.append(o)
    return cfg, ctx, outs, dict(topk_idx=np_of(topk_idx), topk_val=np_of(topk_val), logits=np_of(logits),
                                sal_kv=sal_kv, sal_len=np_of(sal_len_d), Ls=Ls, keep=(dwd, dstruct))


def check_draft(cfg, outs, got, n_stages=2):
    tol = TOL[cfg.dtype]
    Ls = got["Ls"]
    for b, o in enumerate(outs):
        worst = assert_rows_close(got["logits"][b], o["logits"], tol, f"draft logits b={b}")
        say(f"  b={b} worst logit row error {worst:.2e}")
        for k in range(cfg.K):
            tol_abs = tol * np.abs(o["logits"][k]).max()
            ok, bad = topk_consistent(got["topk_idx"][b, k], o["logits"][k], cfg.topk, tol_abs)
            assert ok, f"top-k of head {k}: ranks {bad} disagree beyond the tolerance"
            # returned values are the logits at the returned indices, in descending order
            np.testing.assert_allclose(got["topk_val"][b, k], got["logits"][b, k][got["topk_idx"][b, k]], rtol=0, atol=0)
            assert np.all(np.diff(got["topk_val"][b, k]) <= 0)
        # the new cache rows (keys after RoPE at position Ls, values) of both stages
        for s in range(n_stages):
            kc = np_of(got["sal_kv"][s, b, 0, :, Ls])
            vc = np_of(got["sal_kv"][s, b, 1, :, Ls])
            assert_rows_close(kc, o["k_new"][s], tol, f"SAL{s + 1} new key row")
            assert_rows_close(vc, o["v_new"][s], tol, f"SAL{s + 1} new value row")
        if n_stages == 1:                              # the second stage's cache is never touched
            assert torch.isnan(got["sal_kv"][1, b, :, :, Ls].float()).all()
    assert np.all(got["sal_len"] == Ls + 1)


@pytest.mark.parametrize("cfg,sal_len", [(si.TINY, None), (si.TINY, 0), (si.MINI, None), (si.MINI, 300)])
def test_draft_matches_oracle(cfg, sal_len):
    say(f"draft {cfg.name} sal_len={sal_len}")
    cfgx, ctx, outs, got = run_draft(cfg, sal_len=sal_len)
    check_draft(cfgx, outs, got)


def test_draft_most_heads_and_candidates():
    """K = 8 heads and top-16 candidates: the largest values the library takes (five heads read the second
    stage's state with K = 8; with K odd the extra head does, see the next case)."""
    say("draft mini K=8 top-16")
    cfgx, ctx, outs, got = run_draft(si.with_(si.MINI, K=8, topk=16))
    check_draft(cfgx, outs, got)
    say("draft tiny K=5 (odd: heads 1-2 read the first stage, 3-5 the second)")
    cfgx, ctx, outs, got = run_draft(si.with_(si.TINY, K=5, topk=4))
    check_draft(cfgx, outs, got)
    say("draft tiny K=1")
    cfgx, ctx, outs, got = run_draft(si.with_(si.TINY, K=1, topk=4))
    check_draft(cfgx, outs, got)


@pytest.mark.parametrize("cfg", [si.TINY, si.MINI])
@pytest.mark.parametrize("variant", [dict(one_stage=True), dict(no_pe=True), dict(alpha=True), dict(lm_rank=64),
                                     dict(one_stage=True, no_pe=True, alpha=True, lm_rank=256)],
                         ids=["one-adaptation-layer", "no-position-encoding", "two-attention-layers", "low-rank-head", "all-four"])
def test_draft_structural_variants(cfg, variant):
    """The ablation variants of Sec. 4.3 and the Appendix as configuration switches."""
    say(f"draft {cfg.name} variant {variant}")
    cfgx, ctx, outs, got = run_draft(cfg, variant=variant)
    check_draft(cfgx, outs, got, n_stages=1 if variant.get("one_stage") else 2)


def test_draft_batch_of_two():
    say("draft mini batch=2")
    cfgx, ctx, outs, got = run_draft(si.MINI, Bsz=2)
    check_draft(cfgx, outs, got)


def test_draft_vicuna7b_shape():
    """Configuration 2: the 7B-shaped draft module (d 4096, 32 x 128 heads, V 32000, K 4, top-10, SAL cache 1024)."""
    say("draft vicuna7b")
    cfgx, ctx, outs, got = run_draft(si.V7B)
    check_draft(cfgx, outs, got)
    # the same call again (fresh context and caches): the same bits
    got2 = run_draft(si.V7B)[3]
    assert np.array_equal(got["logits"], got2["logits"]) and np.array_equal(got["topk_idx"], got2["topk_idx"])
    assert np.array_equal(got["topk_val"], got2["topk_val"])


def test_draft_vicuna13b_shape():
    """Configuration 4's draft module (d 5120, 40 x 128 heads, FFN 13824, SAL cache 2048)."""
    say("draft vicuna13b")
    cfgx, ctx, outs, got = run_draft(si.V13B)
    check_draft(cfgx, outs, got)


def test_draft_vicuna33b_shape_batch4():
    """Configuration 5's draft module (d 6656, 52 x 128 heads, FFN 17920, K 5, batch 4, SAL cache 4096): the
    float32 activation rows of a launch no longer fit in LDS for the widest matrices, so fc, W_down and the
    head MLPs run as several launches over row ranges, and the 20 head rows as three groups."""
    say("draft vicuna33b batch 4")
    cfgx, ctx, outs, got = run_draft(si.V33B, Bsz=4)
    check_draft(cfgx, outs, got)


def test_draft_is_deterministic_and_flags_overflow():
    say("draft determinism / overflow")
    cfg = si.TINY
    cfgx, ctx, outs, got1 = run_draft(cfg, seed=3)
    cfgx, ctx2, outs, got2 = run_draft(cfg, seed=3)
    assert np.array_equal(got1["logits"], got2["logits"]) and np.array_equal(got1["topk_idx"], got2["topk_idx"])
    # sal_len at capacity: the call must flag it and leave the cache alone
    dwd, dstruct = got1["keep"]
    max_kv = got1["sal_kv"].shape[4]
    before = got1["sal_kv"].clone()
    full = i32_to_dev([max_kv])
    h = torch.zeros((1, cfg.d_model), dtype=torch.float32, device=DEV)
    tok = i32_to_dev([1])
    idx = torch.zeros((1, cfg.K, cfg.topk), dtype=torch.int32, device=DEV)
    val = torch.zeros((1, cfg.K, cfg.topk), dtype=torch.float32, device=DEV)
    ctx.amph_draft(dstruct, h, tok, got1["sal_kv"], full, idx, val, None)
    assert ctx.device_status() & B.AMPH_DEV_SAL_OVERFLOW
    assert torch.equal(torch.nan_to_num(before.float()), torch.nan_to_num(got1["sal_kv"].float()))


# ---------------------------------------------------------------------------- amph_target_forward (A7-A9)
def run_target(cfg: si.Config, n_layers, T, caps, L, seed=0, Bsz=1, tiled=False, oracle=True, tiled_keys=None, model=False,
               keep_all=False):
    cfg = si.with_(cfg, batch=Bsz, K=len(caps), topk=min(16, max(caps)))
    n_h, d_h, d, V = cfg.n_heads, cfg.head_dim, cfg.d_model, cfg.vocab
    max_kv = (L + T + 31) // 32 * 32
    ctx = make_ctx(cfg, T=T, batch=Bsz, max_kv=max_kv)
    tw = si.target_weights(cfg, seed, n_layers)
    layers_d = [D.layer_to_device(lw, DEV) for lw in tw["layers"]]
    structs = [B.Context.layer_struct(l) for l in layers_d]
    embed_d, fn_d, lm_d = cfg_tensor_to_dev(tw["embed"]), cfg_tensor_to_dev(tw["final_norm"]), cfg_tensor_to_dev(tw["lm_head"])
    paths = si.tree_paths(T, caps)
    tree = B.Tree(paths, cfg.K)
    otree = orc.tree_from_paths(paths, cfg.K)
    tdt = D.torch_dtype(cfg.dtype)
    kcs = [si.normal(cfg, seed, f"tkv{li}.k", (Bsz, n_h, L, d_h), 1.0) for li in range(n_layers)]
    vcs = [si.normal(cfg, seed, f"tkv{li}.v", (Bsz, n_h, L, d_h), 1.0) for li in range(n_layers)]
    k_caches = torch.full((max(n_layers, 1), Bsz, n_h, max_kv, d_h), float("nan"), dtype=tdt, device=DEV)
    v_caches = torch.full((max(n_layers, 1), Bsz, n_h, max_kv, d_h), float("nan"), dtype=tdt, device=DEV)
    for li in range(n_layers):
        k_caches[li, :, :, :L] = cfg_tensor_to_dev(kcs[li])
        v_caches[li, :, :, :L] = cfg_tensor_to_dev(vcs[li])
    k_caches, v_caches = D.pack_kv(ctx, k_caches, v_caches)      # rows -> step-tiled storage
    tok = si.tokens(cfg, seed, "tree.tok", (Bsz, T))
    pos = np.stack([L + otree.depth for _ in range(Bsz)]).astype(np.int32)
    hidden = torch.full((Bsz, T, d), float("nan"), dtype=torch.float32, device=DEV)
    logits = torch.full((Bsz, T, V), float("nan"), dtype=torch.float32, device=DEV)
    tgt = torch.full((Bsz, T), -1, dtype=torch.int32, device=DEV)
    tiled_structs = lm_t = keep = None
    if tiled:
        # tiled copies of every matrix; the row-major pointers are withheld to show that nothing reads them
        packed = [D.pack_layer(ctx, l) for l in layers_d]
        tiled_structs, keep = [p[0] for p in packed], [p[1] for p in packed]
        lm_t = D.pack_lm_head(ctx, lm_d)
        if tiled_keys is None:
            structs = [B.amph_layer_w(rms1=l["rms1"].data_ptr(), rms2=l["rms2"].data_ptr()) for l in layers_d]
        else:
            # only the matrices named in tiled_keys get their tiled copy; the others stay row-major
            for ts in tiled_structs:
                for name in ("qkv", "wo", "gate_up", "down"):
                    if name not in tiled_keys:
                        setattr(ts, name, None)
    ctx.amph_target_forward(tree, structs, embed_d, fn_d, None if tiled else lm_d, i32_to_dev(tok), i32_to_dev(pos),
                            k_caches, v_caches, i32_to_dev(np.full(Bsz, L)), hidden, logits, tgt,
                            tiled_structs=tiled_structs, lm_head_tiled=lm_t)
    torch.cuda.synchronize()
    assert ctx.device_status() == 0
    dev = dict(structs=structs, tiled_structs=tiled_structs, lm_t=lm_t, embed_d=embed_d, fn_d=fn_d, lm_d=None if tiled else lm_d,
               keep=(keep, layers_d))       # what a further pass on the same weights needs (kept alive with the result)
    if not oracle:
        return cfg, None, dict(hidden=np_of(hidden), logits=np_of(logits), tgt=np_of(tgt), k_caches=k_caches,
                               v_caches=v_caches, L=L, T=T, ctx=ctx, dev=dev), (ctx, tree, otree)
    two = dict(embed=tw["embed"].f32, layers=f32_layers(tw["layers"]), final_norm=tw["final_norm"].f32, lm_head=tw["lm_head"].f32)
    refs = [orc.target_forward(two, tok[b], pos[b], otree.mask, [kcs[li].f32[b] for li in range(n_layers)],
                               [vcs[li].f32[b] for li in range(n_layers)], n_h, cfg.rms_eps, cfg.rope_theta, keep=True)
            for b in range(Bsz)]
    models = None
    if model:      # the oracle with its values rounded where the device stores bf16 (tests/bf16_noise_model.py)
        models = []
        for b in range(Bsz):
            m = nm.target_forward(two, tok[b], pos[b], otree.mask, [kcs[li].f32[b] for li in range(n_layers)],
                                  [vcs[li].f32[b] for li in range(n_layers)], n_h, cfg.rms_eps, cfg.rope_theta, nm.bf16)
            m["tgt"] = np.array([orc.row_argmax(r) for r in m["logits"]])
            models.append(m)
    host = None
    if keep_all:   # the last layer's host-side weights and cache rows, the final norm and the LM head, as float arrays
        host = (two["layers"][-1], [x for x in kcs[-1].f32], [x for x in vcs[-1].f32], two["final_norm"], two["lm_head"])
    return cfg, refs, dict(hidden=np_of(hidden), logits=np_of(logits), tgt=np_of(tgt), k_caches=k_caches, v_caches=v_caches,
                           L=L, T=T, ctx=ctx, model=models, dev=dev, host=host), (ctx, tree, otree)


HEAD_ROW_SCALE = 1.0      # (head, node) rows of the tree K/V are held to the same bound as whole node rows (worst measured: 1.6e-2 at the 33B width)


def check_target(cfg, refs, got, tol_scale=1.0):
    tol = TOL[cfg.dtype] * tol_scale
    L, T = got["L"], got["T"]
    for b, r in enumerate(refs):
        w1 = assert_rows_close(got["hidden"][b], r["hidden"], tol, "final hidden")
        w2 = assert_rows_close(got["logits"][b], r["logits"], tol, "target logits")
        say(f"  b={b} worst row error: hidden {w1:.2e}, logits {w2:.2e}")
        # argmax: equal wherever the oracle's top-1/top-2 gap exceeds the tolerance; elsewhere the GPU's
        # choice must still be within the tolerance of the oracle's maximum
        undecided = 0
        for i in range(T):
            o = r["logits"][i]
            srt = np.sort(o)
            tol_abs = tol * np.abs(o).max()
            if srt[-1] - srt[-2] > 2 * tol_abs:
                assert got["tgt"][b, i] == r["tgt"][i], f"argmax differs at node {i} despite a clear gap"
            else:
                undecided += 1
                assert o[got["tgt"][b, i]] >= srt[-1] - 2 * tol_abs
            # and the GPU's argmax is the exact argmax of the GPU's own logits (ties -> lowest id)
            assert got["tgt"][b, i] == orc.row_argmax(got["logits"][b, i])
        say(f"  b={b} nodes with an oracle top-1/top-2 gap below tolerance: {undecided}/{T}")
        # tree K/V rows written by every layer at rows [L, L+T), read back through amph_unpack_kv.  Two row
        # definitions: (i) one tree node's whole key (value) vector = one output row of the projection GEMM, held to
        # the tolerance; (ii) one (head, node) row of d_h values = what the attention consumes.  The absolute error of
        # a GEMM output does not depend on the head, but a single head's largest value is smaller than the largest of
        # all n_h heads together, so (ii) reads higher than (i) by that ratio; it still fits the plain tolerance at every
        # shape tested (HEAD_ROW_SCALE = 1) and its worst value is printed.
        k_rows, v_rows = D.unpack_kv(got["ctx"], got["k_caches"], got["v_caches"])
        worst_head = 0.0
        for li, lay in enumerate(r["layers"]):
            per_node = lambda a: np.transpose(a, (1, 0, 2)).reshape(a.shape[1], -1)             # [n_h, T, d_h] -> [T, d]
            per_head = lambda a: a.reshape(-1, a.shape[-1])                                      # [n_h, T, d_h] -> [n_h*T, d_h]
            kc, vc = np_of(k_rows[li, b][:, L:L + T]), np_of(v_rows[li, b][:, L:L + T])
            assert_rows_close(per_node(kc), per_node(lay["k_new"]), tol, f"layer {li} tree keys")
            assert_rows_close(per_node(vc), per_node(lay["v_new"]), tol, f"layer {li} tree values")
            wk = assert_rows_close(per_head(kc), per_head(lay["k_new"]), HEAD_ROW_SCALE * tol, f"layer {li} tree keys per head")
            wv = assert_rows_close(per_head(vc), per_head(lay["v_new"]), HEAD_ROW_SCALE * tol, f"layer {li} tree values per head")
            worst_head = max(worst_head, wk, wv)
        say(f"  b={b} worst (head, node) K/V row error {worst_head:.2e} (bound {HEAD_ROW_SCALE * tol:.1e})")


@pytest.mark.parametrize("tiled", [False, True], ids=["rowmajor", "tiled"])
@pytest.mark.parametrize("cfg,n_layers,T,caps,L", [
    (si.TINY, 2, 16, (4, 2, 2, 2), 128),
    (si.TINY, 0, 16, (4, 2, 2, 2), 128),           # embedding -> final norm -> LM head only
    (si.TINY, 1, 22, (10,) * 4, 5),
    (si.MINI, 2, 64, (10,) * 4, 200),
    (si.MINI, 3, 35, (10,) * 4, 61),
])
def test_target_forward_matches_oracle(cfg, n_layers, T, caps, L, tiled):
    say(f"target_forward {cfg.name} layers={n_layers} T={T} L={L} tiled={tiled}")
    cfgx, refs, got, _ = run_target(cfg, n_layers, T, caps, L, tiled=tiled)
    check_target(cfgx, refs, got)


def test_target_forward_batch_two():
    say("target_forward mini batch=2")
    cfgx, refs, got, _ = run_target(si.MINI, 2, 64, (10,) * 4, 100, Bsz=2)
    check_target(cfgx, refs, got)


@pytest.mark.parametrize("cfg,n_layers,T,caps,L,Bsz", [
    (si.MINI, 2, 64, (10,) * 4, 100, 2),           # M = 128: two blocks of 64 rows, still the skinny kernel
    (si.MINI, 2, 64, (10,) * 4, 90, 3),            # M = 192: 6 tiles of 32 rows, the smallest case of the wide kernel
    (si.MINI, 2, 64, (10,) * 4, 77, 5),            # M = 320: 10 tiles, two math waves per SIMD, two of them with 2 tiles
    (si.MINI, 1, 35, (10,) * 4, 61, 10),           # M = 350: 11 tiles, the last one ragged
    (si.MINI, 1, 64, (10,) * 4, 40, 7),            # M = 448: 14 tiles in one group
    (si.TINY, 2, 64, (10,) * 4, 5, 6),             # float32, M = 384: 12 tiles
    (si.MINI, 1, 96, (10,) * 5, 30, 3),            # M = 288: 9 tiles, only the first wave has two
    (si.MINI, 1, 64, (10,) * 4, 20, 8),            # M = 512: 16 tiles, every wave two
    (si.MINI, 1, 64, (10,) * 4, 12, 9),            # M = 576: 18 tiles, two groups of 9
])
def test_target_forward_batches_on_tiled_weights(cfg, n_layers, T, caps, L, Bsz):
    """Three blocks of 64 activation rows or more with tiled weights take the wide GEMM (groups of up to 16 tiles of 32
    rows of a weight tile in one workgroup, 32 x 32 matrix-core tiles, one or two math waves per SIMD); the same inputs
    with row-major weights take the skinny one.  Both against the oracle."""
    say(f"target_forward {cfg.name} layers={n_layers} T={T} L={L} batch={Bsz} (M = {T * Bsz}), tiled weights")
    cfgx, refs, got, _ = run_target(cfg, n_layers, T, caps, L, Bsz=Bsz, tiled=True)
    check_target(cfgx, refs, got)
    say("  row-major weights")
    cfgx, refs, got, _ = run_target(cfg, n_layers, T, caps, L, Bsz=Bsz, tiled=False)
    check_target(cfgx, refs, got)


@pytest.mark.parametrize("cfg,n_layers,T,caps,L,Bsz", [(si.MINI, 2, 64, (10,) * 4, 200, 1), (si.V7B, 2, 64, (10,) * 4, 1024, 1),
                                                       (si.MINI, 2, 64, (10,) * 4, 77, 4)], ids=["mini", "7b", "mini-batch4"])
def test_target_forward_is_bit_reproducible(cfg, n_layers, T, caps, L, Bsz):
    """Split reductions are folded in a fixed order and nothing is accumulated with atomics, so two passes over the same
    inputs (fresh contexts, fresh caches) give the same bits: hidden states, logits, argmax and the tree's K/V rows."""
    say(f"target_forward twice on {cfg.name}, {n_layers} layers, batch {Bsz}")
    runs = [run_target(cfg, n_layers, T, caps, L, seed=5, Bsz=Bsz, tiled=True, oracle=False)[2] for _ in range(2)]
    a, b = runs
    for key in ("hidden", "logits", "tgt"):
        assert np.array_equal(a[key], b[key]), key
    bits = lambda t: t.view(torch.int16 if t.element_size() == 2 else torch.int32)      # compare bits (NaN-safe)
    rows_a, rows_b = D.unpack_kv(a["ctx"], a["k_caches"], a["v_caches"]), D.unpack_kv(b["ctx"], b["k_caches"], b["v_caches"])
    for ra, rb, name in zip(rows_a, rows_b, ("keys", "values")):
        assert torch.equal(bits(ra[:, :, :, :L + T]), bits(rb[:, :, :, :L + T])), name


@pytest.mark.parametrize("tiled_keys", [("qkv",), ("wo", "down"), ("gate_up",), ("qkv", "gate_up", "down")])
def test_target_forward_partially_tiled_weights(tiled_keys):
    """Some matrices tiled, the others row-major, with enough rows (M = 256) that the tiled ones take the wide GEMM: its
    input then comes either from a producer that wrote the tiled activation layout or from the fallback copy."""
    say(f"target_forward mini batch=4, tiled copies only of {tiled_keys}")
    cfgx, refs, got, _ = run_target(si.MINI, 2, 64, (10,) * 4, 50, Bsz=4, tiled=True, tiled_keys=tiled_keys)
    check_target(cfgx, refs, got)


def test_target_forward_vicuna7b_two_layers():
    """Configuration 3 at full width (d 4096, FFN 11008, 32 x 128 heads, V 32000, L 1024, T 64) with two
    layers: the per-layer launch configuration is the one the bench times."""
    say("target_forward vicuna7b 2 layers (tiled weights, as the bench runs them)")
    cfgx, refs, got, _ = run_target(si.V7B, 2, 64, (10,) * 4, 1024, tiled=True)
    check_target(cfgx, refs, got)
    say("  same inputs with row-major weights: results must be bit-identical")
    _, _, got_rm, _ = run_target(si.V7B, 2, 64, (10,) * 4, 1024, tiled=False, oracle=False)
    assert np.array_equal(got["logits"], got_rm["logits"]) and np.array_equal(got["tgt"], got_rm["tgt"])
    assert np.array_equal(got["hidden"], got_rm["hidden"])
    for name in ("k_caches", "v_caches"):       # tree rows 1024..1087 = the last two key steps of the tiled storage
        assert torch.equal(got[name][:, :, :, 1024:1088].view(torch.int16), got_rm[name][:, :, :, 1024:1088].view(torch.int16))


def test_target_forward_vicuna13b_two_layers():
    """Configuration 4 at full width (d 5120, FFN 13824, 40 x 128 heads, L 2048, T 64), two layers, tiled
    weights: the per-layer launch configuration (tile heights 4 / 5 / 7 / 5 blocks) differs from 7B's."""
    say("target_forward vicuna13b 2 layers (tiled weights)")
    cfgx, refs, got, _ = run_target(si.V13B, 2, 64, (10,) * 4, 2048, tiled=True)
    check_target(cfgx, refs, got)


@pytest.mark.parametrize("seed", [0, 1])
def test_target_forward_vicuna33b_one_layer_batch4(seed):
    """Configuration 5 at full width (d 6656, FFN 17920, 52 x 128 heads, L 4096, T 96, batch 4: M = 384 rows, six
    blocks of 64 rows per weight tile), one sampled layer + final norm + LM head, tiled weights."""
    say(f"target_forward vicuna33b 1 layer (seed {seed}), batch 4 (tiled weights)")
    cfgx, refs, got, _ = run_target(si.V33B, 1, 96, (10,) * 5, 4096, seed=seed, Bsz=4, tiled=True)
    check_target(cfgx, refs, got)


def test_target_forward_vicuna33b_two_layers_batch4():
    """The same configuration end to end through two layers.  At this width the rounding of the bf16 activations
    between kernels alone (emulated on the CPU: tests/test_bf16_noise_cpu.py, 1.6e-2 for one layer of this shape)
    nearly uses up the 2e-2 bound in ONE layer and passes it in two.  So the stated 2e-2 is held per layer (the
    first layer by the one-layer tests above, the second one here, teacher-forced: it gets the oracle's input to
    it), and the two-layer chain against the exact oracle is bounded by 1.5 x the drift of the oracle with its own
    values rounded at the device's five rounding points (tests/bf16_noise_model.py) on the same inputs."""
    say("target_forward vicuna33b 2 layers, batch 4 (tiled weights)")
    T, L, Bsz = 96, 4096, 4
    cfgx, refs, got, (ctx, tree, otree) = run_target(si.V33B, 2, T, (10,) * 5, L, Bsz=Bsz, tiled=True, model=True, keep_all=True)
    tol = TOL[cfgx.dtype]
    for b, (r, m) in enumerate(zip(refs, got["model"])):
        d_h, d_l = nm.worst_row(m["hidden"], r["hidden"]), nm.worst_row(m["logits"], r["logits"])
        e_h, e_l = nm.worst_row(got["hidden"][b], r["hidden"]), nm.worst_row(got["logits"][b], r["logits"])
        say(f"  b={b} two-layer chain against the exact oracle: hidden {e_h:.2e}, logits {e_l:.2e}; the rounding model's own drift: "
            f"{d_h:.2e}, {d_l:.2e}")
        assert e_h <= 1.5 * d_h and e_l <= 1.5 * d_l
    # the second layer alone on the oracle's first-layer output (rounded to bf16, as both sides then see it)
    dev = got["dev"]
    n_h, d = cfgx.n_heads, cfgx.d_model
    x1 = np.stack([nm.bf16(r["layers"][0]["x"]) for r in refs])                     # [B, T, d]
    x_dev = torch.from_numpy(x1.reshape(Bsz * T, d).astype(np.float32)).to(DEV).to(torch.bfloat16)
    rows = i32_to_dev(np.arange(Bsz * T).reshape(Bsz, T))
    pos = i32_to_dev(np.stack([L + otree.depth for _ in range(Bsz)]))
    hidden = torch.zeros((Bsz, T, d), dtype=torch.float32, device=DEV)
    logits = torch.zeros((Bsz, T, cfgx.vocab), dtype=torch.float32, device=DEV)
    tgt = torch.zeros((Bsz, T), dtype=torch.int32, device=DEV)
    ctx.amph_target_forward(tree, dev["structs"][1:2], x_dev, dev["fn_d"], None, rows, pos, got["k_caches"][1:2], got["v_caches"][1:2],
                            i32_to_dev(np.full(Bsz, L)), hidden, logits, tgt, tiled_structs=dev["tiled_structs"][1:2],
                            lm_head_tiled=dev["lm_t"])
    torch.cuda.synchronize()
    assert ctx.device_status() == 0
    lw1, kcs1, vcs1, fn, lm = got["host"]
    forced = []
    for b in range(Bsz):
        o, k_new, v_new, _, _ = orc.decoder_layer_rows(x1[b], lw1, kcs1[b], vcs1[b], list(L + otree.depth), otree.mask, n_h,
                                                       cfgx.rms_eps, cfgx.rope_theta)
        hid = orc.rmsnorm(o, fn, cfgx.rms_eps)
        lg = orc.linear(lm, hid)
        forced.append(dict(hidden=hid, logits=lg, tgt=np.array([orc.row_argmax(x) for x in lg]), layers=[dict(k_new=k_new, v_new=v_new)]))
    got2 = dict(hidden=np_of(hidden), logits=np_of(logits), tgt=np_of(tgt), k_caches=got["k_caches"][1:2], v_caches=got["v_caches"][1:2],
                L=L, T=T, ctx=ctx)
    say("  second layer alone, teacher-forced, at the plain tolerance:")
    check_target(cfgx, forced, got2)


# ---------------------------------------------------------------------------- one whole step (A1-A10)
@pytest.mark.parametrize("cfg,n_layers,tiled", [(si.TINY, None, False), (si.MINI, None, False), (si.V7B, 2, True), (si.V13B, 2, True)],
                         ids=["tiny", "mini", "vicuna7b-2-layers-tiled", "vicuna13b-2-layers-tiled"])
def test_full_step_matches_oracle(cfg, n_layers, tiled):
    """amph_draft -> amph_tree_build -> amph_target_forward -> amph_accept on the device, with the
    integer decisions compared exactly wherever the oracle's own margins are clear.  At the 7B and 13B shapes this
    is the call sequence the bench times (tiled target weights, the draft's own top-k through the tree), at reduced
    depth; the target's logits are also compared with the oracle run on the tree the device built."""
    say(f"full step {cfg.name}")
    seed = 4
    n_h, d_h, d, V, K, T, L = cfg.n_heads, cfg.head_dim, cfg.d_model, cfg.vocab, cfg.K, cfg.T, cfg.kv_len
    max_kv = cfg.max_kv
    ctx = make_ctx(cfg)
    nl = cfg.n_layers if n_layers is None else n_layers
    dw, tw = si.draft_weights(cfg, seed), si.target_weights(cfg, seed, nl)
    dwd = D.draft_to_device(dw, DEV)
    dstruct = B.Context.draft_struct(dwd)
    layers_d = [D.layer_to_device(lw, DEV) for lw in tw["layers"]]
    structs = [B.Context.layer_struct(l) for l in layers_d]
    fn_d, lm_d = cfg_tensor_to_dev(tw["final_norm"]), cfg_tensor_to_dev(tw["lm_head"])
    tiled_structs = lm_t = keep = None
    if tiled:
        packed = [D.pack_layer(ctx, l) for l in layers_d]
        tiled_structs, keep = [p[0] for p in packed], [p[1] for p in packed]
        lm_t = D.pack_lm_head(ctx, lm_d)
        structs = [B.amph_layer_w(rms1=l["rms1"].data_ptr(), rms2=l["rms2"].data_ptr()) for l in layers_d]
    paths = si.tree_paths(T, cfg.tree_caps)
    tree = B.Tree(paths, K)
    otree = orc.tree_from_paths(paths, K)
    tdt = D.torch_dtype(cfg.dtype)
    h = si.as_f32_exact(cfg, seed, "step.h", (1, d), 1.0)
    tok = si.tokens(cfg, seed, "step.tok", (1,))
    Ls = cfg.sal_len
    sal_k = [si.normal(cfg, seed, f"sal{s}.k", (1, n_h, Ls, d_h), 1.0) for s in range(2)]
    sal_v = [si.normal(cfg, seed, f"sal{s}.v", (1, n_h, Ls, d_h), 1.0) for s in range(2)]
    sal_kv = torch.zeros((2, 1, 2, n_h, max_kv, d_h), dtype=tdt, device=DEV)
    for s in range(2):
        sal_kv[s, :, 0, :, :Ls] = cfg_tensor_to_dev(sal_k[s])
        sal_kv[s, :, 1, :, :Ls] = cfg_tensor_to_dev(sal_v[s])
    kcs = [si.normal(cfg, seed, f"tkv{li}.k", (1, n_h, L, d_h), 1.0) for li in range(nl)]
    vcs = [si.normal(cfg, seed, f"tkv{li}.v", (1, n_h, L, d_h), 1.0) for li in range(nl)]
    k_caches = torch.zeros((nl, 1, n_h, max_kv, d_h), dtype=tdt, device=DEV)
    v_caches = torch.zeros((nl, 1, n_h, max_kv, d_h), dtype=tdt, device=DEV)
    for li in range(nl):
        k_caches[li, :, :, :L] = cfg_tensor_to_dev(kcs[li])
        v_caches[li, :, :, :L] = cfg_tensor_to_dev(vcs[li])
    k_caches, v_caches = D.pack_kv(ctx, k_caches, v_caches)
    i32 = lambda *shape: torch.full(shape, -9, dtype=torch.int32, device=DEV)
    topk_idx, topk_val = i32(1, K, cfg.topk), torch.zeros((1, K, cfg.topk), dtype=torch.float32, device=DEV)
    tree_tok, tree_pos, tgt = i32(1, T), i32(1, T), i32(1, T)
    a_len, a_path, nxt, best = i32(1), i32(1, K + 1), i32(1), i32(1)
    tok_d, kv_len_d, sal_len_d = i32_to_dev(tok), i32_to_dev([L]), i32_to_dev([Ls])
    ctx.amph_draft(dstruct, f32_to_dev(h), tok_d, sal_kv, sal_len_d, topk_idx, topk_val, None)
    ctx.amph_tree_build(tree, tok_d, topk_idx, kv_len_d, tree_tok, tree_pos)
    t_logits = torch.full((1, T, V), float("nan"), dtype=torch.float32, device=DEV)
    ctx.amph_target_forward(tree, structs, dwd["embed"], fn_d, None if tiled else lm_d, tree_tok, tree_pos, k_caches, v_caches,
                            kv_len_d, None, t_logits, tgt, tiled_structs=tiled_structs, lm_head_tiled=lm_t)
    ctx.amph_accept(tree, tree_tok, tgt, None, a_len, a_path, nxt, best)
    torch.cuda.synchronize()
    assert ctx.device_status() == 0
    del keep

    two = dict(embed=tw["embed"].f32, layers=f32_layers(tw["layers"]), final_norm=tw["final_norm"].f32, lm_head=tw["lm_head"].f32)
    o = orc.step(draft_f32(dw), two, otree, h[0], int(tok[0]), [x.f32[0] for x in sal_k], [x.f32[0] for x in sal_v],
                 [x.f32[0] for x in kcs], [x.f32[0] for x in vcs], n_h, cfg.topk, cfg.rms_eps, cfg.rope_theta)
    tol = TOL[cfg.dtype]
    g_topk = np_of(topk_idx)[0]
    same_topk = np.array_equal(g_topk, o["draft"]["topk_idx"])
    for k in range(K):
        ok, bad = topk_consistent(g_topk[k], o["draft"]["logits"][k], cfg.topk, tol * np.abs(o["draft"]["logits"][k]).max())
        assert ok, (k, bad)
    # tree construction is integer work on the GPU's own top-k: exact against the oracle's rule
    g_tok, g_pos = np_of(tree_tok)[0], np_of(tree_pos)[0]
    e_tok, e_pos = orc.tree_tokens(otree, int(tok[0]), g_topk, L)
    np.testing.assert_array_equal(g_tok, e_tok)
    np.testing.assert_array_equal(g_pos, e_pos)
    # the target's logits against the oracle run on the tree the device built (equal to the oracle's own tree when
    # the draft's candidates agree)
    t_ref = orc.target_forward(two, g_tok, e_pos, otree.mask, [x.f32[0] for x in kcs], [x.f32[0] for x in vcs], n_h,
                               cfg.rms_eps, cfg.rope_theta)
    w_t = assert_rows_close(np_of(t_logits)[0], t_ref["logits"], tol, "target logits on the device's own tree")
    say(f"  target logits on the device's tree: worst row error {w_t:.2e}")
    # acceptance is integer work on the GPU's own target argmax: exact against the oracle's rule
    g_tgt = np_of(tgt)[0]
    ea, epath, enxt, ebest = orc.accept_greedy(otree, g_tok, g_tgt)
    assert (int(a_len[0]), int(best[0]), int(nxt[0])) == (ea, ebest, enxt)
    np.testing.assert_array_equal(np_of(a_path)[0], epath)
    # end to end: when the draft candidates agree and every target decision on the way has a clear margin,
    # the accepted length and the emitted token equal the oracle's
    if same_topk:
        clear = True
        for i in range(T):
            srt = np.sort(o["target"]["logits"][i])
            if srt[-1] - srt[-2] <= 2 * tol * np.abs(o["target"]["logits"][i]).max():
                clear = False
        say(f"  same top-k as the oracle; all target margins clear: {clear}; oracle accept_len {o['accept_len']}")
        if clear:
            np.testing.assert_array_equal(g_tgt, o["target"]["tgt"])
            assert int(a_len[0]) == o["accept_len"] and int(nxt[0]) == o["next_tok"]
    else:
        say("  top-k differs from the oracle within tolerance (near-ties); end-to-end equality not applicable")


@pytest.mark.parametrize("cfg,n_layers,T,caps,L,tiled", [
    (si.TINY, 2, 16, (4, 2, 2, 2), 64, False),
    (si.V7B, 2, 64, (10,) * 4, 1024, True),
    (si.V13B, 2, 64, (10,) * 4, 2048, True),
], ids=["tiny", "vicuna7b-2-layers-tiled", "vicuna13b-2-layers-tiled"])
def test_planted_drafts_are_fully_accepted_on_the_gpu(cfg, n_layers, T, caps, L, tiled):
    """Invariant: drafts set to the target's argmax along a path are accepted to that path's depth.  The
    tokens are planted depth by depth from the GPU's own target argmax (a node's logits depend only on
    its ancestors), then one more forward pass must accept the whole path: accept_len = K at full width, through
    the kernels and the launch configuration of the 7B and 13B steps."""
    say(f"planted path {cfg.name}")
    seed, K = 9, len(caps)
    cfgx, _, got, (ctx, tree, otree) = run_target(cfg, n_layers, T, caps, L, seed=seed, tiled=tiled, oracle=False)
    dev = got["dev"]
    k_caches, v_caches = got["k_caches"], got["v_caches"]
    leaf = [int(n) for n in otree.retrieve[np.argmax((otree.retrieve >= 0).sum(axis=1))] if n >= 0]
    assert len(leaf) == K + 1
    tok = si.tokens(cfgx, seed, "tree.tok", (1, T)).copy()
    pos = i32_to_dev((L + otree.depth)[None])
    kv_len = i32_to_dev([L])
    tgt = torch.zeros((1, T), dtype=torch.int32, device=DEV)
    a_len, a_path = torch.zeros(1, dtype=torch.int32, device=DEV), torch.zeros((1, K + 1), dtype=torch.int32, device=DEV)
    nxt, best = torch.zeros(1, dtype=torch.int32, device=DEV), torch.zeros(1, dtype=torch.int32, device=DEV)

    def forward(tok_d):
        ctx.amph_target_forward(tree, dev["structs"], dev["embed_d"], dev["fn_d"], dev["lm_d"], tok_d, pos, k_caches, v_caches,
                                kv_len, None, None, tgt, tiled_structs=dev["tiled_structs"], lm_head_tiled=dev["lm_t"])
        torch.cuda.synchronize()

    for m in range(1, K + 1):
        forward(i32_to_dev(tok))
        tok[0, leaf[m]] = int(tgt[0, leaf[m - 1]])
        # a sibling that happens to carry the same token would be an equally valid accepted node: make it differ
        for j in range(1, T):
            if j != leaf[m] and otree.parent[j] == otree.parent[leaf[m]] and tok[0, j] == tok[0, leaf[m]]:
                tok[0, j] = (tok[0, j] + 1) % cfgx.vocab
    tok_d = i32_to_dev(tok)
    forward(tok_d)
    ctx.amph_accept(tree, tok_d, tgt, None, a_len, a_path, nxt, best)
    torch.cuda.synchronize()
    assert ctx.device_status() == 0
    assert int(a_len[0]) == K
    assert list(np_of(a_path)[0]) == leaf
    assert int(nxt[0]) == int(tgt[0, leaf[-1]])
    # one wrong token in the middle of the path stops the acceptance there
    tok[0, leaf[2]] = (tok[0, leaf[2]] + 1) % cfgx.vocab
    sib = [j for j in range(1, T) if j != leaf[2] and otree.parent[j] == otree.parent[leaf[2]]]
    for j in sib:                                          # no sibling may pick up the planted token
        if tok[0, j] == int(tgt[0, leaf[1]]):
            tok[0, j] = (tok[0, j] + 2) % cfgx.vocab
    tok_d = i32_to_dev(tok)
    forward(tok_d)
    ctx.amph_accept(tree, tok_d, tgt, None, a_len, a_path, nxt, best)
    torch.cuda.synchronize()
    assert int(a_len[0]) == 1 and list(np_of(a_path)[0][:2]) == leaf[:2]
