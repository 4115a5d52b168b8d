"""GPU parity of amph_accept_typical (acceptance under random sampling, Table 2) against the oracle.

The rule is a reading (the paper names none); what is compared is the HIP path against the oracle's statement of
that rule on the same float32 logits.  Integer outputs must agree exactly unless the oracle's float64 margin of a
decision is within float32 rounding of zero (none of the seeded cases has one: the test says so if that changes),
and the drawn token must be one whose cumulative-probability interval contains u up to float32 rounding."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import amphista_oracle as orc
from paper_2406_13170_amd import binding as B

from gpu_common import DEV, f32_to_dev, i32_to_dev, make_ctx, np_of, say

pytestmark = pytest.mark.gpu

REL_TIE = 2e-4          # |p - threshold| below this fraction of the threshold counts as a near tie
CDF_TOL = 2e-5          # float32 rounding of a cumulative sum of V terms, in probability


def synthetic_logits(rng, Bn, T, V, spread):
    """Peaked rows as a language model's: a few large logits over a wide bulk."""
    lg = rng.standard_normal((Bn, T, V)) * spread
    hot = rng.integers(0, V, size=(Bn, T, 6))
    for b in range(Bn):
        for j in range(T):
            lg[b, j, hot[b, j]] += rng.uniform(2.0, 9.0, size=6)
    return lg.astype(np.float32)


def plant_tokens(rng, otree, logits_b, V, temp):
    """Every node carries a token of its parent's distribution: mostly one of its likeliest, sometimes any."""
    T = otree.T
    tok = np.zeros(T, dtype=np.int32)
    tok[0] = rng.integers(0, V)
    for i in range(1, T):
        j = otree.parent[i]
        if rng.random() < 0.8:
            order = np.argsort(-logits_b[j])
            tok[i] = order[min(int(rng.geometric(0.45)) - 1, V - 1)]
        else:
            tok[i] = rng.integers(0, V)
    return tok


def run_case(V, T, caps, Bn, seed, temp, eps, delta, spread=2.5, logits=None, toks=None, us=None):
    K = len(caps)
    cfg = si.with_(si.TINY, vocab=V, batch=Bn, K=K, topk=min(16, max(caps)))
    ctx = make_ctx(cfg, T=T, batch=Bn)
    paths = si.tree_paths(T, caps)
    tree = B.Tree(paths, K)
    otree = orc.tree_from_paths(paths, K)
    rng = np.random.default_rng(np.random.SeedSequence([seed, V, T, Bn, 0x7a]))
    if logits is None:
        logits = synthetic_logits(rng, Bn, T, V, spread)
    if toks is None:
        toks = np.stack([plant_tokens(rng, otree, logits[b], V, temp) for b in range(Bn)])
    if us is None:
        us = rng.random(Bn).astype(np.float32)
    a_len = torch.full((Bn,), -7, dtype=torch.int32, device=DEV)
    a_path = torch.full((Bn, K + 1), -7, dtype=torch.int32, device=DEV)
    nxt = torch.full((Bn,), -7, dtype=torch.int32, device=DEV)
    best = torch.full((Bn,), -7, dtype=torch.int32, device=DEV)
    ctx.amph_accept_typical(tree, i32_to_dev(toks), f32_to_dev(logits), temp, eps, delta, f32_to_dev(us), a_len, a_path, nxt, best)
    torch.cuda.synchronize()
    assert ctx.device_status() == 0
    lens = []
    for b in range(Bn):
        oa, opath, onxt, obest, margin, held = orc.accept_typical(otree, toks[b], logits[b], temp, eps, delta, float(us[b]))
        near = [i for i in range(1, T) if abs(margin[i]) <= REL_TIE * held[i]]
        assert not near, f"seed {seed}: nodes {near} of element {b} are near ties; pick another seed"
        assert (int(a_len[b]), int(best[b])) == (oa, obest), f"element {b}"
        np.testing.assert_array_equal(np_of(a_path)[b], opath)
        g = int(nxt[b])
        if g != onxt:                                         # allowed only when u sits on an interval boundary
            p = orc.softmax(logits[b, obest].astype(np.float64) / temp)
            cdf = np.cumsum(p)
            lo = cdf[g - 1] if g > 0 else 0.0
            assert p[g] > 0 and lo - CDF_TOL <= us[b] < cdf[g] + CDF_TOL, f"element {b}: drew {g}, oracle {onxt}, u {us[b]}"
        lens.append(oa)
    return lens


@pytest.mark.parametrize("V,T,caps,Bn,temp,eps,delta", [
    (1024, 16, (4, 2, 2, 2), 1, 0.7, 0.09, 0.3),
    (1024, 16, (4, 2, 2, 2), 3, 1.0, 0.05, 0.6),
    (1000, 22, (10,) * 4, 2, 0.7, 0.09, 0.3),            # V not a multiple of the thread count or of four
    (37, 5, (1, 1, 1, 1), 2, 0.5, 0.2, 0.9),             # fewer tokens than threads; a chain
    (5000, 64, (10,) * 4, 2, 0.7, 0.09, 0.3),
    (2048, 128, (10,) * 8, 1, 0.7, 0.02, 0.1),           # the largest tree, depth 8
    (1024, 1, (4, 4, 4, 4), 2, 0.7, 0.09, 0.3),          # the root alone: only the draw
])
def test_accept_typical_matches_oracle(V, T, caps, Bn, temp, eps, delta):
    say(f"accept_typical V={V} T={T} B={Bn} temp={temp} eps={eps} delta={delta}")
    seen = set()
    for seed in range(4):
        seen.update(run_case(V, T, caps, Bn, seed, temp, eps, delta))
    say(f"  accept lengths seen: {sorted(seen)}")


@pytest.mark.parametrize("T,caps,Bn", [(64, (10,) * 4, 4), (96, (10,) * 5, 4)])
def test_accept_typical_full_vocabulary(T, caps, Bn):
    """32000 tokens, the 7B / 13B tree of 64 nodes and the 33B tree of 96, batch 4: the sizes the bench runs."""
    say(f"accept_typical V=32000 T={T} B={Bn}")
    lens = run_case(32000, T, caps, Bn, 3, 0.7, 0.09, 0.3, spread=2.0)
    say(f"  accept lengths: {lens}")
    assert max(lens) >= 1


def test_accept_typical_small_temperature_equals_greedy_entry_point():
    """At a vanishing temperature every row is one-hot at its argmax: the outcome must equal amph_accept's on the
    same logits (and the oracle's greedy rule), including the token that follows."""
    V, T, K, Bn = 4096, 64, 4, 3
    caps = (10,) * 4
    cfg = si.with_(si.TINY, vocab=V, batch=Bn, K=K, topk=10)
    ctx = make_ctx(cfg, T=T, batch=Bn)
    paths = si.tree_paths(T, caps)
    tree = B.Tree(paths, K)
    otree = orc.tree_from_paths(paths, K)
    rng = np.random.default_rng(5)
    logits = synthetic_logits(rng, Bn, T, V, 2.5)
    toks = np.zeros((Bn, T), dtype=np.int32)
    for b in range(Bn):
        tgt = np.array([orc.row_argmax(r) for r in logits[b]], dtype=np.int32)
        toks[b] = rng.integers(0, V, size=T)
        for i in range(1, T):
            if rng.random() < 0.7:
                toks[b, i] = tgt[otree.parent[i]]
    outs = []
    for typical in (False, True):
        a_len = torch.empty(Bn, dtype=torch.int32, device=DEV)
        a_path = torch.empty((Bn, K + 1), dtype=torch.int32, device=DEV)
        nxt = torch.empty(Bn, dtype=torch.int32, device=DEV)
        best = torch.empty(Bn, dtype=torch.int32, device=DEV)
        if typical:
            u = f32_to_dev(rng.random(Bn).astype(np.float32))
            ctx.amph_accept_typical(tree, i32_to_dev(toks), f32_to_dev(logits), 1e-4, 0.3, 0.5, u, a_len, a_path, nxt, best)
        else:
            ctx.amph_accept(tree, i32_to_dev(toks), None, f32_to_dev(logits), a_len, a_path, nxt, best)
        torch.cuda.synchronize()
        outs.append((np_of(a_len), np_of(a_path), np_of(nxt), np_of(best)))
    for x, y in zip(outs[0], outs[1]):
        np.testing.assert_array_equal(x, y)
    for b in range(Bn):
        tgt = np.array([orc.row_argmax(r) for r in logits[b]], dtype=np.int32)
        oa, opath, onxt, obest = orc.accept_greedy(otree, toks[b], tgt)
        assert (int(outs[1][0][b]), int(outs[1][3][b]), int(outs[1][2][b])) == (oa, obest, onxt)
    say(f"  accept lengths: {list(outs[1][0])}")


def test_accept_typical_edges():
    V, T, K = 512, 16, 4
    caps = (4, 2, 2, 2)
    rng = np.random.default_rng(9)
    # masked vocabulary: -inf logits are never drawn and never pass; u = 0 and u just below 1
    logits = synthetic_logits(rng, 2, T, V, 2.0)
    logits[:, :, :7] = -np.inf
    logits[:, :, V - 9:] = -np.inf
    otree = orc.tree_from_paths(si.tree_paths(T, caps), K)
    toks = np.stack([plant_tokens(rng, otree, logits[b], V, 0.7) for b in range(2)])
    toks[0, 1] = 3                                         # a masked token as a candidate
    us = np.array([0.0, np.float32(1.0) - np.float32(2.0 ** -24)], dtype=np.float32)
    run_case(V, T, caps, 2, 0, 0.7, 0.09, 0.3, logits=logits, toks=toks, us=us)
    # token ids outside the vocabulary never pass (and are never used as an index)
    toks2 = toks.copy()
    toks2[0, 1], toks2[1, 2] = -5, V + 100
    cfg = si.with_(si.TINY, vocab=V, batch=2, K=K, topk=4)
    ctx = make_ctx(cfg, T=T, batch=2)
    tree = B.Tree(si.tree_paths(T, caps), K)
    a_len = torch.empty(2, dtype=torch.int32, device=DEV)
    a_path = torch.empty((2, K + 1), dtype=torch.int32, device=DEV)
    nxt = torch.empty(2, dtype=torch.int32, device=DEV)
    best = torch.empty(2, dtype=torch.int32, device=DEV)
    ctx.amph_accept_typical(tree, i32_to_dev(toks2), f32_to_dev(logits), 0.7, 0.0, 0.0, f32_to_dev(us), a_len, a_path, nxt, best)
    torch.cuda.synchronize()
    paths_g = np_of(a_path)
    assert 1 not in paths_g[0] and 2 not in paths_g[1]
    assert np.all((np_of(nxt) >= 7) & (np_of(nxt) < V - 9))
    # thresholds at zero accept every token of non-zero probability: the deepest node with live tokens all the way
    # bad arguments are refused before any launch
    for bad in [dict(temperature=0.0), dict(temperature=-1.0), dict(eps=-0.1), dict(delta=float("nan"))]:
        kw = dict(temperature=0.7, eps=0.09, delta=0.3)
        kw.update(bad)
        with pytest.raises(B.AmphError):
            ctx.amph_accept_typical(tree, i32_to_dev(toks), f32_to_dev(logits), kw["temperature"], kw["eps"], kw["delta"],
                                    f32_to_dev(us), a_len, a_path, nxt, best)


def test_accept_typical_on_the_target_forward_logits():
    """The Tiny target's own logits (written by amph_target_forward) decide: the oracle applies the rule to the same
    float32 logits."""
    from test_gpu_step import run_target
    T, caps, Bn, seed = 16, (4, 2, 2, 2), 2, 2
    cfg, _, got, (ctx, tree, otree) = run_target(si.TINY, 2, T, caps, 40, seed=seed, Bsz=Bn, oracle=False)
    K = otree.K
    tk = si.tokens(cfg, seed, "tree.tok", (Bn, T)).astype(np.int32)
    lg = got["logits"]
    rng = np.random.default_rng(4)
    us = rng.random(Bn).astype(np.float32)
    a_len = torch.empty(Bn, dtype=torch.int32, device=DEV)
    a_path = torch.empty((Bn, K + 1), dtype=torch.int32, device=DEV)
    nxt = torch.empty(Bn, dtype=torch.int32, device=DEV)
    best = torch.empty(Bn, dtype=torch.int32, device=DEV)
    # random weights give nearly flat distributions (H close to ln V): delta below one accepts, above one rejects
    for delta in (0.5, 1.5):
        ctx.amph_accept_typical(tree, i32_to_dev(tk), f32_to_dev(lg), 0.7, 0.09, delta, f32_to_dev(us), a_len, a_path, nxt, best)
        torch.cuda.synchronize()
        for b in range(Bn):
            oa, opath, onxt, obest, margin, held = orc.accept_typical(otree, tk[b], lg[b], 0.7, 0.09, delta, float(us[b]))
            if any(abs(margin[i]) <= REL_TIE * held[i] for i in range(1, T)):
                continue
            assert (int(a_len[b]), int(best[b])) == (oa, obest)
            np.testing.assert_array_equal(np_of(a_path)[b], opath)
        say(f"  delta={delta}: accept lengths {list(np_of(a_len))}")


def test_generator_with_typical_acceptance():
    """Six steps of the whole loop on the device (draft, tree, target pass, acceptance under sampling, commit, catch-up),
    float32 Tiny configuration with a vocabulary of 8.  There is no oracle generator for this rule (it is not
    lossless, so no autoregressive sequence pins it); each step's decision is checked by giving the oracle's rule the
    device's own float32 logits and tree tokens, and the chain around it by its bookkeeping: the committed length grows
    by the accepted tokens plus one, the adaptation layers have seen every position before the step, the next root is
    the drawn token."""
    from test_gpu_loop import generator_state
    n_steps = 6
    st = generator_state(n_steps)
    cfg, otree, P, n_layers = st["cfg"], st["otree"], st["P"], st["n_layers"]
    K, T, V = cfg.K, cfg.T, cfg.vocab
    ctx, tree = st["ctx"], st["tree"]
    logits = torch.zeros((1, T, V), dtype=torch.float32, device=DEV)
    rng = np.random.default_rng(12)
    us = rng.random(n_steps).astype(np.float32)
    temp, eps, delta = 0.7, 0.09, 0.3
    committed, lens = P, []
    for step in range(n_steps):
        ctx.amph_draft(st["dstruct"], st["h_new"], st["tok_new"], st["sal_kv"], st["sal_len"], st["topk_idx"], st["topk_val"], None,
                       n_new=K + 1, n_valid=st["n_new"])
        ctx.amph_tree_build(tree, st["root"], st["topk_idx"], st["kv_len"], st["tree_tok"], st["tree_pos"])
        ctx.amph_target_forward(tree, st["structs"], st["dwd"]["embed"], st["fn_d"], st["lm_d"], st["tree_tok"], st["tree_pos"],
                                st["k_caches"], st["v_caches"], st["kv_len"], st["hidden"], logits, st["tgt"])
        ctx.amph_accept_typical(tree, st["tree_tok"], logits, temp, eps, delta, f32_to_dev(us[step:step + 1]), st["a_len"],
                                st["a_path"], st["nxt"], st["best"])
        tt, lg = np_of(st["tree_tok"])[0], np_of(logits)[0]
        al, ap, nx, bn = int(np_of(st["a_len"])[0]), np_of(st["a_path"])[0], int(np_of(st["nxt"])[0]), int(np_of(st["best"])[0])
        ctx.amph_commit(tree, n_layers, st["k_caches"], st["v_caches"], st["kv_len"], st["a_len"], st["a_path"], st["nxt"],
                        st["tree_tok"], st["hidden"], st["h_new"], st["tok_new"], st["n_new"])
        st["root"].copy_(st["nxt"])
        torch.cuda.synchronize()
        assert ctx.device_status() == 0
        oa, opath, onxt, obest, margin, held = orc.accept_typical(otree, tt, lg, temp, eps, delta, float(us[step]))
        near = [i for i in range(1, T) if abs(margin[i]) <= REL_TIE * held[i]]
        assert not near, f"step {step}: nodes {near} are near ties; pick another seed"
        assert (al, bn) == (oa, obest), f"step {step}"
        np.testing.assert_array_equal(ap, opath)
        if nx != onxt:
            p = orc.softmax(lg[obest].astype(np.float64) / temp)
            cdf = np.cumsum(p)
            lo = cdf[nx - 1] if nx > 0 else 0.0
            assert p[nx] > 0 and lo - CDF_TOL <= us[step] < cdf[nx] + CDF_TOL
        assert int(np_of(st["kv_len"])[0]) == committed + al + 1 and int(np_of(st["sal_len"])[0]) == committed
        assert int(np_of(st["n_new"])[0]) == al + 1 and int(np_of(st["root"])[0]) == nx
        committed += al + 1
        lens.append(al)
        say(f"  step {step}: accepted {al}, drew {nx}")
    assert max(lens) >= 1, "the seed should accept at least one draft token somewhere"
