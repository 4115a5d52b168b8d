#!/usr/bin/env python3
"""Benchmark of the Amphista draft+verify step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input, all through the C ABI:
amph_draft (Eq. 1-6) -> amph_tree_build -> amph_target_forward (32 decoder layers with tree attention,
final norm, LM head, argmax) -> amph_accept.  Workload at N = 1: Vicuna-7B shapes (configurations 2 + 3:
hidden 4096, 32 x 128 heads, FFN 11008, vocab 32000, K = 4 heads, top-10, 64-node tree, KV length 1024,
SAL cache 1024, batch 1, bf16 weights N(0, 0.02^2) generated on the device, seed 0).

Prints one JSON line with steps/s, the roofline of the dominant kernel (timed live with HIP events
around each of its launches inside the timed region) and the CPU oracle's rate on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PROF_EVERY = 31
HBM_PEAK_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algo_bytes(kind: str, c, M: int) -> float:
    """Algorithmic bytes one launch of `kind` must move: every weight/cache byte once plus the
    activations it reads and writes (bf16 = 2 B, float32 = 4 B)."""
    e = 2 if c.dtype == "bf16" else 4
    d, f, V, K, L, T, B = c.d_model, c.d_ffn, c.vocab, c.K, c.kv_len, c.T, c.batch
    Ls = c.sal_len
    return {
        "fc": 2 * d * d * e + B * (3 * d) * 4,
        "sal_qkv": 3 * d * d * e + B * d * 4 * 2 + 2 * B * d * e,
        "sal_attn": 2 * B * (Ls + 1) * d * e + 2 * B * d * 4,
        "sal_wo": d * d * e + 3 * B * d * 4,
        "sal_gateup": 2 * f * d * e + B * (d + f) * 4,
        "sal_down": d * f * e + B * (f + 2 * d) * 4,
        "head_mlp": K * d * d * e + B * (2 * d + K * d) * 4,
        "aeb_qkv": 3 * d * d * e + 4 * B * K * d * 4,
        "aeb_attn": 4 * B * K * d * 4,
        "aeb_wo": d * d * e + 2 * B * K * d * 4,
        "lm_head": V * d * e + B * K * d * 4,                 # candidates instead of logits: a few hundred KB
        "topk": B * K * 512 * c.topk * 8,                     # (value, token) candidates of about 512 workgroups per row
        "t_rmsnorm": M * d * (4 + e),
        "t_qkv": 3 * d * d * e + M * d * e + 3 * M * d * e,
        "verify": 2 * B * (L + T) * d * e + 2 * M * d * e,
        "t_wo": d * d * e + M * d * e + 2 * M * d * 4,
        "t_gateup": 2 * f * d * e + M * d * e + M * f * e,
        "t_down": d * f * e + M * f * e + 2 * M * d * 4,
        "t_lmhead": V * d * e + M * d * e + M * 4,
    }[kind]


def step_bytes(c, M: int, n_layers: int) -> float:
    per_layer = sum(algo_bytes(k, c, M) for k in ("t_qkv", "verify", "t_wo", "t_gateup", "t_down")) + 2 * algo_bytes("t_rmsnorm", c, M)
    draft = 2 * sum(algo_bytes(k, c, M) for k in ("fc", "sal_qkv", "sal_attn", "sal_wo", "sal_gateup", "sal_down")) + \
        sum(algo_bytes(k, c, M) for k in ("head_mlp", "aeb_qkv", "aeb_attn", "aeb_wo", "lm_head", "topk"))
    return draft + n_layers * per_layer + algo_bytes("t_rmsnorm", c, M) + algo_bytes("t_lmhead", c, M)


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


CPU_BUDGET_S = 90.0      # oracle time above which the target layers are sampled instead of all run


def cpu_baseline(cfg, n_layers: int):
    """The oracle as it stands, timed on the host cores over ONE whole step of the same workload: the draft, every
    one of the n_layers target layers over the tree tokens (each fed the previous one's output), the final norm,
    the LM head, the argmax and the acceptance.  The oracle's time does not depend on the weights' values, so the
    seeded weights of ONE layer (and one layer's cache rows) serve all n_layers layers: generating 32 distinct
    layers on the host would take minutes and add nothing to the timing.  If the first layer shows that the whole
    stack would take more than CPU_BUDGET_S (the 33B shapes), the layers are sampled instead and the result says so."""
    import numpy as np
    import synth_inputs as si
    from oracle import amphista_oracle as orc
    f32l = lambda lw: {k: v.f32 for k, v in lw.items()}
    t0 = time.time()
    dw = si.draft_weights(cfg, 0)
    dwo = dict(embed=dw["embed"].f32, fc=[x.f32 for x in dw["fc"]], sal=[f32l(l) for l in dw["sal"]], mlp=dw["mlp"].f32,
               pe=dw["pe"].f32, aeb_wq=dw["aeb_wq"].f32, aeb_wk=dw["aeb_wk"].f32, aeb_wv=dw["aeb_wv"].f32,
               aeb_wo=dw["aeb_wo"].f32, lm_head=dw["lm_head"].f32)
    n_h, d_h, d, L, Ls, T = cfg.n_heads, cfg.head_dim, cfg.d_model, cfg.kv_len, cfg.sal_len, cfg.T
    h = si.as_f32_exact(cfg, 0, "bench.h", (d,), 1.0)
    tok = int(si.tokens(cfg, 0, "bench.tok", (1,))[0])
    sal_k = [si.normal(cfg, 0, f"sal{s}.k", (n_h, Ls, d_h), 1.0).f32 for s in range(2)]
    sal_v = [si.normal(cfg, 0, f"sal{s}.v", (n_h, Ls, d_h), 1.0).f32 for s in range(2)]
    tree = orc.tree_from_paths(si.tree_paths(T, cfg.tree_caps), cfg.K)
    lw = f32l(si.decoder_layer(cfg, 0, "target.layer0"))
    kc = si.normal(cfg, 0, "tkv0.k", (n_h, L, d_h), 1.0).f32
    vc = si.normal(cfg, 0, "tkv0.v", (n_h, L, d_h), 1.0).f32
    lm = si.normal(cfg, 0, "target.lm_head", (cfg.vocab, d), si.W_STD).f32
    log(f"[cpu_baseline] seeded inputs generated in {time.time() - t0:.1f}s")
    t1 = time.time()
    dr = orc.draft(dwo, h, tok, sal_k, sal_v, n_h, cfg.topk, cfg.rms_eps, cfg.rope_theta)
    tree_tok, tree_pos = orc.tree_tokens(tree, tok, dr["topk_idx"], L)
    t_draft = time.time() - t1
    x = dwo["embed"][tree_tok]
    t2 = time.time()
    x, _, _, _, _ = orc.decoder_layer_rows(x, lw, kc, vc, list(tree_pos), tree.mask, n_h, cfg.rms_eps, cfg.rope_theta)
    t_first = time.time() - t2
    full = t_first * n_layers <= CPU_BUDGET_S
    n_run = n_layers if full else max(2, int(CPU_BUDGET_S / 3 / t_first))
    for _ in range(n_run - 1):
        x, _, _, _, _ = orc.decoder_layer_rows(x, lw, kc, vc, list(tree_pos), tree.mask, n_h, cfg.rms_eps, cfg.rope_theta)
    t_layers = time.time() - t2
    t3 = time.time()
    hidden = orc.rmsnorm(x, np.ones(d), cfg.rms_eps)
    logits = orc.linear(lm, hidden)
    tgt = np.array([orc.row_argmax(r) for r in logits], dtype=np.int32)
    orc.accept_greedy(tree, tree_tok, tgt)
    t_head = time.time() - t3
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    if full:
        total = t_draft + t_layers + t_head
        sample = (f"full step, 1 run: draft + tree + all {n_layers} target layers (T={T}, L={L}) + final norm / LM head / argmax / "
                  f"accept = {total:.1f} s of oracle time (draft {t_draft:.2f} s, layers {t_layers:.2f} s, head {t_head:.2f} s); "
                  f"one layer's seeded weights serve every layer (the oracle's time does not depend on the values)")
    else:
        total = t_draft + t_layers / n_run * n_layers + t_head
        sample = (f"SCALED, not a full run: all {n_layers} layers would take {t_first * n_layers:.0f} s (> {CPU_BUDGET_S:.0f} s): whole draft + "
                  f"{n_run} of {n_layers} target layers (T={T}, L={L}) + final norm / LM head / argmax / accept, "
                  f"t_draft + {n_layers} * t_layer + t_head = {total:.1f} s per step; {t_draft + t_layers + t_head:.0f} s of oracle time")
    log(f"[cpu_baseline] draft {t_draft:.2f}s, {n_run} layers {t_layers:.2f}s, head {t_head:.2f}s -> step {total:.1f}s on {cores} threads, {cpu_model()}")
    return {"value": 1.0 / total, "unit": "steps/s", "cores": cores, "kind": "oracle", "sample": sample, "cpu_model": cpu_model(),
            "seconds_per_step": total}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="vicuna7b", choices=["vicuna7b", "vicuna13b", "vicuna33b", "tiny", "mini_bf16"])
    ap.add_argument("--layers", type=int, default=None, help="target layers (default: the configuration's)")
    ap.add_argument("--batch", type=int, default=None, help="independent sequences per step (default: the configuration's)")
    ap.add_argument("--tree-nodes", type=int, default=None, help="nodes of the candidate tree (default: the configuration's)")
    ap.add_argument("--unequal-kv", action="store_true",
                    help="batch elements get committed lengths spread over [L/4, L] instead of all L")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-loop", action="store_true",
                    help="skip the second timed region (the loop iteration: catch-up draft + step + commit)")
    ap.add_argument("--breakdown", action="store_true", help="time every kernel kind (one extra step each) and print it")
    ap.add_argument("--row-major", action="store_true",
                    help="feed the target's GEMMs the row-major matrices instead of their tiled copies (slower; for comparison)")
    ap.add_argument("--aeb-layers", type=int, default=1, choices=[1, 2], help="self-attention layers in the Auto-embedding Block (2 = the alpha variant)")
    ap.add_argument("--lm-rank", type=int, default=0, help="rank of the low-rank LM head of the draft (0 = full head)")
    ap.add_argument("--one-stage", action="store_true", help="one adaptation layer for all heads")
    ap.add_argument("--no-pe", action="store_true", help="no position encoding")
    ap.add_argument("--temperature", type=float, default=0.0,
                    help="0: greedy acceptance (the headline); above 0: acceptance under random sampling (typical acceptance, "
                         "eps 0.09, delta 0.3) on the target's logits")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain streaming copy (read 256 MiB, write 256 MiB) so that a counter run can "
                         "scale FETCH_SIZE / WRITE_SIZE by what they read for a kernel of known traffic")
    ap.add_argument("--profile-kind", default=None, help="kernel kind to time live (default: the one with the largest share)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth_inputs as si
    from paper_2406_13170_amd import binding as B
    from paper_2406_13170_amd import device as D

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    cfg = si.CONFIGS[args.workload]
    if args.batch is not None:
        cfg = si.with_(cfg, batch=args.batch)
    if args.tree_nodes is not None:
        cfg = si.with_(cfg, T=args.tree_nodes)
    n_layers = cfg.n_layers if args.layers is None else args.layers
    n_h, d_h, d, f, V, K, T, L, Ls, Bsz = (cfg.n_heads, cfg.head_dim, cfg.d_model, cfg.d_ffn, cfg.vocab, cfg.K, cfg.T,
                                           cfg.kv_len, cfg.sal_len, cfg.batch)
    max_kv = cfg.max_kv
    tdt = D.torch_dtype(cfg.dtype)
    gen = torch.Generator(device=dev)
    gen.manual_seed(0)

    def randn(shape, std):
        t = torch.randn(shape, generator=gen, device=dev, dtype=torch.float32)
        return (t * std).to(tdt) if std != 1.0 else t.to(tdt)

    def layer():
        return dict(rms1=torch.ones(d, dtype=tdt, device=dev), rms2=torch.ones(d, dtype=tdt, device=dev),
                    wq=randn((d, d), 0.02), wk=randn((d, d), 0.02), wv=randn((d, d), 0.02), wo=randn((d, d), 0.02),
                    w_gate=randn((f, d), 0.02), w_up=randn((f, d), 0.02), w_down=randn((d, f), 0.02))

    t0 = time.time()
    dw = dict(embed=randn((V, d), 0.02), fc=[randn((d, 2 * d), 0.02) for _ in range(2)], sal=[layer() for _ in range(2)],
              mlp=randn((K, d, d), 0.02), pe=randn((K, d), 0.02), aeb_wq=randn((d, d), 0.02), aeb_wk=randn((d, d), 0.02),
              aeb_wv=randn((d, d), 0.02), aeb_wo=randn((d, d), 0.02), lm_head=randn((V, d), 0.02))
    n_stages = 1 if args.one_stage else 2
    if args.one_stage:
        dw["sal"], dw["fc"] = dw["sal"][:1], dw["fc"][:1]
    if args.no_pe:
        dw["pe"] = None
    if args.aeb_layers == 2:
        for k in ("wq", "wk", "wv", "wo"):
            dw["aeb2_" + k] = randn((d, d), 0.02)
    if args.lm_rank:
        dw["lm_a"], dw["lm_b"], dw["lm_head"] = randn((args.lm_rank, d), 0.02), randn((V, args.lm_rank), 0.02), None
    layers = [layer() for _ in range(n_layers)]
    final_norm = torch.ones(d, dtype=tdt, device=dev)
    t_lm_head = randn((V, d), 0.02)
    k_caches = torch.zeros((max(n_layers, 1), Bsz, n_h, max_kv, d_h), dtype=tdt, device=dev)
    v_caches = torch.zeros((max(n_layers, 1), Bsz, n_h, max_kv, d_h), dtype=tdt, device=dev)
    for li in range(n_layers):      # random rows: the step-tiled storage order does not matter for throughput
        k_caches[li, :, :, :L] = randn((Bsz, n_h, L, d_h), 1.0)
        v_caches[li, :, :, :L] = randn((Bsz, n_h, L, d_h), 1.0)
    sal_kv = torch.zeros((2, Bsz, 2, n_h, max_kv, d_h), dtype=tdt, device=dev)
    sal_kv[:, :, :, :, :Ls] = randn((2, Bsz, 2, n_h, Ls, d_h), 1.0)
    h = torch.randn((Bsz, d), generator=gen, device=dev, dtype=torch.float32).to(tdt).float()
    tok = torch.randint(0, V, (Bsz,), generator=gen, device=dev, dtype=torch.int32)
    torch.cuda.synchronize()
    log(f"[bench] {args.workload}: {n_layers} layers, weights on device in {time.time() - t0:.1f}s")

    ctx = B.Context(d_model=d, n_heads=n_h, head_dim=d_h, d_ffn=f, vocab=V, K=K, topk=cfg.topk, max_tree=T, max_kv=max_kv,
                    batch=Bsz, dtype=D.dtype_code(cfg.dtype), rms_eps=cfg.rms_eps, rope_theta=cfg.rope_theta, device=dev,
                    n_stages=n_stages, aeb_layers=args.aeb_layers, lm_rank=args.lm_rank)
    tree = B.Tree(si.tree_paths(T, cfg.tree_caps), K)
    dstruct = B.Context.draft_struct(dw)
    structs = [B.Context.layer_struct(l) for l in layers]
    tiled_structs = lm_tiled = tiled_keep = None
    if not args.row_major:
        # The target's matrices in the tiled layout the matrix-core GEMM streams (amph_pack_weights, once at load
        # time); the row-major copies are dropped, as a server would.
        tiled_structs, tiled_keep = [], []
        for li, l in enumerate(layers):
            ts, tt = D.pack_layer(ctx, l)
            tiled_structs.append(ts)
            tiled_keep.append(tt)
            structs[li] = B.amph_layer_w(rms1=l["rms1"].data_ptr(), rms2=l["rms2"].data_ptr())
            torch.cuda.synchronize()
            for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
                del l[k]
        lm_tiled = D.pack_lm_head(ctx, t_lm_head)
        torch.cuda.synchronize()
        t_lm_head = None
    i32 = lambda *shape: torch.zeros(shape, dtype=torch.int32, device=dev)
    topk_idx, topk_val = i32(Bsz, K, cfg.topk), torch.zeros((Bsz, K, cfg.topk), dtype=torch.float32, device=dev)
    tree_tok, tree_pos, tgt = i32(Bsz, T), i32(Bsz, T), i32(Bsz, T)
    a_len, a_path, nxt, best = i32(Bsz), i32(Bsz, K + 1), i32(Bsz), i32(Bsz)
    kv_lens = [L - (3 * L // 4) * b // max(Bsz - 1, 1) for b in range(Bsz)] if args.unequal_kv else [L] * Bsz
    kv_len = torch.tensor(kv_lens, dtype=torch.int32, device=dev)
    sal_len0 = torch.full((Bsz,), Ls, dtype=torch.int32, device=dev)
    sal_len = sal_len0.clone()

    sampling = args.temperature > 0.0
    t_logits = torch.zeros((Bsz, T, cfg.vocab), dtype=torch.float32, device=dev) if sampling else None
    u_draws = torch.rand((Bsz,), generator=torch.Generator(device=dev).manual_seed(1), device=dev) if sampling else None

    def step():
        sal_len.copy_(sal_len0)          # every step repeats the same work: the SAL cache does not grow across steps
        ctx.amph_draft(dstruct, h, tok, sal_kv, sal_len, topk_idx, topk_val, None)
        ctx.amph_tree_build(tree, tok, topk_idx, kv_len, tree_tok, tree_pos)
        ctx.amph_target_forward(tree, structs, dw["embed"], final_norm, t_lm_head, tree_tok, tree_pos, k_caches, v_caches,
                                kv_len, None, t_logits, tgt, tiled_structs=tiled_structs, lm_head_tiled=lm_tiled)
        if sampling:
            ctx.amph_accept_typical(tree, tree_tok, t_logits, args.temperature, 0.09, 0.3, u_draws, a_len, a_path, nxt, best)
        else:
            ctx.amph_accept(tree, tree_tok, tgt, None, a_len, a_path, nxt, best)

    # The iteration of the decode loop (Sec. 2 "Speculative Decoding"): what a serving loop runs between two emitted
    # chunks.  The draft catches up over the K + 1 rows amph_commit gathered (n_valid of them live), the target also
    # writes its final-normed hidden states, and amph_commit compacts the accepted rows in every layer and gathers the
    # next draft's inputs.  Lengths are reset every iteration so that each one does the same work.
    hidden = torch.zeros((Bsz, T, d), dtype=torch.float32, device=dev)
    h_new = torch.zeros((Bsz, K + 1, d), dtype=torch.float32, device=dev)
    h_new[:, 0] = h
    tok_new = i32(Bsz, K + 1)
    tok_new[:, 0] = tok
    n_new = torch.ones((Bsz,), dtype=torch.int32, device=dev)
    root = tok.clone()
    kv_len0 = kv_len.clone()
    kv_len_loop = kv_len.clone()

    def loop_iteration():
        sal_len.copy_(sal_len0)
        kv_len_loop.copy_(kv_len0)
        ctx.amph_draft(dstruct, h_new, tok_new, sal_kv, sal_len, topk_idx, topk_val, None, n_new=K + 1, n_valid=n_new)
        ctx.amph_tree_build(tree, root, topk_idx, kv_len_loop, tree_tok, tree_pos)
        ctx.amph_target_forward(tree, structs, dw["embed"], final_norm, t_lm_head, tree_tok, tree_pos, k_caches, v_caches,
                                kv_len_loop, hidden, t_logits, tgt, tiled_structs=tiled_structs, lm_head_tiled=lm_tiled)
        if sampling:
            ctx.amph_accept_typical(tree, tree_tok, t_logits, args.temperature, 0.09, 0.3, u_draws, a_len, a_path, nxt, best)
        else:
            ctx.amph_accept(tree, tree_tok, tgt, None, a_len, a_path, nxt, best)
        ctx.amph_commit(tree, n_layers, k_caches, v_caches, kv_len_loop, a_len, a_path, nxt, tree_tok, hidden, h_new, tok_new, n_new)
        root.copy_(nxt)

    if args.calibrate_copy:
        n_cal = 64 * 2 ** 20                                   # float32 elements: 256 MiB in, 256 MiB out
        cal_src = torch.ones(n_cal, dtype=torch.float32, device=dev)
        cal_dst = torch.empty_like(cal_src)
        torch.cuda.synchronize()
        torch.mul(cal_src, 1.0, out=cal_dst)                   # one elementwise kernel over n_cal elements
        torch.cuda.synchronize()
        log(f"[bench] calibration copy: {n_cal} float32 elements, {n_cal * 4} bytes read and as many written")
        del cal_src, cal_dst

    for _ in range(max(args.warmup, 1)):
        step()
    torch.cuda.synchronize()
    assert ctx.device_status() == 0, "device-side range check failed"

    M = Bsz * T
    kinds = B.KERNEL_KINDS
    per_kind = {}
    if args.breakdown or args.profile_kind is None:
        for ki, name in enumerate(kinds):
            ctx.amph_profile_kind(ki, 4096)
            step()
            ms, n = ctx.amph_profile_read()
            per_kind[name] = (ms, n)
        ctx.amph_profile_kind(-1, 0)
        tot = sum(v[0] for v in per_kind.values())
        log("[bench] per-kind kernel time in one step (HIP events around each launch):")
        for name, (ms, n) in sorted(per_kind.items(), key=lambda kv: -kv[1][0]):
            if n:
                gbs = algo_bytes(name, cfg, M) * n / (ms * 1e-3) / 1e9
                log(f"    {name:11s} {n:4d} launches {ms * 1e3:9.1f} us total {ms * 1e3 / n:8.2f} us avg {gbs:8.0f} GB/s "
                    f"({gbs / HBM_PEAK_GBS * 100:5.1f}% of HBM peak)")
        log(f"    sum of kernel time {tot * 1e3:.1f} us")
    dominant = args.profile_kind or max(per_kind, key=lambda k: per_kind[k][0])
    dom_id = kinds.index(dominant)

    # The matrix-core GEMMs carry their two events in the launch itself (the events take the kernel's own begin and
    # end time stamps); other kinds are bracketed by events on the stream.  Either way a timed launch costs the
    # stream a few microseconds, so only one launch in PROF_EVERY of the dominant kind is timed inside the timed
    # region: about one per step, 3 us of a 4 ms step (31 is coprime to the launches per step, so samples rotate
    # over layers).
    ctx.amph_profile_kind(dom_id, min(65536, 64 * args.steps + 64), PROF_EVERY)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    dom_ms, dom_n = ctx.amph_profile_read()
    ctx.amph_profile_kind(-1, 0)
    # what a bracket reads with nothing inside: the part of avg_launch_us that is the markers, not the kernel
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(64)]
    for e0, e1 in pairs:
        e0.record()
        e1.record()
    torch.cuda.synchronize()
    empty_us = sum(e0.elapsed_time(e1) for e0, e1 in pairs) / len(pairs) * 1e3
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    steps_per_s = 1e3 / ms_per_step
    loop = None
    if not args.no_loop:
        for _ in range(3):
            loop_iteration()
        torch.cuda.synchronize()
        assert ctx.device_status() == 0, "device-side range check failed in the loop iteration"
        tl0 = time.perf_counter()
        for _ in range(args.steps):
            loop_iteration()
        torch.cuda.synchronize()
        loop_ms = (time.perf_counter() - tl0) * 1e3 / args.steps
        loop = {"ms_per_iteration": loop_ms, "iterations_per_s": 1e3 / loop_ms, "iterations": args.steps,
                "what": f"amph_draft over K + 1 = {K + 1} catch-up rows per sequence (n_valid live) + amph_tree_build + "
                        f"amph_target_forward (hidden states out) + accept + amph_commit in all {n_layers} layers; "
                        "lengths reset every iteration",
                "mean_accept_len": float(a_len.float().mean().item())}
        log(f"[bench] loop iteration: {loop_ms:.3f} ms ({1e3 / loop_ms:.1f} per s) against {ms_per_step:.3f} ms for the step alone")
    dom_avg_s = dom_ms * 1e-3 / max(dom_n, 1)
    dom_bytes = algo_bytes(dominant, cfg, M)
    achieved = dom_bytes / dom_avg_s / 1e9
    sb = step_bytes(cfg, M, n_layers)

    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{dominant}_{args.workload}.txt")
    if os.path.exists(tpath):
        for line in open(tpath):
            if line.startswith("hbm_bytes_per_launch"):
                traffic = float(line.split()[1])

    out = {
        "metric": "draft+verify steps/sec at Vicuna-7B shapes, 1 MI355X" if args.workload == "vicuna7b"
                  else f"draft+verify steps/sec, {args.workload}",
        "value": steps_per_s, "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{args.workload} full step: draft (K={K}, top-{cfg.topk}, SAL cache {Ls}) + {n_layers}-layer "
                               f"tree verification (T={T}, L={L}) + "
                               + (f"typical acceptance at temperature {args.temperature}" if sampling else "greedy accept")
                               + f", batch {Bsz}",
                   "layers": n_layers, "tree_nodes": T, "kv_len": L if not args.unequal_kv else kv_lens, "batch": Bsz,
                   "target_weight_layout": "row-major" if args.row_major else "tiled",
                   "draft_variant": {"adaptation_layers": n_stages, "position_encoding": not args.no_pe,
                                     "self_attention_layers": args.aeb_layers, "lm_head_rank": args.lm_rank or "full"}},
        "step_algorithmic_GB": sb / 1e9,
        "step_hbm_frac": sb * steps_per_s / 1e9 / HBM_PEAK_GBS,
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "launches_timed": dom_n, "timed_one_launch_in": PROF_EVERY,
                     "avg_launch_us": dom_avg_s * 1e6, "empty_event_pair_us": empty_us,
                     "algorithmic_bytes_per_launch": dom_bytes},
    }
    if per_kind:
        # every kernel kind of one step, event-bracketed in its own untimed step (the brackets add the markers' own
        # few microseconds to the short kinds: see roofline.empty_event_pair_us); GB/s = algorithmic bytes / time
        out["per_kind"] = {name: {"launches": n, "avg_us": ms * 1e3 / n,
                                  "GBps": algo_bytes(name, cfg, M) * n / (ms * 1e-3) / 1e9,
                                  "frac_of_hbm_peak": algo_bytes(name, cfg, M) * n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
                           for name, (ms, n) in per_kind.items() if n}
        draft_kinds = ("fc", "sal_qkv", "sal_attn", "sal_wo", "sal_gateup", "sal_down", "head_mlp", "aeb_qkv", "aeb_attn", "aeb_wo",
                       "lm_head", "topk")
        draft_us = sum(per_kind[k][0] for k in draft_kinds if k in per_kind) * 1e3
        draft_b = sum(algo_bytes(k, cfg, M) * per_kind[k][1] for k in draft_kinds if k in per_kind)
        out["draft"] = {"kernel_time_us": draft_us, "algorithmic_GB": draft_b / 1e9,
                        "frac_of_hbm_peak": draft_b / (draft_us * 1e-6) / 1e9 / HBM_PEAK_GBS if draft_us else None}
    if loop is not None:
        out["loop"] = loop
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, n_layers)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
