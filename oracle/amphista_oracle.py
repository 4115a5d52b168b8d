"""CPU oracle for one Amphista speculate-and-verify decode step.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the HIP
path is judged against.  Only tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg may import it; it imports nothing from the HIP package and
shares no code with it.

Everything is float64 NumPy written straight from the paper's formulas, with no
blocking, fusion, online softmax or reordering:

  * Staged Adaptation Layers         -- Sec. 3.1, Eq. 1
  * head MLPs, concat, positional PE -- Sec. 3.2, Eq. 2-4
  * bi-directional self-attention    -- Sec. 3.2, Eq. 5
  * LM head + per-head top-k         -- Sec. 3.2, Eq. 6
  * draft tree + tree mask           -- Sec. 2 "Tree Attention", Appendix "Draft Tree"
  * tree-attention verification      -- Sec. 2 "Tree Attention", Sec. 3.2 last paragraph
  * greedy acceptance                -- Sec. 2 "Speculative Decoding", Table 1 (Temperature = 0)
  * acceptance under random sampling -- Table 2 (Temperature = 0.7); PARITY UNPINNED by the paper, which
                                        names no rule: see accept_typical for the reading taken

Where the paper is silent the readings are: Llama-style decoder layers (pre-RMSNorm, half-split RoPE, SwiGLU, no
biases) for both the target and the adaptation layers; h before e in the
concat; MLP_k(h) = h + SiLU(W_k h); Eq. 5 is a bare multi-head attention
sublayer (Wq, Wk, Wv, Wo; no mask, no RoPE, no residual, no norm); one LM head
shared by all K positions; a tree node attends to the committed cache, its
ancestors and itself; tree positions are kv_len + depth; ties go to the lowest
token id.

Pins (tests/test_oracle_*.py): brute-force per-path causal attention, chain
tree = causal attention, torch scaled_dot_product_attention, a Hugging Face
Llama decoder stack run with the same weights and tree mask, KV-cache
incremental = full recompute, closed forms of Eq. 5 (K = 1, Wq = 0, row
permutation), full-sort top-k, planted-argmax acceptance and equality with the
target's own autoregressive greedy continuation.  The numeric output of a whole
step is otherwise "parity unpinned": the paper prints no worked numbers.

The decode loop around the step (commit of the accepted path, the adaptation
layers catching up over the newly committed positions -- Eq. 1 keeps one cache
row per position --, and the generator) is written out at the end of the file;
its pin is that N steps emit exactly the target's autoregressive greedy tokens.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


def _f(a) -> np.ndarray:
    return np.asarray(a, dtype=F64)


# ----------------------------------------------------------------------------
# Llama-style building blocks (Fig. 2's caption says the adaptation layers are causal decoder
# layers of the target's kind; read here as the target's own layer shape)
# ----------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, w: np.ndarray, eps: float) -> np.ndarray:
    x = _f(x)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * _f(w)


def silu(z: np.ndarray) -> np.ndarray:
    z = _f(z)
    return z / (1.0 + np.exp(-z))


def rope(x: np.ndarray, pos: int, theta: float) -> np.ndarray:
    """Rotate pairs (i, i + d_h/2) of the last axis by pos * theta^(-2i/d_h)."""
    x = _f(x)
    d_h = x.shape[-1]
    half = d_h // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=F64) / d_h)
    ang = float(pos) * inv_freq
    c, s = np.cos(ang), np.sin(ang)
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def softmax(s: np.ndarray) -> np.ndarray:
    s = _f(s)
    e = np.exp(s - np.max(s))
    return e / np.sum(e)


def linear(W: np.ndarray, x: np.ndarray) -> np.ndarray:
    """y = W x for W [out, in]; x is [in] or [rows, in]."""
    return _f(x) @ _f(W).T


def swiglu_ffn(x: np.ndarray, lw: Dict[str, np.ndarray]) -> np.ndarray:
    return linear(lw["w_down"], silu(linear(lw["w_gate"], x)) * linear(lw["w_up"], x))


def attend(q: np.ndarray, keys: np.ndarray, values: np.ndarray) -> np.ndarray:
    """Single query over a set of keys: sum_j softmax_j(q.k_j / sqrt(d_h)) v_j."""
    return attend_segments(q, [(keys, values)])


def attend_segments(q: np.ndarray, segments) -> np.ndarray:
    """The same single-query attention with the key set given as a list of
    (keys, values) pieces; the softmax runs over the union of all pieces."""
    q = _f(q)
    d_h = q.shape[-1]
    scores = np.concatenate([_f(k) @ q for k, _ in segments]) / np.sqrt(float(d_h))
    p = softmax(scores)
    out = np.zeros(d_h, dtype=F64)
    at = 0
    for k, v in segments:
        n = k.shape[0]
        out += p[at:at + n] @ _f(v)
        at += n
    return out


def decoder_layer_rows(x: np.ndarray, lw: Dict[str, np.ndarray], k_cache: np.ndarray,
                       v_cache: np.ndarray, positions: Sequence[int], visible: np.ndarray,
                       n_heads: int, eps: float, theta: float):
    """One pre-norm decoder layer applied to R new rows on top of a committed cache.

    x [R, d]; k_cache, v_cache [n_heads, L, d_h] (committed rows, keys already
    rotated); positions[r] is the RoPE position of new row r; visible[r, j]
    says whether new row r may attend to new row j (every committed row is
    always visible).  Returns (out [R, d], k_new [n_heads, R, d_h], v_new,
    q [R, n_heads, d_h], attn [R, n_heads, d_h]).
    """
    x = _f(x)
    R, d = x.shape
    d_h = d // n_heads
    n = rmsnorm(x, lw["rms1"], eps)
    q = linear(lw["wq"], n).reshape(R, n_heads, d_h)
    k = linear(lw["wk"], n).reshape(R, n_heads, d_h)
    v = linear(lw["wv"], n).reshape(R, n_heads, d_h)
    for r in range(R):
        q[r] = rope(q[r], positions[r], theta)
        k[r] = rope(k[r], positions[r], theta)
    k_new = np.transpose(k, (1, 0, 2))
    v_new = np.transpose(v, (1, 0, 2))
    attn = np.zeros((R, n_heads, d_h), dtype=F64)
    kc, vc = _f(k_cache), _f(v_cache)
    for h in range(n_heads):
        for r in range(R):
            sel = np.nonzero(visible[r])[0]
            attn[r, h] = attend_segments(q[r, h], [(kc[h], vc[h]), (k_new[h][sel], v_new[h][sel])])
    y = x + linear(lw["wo"], attn.reshape(R, d))
    m = rmsnorm(y, lw["rms2"], eps)
    out = y + swiglu_ffn(m, lw)
    return out, k_new, v_new, q, attn


# ----------------------------------------------------------------------------
# Draft path: Eq. 1-6
# ----------------------------------------------------------------------------
def fc_concat(W_fc: np.ndarray, u: np.ndarray, e: np.ndarray) -> np.ndarray:
    """fc([u; e]) of Eq. 1: concat hidden state first, then the token embedding."""
    return linear(W_fc, np.concatenate([_f(u), _f(e)], axis=-1))


def sal_stage(x: np.ndarray, lw: Dict[str, np.ndarray], k_cache: np.ndarray, v_cache: np.ndarray,
              n_heads: int, eps: float, theta: float):
    """SAL^s of Eq. 1 on the single new position; its RoPE position is the
    number of rows already in that stage's cache, and it attends to them and itself."""
    pos = k_cache.shape[1]
    out, k_new, v_new, _, _ = decoder_layer_rows(
        _f(x)[None, :], lw, k_cache, v_cache, [pos], np.ones((1, 1), dtype=bool), n_heads, eps, theta)
    return out[0], k_new[:, 0, :], v_new[:, 0, :]


def head_mlp(W_k: np.ndarray, h: np.ndarray) -> np.ndarray:
    """MLP_k of Eq. 2 read as one d x d linear, SiLU and a residual."""
    return _f(h) + silu(linear(W_k, h))


def head_inputs(h1: np.ndarray, h2: np.ndarray, W_mlp: np.ndarray, pe: np.ndarray) -> np.ndarray:
    """Eq. 2-4: heads 1..floor(K/2) read h^1, the rest h^2; rows are stacked and PE added."""
    K = W_mlp.shape[0]
    rows = []
    for k in range(1, K + 1):
        src = h1 if k <= K // 2 else h2
        rows.append(head_mlp(W_mlp[k - 1], src))
    return np.stack(rows, axis=0) + _f(pe)


def bi_self_attention(Hp: np.ndarray, wq, wk, wv, wo, n_heads: int) -> np.ndarray:
    """Eq. 5: every one of the K rows attends to all K rows (no mask, no RoPE)."""
    Hp = _f(Hp)
    K, d = Hp.shape
    d_h = d // n_heads
    Q = linear(wq, Hp).reshape(K, n_heads, d_h)
    Kk = linear(wk, Hp).reshape(K, n_heads, d_h)
    V = linear(wv, Hp).reshape(K, n_heads, d_h)
    ctx = np.zeros((K, n_heads, d_h), dtype=F64)
    for h in range(n_heads):
        for i in range(K):
            ctx[i, h] = attend(Q[i, h], Kk[:, h, :], V[:, h, :])
    return linear(wo, ctx.reshape(K, d))


def topk_sorted(logits: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """Top-k by a full stable sort on (-logit, token id): descending value, ties to the lower id."""
    logits = _f(logits)
    order = np.lexsort((np.arange(logits.shape[0]), -logits))
    idx = order[:k].astype(np.int32)
    return idx, logits[idx]


def lm_head_topk(W_lm: np.ndarray, attn_o: np.ndarray, k: int):
    """Eq. 6 with one LM head shared by the K rows."""
    logits = linear(W_lm, attn_o)
    idx = np.zeros((logits.shape[0], k), dtype=np.int32)
    val = np.zeros((logits.shape[0], k), dtype=F64)
    for r in range(logits.shape[0]):
        idx[r], val[r] = topk_sorted(logits[r], k)
    return logits, idx, val


def draft(dw: Dict[str, object], h_t: np.ndarray, tok: int, sal_k: List[np.ndarray],
          sal_v: List[np.ndarray], n_heads: int, topk: int, eps: float, theta: float) -> Dict[str, object]:
    """Eq. 1-6 for one batch element.

    dw holds float arrays: embed [V,d], fc [2][d,2d], sal [2]{layer}, mlp [K,d,d],
    pe [K,d], aeb_wq/wk/wv/wo [d,d], lm_head [V,d].  sal_k[s], sal_v[s] are the
    committed rows [n_heads, L_s, d_h] of stage s.

    The structural variants of the paper's ablations are read off dw:
      * one adaptation layer for all heads (Sec. 4.3, variant 4): len(dw["sal"]) == 1, every head reads h^1;
      * no position encoding (variant 2): dw["pe"] is None;
      * two self-attention layers in the Auto-embedding Block (Appendix, the "alpha" model): dw["aeb2_wq"]
        .. dw["aeb2_wo"] present; the second layer reads the first one's output;
      * LoRA-like LM head (Appendix): dw["lm_a"] [r,d] and dw["lm_b"] [V,r] present; logits = lm_b (lm_a x).
    """
    e = _f(dw["embed"][tok])
    out: Dict[str, object] = {"x": [], "h": [], "k_new": [], "v_new": []}
    u = _f(h_t)
    n_stages = len(dw["sal"])
    for s in range(n_stages):
        x = fc_concat(dw["fc"][s], u, e)
        h, k_new, v_new = sal_stage(x, dw["sal"][s], sal_k[s], sal_v[s], n_heads, eps, theta)
        out["x"].append(x); out["h"].append(h); out["k_new"].append(k_new); out["v_new"].append(v_new)
        u = h
    K, d = dw["mlp"].shape[0], dw["mlp"].shape[1]
    pe = dw.get("pe")
    Hp = head_inputs(out["h"][0], out["h"][-1], dw["mlp"], np.zeros((K, d)) if pe is None else pe)
    attn_o = bi_self_attention(Hp, dw["aeb_wq"], dw["aeb_wk"], dw["aeb_wv"], dw["aeb_wo"], n_heads)
    if dw.get("aeb2_wq") is not None:
        attn_o = bi_self_attention(attn_o, dw["aeb2_wq"], dw["aeb2_wk"], dw["aeb2_wv"], dw["aeb2_wo"], n_heads)
    if dw.get("lm_a") is not None:
        low = linear(dw["lm_a"], attn_o)                       # [K, r]
        logits, idx, val = lm_head_topk(dw["lm_b"], low, topk)
    else:
        logits, idx, val = lm_head_topk(dw["lm_head"], attn_o, topk)
    out.update(Hp=Hp, attn_o=attn_o, logits=logits, topk_idx=idx, topk_val=val)
    return out


# ----------------------------------------------------------------------------
# Draft tree (Appendix "Draft Tree"; Sec. 2 "Tree Attention")
# ----------------------------------------------------------------------------
@dataclass
class Tree:
    K: int
    paths: List[Tuple[int, ...]]      # node i -> rank path (root = ())
    parent: np.ndarray                # [T] int32, root = -1
    depth: np.ndarray                 # [T] int32
    rank: np.ndarray                  # [T] int32, rank within its head's top-k; root = -1
    mask: np.ndarray                  # [T, T] bool: mask[i, j] = j is i or an ancestor of i
    leaves: List[int]
    retrieve: np.ndarray              # [n_leaves, K+1] node ids root..leaf, -1 padded

    @property
    def T(self) -> int:
        return len(self.paths)


def tree_from_paths(paths: Sequence[Sequence[int]], K: int) -> Tree:
    """Node order: root first, then by (depth, rank path).  Every prefix of a
    path must itself be present (a node needs its parent)."""
    ps = sorted({tuple(int(r) for r in p if r >= 0) for p in paths}, key=lambda p: (len(p), p))
    if any(len(p) == 0 for p in ps):
        raise ValueError("the root is implicit")
    if len(ps) != len(paths):
        raise ValueError("duplicate path")
    nodes = [()] + ps
    index = {p: i for i, p in enumerate(nodes)}
    T = len(nodes)
    parent = np.full(T, -1, dtype=np.int32)
    depth = np.zeros(T, dtype=np.int32)
    rank = np.full(T, -1, dtype=np.int32)
    for i, p in enumerate(nodes[1:], start=1):
        if len(p) > K:
            raise ValueError("path deeper than K")
        if p[:-1] not in index:
            raise ValueError("missing parent")
        parent[i] = index[p[:-1]]
        depth[i] = len(p)
        rank[i] = p[-1]
    mask = np.zeros((T, T), dtype=bool)
    for i in range(T):
        j = i
        while j >= 0:
            mask[i, j] = True
            j = parent[j]
    has_child = np.zeros(T, dtype=bool)
    has_child[parent[1:]] = True
    leaves = [i for i in range(T) if not has_child[i]]
    retrieve = np.full((len(leaves), K + 1), -1, dtype=np.int32)
    for li, leaf in enumerate(leaves):
        chain = []
        j = leaf
        while j >= 0:
            chain.append(j)
            j = parent[j]
        chain.reverse()
        retrieve[li, :len(chain)] = chain
    return Tree(K, nodes, parent, depth, rank, mask, leaves, retrieve)


def tree_tokens(tree: Tree, root_tok: int, topk_idx: np.ndarray, kv_len: int):
    """Node i at depth m >= 1 carries the rank[i]-th candidate of head m; the root is
    the token the target just sampled.  Position = committed length + depth."""
    tok = np.zeros(tree.T, dtype=np.int32)
    pos = np.zeros(tree.T, dtype=np.int32)
    for i in range(tree.T):
        m = int(tree.depth[i])
        tok[i] = root_tok if m == 0 else topk_idx[m - 1][tree.rank[i]]
        pos[i] = kv_len + m
    return tok, pos


def tree_attention(q: np.ndarray, k_rows: np.ndarray, v_rows: np.ndarray, L: int, mask: np.ndarray) -> np.ndarray:
    """Tree-masked attention.  q [T, n_h, d_h]; k_rows, v_rows [n_h, L+T, d_h] with the
    tree's own keys/values at rows [L, L+T) in node order.  Node i sees rows
    [0, L) and rows L + j for every j with mask[i, j]."""
    q = _f(q)
    T, n_h, d_h = q.shape
    out = np.zeros_like(q)
    kr, vr = _f(k_rows), _f(v_rows)
    for h in range(n_h):
        for i in range(T):
            sel = L + np.nonzero(mask[i])[0]
            out[i, h] = attend_segments(q[i, h], [(kr[h][:L], vr[h][:L]), (kr[h][sel], vr[h][sel])])
    return out


def target_forward(tw: Dict[str, object], tree_tok: np.ndarray, tree_pos: np.ndarray, mask: np.ndarray,
                   k_caches: List[np.ndarray], v_caches: List[np.ndarray], n_heads: int, eps: float,
                   theta: float, keep: bool = False) -> Dict[str, object]:
    """The target's forward pass over the T tree tokens (tree attention in every layer),
    then the final norm, the LM head and the per-node argmax (ties -> lowest id)."""
    x = _f(tw["embed"])[np.asarray(tree_tok)]
    per_layer = []
    for li, lw in enumerate(tw["layers"]):
        x, k_new, v_new, q, attn = decoder_layer_rows(
            x, lw, k_caches[li], v_caches[li], list(tree_pos), mask, n_heads, eps, theta)
        if keep:
            per_layer.append(dict(x=x.copy(), k_new=k_new, v_new=v_new, q=q, attn=attn))
    hidden = rmsnorm(x, tw["final_norm"], eps)
    logits = linear(tw["lm_head"], hidden)
    tgt = np.array([row_argmax(r) for r in logits], dtype=np.int32)
    return dict(hidden=hidden, logits=logits, tgt=tgt, layers=per_layer)


def row_argmax(v: np.ndarray) -> int:
    """Index of the maximum; the lowest index among exact ties."""
    v = _f(v)
    return int(np.nonzero(v == np.max(v))[0][0])


def accept_greedy(tree: Tree, tree_tok: np.ndarray, tgt: np.ndarray):
    """Greedy verification: a node is accepted iff its parent is accepted and its token
    equals the target's argmax at the parent; the result is the deepest accepted node.
    Returns (accept_len, path node ids [K+1] -1 padded, next_tok, best_node)."""
    T = tree.T
    ok = np.zeros(T, dtype=bool)
    ok[0] = True
    for i in range(1, T):                     # parents precede children in node order
        p = tree.parent[i]
        ok[i] = ok[p] and (tree_tok[i] == tgt[p])
    best = 0
    for i in range(1, T):
        if ok[i] and tree.depth[i] > tree.depth[best]:
            best = i
    path = np.full(tree.K + 1, -1, dtype=np.int32)
    chain = []
    j = best
    while j >= 0:
        chain.append(j)
        j = tree.parent[j]
    chain.reverse()
    path[:len(chain)] = chain
    return int(tree.depth[best]), path, int(tgt[best]), int(best)


def accept_typical(tree: Tree, tree_tok: np.ndarray, logits: np.ndarray, temperature: float, eps: float,
                   delta: float, u: float):
    """Acceptance under random sampling (Table 2, Temperature = 0.7).

    PARITY UNPINNED BY THE PAPER: it reports results at this temperature but states no acceptance rule.  The
    reading taken is the typical-acceptance criterion of the multi-head decoding framework whose tree and
    settings the paper adopts (its reference cai2024medusa): with p_j = softmax(logits_j / temperature) the
    target's distribution after node j and H(p_j) its entropy in nats, a child i of j is accepted iff j is and

        p_j(tree_tok[i]) > min(eps, delta * exp(-H(p_j))).

    The result is the deepest accepted node (the lowest id among equals, as in the greedy rule).  The token
    that follows it is drawn from p_best by inverting its cumulative distribution, taken in vocabulary order,
    at the caller's uniform number u in [0, 1): the first v with sum_{w <= v} p_best(w) > u (the last token of
    non-zero probability if rounding leaves none).

    Returns (accept_len, path [K+1] -1 padded, next_tok, best_node, margin, threshold) where margin[i] = p -
    threshold of node i (margin[0] = +inf) and threshold[i] the threshold it was held against: a test that
    compares a float32 implementation can see which decisions are near ties."""
    T = tree.T
    lg = _f(logits) / float(temperature)
    p = np.stack([softmax(lg[j]) for j in range(T)])
    H = np.array([-np.sum(p[j][p[j] > 0] * np.log(p[j][p[j] > 0])) for j in range(T)])
    thr = np.minimum(float(eps), float(delta) * np.exp(-H))
    margin = np.full(T, np.inf)
    held = np.zeros(T)
    ok = np.zeros(T, dtype=bool)
    ok[0] = True
    for i in range(1, T):                     # parents precede children in node order
        j = tree.parent[i]
        held[i] = thr[j]
        margin[i] = p[j][int(tree_tok[i])] - thr[j]
        ok[i] = ok[j] and margin[i] > 0.0
    best = 0
    for i in range(1, T):
        if ok[i] and tree.depth[i] > tree.depth[best]:
            best = i
    path = np.full(tree.K + 1, -1, dtype=np.int32)
    chain = []
    j = best
    while j >= 0:
        chain.append(j)
        j = tree.parent[j]
    chain.reverse()
    path[:len(chain)] = chain
    acc, nxt = 0.0, -1
    for v in range(p.shape[1]):
        acc += p[best][v]
        if acc > u:
            nxt = v
            break
    if nxt < 0:
        nxt = int(np.nonzero(p[best] > 0)[0][-1])
    return int(tree.depth[best]), path, int(nxt), int(best), margin, held


# ----------------------------------------------------------------------------
# One whole step for one batch element
# ----------------------------------------------------------------------------
def step(dw, tw, tree: Tree, h_t, tok, sal_k, sal_v, k_caches, v_caches, n_heads, topk, eps, theta):
    d = draft(dw, h_t, tok, sal_k, sal_v, n_heads, topk, eps, theta)
    L = k_caches[0].shape[1]
    tree_tok, tree_pos = tree_tokens(tree, tok, d["topk_idx"], L)
    t = target_forward(tw, tree_tok, tree_pos, tree.mask, k_caches, v_caches, n_heads, eps, theta)
    a, path, nxt, best = accept_greedy(tree, tree_tok, t["tgt"])
    return dict(draft=d, tree_tok=tree_tok, tree_pos=tree_pos, target=t,
                accept_len=a, path=path, next_tok=nxt, best_node=best)


# ----------------------------------------------------------------------------
# The decode loop around the step (Sec. 2 "Speculative Decoding"; Eq. 1's kv_{1:t-1})
# ----------------------------------------------------------------------------
def commit_rows(cache_rows: np.ndarray, new_rows: np.ndarray, path_nodes: Sequence[int]) -> np.ndarray:
    """Committed cache after a step: the old rows followed by the tree rows of the accepted path
    (root first), in path order.  cache_rows [n_heads, L, d_h], new_rows [n_heads, T, d_h]."""
    return np.concatenate([_f(cache_rows), _f(new_rows)[:, list(path_nodes), :]], axis=1)


def draft_catchup(dw: Dict[str, object], h_rows: np.ndarray, toks: Sequence[int], sal_k: List[np.ndarray],
                  sal_v: List[np.ndarray], n_heads: int, topk: int, eps: float, theta: float):
    """Eq. 1 applied to several newly committed positions, oldest first: position j contributes
    the pair (h_j, token that follows it) and appends one row to each stage's cache; the heads
    (Eq. 2-6) of the LAST position are the draft.  Returns (draft of the last position, caches).
    The number of stages is the number of adaptation layers in dw (one in the ablation of Sec. 4.3
    that keeps a single adaptation layer): sal_k, sal_v hold one cache per stage."""
    sal_k = [_f(k) for k in sal_k]
    sal_v = [_f(v) for v in sal_v]
    n_stages = len(dw["sal"])
    d = None
    for h_t, tok in zip(h_rows, toks):
        d = draft(dw, h_t, int(tok), sal_k, sal_v, n_heads, topk, eps, theta)
        for s in range(n_stages):
            sal_k[s] = np.concatenate([sal_k[s], d["k_new"][s][:, None, :]], axis=1)
            sal_v[s] = np.concatenate([sal_v[s], d["v_new"][s][:, None, :]], axis=1)
    return d, sal_k, sal_v


def generate(dw, tw, tree: Tree, prompt: Sequence[int], n_steps: int, n_heads: int, topk: int, eps: float,
             theta: float):
    """Speculate-and-verify decoding from a prompt (at least two tokens).  The target runs causally over
    prompt[:-1]; prompt[-1] is the first root.  Every step: draft over the newly committed
    positions, tree, verification, greedy acceptance, commit.  Returns (emitted tokens, per-step
    records); the emitted tokens are the target's own greedy continuation of the prompt."""
    prompt = [int(t) for t in prompt]
    P = len(prompt) - 1
    d_h = _f(tw["embed"]).shape[1] // n_heads
    empty = [np.zeros((n_heads, 0, d_h)) for _ in tw["layers"]]
    pre = target_forward(tw, np.asarray(prompt[:-1]), np.arange(P), np.tril(np.ones((P, P), dtype=bool)),
                         empty, empty, n_heads, eps, theta, keep=True)
    k_caches = [l["k_new"] for l in pre["layers"]]
    v_caches = [l["v_new"] for l in pre["layers"]]
    sal_k = [np.zeros((n_heads, 0, d_h)) for _ in dw["sal"]]
    sal_v = [np.zeros((n_heads, 0, d_h)) for _ in dw["sal"]]
    h_rows, toks, root = pre["hidden"], prompt[1:], prompt[-1]
    emitted, records = [], []
    for _ in range(n_steps):
        d, sal_k, sal_v = draft_catchup(dw, h_rows, toks, sal_k, sal_v, n_heads, topk, eps, theta)
        L = k_caches[0].shape[1]
        tree_tok, tree_pos = tree_tokens(tree, root, d["topk_idx"], L)
        t = target_forward(tw, tree_tok, tree_pos, tree.mask, k_caches, v_caches, n_heads, eps, theta, keep=True)
        a, path, nxt, best = accept_greedy(tree, tree_tok, t["tgt"])
        nodes = [int(n) for n in path[:a + 1]]
        new_toks = [int(tree_tok[n]) for n in nodes[1:]] + [int(nxt)]
        emitted += new_toks
        records.append(dict(draft=d, tree_tok=tree_tok, target=t, accept_len=a, path=path, next_tok=nxt,
                            nodes=nodes, h_rows=h_rows, toks=list(toks), kv_len=L))
        k_caches = [commit_rows(k_caches[li], t["layers"][li]["k_new"], nodes) for li in range(len(k_caches))]
        v_caches = [commit_rows(v_caches[li], t["layers"][li]["v_new"], nodes) for li in range(len(v_caches))]
        h_rows, toks, root = t["hidden"][nodes], new_toks, int(nxt)
    return emitted, records
