// C-ABI layer of libamph: argument checks, the host side of the draft tree, workspace layout, and the
// launch sequences of amph_draft / amph_target_forward.  All arithmetic lives in the kernels.
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <map>
#include <new>
#include <string>
#include <vector>

#include "kernels.h"

using namespace amph;

// Scratch of amph_verify_attn_static: the key-split partials of the verification attention, for callers that
// cannot bring a workspace or allocate one.  Every GPU holds its own copy at its own address; host code never
// uses the array's name as an address, only the pointer hipGetSymbolAddress returns for the current device.
static __device__ __align__(256) unsigned char scratch[AMPH_STATIC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
void *g_scratch_ptr[MAX_DEVICES] = {};      // device address of `scratch` on each device that created a context

// Address of this device's copy of `scratch` (resolved once per device, with that device current).
hipError_t scratch_for_current_device(int *dev_out, void **ptr_out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[dev] = p;
  }
  *dev_out = dev;
  *ptr_out = g_scratch_ptr[dev];
  return hipSuccess;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct WsLayout {   // byte offsets into the caller's workspace
  size_t x, q, att, y, act, h[2], Hp, Qa, Ka, Va, ctxa, attn_o, logits, topk_ws;                 // draft
  size_t xres, xn, qb, attb, actb, slabs, amax_val, amax_idx, ver_part, tgt_tmp, row_stats, rope_cs, xt;  // target
  size_t slabs_floats, ver_part_floats;
  size_t total;
};

}  // namespace

struct amph_ctx {
  amph_config cfg;
  hipStream_t stream = nullptr;
  uint32_t *dev_status = nullptr;     // device, sticky (the context's only device allocation)
  int device = -1;                    // the device that was current in amph_create
  void *static_scratch = nullptr;     // that device's copy of the library's static scratch array
  std::string err = "";
  WsLayout ws;
  int esz = 2;
  int prof_kind = -1;                 // amph_kernel_kind being timed, -1 = none
  std::vector<hipEvent_t> prof_ev;    // start/stop pairs
  size_t prof_used = 0;
  int prof_every = 1;                 // one launch in this many is timed
  long long prof_seen = 0;            // launches of prof_kind since it was selected
  int verify_kernel = -1;             // amph_verify_kernel: -1 by shape, 0 registers, 1 LDS ring
};

struct amph_tree {
  int T = 0, K = 0, n_leaves = 0;
  std::vector<int32_t> parent, depth, rank, retrieve;
  std::vector<uint64_t> mask;
  // device copies, one allocation made by amph_tree_create: mask, then parent, depth, rank
  void *d_block = nullptr;
  int32_t *d_parent = nullptr, *d_depth = nullptr, *d_rank = nullptr;
  uint64_t *d_mask = nullptr;
};

namespace {

amph_status fail(amph_ctx *ctx, amph_status st, const std::string &msg) {
  if (ctx) ctx->err = msg;
  return st;
}
amph_status hip_fail(amph_ctx *ctx, hipError_t e, const char *where) {
  return fail(ctx, AMPH_EHIP, std::string(where) + ": " + hipGetErrorString(e));
}
#define HIP_TRY(ctx, expr)                                  \
  do {                                                      \
    hipError_t e__ = (expr);                                \
    if (e__ != hipSuccess) return hip_fail(ctx, e__, #expr); \
  } while (0)

// Launch `expr`; when its kind is the one being profiled, bracket it with a pair of events on the stream.
#define PROF_TRY(ctx, kind, expr)                                                              \
  do {                                                                                         \
    const bool p__ = ((ctx)->prof_kind == (kind)) && ((ctx)->prof_seen++ % (ctx)->prof_every == 0) && \
                     ((ctx)->prof_used < (ctx)->prof_ev.size() / 2);                                   \
    if (p__) HIP_TRY(ctx, hipEventRecord((ctx)->prof_ev[2 * (ctx)->prof_used], (ctx)->stream));       \
    HIP_TRY(ctx, expr);                                                                        \
    if (p__) {                                                                                 \
      HIP_TRY(ctx, hipEventRecord((ctx)->prof_ev[2 * (ctx)->prof_used + 1], (ctx)->stream));   \
      (ctx)->prof_used++;                                                                      \
    }                                                                                          \
  } while (0)

// The same for a matrix-core GEMM: the launch carries the two events, which then hold the kernel's own begin and
// end time stamps (no marker on the stream, nothing but the kernel between them).
#define PROF_GEMM(ctx, kind, T, st, epi, args)                                                 \
  do {                                                                                         \
    const bool p__ = ((ctx)->prof_kind == (kind)) && ((ctx)->prof_seen++ % (ctx)->prof_every == 0) && \
                     ((ctx)->prof_used < (ctx)->prof_ev.size() / 2);                                   \
    if (p__) {                                                                                 \
      HIP_TRY(ctx, launch_gemm<T>(st, epi, args, (ctx)->prof_ev[2 * (ctx)->prof_used],         \
                                  (ctx)->prof_ev[2 * (ctx)->prof_used + 1]));                  \
      (ctx)->prof_used++;                                                                      \
    } else {                                                                                   \
      HIP_TRY(ctx, launch_gemm<T>(st, epi, args));                                             \
    }                                                                                          \
  } while (0)

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

WsLayout make_layout(const amph_config &c) {
  WsLayout w{};
  const size_t esz = (c.dtype == AMPH_BF16) ? 2 : 4;
  const size_t B = c.batch, d = c.d_model, f = c.d_ffn, V = c.vocab, K = c.K, BK = B * K;
  const size_t M = B * (size_t)c.max_tree;
  size_t at = 0;
  auto take = [&](size_t bytes) { size_t o = at; at = align_up(at + bytes, 256); return o; };
  const size_t Mr = B * (K + 1);                // adaptation-layer rows: (batch element, new position) pairs, n_new <= K + 1
  w.x = take(Mr * d * 4); w.q = take(Mr * d * 4); w.att = take(Mr * d * 4); w.y = take(Mr * d * 4);
  w.act = take(Mr * f * 4); w.h[0] = take(Mr * d * 4); w.h[1] = take(Mr * d * 4);
  w.Hp = take(BK * d * 4); w.Qa = take(BK * d * 4); w.Ka = take(BK * d * 4); w.Va = take(BK * d * 4);
  w.ctxa = take(BK * d * 4); w.attn_o = take(BK * d * 4); w.logits = take(BK * V * 4);
  w.topk_ws = take(std::max(std::max(topk_ws_floats((int)BK, c.vocab, c.topk), topk_ws_floats((int)M, c.vocab, 1)),
                            lmtk_ws_floats((int)BK, c.topk)) * 4);
  const size_t Mp = (M + 31) / 32 * 32;         // activations may be kept in 32-row tiles for the wide GEMM
  w.xres = take(M * d * 4); w.xn = take(Mp * d * esz); w.qb = take(M * d * esz); w.attb = take(Mp * d * esz);
  w.actb = take(Mp * f * esz);
  // partial slabs of the split-K GEMMs (Wo, W_down: up to 8 slabs of [M, d]); amph_gemm may use the same area
  w.slabs_floats = std::max((size_t)8 * M * d, (size_t)8 * 1024 * 1024);
  w.slabs = take(w.slabs_floats * 4);
  const size_t tilesV = (V + 31) / 32 + 1;      // upper bound on the LM head's tiles (at least two 16-row blocks each)
  w.amax_val = take(tilesV * M * 4); w.amax_idx = take(tilesV * M * 4);
  w.xt = take(gemm_xt_bytes((int)M, (int)std::max(d, f), (int)esz));     // fragment-tiled activations of the wide GEMM
  size_t vfl = 0;                                           // any tree size up to max_tree may be used
  for (int t = 1; t <= c.max_tree; ++t) vfl = std::max(vfl, verify_ws_floats(c.batch, t, c.n_heads, c.head_dim, c.max_kv, (int)esz));
  w.ver_part = take(vfl * 4);
  w.ver_part_floats = vfl;
  w.tgt_tmp = take(M * 4);
  w.row_stats = take(M * 16);
  w.rope_cs = take(M * (size_t)(c.head_dim / 2) * 8);
  w.total = at;
  return w;
}

// Device copies of a tree's tables on the current device: one allocation, one blocking copy.  Called from
// amph_tree_create only (a set-up call), so that no call of the step allocates or blocks.
hipError_t tree_upload(amph_tree *t) {
  const size_t n = t->T;
  const size_t bytes = n * 16 + 3 * n * 4;
  hipError_t e = hipMalloc(&t->d_block, bytes);
  if (e != hipSuccess) { t->d_block = nullptr; return e; }
  std::vector<unsigned char> host(bytes);
  std::memcpy(host.data(), t->mask.data(), n * 16);
  std::memcpy(host.data() + n * 16, t->parent.data(), n * 4);
  std::memcpy(host.data() + n * 16 + n * 4, t->depth.data(), n * 4);
  std::memcpy(host.data() + n * 16 + 2 * n * 4, t->rank.data(), n * 4);
  e = hipMemcpy(t->d_block, host.data(), bytes, hipMemcpyHostToDevice);
  if (e != hipSuccess) { (void)hipFree(t->d_block); t->d_block = nullptr; return e; }
  unsigned char *base = (unsigned char *)t->d_block;
  t->d_mask = (uint64_t *)base;
  t->d_parent = (int32_t *)(base + n * 16);
  t->d_depth = (int32_t *)(base + n * 16 + n * 4);
  t->d_rank = (int32_t *)(base + n * 16 + 2 * n * 4);
  return hipSuccess;
}

template <typename T>
amph_status draft_impl(amph_ctx *ctx, const amph_draft_w *w, const float *h_new, const int32_t *tok_new, int R,
                       const int32_t *n_valid, void *sal_kv, int32_t *sal_len, int32_t *topk_idx, float *topk_val,
                       float *logits, void *workspace) {
  const amph_config &c = ctx->cfg;
  const int B = c.batch, d = c.d_model, f = c.d_ffn, V = c.vocab, K = c.K, n_h = c.n_heads, d_h = c.head_dim;
  const int M = B * R;                     // rows of the adaptation layers: (batch element, new position)
  hipStream_t st = ctx->stream;
  char *ws = (char *)workspace;
  auto F = [&](size_t off) { return (float *)(ws + off); };
  float *x = F(ctx->ws.x), *q = F(ctx->ws.q), *att = F(ctx->ws.att), *y = F(ctx->ws.y), *act = F(ctx->ws.act);
  float *h[2] = {F(ctx->ws.h[0]), F(ctx->ws.h[1])};
  const size_t stage_stride = (size_t)B * 2 * n_h * c.max_kv * d_h;      // elements of T
  for (int s = 0; s < c.n_stages; ++s) {
    const float *u = (s == 0) ? h_new : h[0];
    void *kv_stage = (T *)sal_kv + s * stage_stride;
    PROF_TRY(ctx, AMPH_K_FC, launch_fc_concat<T>(st, w->fc[s], u, w->embed, tok_new, V, d, M, x, ctx->dev_status));
    PROF_TRY(ctx, AMPH_K_SAL_QKV, launch_sal_qkv<T>(st, w->sal[s], x, d, n_h, d_h, M, c.rms_eps, c.rope_theta, sal_len, c.max_kv, kv_stage,
                                   q, ctx->dev_status, R, n_valid));
    // Nothing reads the LAST stage's output at any but the last live position of a sequence (the heads read that one;
    // the earlier positions only have to leave their cache rows, which the projections above wrote): there the
    // attention, Wo and the FFN run over one row per sequence instead of R.
    const bool last_rows_only = (R > 1 && s == c.n_stages - 1);
    const int Ms = last_rows_only ? B : M;
    const float *res = x;
    if (last_rows_only) {
      float *x_last = att + (size_t)B * d;        // att holds B * (K + 1) rows and the attention now fills the first B only
      HIP_TRY(ctx, launch_gather_rows(st, x, B, R, d, n_valid, x_last));
      res = x_last;
    }
    PROF_TRY(ctx, AMPH_K_SAL_ATTN, launch_sal_attn<T>(st, q, kv_stage, sal_len, B, n_h, d_h, c.max_kv, att, R, n_valid,
                                                      last_rows_only ? 1 : 0));
    PROF_TRY(ctx, AMPH_K_SAL_WO, launch_linear<T>(st, w->sal[s].wo, nullptr, nullptr, 1, d, d, att, d, Ms, res, y, nullptr, nullptr, d));
    PROF_TRY(ctx, AMPH_K_SAL_GATEUP, launch_gate_up<T>(st, w->sal[s], y, d, f, Ms, c.rms_eps, act));
    PROF_TRY(ctx, AMPH_K_SAL_DOWN, launch_linear<T>(st, w->sal[s].w_down, nullptr, nullptr, 1, d, f, act, f, Ms, y, h[s], nullptr, nullptr, d));
  }
  // the heads (Eq. 2-6) read the last live position of every batch element; with one adaptation layer every
  // head reads that layer's output.  After a catch-up the last stage's output already is one row per sequence.
  const float *h1 = h[0], *h2 = h[c.n_stages - 1];
  if (R > 1) {
    if (c.n_stages == 2) {
      HIP_TRY(ctx, launch_gather_rows(st, h[0], B, R, d, n_valid, x));
      h1 = x;
    } else {
      h1 = h2;
    }
  }
  float *Hp = F(ctx->ws.Hp), *Qa = F(ctx->ws.Qa), *Ka = F(ctx->ws.Ka), *Va = F(ctx->ws.Va), *ctxa = F(ctx->ws.ctxa);
  float *attn_o = F(ctx->ws.attn_o);
  PROF_TRY(ctx, AMPH_K_HEAD_MLP, launch_head_mlp<T>(st, w->mlp, w->pe, h1, h2, d, K, B, Hp));
  const int BK = B * K;
  // Eq. 5, once or twice: q/k/v projections of the K rows, K x K attention per head, output projection
  auto self_attention = [&](const void *wq, const void *wk, const void *wv, const void *wo, const float *in,
                            float *out_rows) -> amph_status {
    for (int r0 = 0; r0 < BK; r0 += 8) {
      const int m = std::min(8, BK - r0);
      const size_t o = (size_t)r0 * d;
      PROF_TRY(ctx, AMPH_K_AEB_QKV, launch_linear<T>(st, wq, wk, wv, 3, d, d, in + o, d, m, nullptr, Qa + o, Ka + o, Va + o, d));
    }
    PROF_TRY(ctx, AMPH_K_AEB_ATTN, launch_aeb_attn(st, Qa, Ka, Va, B, K, n_h, d_h, ctxa));
    for (int r0 = 0; r0 < BK; r0 += 8) {
      const int m = std::min(8, BK - r0);
      const size_t o = (size_t)r0 * d;
      PROF_TRY(ctx, AMPH_K_AEB_WO, launch_linear<T>(st, wo, nullptr, nullptr, 1, d, d, ctxa + o, d, m, nullptr, out_rows + o,
                                    nullptr, nullptr, d));
    }
    return AMPH_OK;
  };
  if (amph_status s1 = self_attention(w->aeb_wq, w->aeb_wk, w->aeb_wv, w->aeb_wo, Hp, attn_o)) return s1;
  const float *head_in = attn_o;
  if (c.aeb_layers == 2) {                 // the second layer reads the first one's output; Hp is free by now
    if (amph_status s2 = self_attention(w->aeb2_wq, w->aeb2_wk, w->aeb2_wv, w->aeb2_wo, attn_o, Hp)) return s2;
    head_in = Hp;
  }
  const void *lm_w = w->lm_head;
  int lm_k = d;
  if (c.lm_rank > 0) {                      // low-rank head: [K rows, r] = lm_a x first, then the [V, r] matrix
    for (int r0 = 0; r0 < BK; r0 += 8) {
      const int m = std::min(8, BK - r0);
      PROF_TRY(ctx, AMPH_K_LM_HEAD, launch_linear<T>(st, w->lm_a, nullptr, nullptr, 1, c.lm_rank, d, head_in + (size_t)r0 * d, d, m,
                                    nullptr, Qa + (size_t)r0 * c.lm_rank, nullptr, nullptr, c.lm_rank));
    }
    head_in = Qa; lm_w = w->lm_b; lm_k = c.lm_rank;
  }
  // Eq. 6: the LM head's launches leave per-workgroup top-k candidates (and the logits only if the caller wants them);
  // the merge kernel picks every row's top k and advances the adaptation layers' cache lengths
  float *cand = F(ctx->ws.topk_ws);
  int n_cand = 0;
  PROF_TRY(ctx, AMPH_K_LM_HEAD, launch_lmhead_cands<T>(st, lm_w, V, lm_k, head_in, BK, c.topk, logits, cand, &n_cand));
  PROF_TRY(ctx, AMPH_K_TOPK, launch_topk_merge(st, cand, reinterpret_cast<const int *>(cand + (size_t)BK * n_cand), BK, n_cand, V, c.topk,
                                               topk_idx, topk_val, sal_len, B, R, n_valid, c.max_kv));
  return AMPH_OK;
}

template <typename T>
amph_status verify_impl(amph_ctx *ctx, const amph_tree *tree, const void *q, const void *k_cache, const void *v_cache,
                        const int32_t *kv_len, void *out, float *partials, size_t partials_floats, int out_tiles = 0) {
  const amph_config &c = ctx->cfg;
  VerifyArgs a{};
  a.q = q; a.k_cache = k_cache; a.v_cache = v_cache; a.out = out; a.kv_len = kv_len; a.mask_bits = tree->d_mask;
  a.B = c.batch; a.T = tree->T; a.n_heads = c.n_heads; a.d_h = c.head_dim; a.max_kv = c.max_kv;
  a.partials = partials;
  a.partials_cap = partials_floats;
  a.dev_status = ctx->dev_status;
  a.kernel = ctx->verify_kernel;
  a.out_tiles = out_tiles;
  PROF_TRY(ctx, AMPH_K_VERIFY, launch_verify_attn<T>(ctx->stream, a));
  return AMPH_OK;
}

template <typename T>
amph_status target_impl(amph_ctx *ctx, const amph_tree *tree, const amph_layer_w *layers, const amph_layer_tiled *tiled,
                        int n_layers, const void *embed, const void *final_norm, const void *lm_head,
                        const void *lm_head_tiled, const int32_t *tree_tok, const int32_t *tree_pos,
                        void *k_caches, void *v_caches, const int32_t *kv_len, float *hidden_out, float *logits_out,
                        int32_t *tgt_argmax, void *workspace) {
  const amph_config &c = ctx->cfg;
  const int B = c.batch, d = c.d_model, f = c.d_ffn, V = c.vocab, n_h = c.n_heads, d_h = c.head_dim, Tn = tree->T;
  const int M = B * Tn;
  const int mblocks = (M + 63) / 64;
  hipStream_t st = ctx->stream;
  char *ws = (char *)workspace;
  float *xres = (float *)(ws + ctx->ws.xres);
  float *slabs = (float *)(ws + ctx->ws.slabs);
  float2 *rope_cs = (float2 *)(ws + ctx->ws.rope_cs);
  void *xn = ws + ctx->ws.xn, *qb = ws + ctx->ws.qb, *attb = ws + ctx->ws.attb, *actb = ws + ctx->ws.actb;
  const size_t cache_layer = (size_t)B * n_h * c.max_kv * d_h;     // elements of T per layer
  const size_t slab = (size_t)M * d;
  GemmArgs g{};
  g.dev_status = ctx->dev_status;
  g.M = M; g.T_nodes = Tn; g.n_heads = n_h; g.d_h = d_h; g.max_kv = c.max_kv;
  g.rope_cs = rope_cs; g.kv_len = kv_len; g.split_k = 1;
  g.xt = ws + ctx->ws.xt;
  auto split_for = [&](int rows, int Kd, bool has_tiled) {
    int s = gemm_plan(EPI_STORE, rows, Kd, (int)sizeof(T), M, 0, has_tiled).split;
    while (s > 1 && (size_t)s * slab > ctx->ws.slabs_floats) s /= 2;
    return s;
  };
  RopeTable rope_req;                     // written by the kernel that gathers the embeddings
  rope_req.pos = tree_pos; rope_req.d_h = d_h; rope_req.theta = c.rope_theta; rope_req.cs = rope_cs;
  int pending = 0;                        // slabs of the previous GEMM still to be added to the residual stream
  for (int li = 0; li < n_layers; ++li) {
    const amph_layer_w &lw = layers[li];
    const amph_layer_tiled lt = tiled ? tiled[li] : amph_layer_tiled{nullptr, nullptr, nullptr, nullptr};
    void *kc = (T *)k_caches + (size_t)li * cache_layer, *vc = (T *)v_caches + (size_t)li * cache_layer;
    const int s_wo = split_for(d, d, lt.wo != nullptr), s_down = split_for(d, f, lt.down != nullptr);
    // Where the consumer of an activation tensor is the wide GEMM (enough rows, tiled weights), its producer writes
    // it in that kernel's tiled layout straight away instead of leaving a copy to be made.
    const int xt_tiles = (M + 31) / 32;
    const bool w_qkv = gemm_is_wide(M, lt.qkv != nullptr), w_wo = gemm_is_wide(M, lt.wo != nullptr);
    const bool w_gu = gemm_is_wide(M, lt.gate_up != nullptr), w_down = gemm_is_wide(M, lt.down != nullptr);
    PROF_TRY(ctx, AMPH_K_T_RMSNORM, launch_norm_fold<T>(st, xres, embed, li == 0 ? tree_tok : nullptr, V, slabs, pending,
                                                        slab, lw.rms1, M, d, c.rms_eps, xn, nullptr, ctx->dev_status,
                                                        w_qkv ? xt_tiles : 0, li == 0 ? rope_req : RopeTable{}));
    GemmArgs a = g;
    a.w0 = lw.wq; a.w1 = lw.wk; a.w2 = lw.wv; a.wt = lt.qkv; a.n_seg = 3; a.seg_rows = d; a.Kd = d; a.x = xn;
    a.x_tiled = w_qkv;
    a.q_out = qb; a.k_cache = kc; a.v_cache = vc;
    PROF_GEMM(ctx, AMPH_K_T_QKV, T, st, EPI_QKV_ROPE, a);
    if (amph_status s = verify_impl<T>(ctx, tree, qb, kc, vc, kv_len, attb, (float *)(ws + ctx->ws.ver_part), ctx->ws.ver_part_floats,
                                       w_wo ? xt_tiles : 0))
      return s;
    a = g;
    a.w0 = lw.wo; a.wt = lt.wo; a.n_seg = 1; a.seg_rows = d; a.Kd = d; a.x = attb; a.out = slabs; a.split_k = s_wo;
    a.x_tiled = w_wo;
    PROF_GEMM(ctx, AMPH_K_T_WO, T, st, EPI_STORE, a);
    PROF_TRY(ctx, AMPH_K_T_RMSNORM, launch_norm_fold<T>(st, xres, nullptr, nullptr, V, slabs, s_wo, slab, lw.rms2, M, d,
                                                        c.rms_eps, xn, nullptr, ctx->dev_status, w_gu ? xt_tiles : 0));
    a = g;
    a.w0 = lw.w_gate; a.w1 = lw.w_up; a.wt = lt.gate_up; a.n_seg = 2; a.seg_rows = f; a.Kd = d; a.x = xn; a.act = actb;
    a.x_tiled = w_gu;
    a.act_tiles = (w_gu && w_down) ? xt_tiles : 0;         // only the wide kernel's epilogue can write the tiled form
    PROF_GEMM(ctx, AMPH_K_T_GATEUP, T, st, EPI_SWIGLU, a);
    a = g;
    a.w0 = lw.w_down; a.wt = lt.down; a.n_seg = 1; a.seg_rows = d; a.Kd = f; a.x = actb; a.out = slabs; a.split_k = s_down;
    a.x_tiled = w_gu && w_down;
    PROF_GEMM(ctx, AMPH_K_T_DOWN, T, st, EPI_STORE, a);
    pending = s_down;
  }
  const bool w_lm = gemm_is_wide(M, lm_head_tiled != nullptr);
  PROF_TRY(ctx, AMPH_K_T_RMSNORM, launch_norm_fold<T>(st, xres, embed, n_layers == 0 ? tree_tok : nullptr, V, slabs, pending,
                                                      slab, final_norm, M, d, c.rms_eps, xn, hidden_out, ctx->dev_status,
                                                      w_lm ? (M + 31) / 32 : 0));
  GemmArgs a = g;
  a.w0 = lm_head; a.wt = lm_head_tiled; a.n_seg = 1; a.seg_rows = V; a.Kd = d; a.x = xn;
  a.x_tiled = w_lm;
  a.logits = logits_out;
  a.amax_val = (float *)(ws + ctx->ws.amax_val); a.amax_idx = (int32_t *)(ws + ctx->ws.amax_idx);
  PROF_GEMM(ctx, AMPH_K_T_LMHEAD, T, st, EPI_ARGMAX, a);
  HIP_TRY(ctx, launch_argmax_fold(st, a.amax_val, a.amax_idx, gemm_plan(EPI_ARGMAX, V, d, (int)sizeof(T), M, 1, lm_head_tiled != nullptr).tiles, M,
                                  tgt_argmax));
  return AMPH_OK;
}

}  // namespace

// =====================================================================================================
extern "C" {

amph_status amph_create(const amph_config *cfg, amph_ctx **out) {
  if (out) *out = nullptr;
  if (!cfg || !out) return AMPH_EINVAL;
  const amph_config &c = *cfg;
  if (c.dtype != AMPH_F32 && c.dtype != AMPH_BF16) return AMPH_EINVAL;
  if (c.d_model <= 0 || c.n_heads <= 0 || c.head_dim <= 0 || c.d_ffn <= 0 || c.vocab <= 0 || c.batch <= 0 || c.K <= 0 ||
      c.topk <= 0 || c.max_tree <= 0 || c.max_kv <= 0)
    return AMPH_EINVAL;
  if (!(c.rms_eps >= 0.f) || !(c.rope_theta > 1.f)) return AMPH_EINVAL;
  if (c.head_dim != 64 && c.head_dim != 128) return AMPH_ESHAPE;
  if (c.d_model != c.n_heads * c.head_dim) return AMPH_ESHAPE;
  if (c.d_model % 64 || c.d_ffn % 16 || (c.dtype == AMPH_BF16 && c.d_ffn % 32)) return AMPH_ESHAPE;
  if (c.K > AMPH_MAX_HEADS_K || c.topk > AMPH_MAX_TOPK || c.topk > c.vocab || c.max_tree > AMPH_MAX_TREE) return AMPH_ESHAPE;
  if (c.max_kv % 32 || c.max_kv < c.max_tree || c.max_kv > (1 << 24)) return AMPH_ESHAPE;   // (kernels index key steps in 32 bits)
  if (c.vocab > 65536 || c.batch > 64 || (long long)c.batch * c.n_heads > 1000) return AMPH_ESHAPE;
  if ((c.n_stages != 1 && c.n_stages != 2) || (c.aeb_layers != 1 && c.aeb_layers != 2)) return AMPH_EINVAL;
  if (c.lm_rank < 0 || c.lm_rank % 8 || c.lm_rank > c.d_model) return AMPH_ESHAPE;
  amph_ctx *ctx = new (std::nothrow) amph_ctx();
  if (!ctx) return AMPH_EINVAL;
  ctx->cfg = c;
  ctx->esz = (c.dtype == AMPH_BF16) ? 2 : 4;
  ctx->ws = make_layout(c);
  hipError_t e = scratch_for_current_device(&ctx->device, &ctx->static_scratch);
  if (e == hipSuccess) e = hipMalloc(&ctx->dev_status, 256);
  if (e == hipSuccess) e = hipMemset(ctx->dev_status, 0, 256);
  if (e != hipSuccess) {
    if (ctx->dev_status) (void)hipFree(ctx->dev_status);
    delete ctx;
    return AMPH_EHIP;
  }
  *out = ctx;
  return AMPH_OK;
}

void amph_destroy(amph_ctx *ctx) {
  if (!ctx) return;
  for (hipEvent_t e : ctx->prof_ev) (void)hipEventDestroy(e);
  if (ctx->dev_status) (void)hipFree(ctx->dev_status);
  delete ctx;
}

amph_status amph_set_stream(amph_ctx *ctx, void *hip_stream) {
  if (!ctx) return AMPH_EINVAL;
  ctx->stream = reinterpret_cast<hipStream_t>(hip_stream);
  return AMPH_OK;
}

size_t amph_workspace_bytes(const amph_ctx *ctx) { return ctx ? ctx->ws.total : 0; }

const char *amph_last_error(const amph_ctx *ctx) { return ctx ? ctx->err.c_str() : "null context"; }

amph_status amph_device_status(amph_ctx *ctx, uint32_t *host_bits) {
  if (!ctx || !host_bits) return AMPH_EINVAL;
  HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  HIP_TRY(ctx, hipMemcpy(host_bits, ctx->dev_status, 4, hipMemcpyDeviceToHost));
  HIP_TRY(ctx, hipMemset(ctx->dev_status, 0, 4));
  return AMPH_OK;
}

amph_status amph_draft(amph_ctx *ctx, const amph_draft_w *w, const float *h_new, const int32_t *tok_new, int n_new,
                       const int32_t *n_valid, void *sal_kv, int32_t *sal_len, int32_t *topk_idx, float *topk_val,
                       float *logits, void *workspace) {
  if (!ctx) return AMPH_EINVAL;
  if (!w || !h_new || !tok_new || !sal_kv || !sal_len || !topk_idx || !topk_val || !workspace)
    return fail(ctx, AMPH_EINVAL, "amph_draft: null argument");
  if (n_new < 1 || n_new > ctx->cfg.K + 1)
    return fail(ctx, AMPH_ESHAPE, "amph_draft: need 1 <= n_new <= K + 1");
  const amph_config &cf = ctx->cfg;
  const void *ptrs[] = {w->embed, w->fc[0], w->mlp, w->aeb_wq, w->aeb_wk, w->aeb_wv, w->aeb_wo, h_new, sal_kv, workspace};
  for (const void *p : ptrs)
    if (!p || !aligned16(p)) return fail(ctx, AMPH_EINVAL, "amph_draft: null or misaligned (16 B) pointer");
  if (!aligned16(w->pe)) return fail(ctx, AMPH_EINVAL, "amph_draft: misaligned position encoding");
  if (cf.n_stages == 2 && (!w->fc[1] || !aligned16(w->fc[1]))) return fail(ctx, AMPH_EINVAL, "amph_draft: fc[1] missing");
  if (cf.aeb_layers == 2) {
    const void *p2[] = {w->aeb2_wq, w->aeb2_wk, w->aeb2_wv, w->aeb2_wo};
    for (const void *p : p2)
      if (!p || !aligned16(p)) return fail(ctx, AMPH_EINVAL, "amph_draft: second self-attention layer missing or misaligned");
  }
  if (cf.lm_rank > 0 ? (!w->lm_a || !w->lm_b || !aligned16(w->lm_a) || !aligned16(w->lm_b)) : (!w->lm_head || !aligned16(w->lm_head)))
    return fail(ctx, AMPH_EINVAL, "amph_draft: LM head (or its low-rank pair) missing or misaligned");
  for (int s = 0; s < cf.n_stages; ++s) {
    const amph_layer_w &l = w->sal[s];
    const void *lp[] = {l.rms1, l.wq, l.wk, l.wv, l.wo, l.rms2, l.w_gate, l.w_up, l.w_down};
    for (const void *p : lp)
      if (!p || !aligned16(p)) return fail(ctx, AMPH_EINVAL, "amph_draft: null or misaligned SAL weight");
  }
  if (ctx->cfg.dtype == AMPH_BF16)
    return draft_impl<bf16_t>(ctx, w, h_new, tok_new, n_new, n_valid, sal_kv, sal_len, topk_idx, topk_val, logits, workspace);
  return draft_impl<float>(ctx, w, h_new, tok_new, n_new, n_valid, sal_kv, sal_len, topk_idx, topk_val, logits, workspace);
}

amph_status amph_tree_create(const int32_t *paths, int n, int K, amph_tree **out) {
  if (out) *out = nullptr;
  if (!out || n < 0 || K < 1 || (n > 0 && !paths)) return AMPH_EINVAL;
  if (n + 1 > AMPH_MAX_TREE || K > AMPH_MAX_HEADS_K) return AMPH_ESHAPE;
  std::vector<std::vector<int32_t>> nodes;
  nodes.emplace_back();                                     // root
  for (int i = 0; i < n; ++i) {
    std::vector<int32_t> p;
    bool ended = false;
    for (int j = 0; j < K; ++j) {
      const int32_t r = paths[(size_t)i * K + j];
      if (r < 0) { ended = true; continue; }
      if (ended) return AMPH_ETREE;                         // a rank after the padding began
      if (r >= AMPH_MAX_TOPK) return AMPH_ESHAPE;
      p.push_back(r);
    }
    if (p.empty()) return AMPH_ETREE;                       // the root is implicit
    nodes.push_back(p);
  }
  std::sort(nodes.begin() + 1, nodes.end(), [](const std::vector<int32_t> &a, const std::vector<int32_t> &b) {
    if (a.size() != b.size()) return a.size() < b.size();
    return a < b;
  });
  std::map<std::vector<int32_t>, int> index;
  for (size_t i = 0; i < nodes.size(); ++i) {
    if (!index.emplace(nodes[i], (int)i).second) return AMPH_ETREE;   // duplicate
  }
  amph_tree *t = new (std::nothrow) amph_tree();
  if (!t) return AMPH_EINVAL;
  const int T = (int)nodes.size();
  t->T = T; t->K = K;
  t->parent.assign(T, -1); t->depth.assign(T, 0); t->rank.assign(T, -1); t->mask.assign((size_t)T * 2, 0);
  for (int i = 1; i < T; ++i) {
    std::vector<int32_t> par(nodes[i].begin(), nodes[i].end() - 1);
    auto it = index.find(par);
    if (it == index.end()) { delete t; return AMPH_ETREE; }          // missing parent
    t->parent[i] = it->second;
    t->depth[i] = (int32_t)nodes[i].size();
    t->rank[i] = nodes[i].back();
  }
  std::vector<char> has_child(T, 0);
  for (int i = 0; i < T; ++i) {
    for (int j = i; j >= 0; j = t->parent[j]) t->mask[(size_t)i * 2 + (j >> 6)] |= (uint64_t)1 << (j & 63);
    if (t->parent[i] >= 0) has_child[t->parent[i]] = 1;
  }
  for (int i = 0; i < T; ++i) {
    if (has_child[i]) continue;
    std::vector<int32_t> chain;
    for (int j = i; j >= 0; j = t->parent[j]) chain.push_back(j);
    std::reverse(chain.begin(), chain.end());
    chain.resize(K + 1, -1);
    t->retrieve.insert(t->retrieve.end(), chain.begin(), chain.end());
    t->n_leaves++;
  }
  // With a device visible the tables go to the current device now; without one (host-only use of the tree's
  // tables) the tree stays a host object and every device call that takes it reports AMPH_EINVAL.
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) == hipSuccess && n_dev > 0) {
    if (tree_upload(t) != hipSuccess) { delete t; return AMPH_EHIP; }
  } else {
    (void)hipGetLastError();                                // a failed device query leaves a sticky error behind
  }
  *out = t;
  return AMPH_OK;
}

void amph_tree_destroy(amph_tree *t) {
  if (!t) return;
  if (t->d_block) (void)hipFree(t->d_block);
  delete t;
}

amph_status amph_tree_info(const amph_tree *t, int *T, int *n_leaves, const int32_t **parent, const int32_t **depth,
                           const int32_t **rank, const uint64_t **mask_bits, const int32_t **retrieve) {
  if (!t) return AMPH_EINVAL;
  if (T) *T = t->T;
  if (n_leaves) *n_leaves = t->n_leaves;
  if (parent) *parent = t->parent.data();
  if (depth) *depth = t->depth.data();
  if (rank) *rank = t->rank.data();
  if (mask_bits) *mask_bits = t->mask.data();
  if (retrieve) *retrieve = t->retrieve.data();
  return AMPH_OK;
}

static amph_status check_tree(amph_ctx *ctx, const amph_tree *tree, const char *who) {
  if (!tree) return fail(ctx, AMPH_EINVAL, std::string(who) + ": null tree");
  if (tree->T > ctx->cfg.max_tree) return fail(ctx, AMPH_ESHAPE, std::string(who) + ": tree larger than cfg.max_tree");
  if (tree->K != ctx->cfg.K) return fail(ctx, AMPH_ESHAPE, std::string(who) + ": tree depth K differs from cfg.K");
  for (int i = 1; i < tree->T; ++i)
    if (tree->rank[i] >= ctx->cfg.topk) return fail(ctx, AMPH_ESHAPE, std::string(who) + ": tree uses a rank >= cfg.topk");
  if (!tree->d_block) return fail(ctx, AMPH_EINVAL, std::string(who) + ": the tree was created without a visible device");
  return AMPH_OK;
}

amph_status amph_tree_build(amph_ctx *ctx, const amph_tree *tree, const int32_t *root_tok, const int32_t *topk_idx,
                            const int32_t *kv_len, int32_t *tree_tok, int32_t *tree_pos) {
  if (!ctx) return AMPH_EINVAL;
  if (!root_tok || !topk_idx || !kv_len || !tree_tok || !tree_pos) return fail(ctx, AMPH_EINVAL, "amph_tree_build: null argument");
  if (amph_status s = check_tree(ctx, tree, "amph_tree_build")) return s;
  HIP_TRY(ctx, launch_tree_build(ctx->stream, tree->d_depth, tree->d_rank, tree->T, ctx->cfg.batch, ctx->cfg.K,
                                 ctx->cfg.topk, root_tok, topk_idx, kv_len, tree_tok, tree_pos));
  return AMPH_OK;
}

amph_status amph_verify_attn(amph_ctx *ctx, const amph_tree *tree, const void *q, const void *k_cache, const void *v_cache,
                             const int32_t *kv_len, void *out, void *workspace) {
  if (!ctx) return AMPH_EINVAL;
  if (!q || !k_cache || !v_cache || !kv_len || !out || !workspace) return fail(ctx, AMPH_EINVAL, "amph_verify_attn: null argument");
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out) || !aligned16(workspace))
    return fail(ctx, AMPH_EINVAL, "amph_verify_attn: pointers must be 16-byte aligned");
  if (q == out) return fail(ctx, AMPH_EINVAL, "amph_verify_attn: out must not alias q");
  if (amph_status s = check_tree(ctx, tree, "amph_verify_attn")) return s;
  float *partials = (float *)((char *)workspace + ctx->ws.ver_part);
  if (ctx->cfg.dtype == AMPH_BF16)
    return verify_impl<bf16_t>(ctx, tree, q, k_cache, v_cache, kv_len, out, partials, ctx->ws.ver_part_floats);
  return verify_impl<float>(ctx, tree, q, k_cache, v_cache, kv_len, out, partials, ctx->ws.ver_part_floats);
}

// The same call with the key-split partials in the library's static device array instead of a workspace: no
// hipMalloc, no hipFree, no allocating library routine anywhere on this path (the tree's tables and the context's
// status word were allocated by their _create calls).
amph_status amph_verify_attn_static(amph_ctx *ctx, const amph_tree *tree, const void *q, const void *k_cache,
                                    const void *v_cache, const int32_t *kv_len, void *out) {
  if (!ctx) return AMPH_EINVAL;
  if (!q || !k_cache || !v_cache || !kv_len || !out) return fail(ctx, AMPH_EINVAL, "amph_verify_attn_static: null argument");
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out))
    return fail(ctx, AMPH_EINVAL, "amph_verify_attn_static: pointers must be 16-byte aligned");
  if (q == out) return fail(ctx, AMPH_EINVAL, "amph_verify_attn_static: out must not alias q");
  if (amph_status s = check_tree(ctx, tree, "amph_verify_attn_static")) return s;
  int dev = -1;
  HIP_TRY(ctx, hipGetDevice(&dev));
  if (dev != ctx->device || !ctx->static_scratch)
    return fail(ctx, AMPH_EINVAL, "amph_verify_attn_static: the current device is not the one the context was created on");
  const amph_config &c = ctx->cfg;
  const size_t need = 4 * verify_partials_floats(c.batch, tree->T, c.n_heads, c.head_dim, c.max_kv, ctx->esz, ctx->verify_kernel);
  if (need > (size_t)AMPH_STATIC_SCRATCH_BYTES) {
    char msg[192];
    std::snprintf(msg, sizeof msg, "amph_verify_attn_static: this shape needs %zu bytes of key-split partials, the static scratch holds %u",
                  need, (unsigned)AMPH_STATIC_SCRATCH_BYTES);
    return fail(ctx, AMPH_ESHAPE, msg);
  }
  float *partials = (float *)ctx->static_scratch;
  const size_t cap = (size_t)AMPH_STATIC_SCRATCH_BYTES / 4;
  if (c.dtype == AMPH_BF16) return verify_impl<bf16_t>(ctx, tree, q, k_cache, v_cache, kv_len, out, partials, cap);
  return verify_impl<float>(ctx, tree, q, k_cache, v_cache, kv_len, out, partials, cap);
}

amph_status amph_accept(amph_ctx *ctx, const amph_tree *tree, const int32_t *tree_tok, const int32_t *tgt_argmax,
                        const float *tgt_logits, int32_t *accept_len, int32_t *accept_path, int32_t *next_tok,
                        int32_t *best_node, void *workspace) {
  if (!ctx) return AMPH_EINVAL;
  if (!tree_tok || !accept_len || !accept_path || !next_tok || !best_node) return fail(ctx, AMPH_EINVAL, "amph_accept: null argument");
  if ((tgt_argmax == nullptr) == (tgt_logits == nullptr))
    return fail(ctx, AMPH_EINVAL, "amph_accept: exactly one of tgt_argmax and tgt_logits must be given");
  if (amph_status s = check_tree(ctx, tree, "amph_accept")) return s;
  const int32_t *tgt = tgt_argmax;
  if (tgt_logits) {
    if (!workspace) return fail(ctx, AMPH_EINVAL, "amph_accept: workspace needed with tgt_logits");
    int32_t *tmp = (int32_t *)((char *)workspace + ctx->ws.tgt_tmp);
    HIP_TRY(ctx, launch_row_argmax(ctx->stream, tgt_logits, ctx->cfg.batch * tree->T, ctx->cfg.vocab, tmp,
                                   (float *)((char *)workspace + ctx->ws.topk_ws)));
    tgt = tmp;
  }
  HIP_TRY(ctx, launch_accept(ctx->stream, tree->d_parent, tree->d_depth, tree->T, ctx->cfg.batch, ctx->cfg.K, tree_tok, tgt,
                             accept_len, accept_path, next_tok, best_node));
  return AMPH_OK;
}

amph_status amph_accept_typical(amph_ctx *ctx, const amph_tree *tree, const int32_t *tree_tok, const float *tgt_logits,
                                float temperature, float eps, float delta, const float *u, int32_t *accept_len,
                                int32_t *accept_path, int32_t *next_tok, int32_t *best_node, void *workspace) {
  if (!ctx) return AMPH_EINVAL;
  if (!tree_tok || !tgt_logits || !u || !accept_len || !accept_path || !next_tok || !best_node || !workspace)
    return fail(ctx, AMPH_EINVAL, "amph_accept_typical: null argument");
  if (!(temperature > 0.f) || !(eps >= 0.f) || !(delta >= 0.f))      // (also rejects NaN)
    return fail(ctx, AMPH_EINVAL, "amph_accept_typical: temperature must be positive, eps and delta non-negative");
  if (!aligned16(workspace)) return fail(ctx, AMPH_EINVAL, "amph_accept_typical: workspace must be 16-byte aligned");
  if (amph_status s = check_tree(ctx, tree, "amph_accept_typical")) return s;
  HIP_TRY(ctx, launch_accept_typical(ctx->stream, tree->d_parent, tree->d_depth, tree->T, ctx->cfg.batch, ctx->cfg.K,
                                     ctx->cfg.vocab, tree_tok, tgt_logits, temperature, eps, delta, u, accept_len, accept_path,
                                     next_tok, best_node, (float *)((char *)workspace + ctx->ws.row_stats)));
  return AMPH_OK;
}

amph_status amph_target_forward(amph_ctx *ctx, const amph_tree *tree, const amph_layer_w *layers,
                                const amph_layer_tiled *tiled, int n_layers, const void *embed, const void *final_norm,
                                const void *lm_head, const void *lm_head_tiled, const int32_t *tree_tok,
                                const int32_t *tree_pos, void *k_caches, void *v_caches, const int32_t *kv_len,
                                float *hidden_out, float *logits_out, int32_t *tgt_argmax, void *workspace) {
  if (!ctx) return AMPH_EINVAL;
  if (n_layers < 0 || (n_layers > 0 && !layers)) return fail(ctx, AMPH_EINVAL, "amph_target_forward: bad layers");
  if (!embed || !final_norm || (!lm_head && !lm_head_tiled) || !tree_tok || !tree_pos || !kv_len || !tgt_argmax ||
      !workspace || (n_layers > 0 && (!k_caches || !v_caches)))
    return fail(ctx, AMPH_EINVAL, "amph_target_forward: null argument");
  for (int i = 0; i < n_layers; ++i) {
    const amph_layer_w &l = layers[i];
    const amph_layer_tiled t = tiled ? tiled[i] : amph_layer_tiled{nullptr, nullptr, nullptr, nullptr};
    // every GEMM needs either its tiled copy or all of its row-major matrices
    const bool ok = l.rms1 && l.rms2 && (t.qkv || (l.wq && l.wk && l.wv)) && (t.wo || l.wo) &&
                    (t.gate_up || (l.w_gate && l.w_up)) && (t.down || l.w_down);
    if (!ok) return fail(ctx, AMPH_EINVAL, "amph_target_forward: a layer lacks a weight in both layouts");
    const void *lp[] = {l.rms1, l.wq, l.wk, l.wv, l.wo, l.rms2, l.w_gate, l.w_up, l.w_down, t.qkv, t.wo, t.gate_up, t.down};
    for (const void *p : lp)
      if (p && !aligned16(p)) return fail(ctx, AMPH_EINVAL, "amph_target_forward: misaligned layer weight");
  }
  if (!aligned16(embed) || !aligned16(lm_head) || !aligned16(lm_head_tiled) || !aligned16(workspace) ||
      (k_caches && !aligned16(k_caches)) || (v_caches && !aligned16(v_caches)))
    return fail(ctx, AMPH_EINVAL, "amph_target_forward: pointers must be 16-byte aligned");
  if (amph_status s = check_tree(ctx, tree, "amph_target_forward")) return s;
  if (ctx->cfg.dtype == AMPH_BF16)
    return target_impl<bf16_t>(ctx, tree, layers, tiled, n_layers, embed, final_norm, lm_head, lm_head_tiled, tree_tok,
                               tree_pos, k_caches, v_caches, kv_len, hidden_out, logits_out, tgt_argmax, workspace);
  return target_impl<float>(ctx, tree, layers, tiled, n_layers, embed, final_norm, lm_head, lm_head_tiled, tree_tok,
                            tree_pos, k_caches, v_caches, kv_len, hidden_out, logits_out, tgt_argmax, workspace);
}

amph_status amph_commit(amph_ctx *ctx, const amph_tree *tree, int n_layers, void *k_caches, void *v_caches,
                        int32_t *kv_len, const int32_t *accept_len, const int32_t *accept_path, const int32_t *next_tok,
                        const int32_t *tree_tok, const float *hidden, float *h_new, int32_t *tok_new, int32_t *n_new) {
  if (!ctx) return AMPH_EINVAL;
  if (n_layers < 0 || !kv_len || !accept_len || !accept_path || (n_layers > 0 && (!k_caches || !v_caches)))
    return fail(ctx, AMPH_EINVAL, "amph_commit: null argument");
  if (h_new && (!tok_new || !n_new || !next_tok || !tree_tok || !hidden || !aligned16(h_new) || !aligned16(hidden)))
    return fail(ctx, AMPH_EINVAL, "amph_commit: the draft's next inputs need tok_new, n_new, next_tok, tree_tok and hidden");
  if (!aligned16(k_caches) || !aligned16(v_caches)) return fail(ctx, AMPH_EINVAL, "amph_commit: misaligned cache");
  if (amph_status s = check_tree(ctx, tree, "amph_commit")) return s;
  const amph_config &c = ctx->cfg;
  if (ctx->cfg.dtype == AMPH_BF16)
    HIP_TRY(ctx, launch_commit<bf16_t>(ctx->stream, k_caches, v_caches, n_layers, c.batch, c.n_heads, c.head_dim, c.max_kv,
                                       tree->T, c.d_model, c.K, kv_len, accept_len, accept_path, next_tok, tree_tok, hidden,
                                       h_new, tok_new, n_new));
  else
    HIP_TRY(ctx, launch_commit<float>(ctx->stream, k_caches, v_caches, n_layers, c.batch, c.n_heads, c.head_dim, c.max_kv,
                                      tree->T, c.d_model, c.K, kv_len, accept_len, accept_path, next_tok, tree_tok, hidden,
                                      h_new, tok_new, n_new));
  return AMPH_OK;
}

// shape of the GEMM a packing role belongs to: epilogue kind, stacked matrices, rows per matrix, reduction length
static bool pack_shape(const amph_config &c, int role, int *epi, int *n_seg, int *rows, int *Kd) {
  switch (role) {
    case AMPH_PACK_QKV: *epi = EPI_QKV_ROPE; *n_seg = 3; *rows = c.d_model; *Kd = c.d_model; return true;
    case AMPH_PACK_WO: *epi = EPI_STORE; *n_seg = 1; *rows = c.d_model; *Kd = c.d_model; return true;
    case AMPH_PACK_GATEUP: *epi = EPI_SWIGLU; *n_seg = 2; *rows = c.d_ffn; *Kd = c.d_model; return true;
    case AMPH_PACK_DOWN: *epi = EPI_STORE; *n_seg = 1; *rows = c.d_model; *Kd = c.d_ffn; return true;
    case AMPH_PACK_LMHEAD: *epi = EPI_ARGMAX; *n_seg = 1; *rows = c.vocab; *Kd = c.d_model; return true;
    default: return false;
  }
}

amph_status amph_tiled_bytes(const amph_ctx *ctx, int role, size_t *bytes) {
  if (!ctx || !bytes) return AMPH_EINVAL;
  int epi, n_seg, rows, Kd;
  if (!pack_shape(ctx->cfg, role, &epi, &n_seg, &rows, &Kd)) return AMPH_EINVAL;
  *bytes = gemm_tiled_bytes(epi, rows, Kd, (int)ctx->esz);
  return AMPH_OK;
}

amph_status amph_pack_weights(amph_ctx *ctx, int role, const void *w0, const void *w1, const void *w2, void *dst) {
  if (!ctx) return AMPH_EINVAL;
  int epi, n_seg, rows, Kd;
  if (!pack_shape(ctx->cfg, role, &epi, &n_seg, &rows, &Kd)) return fail(ctx, AMPH_EINVAL, "amph_pack_weights: bad role");
  if (!w0 || (n_seg >= 2 && !w1) || (n_seg >= 3 && !w2) || !dst)
    return fail(ctx, AMPH_EINVAL, "amph_pack_weights: null argument");
  if (!aligned16(w0) || !aligned16(w1) || !aligned16(w2) || !aligned16(dst))
    return fail(ctx, AMPH_EINVAL, "amph_pack_weights: pointers must be 16-byte aligned");
  if ((Kd * (int)ctx->esz) % 64) return fail(ctx, AMPH_ESHAPE, "amph_pack_weights: a weight row must be a multiple of 64 bytes");
  GemmArgs a{};
  a.w0 = w0; a.w1 = w1; a.w2 = w2; a.n_seg = n_seg; a.seg_rows = rows; a.Kd = Kd;
  a.n_heads = ctx->cfg.n_heads; a.d_h = ctx->cfg.head_dim;
  if (ctx->cfg.dtype == AMPH_BF16) HIP_TRY(ctx, launch_pack_weights<bf16_t>(ctx->stream, epi, a, dst));
  else HIP_TRY(ctx, launch_pack_weights<float>(ctx->stream, epi, a, dst));
  return AMPH_OK;
}

static amph_status kv_layout(amph_ctx *ctx, const char *who, const void *k_src, const void *v_src, void *k_dst, void *v_dst,
                             int n_caches, bool to_tiled) {
  if (!ctx) return AMPH_EINVAL;
  if (n_caches < 1 || (!k_src && !v_src) || (k_src != nullptr) != (k_dst != nullptr) || (v_src != nullptr) != (v_dst != nullptr))
    return fail(ctx, AMPH_EINVAL, std::string(who) + ": need n_caches >= 1 and source and destination of keys, values or both");
  if (!aligned16(k_src) || !aligned16(v_src) || !aligned16(k_dst) || !aligned16(v_dst))
    return fail(ctx, AMPH_EINVAL, std::string(who) + ": pointers must be 16-byte aligned");
  if ((k_src && k_src == k_dst) || (v_src && v_src == v_dst)) return fail(ctx, AMPH_EINVAL, std::string(who) + ": in-place conversion is not supported");
  if (n_caches > 65535 * 16) return fail(ctx, AMPH_ESHAPE, std::string(who) + ": more than 65535 * 16 caches in one call");
  const amph_config &c = ctx->cfg;
  if (c.dtype == AMPH_BF16) HIP_TRY(ctx, launch_kv_layout<bf16_t>(ctx->stream, k_src, v_src, k_dst, v_dst, n_caches, c.max_kv, c.head_dim, to_tiled));
  else HIP_TRY(ctx, launch_kv_layout<float>(ctx->stream, k_src, v_src, k_dst, v_dst, n_caches, c.max_kv, c.head_dim, to_tiled));
  return AMPH_OK;
}

amph_status amph_pack_kv(amph_ctx *ctx, const void *k_rows, const void *v_rows, void *k_tiled, void *v_tiled, int n_caches) {
  return kv_layout(ctx, "amph_pack_kv", k_rows, v_rows, k_tiled, v_tiled, n_caches, true);
}

amph_status amph_unpack_kv(amph_ctx *ctx, const void *k_tiled, const void *v_tiled, void *k_rows, void *v_rows, int n_caches) {
  return kv_layout(ctx, "amph_unpack_kv", k_tiled, v_tiled, k_rows, v_rows, n_caches, false);
}

amph_status amph_verify_kernel(amph_ctx *ctx, int kernel) {
  if (!ctx) return AMPH_EINVAL;
  if (kernel < -1 || kernel > 1) return fail(ctx, AMPH_EINVAL, "amph_verify_kernel: kernel must be -1, 0 or 1");
  ctx->verify_kernel = kernel;
  return AMPH_OK;
}

amph_status amph_profile_kind(amph_ctx *ctx, int kind, int max_launches, int every) {
  if (!ctx) return AMPH_EINVAL;
  if (kind < -1 || kind >= AMPH_K_COUNT || max_launches < 0 || max_launches > 65536 || every < 1)
    return fail(ctx, AMPH_EINVAL, "amph_profile_kind: bad kind, max_launches or every");
  while (ctx->prof_ev.size() < (size_t)2 * max_launches) {
    hipEvent_t e;
    HIP_TRY(ctx, hipEventCreate(&e));
    ctx->prof_ev.push_back(e);
  }
  ctx->prof_kind = kind;
  ctx->prof_used = 0;
  ctx->prof_every = every;
  ctx->prof_seen = 0;
  return AMPH_OK;
}

amph_status amph_profile_read(amph_ctx *ctx, double *total_ms, int *launches) {
  if (!ctx || !total_ms || !launches) return AMPH_EINVAL;
  HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  double tot = 0.0;
  for (size_t i = 0; i < ctx->prof_used; ++i) {
    float ms = 0.f;
    HIP_TRY(ctx, hipEventElapsedTime(&ms, ctx->prof_ev[2 * i], ctx->prof_ev[2 * i + 1]));
    tot += ms;
  }
  *total_ms = tot;
  *launches = (int)ctx->prof_used;
  ctx->prof_used = 0;
  return AMPH_OK;
}

amph_status amph_gemv(amph_ctx *ctx, const float *x, const void *W, float *y, int M, int N, int Kd) {
  if (!ctx) return AMPH_EINVAL;
  if (!x || !W || !y || !aligned16(W)) return fail(ctx, AMPH_EINVAL, "amph_gemv: null or misaligned argument");
  if (M < 1 || M > 8 || N < 1 || Kd < 8 || Kd % 8) return fail(ctx, AMPH_ESHAPE, "amph_gemv: need 1 <= M <= 8, Kd % 8 == 0");
  if (ctx->cfg.dtype == AMPH_BF16)
    HIP_TRY(ctx, launch_linear<bf16_t>(ctx->stream, W, nullptr, nullptr, 1, N, Kd, x, Kd, M, nullptr, y, nullptr, nullptr, N));
  else
    HIP_TRY(ctx, launch_linear<float>(ctx->stream, W, nullptr, nullptr, 1, N, Kd, x, Kd, M, nullptr, y, nullptr, nullptr, N));
  return AMPH_OK;
}

amph_status amph_gemm(amph_ctx *ctx, const void *x, const void *W, float *y, int M, int N, int Kd, int split_k,
                      void *workspace) {
  if (!ctx) return AMPH_EINVAL;
  if (!x || !W || !y || !workspace || !aligned16(x) || !aligned16(W) || !aligned16(workspace))
    return fail(ctx, AMPH_EINVAL, "amph_gemm: null or misaligned argument");
  if (M < 1 || N < 1 || Kd < 1 || (Kd * ctx->esz) % 64) return fail(ctx, AMPH_ESHAPE, "amph_gemm: a row of x must be a multiple of 64 bytes");
  if (split_k == 0) split_k = gemm_plan(EPI_STORE, N, Kd, ctx->esz, M, 0, false).split;
  if (split_k != 1 && split_k != 2 && split_k != 4 && split_k != 8) return fail(ctx, AMPH_ESHAPE, "amph_gemm: split_k");
  if (split_k > 1 && (size_t)split_k * M * N > ctx->ws.slabs_floats)
    return fail(ctx, AMPH_ESHAPE, "amph_gemm: split_k * M * N exceeds the workspace's slab area");
  float *slabs = (float *)((char *)workspace + ctx->ws.slabs);
  GemmArgs a{};
  a.w0 = W; a.n_seg = 1; a.seg_rows = N; a.Kd = Kd; a.x = x; a.M = M; a.split_k = split_k;
  a.out = (split_k > 1) ? slabs : y; a.dev_status = ctx->dev_status;
  if (ctx->cfg.dtype == AMPH_BF16) HIP_TRY(ctx, launch_gemm<bf16_t>(ctx->stream, EPI_STORE, a));
  else HIP_TRY(ctx, launch_gemm<float>(ctx->stream, EPI_STORE, a));
  if (split_k > 1) HIP_TRY(ctx, launch_sum_slabs(ctx->stream, slabs, split_k, (size_t)M * N, y));
  return AMPH_OK;
}

}  // extern "C"
