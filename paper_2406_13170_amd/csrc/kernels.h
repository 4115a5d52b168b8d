// Internal launcher declarations shared by the kernel files and the C-ABI layer.
#pragma once
#include "../../include/amph.h"
#include "common.h"

namespace amph {

constexpr size_t GV_MAX_SMEM = 128 * 1024;    // dynamic LDS a GEMV workgroup may ask for (gfx950: 160 KB per workgroup)

// ---- gemv.hip (draft path, M <= 8 rows) ----
template <typename T>
hipError_t launch_fc_concat(hipStream_t st, const void *W, const float *u, const void *embed, const int32_t *tok,
                            int vocab, int d, int M, float *out, uint32_t *dev_status);
template <typename T>
hipError_t launch_sal_qkv(hipStream_t st, const amph_layer_w &lw, const float *x, int d, int n_heads, int d_h, int M,
                          float eps, float theta, const int32_t *sal_len, int max_kv, void *kv_stage, float *qbuf,
                          uint32_t *dev_status, int R, const int32_t *n_valid);   // rows = (batch element, new position < R)
template <typename T>
hipError_t launch_linear(hipStream_t st, const void *w0, const void *w1, const void *w2, int n_seg, int seg_rows, int Kd,
                         const float *x, int ldx, int M, const float *res, float *o0, float *o1, float *o2, int ldo);
template <typename T>
hipError_t launch_gate_up(hipStream_t st, const amph_layer_w &lw, const float *x, int d, int f, int M, float eps,
                          float *act);
template <typename T>
hipError_t launch_head_mlp(hipStream_t st, const void *w_mlp, const void *pe, const float *h1, const float *h2, int d,
                           int K, int M, float *Hp);

// The shared LM head of Eq. 6 with the top-k candidates taken in its epilogue: every workgroup leaves its k best
// (value, token) pairs per row in ws (lmtk_ws_floats(M, k) floats: values [M][n_cand], then tokens [M][n_cand]);
// logits are written only if `logits` is non-NULL.  launch_topk_merge then picks each row's top k.
constexpr int LMTK_MAX_WG = 1024;
size_t lmtk_ws_floats(int rows, int k);
template <typename T>
hipError_t launch_lmhead_cands(hipStream_t st, const void *W, int V, int Kd, const float *x, int M, int k, float *logits,
                               float *ws, int *n_cand);

// ---- small.hip (attention of the draft path, top-k, tree, accept, norms) ----
template <typename T>
hipError_t launch_sal_attn(hipStream_t st, const float *qbuf, const void *kv_stage, const int32_t *sal_len, int B,
                           int n_heads, int d_h, int max_kv, float *out, int R, const int32_t *n_valid, int last_only = 0);
hipError_t launch_aeb_attn(hipStream_t st, const float *Q, const float *Kk, const float *V, int B, int K, int n_heads,
                           int d_h, float *ctx);
// ws: topk_ws_floats(rows, V, k) floats of scratch for the per-wave candidates
size_t topk_ws_floats(int rows, int V, int k);
hipError_t launch_topk_rows(hipStream_t st, const float *logits, int rows, int V, int k, int32_t *idx, float *val,
                            int32_t *advance, int n_advance, int advance_by, const int32_t *advance_each, int advance_limit,
                            float *ws);   // advance[i] += advance_each ? advance_each[i] : advance_by where the sum stays <= advance_limit
// top-k of n_cand (value, token) candidates per row (cand_i < 0: no candidate), one workgroup per row
hipError_t launch_topk_merge(hipStream_t st, const float *cand_v, const int *cand_i, int rows, int n_cand, int V, int k,
                             int32_t *idx, float *val, int32_t *advance, int n_advance, int advance_by,
                             const int32_t *advance_each, int advance_limit);
hipError_t launch_row_argmax(hipStream_t st, const float *logits, int rows, int V, int32_t *out, float *ws);
hipError_t launch_tree_build(hipStream_t st, const int32_t *depth, const int32_t *rank, int T, int B, int K, int topk,
                             const int32_t *root_tok, const int32_t *topk_idx, const int32_t *kv_len, int32_t *tree_tok,
                             int32_t *tree_pos);
// stats_ws: B * T * 4 floats (16-byte aligned)
hipError_t launch_accept_typical(hipStream_t st, const int32_t *parent, const int32_t *depth, int T, int B, int K, int V,
                                 const int32_t *tree_tok, const float *logits, float temperature, float eps, float delta,
                                 const float *u, int32_t *accept_len, int32_t *accept_path, int32_t *next_tok,
                                 int32_t *best_node, float *stats_ws);
hipError_t launch_accept(hipStream_t st, const int32_t *parent, const int32_t *depth, int T, int B, int K,
                         const int32_t *tree_tok, const int32_t *tgt, int32_t *accept_len, int32_t *accept_path,
                         int32_t *next_tok, int32_t *best_node);
// the loop around the step: compaction of the accepted path's K/V rows in every layer, the rows the draft
// consumes next (h_new may be NULL: then only the caches and kv_len are updated), kv_len += accepted + 1
template <typename T>
hipError_t launch_commit(hipStream_t st, void *k_caches, void *v_caches, int n_layers, int B, int n_heads, int d_h, int max_kv,
                         int T_nodes, int d, int K, int32_t *kv_len, const int32_t *accept_len, const int32_t *accept_path,
                         const int32_t *next_tok, const int32_t *tree_tok, const float *hidden, float *h_new, int32_t *tok_new,
                         int32_t *n_new);
// n_caches row-major [max_kv, d_h] caches <-> their step-tiled storage; a NULL source skips keys or values
template <typename T>
hipError_t launch_kv_layout(hipStream_t st, const void *k_src, const void *v_src, void *k_dst, void *v_dst, int n_caches,
                            int max_kv, int d_h, bool to_tiled);
hipError_t launch_gather_rows(hipStream_t st, const float *rows, int B, int R, int d, const int32_t *n_valid, float *out);
// x[m] (+)= sum_s slabs[s][m] (or x[m] = embed[tok[m]] when tok != NULL); xn[m] = RMSNorm(x[m]) * g as T;
// hidden_out (float32, optional) receives the same normalised rows.  xn_tiles != 0: xn is written in the tiled
// activation layout of the wide GEMM (xn_tiles = number of 32-row tiles).
// optional by-product of the embedding instance of k_norm_fold: cs[row][e] = (cos, sin)(pos[row] * theta^(-2e/d_h))
struct RopeTable { const int32_t *pos = nullptr; int d_h = 0; float theta = 0.f; float2 *cs = nullptr; };
template <typename T>
hipError_t launch_norm_fold(hipStream_t st, float *x, const void *embed, const int32_t *tok, int vocab,
                            const float *slabs, int S, size_t slab_stride, const void *g, int rows, int d, float eps,
                            void *xn, float *hidden_out, uint32_t *dev_status, int xn_tiles = 0, RopeTable rope = RopeTable{});

// ---- gemm_skinny.hip (target path, rows on the matrix cores) ----
enum GemmEpi { EPI_STORE = 0, EPI_QKV_ROPE = 2, EPI_SWIGLU = 3, EPI_ARGMAX = 4 };
struct GemmArgs {
  const void *w0, *w1, *w2;   // stacked matrices (q,k,v | gate,up | single), row-major [seg_rows, Kd]
  const void *wt;             // the same matrices in the tiled layout (launch_pack_weights), or NULL: then w0..w2 are read
  int n_seg, seg_rows;        // rows per matrix
  int Kd;
  const void *x;              // [M, Kd] T
  void *xt;                   // scratch of gemm_xt_bytes(M, Kd): fragment-tiled copy of x for the wide kernel, or NULL
  bool x_tiled;               // x itself is already in that tiled layout (its producer wrote it so): no copy is made
  int act_tiles;              // EPI_SWIGLU: 0 = act is row-major [M, f]; else its 32-row tile count, act is written tiled
  int M;
  int split_k;                // 1, 2, 4, 8 (fused epilogues: 1)
  int nb;                     // row blocks per workgroup: filled in by launch_gemm from gemm_plan
  // epilogue operands
  float *out;                 // EPI_STORE: [split_k][M, seg_rows] float32 partial slabs
  float *logits;              // EPI_ARGMAX: optional [M, seg_rows]
  void *act;                  // EPI_SWIGLU: [M, f] T
  // QKV
  void *q_out;                // [M, d] T
  void *k_cache, *v_cache;    // this layer: [B, n_h] step-tiled caches of max_kv * d_h elements each
  const float2 *rope_cs;      // [M, d_h/2] (cos, sin) of each row's position
  const int32_t *kv_len;      // [B]
  int T_nodes, n_heads, d_h, max_kv;
  // ARGMAX
  float *amax_val;            // [tiles_n][M] per-tile maxima
  int32_t *amax_idx;          // [tiles_n][M]
  uint32_t *dev_status;
};
// Tile height (row blocks per workgroup), reduction split and resulting tile count of one GEMM.  split_req: 0 lets
// the plan choose (fused epilogues always 1), else the caller's split; tiled: the launch will have both GemmArgs::wt
// and GemmArgs::xt (then 128 rows or more go to the wide kernel).  The same call must be used to size
// whatever depends on the plan (partial slabs: split; per-tile argmax candidates: tiles).
struct GemmPlan { int nb, split, tiles, blocks; bool wide; int mgroups, nw, tw, gt; };   // wide: mgroups groups of gt tiles of 32 rows, nw math waves x up to tw tiles
GemmPlan gemm_plan(int epi, int seg_rows, int Kd, int elem_bytes, int M, int split_req, bool tiled);
size_t gemm_xt_bytes(int M, int Kd, int elem_bytes);
bool gemm_is_wide(int M, bool tiled);       // whether gemm_plan sends this many rows to the wide kernel
// ev_start / ev_stop (both or neither): events that receive the kernel's own begin and end time stamps
template <typename T> hipError_t launch_gemm(hipStream_t st, int epi, const GemmArgs &a, hipEvent_t ev_start = nullptr,
                                             hipEvent_t ev_stop = nullptr);
// bytes of the tiled copy of the matrices of one GEMM, and the kernel that writes it (w0..w2, seg_rows, Kd, n_heads, d_h of a)
size_t gemm_tiled_bytes(int epi, int seg_rows, int Kd, int elem_bytes);
template <typename T> hipError_t launch_pack_weights(hipStream_t st, int epi, const GemmArgs &a, void *dst);
hipError_t launch_sum_slabs(hipStream_t st, const float *slabs, int S, size_t n, float *out);
hipError_t launch_argmax_fold(hipStream_t st, const float *amax_val, const int32_t *amax_idx, int tiles, int M,
                              int32_t *tgt);

// ---- verify_attn.hip ----
struct VerifyArgs {
  const void *q; const void *k_cache; const void *v_cache; void *out;
  const int32_t *kv_len; const uint64_t *mask_bits;
  int B, T, n_heads, d_h, max_kv;
  float *partials; size_t partials_cap; uint32_t *dev_status;
  int out_tiles;    // 0: out is row-major [B*T, n_heads*d_h]; else the 32-row tile count of the tiled activation layout
  int kernel;       // -1: chosen by shape; 0: operands through registers; 1: operands through an LDS ring
};
size_t verify_ws_floats(int B, int T, int n_heads, int d_h, int max_kv, int elem_bytes);
// floats of key-split partials one call writes with the given kernel choice (VerifyArgs::kernel); 0 without key splits
size_t verify_partials_floats(int B, int T, int n_heads, int d_h, int max_kv, int elem_bytes, int kernel);
template <typename T> hipError_t launch_verify_attn(hipStream_t st, const VerifyArgs &a);

}  // namespace amph
