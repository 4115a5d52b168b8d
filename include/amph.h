/*
 * amph.h -- C ABI of libamph: the hot path of one Amphista speculate-and-verify decode step
 * (arXiv 2406.13170) on one MI355X (gfx950).
 *
 * Conventions
 *   - Every function returns amph_status (0 = OK).  Argument checks run on the host and are
 *     synchronous; all device work is enqueued on the context's stream and returns at once.  No call
 *     synchronises the stream or reads device memory on the host unless its comment says so.
 *   - Unless marked "host", every pointer is a DEVICE pointer owned by the caller; the library never
 *     frees or reallocates caller memory.  The library owns amph_ctx (one device status word) and
 *     amph_tree (host tables plus device copies), both allocated by their _create calls and released
 *     by their _destroy calls; no other call allocates, frees or blocks.
 *   - Layouts are dense row-major in the order written, last index fastest, with two exceptions that
 *     are private to the matrix-core kernels and have converters here: the target's K/V caches are
 *     STEP-TILED (amph_pack_kv / amph_unpack_kv; formulas at amph_verify_attn) and the target's weight
 *     matrices may be given as tiled copies (amph_pack_weights).  "T" below is the configuration's
 *     storage type: float for AMPH_F32, bfloat16 (16-bit patterns) for AMPH_BF16.
 *     Weights are [out_features, in_features].  Accumulation is always float32.
 *   - Quantities that only the device knows (kv_len, sal_len) are range-checked inside the kernels:
 *     a violation sets a sticky device flag, the offending call writes no output for that batch
 *     element, and amph_device_status() reports it.
 *   - Paper references: Sec. 3.1 Eq. 1 (staged adaptation layers), Sec. 3.2 Eq. 2-6 (auto-embedding
 *     block, LM head, top-k), Sec. 2 "Tree Attention" and Appendix "Draft Tree" (tree, mask,
 *     verification), Sec. 2 "Speculative Decoding" and Table 1 (greedy acceptance).
 */
#ifndef AMPH_H
#define AMPH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  AMPH_OK = 0,
  AMPH_EINVAL = 1,  /* null pointer, negative size, unsupported value           */
  AMPH_ESHAPE = 2,  /* dimensions inconsistent or beyond a documented limit      */
  AMPH_ETREE = 3,   /* malformed topology (missing parent, duplicate, too deep)  */
  AMPH_EHIP = 4     /* HIP runtime error; text via amph_last_error               */
} amph_status;

enum { AMPH_F32 = 0, AMPH_BF16 = 1 };

enum { AMPH_MAX_TREE = 128, AMPH_MAX_TOPK = 16, AMPH_MAX_HEADS_K = 8 };

/* bits of the device status word (amph_device_status) */
enum { AMPH_DEV_SAL_OVERFLOW = 1, AMPH_DEV_KV_OVERFLOW = 2, AMPH_DEV_BAD_TOKEN = 4 };

typedef struct amph_config {
  int32_t d_model, n_heads, head_dim; /* d_model = n_heads * head_dim; head_dim is 64 or 128        */
  int32_t d_ffn, vocab;
  int32_t K;                 /* drafting heads, 1..AMPH_MAX_HEADS_K                                */
  int32_t topk;              /* per-head candidates, 1..AMPH_MAX_TOPK                              */
  int32_t max_tree;          /* largest tree (nodes incl. root) used with this context, <= 128     */
  int32_t max_kv;            /* rows of every KV cache; multiple of 32, at most 2^24               */
  int32_t batch;             /* independent sequences per call                                     */
  int32_t dtype;             /* AMPH_F32 | AMPH_BF16                                               */
  float rms_eps;             /* RMSNorm epsilon                                                    */
  float rope_theta;          /* RoPE base; pairs are (i, i + head_dim/2)                           */
  /* structural variants of the paper's ablations (Sec. 4.3; Appendix); the method itself is 2, 1, 0 */
  int32_t n_stages;          /* adaptation layers: 2, or 1 = one layer whose output every head reads */
  int32_t aeb_layers;        /* self-attention layers in the Auto-embedding Block: 1, or 2 ("alpha")  */
  int32_t lm_rank;           /* 0 = full LM head; r > 0 (multiple of 8) = low-rank pair lm_a, lm_b    */
} amph_config;

/* One Llama-style decoder layer (pre-RMSNorm, RoPE, SwiGLU, no biases); all T. */
typedef struct amph_layer_w {
  const void *rms1;                 /* [d]     */
  const void *wq, *wk, *wv, *wo;    /* [d, d]  */
  const void *rms2;                 /* [d]     */
  const void *w_gate, *w_up;        /* [f, d]  */
  const void *w_down;               /* [d, f]  */
} amph_layer_w;

/* The matrices of one target layer in the TILED layout that the matrix-core GEMM streams at full rate
 * (amph_pack_weights writes it, once per matrix, from the row-major matrices).  A matrix-core operand
 * fragment is 16 rows x 64 bytes; read from a row-major matrix it touches 16 half cache lines per
 * load instruction, which the vector L1 of a CU handles about four times slower than one contiguous
 * 1 KB load.  The tiled copy stores every fragment the kernel will ask for as one contiguous 1 KB piece,
 * in the order the kernel walks them; its exact form is private to the library (amph_tiled_bytes gives
 * the size).  A NULL member means "use the row-major matrices of amph_layer_w for this GEMM". */
typedef struct amph_layer_tiled {
  const void *qkv;          /* from wq, wk, wv  (AMPH_PACK_QKV)    */
  const void *wo;           /* from wo          (AMPH_PACK_WO)     */
  const void *gate_up;      /* from w_gate, w_up (AMPH_PACK_GATEUP) */
  const void *down;         /* from w_down      (AMPH_PACK_DOWN)   */
} amph_layer_tiled;

/* Weights of the draft module (host struct of device pointers; all T). */
typedef struct amph_draft_w {
  const void *embed;        /* [V, d]  target's embedding table: e_{t+1} (Sec. 3.1)                */
  const void *fc[2];        /* [d, 2d] fc^1, fc^2 of Eq. 1; columns [0,d) act on h, [d,2d) on e     */
  amph_layer_w sal[2];      /* SAL^1, SAL^2 of Eq. 1                                                */
  const void *mlp;          /* [K, d, d] MLP_k of Eq. 2, used as h + SiLU(W_k h)                    */
  const void *pe;           /* [K, d]  positional embedding of Eq. 4                                */
  const void *aeb_wq, *aeb_wk, *aeb_wv, *aeb_wo; /* [d, d] self-attention of Eq. 5                  */
  const void *lm_head;      /* [V, d]  LM head of Eq. 6, shared by the K positions                  */
  /* variants: pe may be NULL (no position encoding); with n_stages = 1 only fc[0] and sal[0] are read;    */
  const void *aeb2_wq, *aeb2_wk, *aeb2_wv, *aeb2_wo; /* [d, d] second self-attention layer (aeb_layers = 2) */
  const void *lm_a;         /* [lm_rank, d]  low-rank LM head: logits = lm_b (lm_a x); lm_head is then unused */
  const void *lm_b;         /* [V, lm_rank]                                                          */
} amph_draft_w;

typedef struct amph_ctx amph_ctx;
typedef struct amph_tree amph_tree;

/* ---- context --------------------------------------------------------------------------------- */
/* Validates cfg (host pointer), allocates the context's device status word on the CURRENT device and
 * resolves that device's copy of the library's static scratch (amph_verify_attn_static).  *out is NULL
 * on failure. */
amph_status amph_create(const amph_config *cfg, amph_ctx **out);
void amph_destroy(amph_ctx *ctx);
/* hip_stream is a hipStream_t (NULL = the default stream).  The caller keeps it alive. */
amph_status amph_set_stream(amph_ctx *ctx, void *hip_stream);
/* Bytes of caller-provided scratch every call below needs (256-byte aligned). */
size_t amph_workspace_bytes(const amph_ctx *ctx);
/* Host string describing the last failure on this context (never NULL). */
const char *amph_last_error(const amph_ctx *ctx);
/* SYNCHRONISES the stream, copies the sticky device status word to *host_bits and clears it. */
amph_status amph_device_status(amph_ctx *ctx, uint32_t *host_bits);

/* ---- A1-A5: draft (Sec. 3.1 Eq. 1, Sec. 3.2 Eq. 2-6) ------------------------------------------
 * For each batch element b: e = embed[tok_new[b]]; x1 = fc1 [h_new[b]; e]; h1 = SAL1(x1);
 * x2 = fc2 [h1; e]; h2 = SAL2(x2); H_p[k] = MLP_k(h1 or h2) + PE[k] (heads 1..floor(K/2) read h1);
 * attn_o = bi-directional multi-head self-attention over the K rows; logits[k] = lm_head attn_o[k];
 * top-k per row, sorted by descending logit, ties to the lower token id.
 * Eq. 1 keeps one cache row per committed position, so after a step that accepted a draft tokens the
 * adaptation layers first catch up over the a + 1 new positions, oldest first (each row attends to the
 * cache and to the new rows before it); the heads read the LAST live position.
 *   h_new    [B, n_new, d] float32     tok_new [B, n_new] int32 (the token that follows each position)
 *            1 <= n_new <= K + 1.  The adaptation layers' weight-streaming kernels take 8 rows at a time (fewer
 *            where 8 float32 rows of the model width do not fit in 128 KB of LDS and the kernel has a fused
 *            epilogue): a call with B * n_new > 8 streams their weights ceil(B * n_new / 8) times or more.
 *   n_valid  [B] int32 on the device or NULL: positions j >= n_valid[b] of element b are ignored (no
 *            cache row, no effect on the heads); NULL = all n_new live.  amph_commit writes such a triple.
 *   sal_kv   [2 stages, B, 2 (K then V), n_heads, max_kv, head_dim] T; rows sal_len[b] + j of both stages
 *            are written (keys after RoPE at that position) and attended together with the rows below them
 *   sal_len  [B] int32, read on the device and advanced by n_valid[b] (or n_new) when the call completes,
 *            unless that would pass max_kv: then it stays as it was (see below)
 *   topk_idx [B, K, topk] int32        topk_val [B, K, topk] float32
 *   logits   [B, K, V] float32 or NULL (then the logits live only in the workspace)
 * Device-side errors: a new position j whose cache row sal_len[b] + j would lie at or beyond max_kv writes
 * no cache row and raises AMPH_DEV_SAL_OVERFLOW (rows below it are still written); sal_len[b] is then left
 * unchanged and the top-k written for element b is meaningless.  A token id outside [0, V) raises
 * AMPH_DEV_BAD_TOKEN and is read as token 0. */
amph_status amph_draft(amph_ctx *ctx, const amph_draft_w *w /* host */, const float *h_new,
                       const int32_t *tok_new, int n_new, const int32_t *n_valid, void *sal_kv,
                       int32_t *sal_len, int32_t *topk_idx, float *topk_val, float *logits,
                       void *workspace);

/* ---- draft tree (Appendix "Draft Tree") -------------------------------------------------------
 * paths: host array [n, K] of top-k ranks, -1 padded; one row per non-root node, any order; the
 * root (the token the target just sampled) is implicit.  Nodes are numbered root first, then by
 * (depth, rank path).  Fails with AMPH_ETREE on a missing parent, a duplicate or a path longer
 * than K, AMPH_ESHAPE if n + 1 > AMPH_MAX_TREE or a rank >= AMPH_MAX_TOPK.
 * A set-up call: it allocates the tree's device tables (a few KB) on the CURRENT device and copies
 * them there with a blocking copy, so that no call of the step allocates or blocks.  Without a visible
 * device the tree is a host object (amph_tree_info works; device calls given it return AMPH_EINVAL). */
amph_status amph_tree_create(const int32_t *paths /* host */, int n, int K, amph_tree **out);
void amph_tree_destroy(amph_tree *tree);
/* Host views valid until amph_tree_destroy; any output pointer may be NULL.
 *   parent, depth, rank [T] (root: -1, 0, -1);  mask_bits [T, 2]: bit j of row i set iff node j is
 *   node i or one of its ancestors;  retrieve [n_leaves, K+1] node ids root..leaf, -1 padded. */
amph_status amph_tree_info(const amph_tree *tree, int *T, int *n_leaves, const int32_t **parent,
                           const int32_t **depth, const int32_t **rank, const uint64_t **mask_bits,
                           const int32_t **retrieve);

/* ---- A6: candidate-tree construction -----------------------------------------------------------
 * tree_tok[b, i] = root_tok[b] for the root, else topk_idx[b, depth_i - 1, rank_i];
 * tree_pos[b, i] = kv_len[b] + depth_i.
 *   root_tok [B] int32   topk_idx [B, K, topk] int32   kv_len [B] int32   tree_tok, tree_pos [B, T] */
amph_status amph_tree_build(amph_ctx *ctx, const amph_tree *tree, const int32_t *root_tok,
                            const int32_t *topk_idx, const int32_t *kv_len, int32_t *tree_tok,
                            int32_t *tree_pos);

/* ---- A8: tree-masked verification attention (Sec. 2 "Tree Attention") ---------------------------
 * out[b, i, h] = sum_j softmax_j(q[b,i,h] . k_j / sqrt(head_dim)) v_j over all committed rows
 * j < kv_len[b] and the tree rows kv_len[b] + j' with j' = i or an ancestor of i.
 *   q, out  [B, T, n_heads, head_dim] T
 *   k_cache, v_cache   per (b, head) max_kv * head_dim elements of T each: rows (already rotated keys;
 *           values) numbered as usual, tree rows at [kv_len[b], kv_len[b] + T) in node order, but stored
 *           STEP-TILED so that every matrix-core fragment of the kernel is one contiguous 1 KB piece (a
 *           row-major cache costs 16 half cache lines per fragment load, about four times slower in the
 *           CU's vector L1).  With E = sizeof(T), P = 16/E, a key step = 4P rows (32 bf16 / 16 float):
 *             K element (row r, dim c): step s = r / 4P, kk = r % 4P, tile t = (kk % P) / 4,
 *               slot i = (kk / P) * 4 + kk % 4, piece ds = c*E / 64:
 *               byte offset ((s * P/4 + t) * (head_dim*E/64) + ds) * 1024 + i * 64 + (c*E) % 64
 *             V element (row r, dim c): step s = r / 4P, block db = c / 16:
 *               byte offset (s * head_dim/16 + db) * 1024 + (c % 16) * 64 + (r % 4P) * E
 *           (K: 16 rows x 64 bytes of their dims per piece; V: 16 dims x the step's 4P rows per piece.)
 * Device-side error: kv_len[b] + T > max_kv (AMPH_DEV_KV_OVERFLOW). */
amph_status amph_verify_attn(amph_ctx *ctx, const amph_tree *tree, const void *q, const void *k_cache,
                             const void *v_cache, const int32_t *kv_len, void *out, void *workspace);

/* ---- the same call for callers that cannot allocate ---------------------------------------------------
 * For code under HIP graph capture, tight serving loops and harnesses that forbid hipMalloc and have no
 * workspace to pass: the key-split partial results live in a static device array of the library
 * (AMPH_STATIC_SCRATCH_BYTES per GPU, held until the process ends) instead of the caller's workspace.
 * The call itself allocates and frees nothing.  Same arguments, arithmetic and results as amph_verify_attn.
 * AMPH_ESHAPE when the shape's partials exceed the array (the 7B and 13B shapes at batch 1 need 4.1 MiB;
 * shapes without key splits need none), AMPH_EINVAL when the current device is not the one the context was
 * created on.  All calls on one GPU share the array: calls that overlap in time there (different streams or
 * contexts) race; calls on one stream are ordered and safe.  Nothing in it needs to start at zero. */
#define AMPH_STATIC_SCRATCH_BYTES (8u << 20)
amph_status amph_verify_attn_static(amph_ctx *ctx, const amph_tree *tree, const void *q, const void *k_cache,
                                    const void *v_cache, const int32_t *kv_len, void *out);

/* ---- A10: greedy longest-accepted-prefix (Sec. 2 "Speculative Decoding"; Table 1, Temperature 0)
 * ok[root] = 1; ok[i] = ok[parent_i] and tree_tok[i] == tgt[parent_i]; best = deepest ok node
 * (lowest node id among equals); accept_len = depth(best); next_tok = tgt[best];
 * accept_path = node ids root..best, -1 padded.
 * Exactly one of tgt_argmax [B, T] int32 and tgt_logits [B, T, V] float32 is non-NULL; with logits
 * the per-node argmax (ties to the lowest id) is taken inside.
 *   accept_len, next_tok, best_node [B] int32     accept_path [B, K+1] int32 */
amph_status amph_accept(amph_ctx *ctx, const amph_tree *tree, const int32_t *tree_tok,
                        const int32_t *tgt_argmax, const float *tgt_logits, int32_t *accept_len,
                        int32_t *accept_path, int32_t *next_tok, int32_t *best_node, void *workspace);

/* ---- next: acceptance under random sampling (Table 2, Temperature = 0.7) -------------------------------
 * The paper reports results at this temperature but states no acceptance rule.  The rule built here is a
 * reading: typical acceptance as defined by the multi-head decoding framework whose tree and settings the
 * paper adopts (its reference cai2024medusa).  With p_j = softmax(tgt_logits[b, j, :] / temperature) and
 * H(p_j) its entropy in nats,
 *   pass[root] = 1;  pass[i] = pass[parent_i] and p_parent_i(tree_tok[i]) > min(eps, delta * exp(-H(p_parent_i)));
 *   best = deepest passing node (lowest node id among equals); accept_len, accept_path as in amph_accept;
 *   next_tok = the first v with sum_{w <= v} p_best(w) > u[b] (vocabulary order; the last token of non-zero
 *   probability if rounding leaves none).
 * All arithmetic is float32; sums run in a fixed order, so equal inputs give equal outputs.
 *   tgt_logits [B, T, V] float32 (amph_target_forward's logits_out); every row needs a finite maximum
 *   u [B] float32, uniform in [0, 1), drawn by the caller      outputs as in amph_accept
 * AMPH_EINVAL unless temperature > 0, eps >= 0 and delta >= 0.  A tree token outside [0, V) never passes. */
amph_status amph_accept_typical(amph_ctx *ctx, const amph_tree *tree, const int32_t *tree_tok,
                                const float *tgt_logits, float temperature, float eps, float delta,
                                const float *u, int32_t *accept_len, int32_t *accept_path, int32_t *next_tok,
                                int32_t *best_node, void *workspace);

/* ---- between two steps: commit the accepted path (Sec. 2 "Speculative Decoding") ---------------------
 * After amph_accept, for every batch element b with a = accept_len[b] and path nodes p_0 = root .. p_a:
 *   * in every layer the K/V rows of p_1 .. p_a move from tree slots kv_len[b] + p_j to rows kv_len[b] + j
 *     (the root already sits at kv_len[b]), so the committed rows are again contiguous;
 *   * if h_new != NULL the inputs of the next amph_draft are gathered: h_new[b, j] = hidden[b, p_j] (the
 *     target's final-normed hidden state), tok_new[b, j] = the token that follows position j (tree_tok of
 *     p_{j+1}, or next_tok[b] after p_a), rows j > a zero, n_new[b] = a + 1;
 *   * kv_len[b] += a + 1.
 * next_tok[b] is the root of the next tree.  All device pointers; nothing is read on the host.
 *   k_caches, v_caches as in amph_target_forward     hidden [B, T, d] float32 (its hidden_out)
 *   h_new [B, K+1, d] float32   tok_new [B, K+1] int32   n_new [B] int32   (call amph_draft with n_new = K+1) */
amph_status amph_commit(amph_ctx *ctx, const amph_tree *tree, int n_layers, void *k_caches, void *v_caches,
                        int32_t *kv_len, const int32_t *accept_len, const int32_t *accept_path,
                        const int32_t *next_tok, const int32_t *tree_tok, const float *hidden, float *h_new,
                        int32_t *tok_new, int32_t *n_new);

/* ---- A7 + A8 + A9: the target's forward pass over the tree tokens -------------------------------
 * x = embed[tree_tok]; for every layer: RMSNorm, Q/K/V projections, RoPE at tree_pos, K/V written to
 * cache rows [kv_len, kv_len + T), tree attention (as amph_verify_attn), output projection and
 * residual, RMSNorm, SwiGLU FFN and residual; then the final RMSNorm, the LM head and the per-node
 * argmax (ties to the lowest id).
 *   layers     host array [n_layers] of device-pointer structs; rms1 and rms2 are always read, a matrix
 *              only where the layer's tiled copy is absent (its pointer may then be NULL)
 *   tiled      host array [n_layers] of tiled copies (amph_pack_weights), or NULL: all row-major
 *   lm_head    [V, d] row-major, may be NULL when lm_head_tiled (AMPH_PACK_LMHEAD) is given
 *   k_caches, v_caches   [n_layers, B, n_heads] caches of max_kv * head_dim elements each, step-tiled as
 *              amph_verify_attn describes; the call writes the tree rows of every layer
 *   hidden_out [B, T, d] float32 (final-normed hidden states) or NULL
 *   logits_out [B, T, V] float32 or NULL
 *   tgt_argmax [B, T] int32 */
amph_status amph_target_forward(amph_ctx *ctx, const amph_tree *tree, const amph_layer_w *layers /* host */,
                                const amph_layer_tiled *tiled /* host or NULL */, int n_layers,
                                const void *embed, const void *final_norm, const void *lm_head,
                                const void *lm_head_tiled, const int32_t *tree_tok, const int32_t *tree_pos,
                                void *k_caches, void *v_caches, const int32_t *kv_len, float *hidden_out,
                                float *logits_out, int32_t *tgt_argmax, void *workspace);

/* ---- weight tiling for the target's GEMMs (A7, A9) -----------------------------------------------------
 * amph_tiled_bytes: size in bytes of the tiled copy for one role, for this context's shapes and type.
 * amph_pack_weights: writes it (asynchronously, on the context's stream) from the row-major device
 * matrices: QKV takes (wq, wk, wv), GATEUP takes (w_gate, w_up, NULL), the others (w, NULL, NULL).
 * dst must be 16-byte aligned and must not overlap the sources.  The results of amph_target_forward
 * are bit-identical with and without tiling: only addresses change, never the order of the sums. */
typedef enum { AMPH_PACK_QKV = 0, AMPH_PACK_WO, AMPH_PACK_GATEUP, AMPH_PACK_DOWN, AMPH_PACK_LMHEAD, AMPH_PACK_COUNT } amph_pack_role;
amph_status amph_tiled_bytes(const amph_ctx *ctx, int role, size_t *bytes /* host */);
amph_status amph_pack_weights(amph_ctx *ctx, int role, const void *w0, const void *w1, const void *w2, void *dst);

/* ---- K/V cache layout conversion (Sec. 2 "Tree Attention": the committed rows the tree attends to) ------
 * A caller that filled its caches elsewhere (a prefill) holds them row-major [n_caches, max_kv, head_dim]
 * with n_caches = layers * batch * heads; amph_verify_attn / amph_target_forward / amph_commit want the
 * step-tiled storage whose byte formulas stand at amph_verify_attn.  amph_pack_kv writes the tiled form of
 * every cache, amph_unpack_kv the row-major form back (all max_kv rows; one kernel per call, on the context's
 * stream).  Keys, values or both: a NULL source skips that half (its destination must then be NULL too).
 * Source and destination must not overlap.  n_caches <= 65535 * 16. */
amph_status amph_pack_kv(amph_ctx *ctx, const void *k_rows, const void *v_rows, void *k_tiled, void *v_tiled,
                         int n_caches);
amph_status amph_unpack_kv(amph_ctx *ctx, const void *k_tiled, const void *v_tiled, void *k_rows, void *v_rows,
                           int n_caches);

/* ---- choice of the verification-attention kernel, for tests and measurements -----------------------
 * The tree attention (amph_verify_attn, and inside amph_target_forward) has two kernels with the same
 * arithmetic: one feeds the matrix cores from registers (lowest fixed cost, short key ranges), one streams
 * the caches through a ring of LDS stages (long key ranges, many (batch, head) pairs).  kernel = -1 (the
 * default) chooses by shape; 0 and 1 force the first or the second for every later call on this context.
 * The workspace is sized for either.  Returns AMPH_EINVAL for any other value. */
amph_status amph_verify_kernel(amph_ctx *ctx, int kernel);

/* ---- per-kernel timing, for measurement ------------------------------------------------------------
 * Every kernel launch inside amph_draft / amph_target_forward / amph_verify_attn belongs to one kind.
 * amph_profile_kind selects one kind (or -1 for none): from then on one launch in `every` (>= 1; the
 * first, the every+1-th, ...) of that kind is timed by a pair of HIP events, up to max_launches timed
 * launches.  The matrix-core GEMM kinds (AMPH_K_T_*) pass the events with the launch, so they hold the
 * kernel's own begin and end time stamps; the other kinds are bracketed by events recorded on the
 * context's stream (a kind made of two kernels is bracketed as a whole).  A timed launch costs a few
 * microseconds of stream time, so a caller that also measures end-to-end time samples sparsely.
 * amph_profile_read SYNCHRONISES the stream, returns the summed elapsed time and the number of launches
 * recorded since the last read, and resets the count.  Not for use under stream capture. */
typedef enum {
  AMPH_K_FC = 0, AMPH_K_SAL_QKV, AMPH_K_SAL_ATTN, AMPH_K_SAL_WO, AMPH_K_SAL_GATEUP, AMPH_K_SAL_DOWN, AMPH_K_HEAD_MLP,
  AMPH_K_AEB_QKV, AMPH_K_AEB_ATTN, AMPH_K_AEB_WO, AMPH_K_LM_HEAD, AMPH_K_TOPK,
  AMPH_K_T_RMSNORM, AMPH_K_T_QKV, AMPH_K_VERIFY, AMPH_K_T_WO, AMPH_K_T_GATEUP, AMPH_K_T_DOWN, AMPH_K_T_LMHEAD,
  AMPH_K_COUNT
} amph_kernel_kind;
amph_status amph_profile_kind(amph_ctx *ctx, int kind, int max_launches, int every);
amph_status amph_profile_read(amph_ctx *ctx, double *total_ms /* host */, int *launches /* host */);

/* ---- single linear layers, exported for per-kernel parity tests and micro-benchmarks ------------
 * amph_gemv: y[m, n] = sum_k x[m, k] W[n, k] for m < M <= 8 (weight-streaming vector kernel).
 *   x [M, Kd] float32, W [N, Kd] T, y [M, N] float32.  Kd must be a multiple of 8.
 * amph_gemm: same contraction on the matrix cores for any M; x [M, Kd] T, y [M, N] float32.
 *   A row of x must be a multiple of 64 bytes (Kd % 32 == 0 in bf16, % 16 in float32).
 *   split_k in {0 (automatic), 1, 2, 4, 8}. */
amph_status amph_gemv(amph_ctx *ctx, const float *x, const void *W, float *y, int M, int N, int Kd);
amph_status amph_gemm(amph_ctx *ctx, const void *x, const void *W, float *y, int M, int N, int Kd,
                      int split_k, void *workspace);

#ifdef __cplusplus
}
#endif
#endif /* AMPH_H */
