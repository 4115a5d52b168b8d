// The small kernels of the step: single-query attention of the adaptation layers over their caches
// (Eq. 1), the K x K bi-directional attention of Eq. 5, per-row top-k / argmax (Eq. 6), candidate-tree
// construction, greedy acceptance, and the row-wise RMSNorm of the target path.
#include "kernels.h"

namespace amph {

// =====================================================================================================
// Single-query attention over a SAL cache: one new position per (batch, head) against rows
// [0, sal_len] of the cache (the new row included).  grid = (splits, heads, batch).  Each 16-byte
// fragment of a key/value row belongs to one lane; LPR lanes share a row, so a wave covers 64/LPR
// rows per load.  Running (max, sum, weighted values) are merged lane group -> wave -> workgroup ->
// key splits; the last workgroup of a (batch, head) to arrive folds the splits and writes the result.
// kv_stage: [B, 2, n_heads, max_kv, DH] T.   partials: [B, n_heads, splits, DH + 2] float32.
// =====================================================================================================
template <typename T, int DH>
__global__ __launch_bounds__(256) void k_sal_attn(const float *qbuf, const T *kv_stage, const int32_t *sal_len,
                                                  int n_heads, int max_kv, float *partials, unsigned int *counters,
                                                  float *out) {
  constexpr int PER = Elem<T>::PER;
  constexpr int LPR = DH / PER;          // lanes per row
  constexpr int G = WAVE / LPR;          // rows per wave load
  constexpr int U = 4;
  __shared__ float sm_m[4], sm_l[4];
  __shared__ float sm_o[4][DH];
  __shared__ int s_flag;
  const int b = blockIdx.z, h = blockIdx.y, s = blockIdx.x, S = gridDim.x;
  const int d = n_heads * DH;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int grp = lane / LPR, li = lane % LPR;
  int len = sal_len[b];
  int n = (len < 0 || len + 1 > max_kv) ? 0 : len + 1;
  const int per = (n + S - 1) / S;
  const int k0 = s * per, k1 = min(n, k0 + per);
  const float scale = 1.4426950408889634f * rsqrtf((float)DH);
  float qv[PER];
  #pragma unroll
  for (int j = 0; j < PER; ++j) qv[j] = qbuf[(size_t)b * d + h * DH + li * PER + j] * scale;
  const T *kbase = kv_stage + (((size_t)b * 2 + 0) * n_heads + h) * (size_t)max_kv * DH;
  const T *vbase = kv_stage + (((size_t)b * 2 + 1) * n_heads + h) * (size_t)max_kv * DH;
  float m = NEG_BIG, l = 0.f, o[PER];
  #pragma unroll
  for (int j = 0; j < PER; ++j) o[j] = 0.f;
  for (int jb = k0 + wave * (U * G); jb < k1; jb += 4 * U * G) {
    uint4 kf[U], vf[U];
    #pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = jb + u * G + grp;
      if (j < k1) {
        kf[u] = ldg16(kbase + (size_t)j * DH + li * PER);
        vf[u] = ldg16(vbase + (size_t)j * DH + li * PER);
      } else {
        kf[u] = make_uint4(0u, 0u, 0u, 0u);
        vf[u] = kf[u];
      }
    }
    #pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = jb + u * G + grp;
      float kk[PER], vv[PER];
      Elem<T>::unpack(kf[u], kk);
      Elem<T>::unpack(vf[u], vv);
      float sc = 0.f;
      #pragma unroll
      for (int e = 0; e < PER; ++e) sc = fmaf(qv[e], kk[e], sc);
      #pragma unroll
      for (int off = 1; off < LPR; off <<= 1) sc += __shfl_xor(sc, off, WAVE);
      if (j < k1) {
        const float mn = fmaxf(m, sc);
        const float corr = exp2f(m - mn), p = exp2f(sc - mn);
        l = l * corr + p;
        #pragma unroll
        for (int e = 0; e < PER; ++e) o[e] = o[e] * corr + p * vv[e];
        m = mn;
      }
    }
  }
  // lane groups -> wave
  #pragma unroll
  for (int off = LPR; off < WAVE; off <<= 1) {
    const float m2 = __shfl_xor(m, off, WAVE), l2 = __shfl_xor(l, off, WAVE);
    const float mn = fmaxf(m, m2);
    const float c1 = exp2f(m - mn), c2 = exp2f(m2 - mn);
    l = l * c1 + l2 * c2;
    #pragma unroll
    for (int e = 0; e < PER; ++e) {
      const float o2 = __shfl_xor(o[e], off, WAVE);
      o[e] = o[e] * c1 + o2 * c2;
    }
    m = mn;
  }
  if (grp == 0) {
    #pragma unroll
    for (int e = 0; e < PER; ++e) sm_o[wave][li * PER + e] = o[e];
    if (li == 0) { sm_m[wave] = m; sm_l[wave] = l; }
  }
  __syncthreads();
  // waves -> workgroup
  const float mw = fmaxf(fmaxf(sm_m[0], sm_m[1]), fmaxf(sm_m[2], sm_m[3]));
  float lw = 0.f;
  #pragma unroll
  for (int w = 0; w < 4; ++w) lw += sm_l[w] * exp2f(sm_m[w] - mw);
  float ow = 0.f;
  if (threadIdx.x < DH) {
    #pragma unroll
    for (int w = 0; w < 4; ++w) ow += sm_o[w][threadIdx.x] * exp2f(sm_m[w] - mw);
  }
  float *dst = out + (size_t)b * d + h * DH;
  if (S == 1) {
    if (threadIdx.x < DH) dst[threadIdx.x] = (lw > 0.f) ? ow / lw : 0.f;
    return;
  }
  float *part = partials + (((size_t)b * n_heads + h) * S + s) * (DH + 2);
  if (threadIdx.x < DH) part[2 + threadIdx.x] = ow;
  if (threadIdx.x == 0) { part[0] = mw; part[1] = lw; }
  if (!arrive_and_is_last(counters + (size_t)b * n_heads + h, (unsigned)S, &s_flag)) return;
  const float *p0 = partials + ((size_t)b * n_heads + h) * S * (DH + 2);
  float mt = NEG_BIG;
  for (int i = 0; i < S; ++i) mt = fmaxf(mt, p0[(size_t)i * (DH + 2)]);
  float lt = 0.f, ot = 0.f;
  for (int i = 0; i < S; ++i) {
    const float wgt = exp2f(p0[(size_t)i * (DH + 2)] - mt);
    lt += p0[(size_t)i * (DH + 2) + 1] * wgt;
    if (threadIdx.x < DH) ot += p0[(size_t)i * (DH + 2) + 2 + threadIdx.x] * wgt;
  }
  if (threadIdx.x < DH) dst[threadIdx.x] = (lt > 0.f) ? ot / lt : 0.f;
}

int sal_attn_splits(int n_heads, int batch, int max_kv) {
  int s = 256 / (n_heads * batch);
  const int cap = (max_kv + 63) / 64;
  if (s > cap) s = cap;
  if (s > 16) s = 16;
  return s < 1 ? 1 : s;
}
size_t sal_attn_ws_floats(int n_heads, int batch, int d_h, int max_kv) {
  return (size_t)batch * n_heads * sal_attn_splits(n_heads, batch, max_kv) * (d_h + 2);
}

template <typename T>
hipError_t launch_sal_attn(hipStream_t st, const float *qbuf, const void *kv_stage, const int32_t *sal_len, int B,
                           int n_heads, int d_h, int max_kv, float *partials, unsigned int *counters, float *out) {
  const dim3 grid(sal_attn_splits(n_heads, B, max_kv), n_heads, B);
  if (d_h == 64)
    hipLaunchKernelGGL((k_sal_attn<T, 64>), grid, dim3(256), 0, st, qbuf, (const T *)kv_stage, sal_len, n_heads, max_kv,
                       partials, counters, out);
  else if (d_h == 128)
    hipLaunchKernelGGL((k_sal_attn<T, 128>), grid, dim3(256), 0, st, qbuf, (const T *)kv_stage, sal_len, n_heads, max_kv,
                       partials, counters, out);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}
template hipError_t launch_sal_attn<float>(hipStream_t, const float *, const void *, const int32_t *, int, int, int, int,
                                           float *, unsigned int *, float *);
template hipError_t launch_sal_attn<bf16_t>(hipStream_t, const float *, const void *, const int32_t *, int, int, int,
                                            int, float *, unsigned int *, float *);

// =====================================================================================================
// Eq. 5 core: for one (batch, head) the K x K score matrix of the K head positions, a row softmax
// with no mask, and the weighted sum of the value rows.  Q, Kk, V, ctx: [B * K, d] float32.
// =====================================================================================================
__global__ __launch_bounds__(128) void k_aeb_attn(const float *Q, const float *Kk, const float *V, int K, int n_heads,
                                                  int d_h, float *ctx) {
  __shared__ float sc[AMPH_MAX_HEADS_K * AMPH_MAX_HEADS_K];
  const int h = blockIdx.x, b = blockIdx.y;
  const int d = n_heads * d_h;
  const size_t base = (size_t)b * K * d + (size_t)h * d_h;
  const int t = threadIdx.x;
  if (t < K * K) {
    const int i = t / K, j = t % K;
    float s = 0.f;
    for (int e = 0; e < d_h; ++e) s = fmaf(Q[base + (size_t)i * d + e], Kk[base + (size_t)j * d + e], s);
    sc[t] = s * rsqrtf((float)d_h);
  }
  __syncthreads();
  if (t < K) {
    float mx = sc[t * K];
    for (int j = 1; j < K; ++j) mx = fmaxf(mx, sc[t * K + j]);
    float sum = 0.f;
    for (int j = 0; j < K; ++j) { const float e = __expf(sc[t * K + j] - mx); sc[t * K + j] = e; sum += e; }
    const float inv = 1.0f / sum;
    for (int j = 0; j < K; ++j) sc[t * K + j] *= inv;
  }
  __syncthreads();
  for (int e = t; e < d_h; e += blockDim.x) {
    for (int i = 0; i < K; ++i) {
      float o = 0.f;
      for (int j = 0; j < K; ++j) o = fmaf(sc[i * K + j], V[base + (size_t)j * d + e], o);
      ctx[base + (size_t)i * d + e] = o;
    }
  }
}

hipError_t launch_aeb_attn(hipStream_t st, const float *Q, const float *Kk, const float *V, int B, int K, int n_heads,
                           int d_h, float *ctx) {
  if (K < 1 || K > AMPH_MAX_HEADS_K) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_aeb_attn, dim3(n_heads, B), dim3(128), 0, st, Q, Kk, V, K, n_heads, d_h, ctx);
  return hipGetLastError();
}

// =====================================================================================================
// Per-row top-k (Eq. 6) by repeated selection.  One 1024-thread workgroup per row; thread t owns
// elements t, t + 1024, ... in registers.  Each round picks the best remaining element of the row:
// thread-local best -> wave butterfly -> 16 wave winners in LDS, read by everybody.  "Better" means a
// larger value, or the same value and a smaller index, so the result is sorted and ties are
// deterministic.  Block 0 also advances the caller's length counters (used by the draft call).
// =====================================================================================================
struct Cand { float v; int i; };
__device__ __forceinline__ bool better(float v1, int i1, float v2, int i2) {
  return (v1 > v2) || (v1 == v2 && i1 < i2);
}

template <int NPT>
__global__ __launch_bounds__(1024) void k_topk_rows(const float *logits, int V, int k, int32_t *idx, float *val,
                                                    int32_t *advance, int n_advance, int advance_by) {
  __shared__ float s_v[2][16];
  __shared__ int s_i[2][16];
  const int row = blockIdx.x, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const float *src = logits + (size_t)row * V;
  const float NEG_INF = -__builtin_huge_valf();
  float x[NPT];
  #pragma unroll
  for (int j = 0; j < NPT; ++j) {
    const int e = t + j * 1024;
    x[j] = (e < V) ? src[e] : NEG_INF;
  }
  // thread-local best; index V marks "nothing left"
  float bv = NEG_INF; int bi = V;
  #pragma unroll
  for (int j = 0; j < NPT; ++j) {
    const int e = t + j * 1024;
    if (e < V && better(x[j], e, bv, bi)) { bv = x[j]; bi = e; }
  }
  for (int r = 0; r < k; ++r) {
    float wv = bv; int wi = bi;
    #pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const float ov = __shfl_xor(wv, off, WAVE);
      const int oi = __shfl_xor(wi, off, WAVE);
      if (better(ov, oi, wv, wi)) { wv = ov; wi = oi; }
    }
    const int buf = r & 1;
    if (lane == 0) { s_v[buf][wave] = wv; s_i[buf][wave] = wi; }
    __syncthreads();
    float gv = s_v[buf][0]; int gi = s_i[buf][0];
    #pragma unroll
    for (int w = 1; w < 16; ++w) {
      const float ov = s_v[buf][w]; const int oi = s_i[buf][w];
      if (better(ov, oi, gv, gi)) { gv = ov; gi = oi; }
    }
    if (t == 0) {
      if (idx) idx[(size_t)row * k + r] = (gi < V) ? gi : -1;
      if (val) val[(size_t)row * k + r] = gv;
    }
    if (gi < V && (gi & 1023) == t) {          // the owner retires the element and rescans its own
      const int jj = gi >> 10;
      bv = NEG_INF; bi = V;
      #pragma unroll
      for (int j = 0; j < NPT; ++j) {
        if (j == jj) x[j] = NEG_INF;
        const int e = t + j * 1024;
        if (e < V && j != jj && x[j] > NEG_INF && better(x[j], e, bv, bi)) { bv = x[j]; bi = e; }
      }
    }
  }
  if (row == 0 && advance && t < n_advance) advance[t] += advance_by;
}

hipError_t launch_topk_rows(hipStream_t st, const float *logits, int rows, int V, int k, int32_t *idx, float *val,
                            int32_t *advance, int n_advance, int advance_by) {
  if (rows < 1 || V < 1 || k < 1 || k > V || n_advance > 1024) return hipErrorInvalidValue;
  if (V <= 32 * 1024)
    hipLaunchKernelGGL((k_topk_rows<32>), dim3(rows), dim3(1024), 0, st, logits, V, k, idx, val, advance, n_advance,
                       advance_by);
  else if (V <= 64 * 1024)
    hipLaunchKernelGGL((k_topk_rows<64>), dim3(rows), dim3(1024), 0, st, logits, V, k, idx, val, advance, n_advance,
                       advance_by);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_row_argmax(hipStream_t st, const float *logits, int rows, int V, int32_t *out) {
  return launch_topk_rows(st, logits, rows, V, 1, out, nullptr, nullptr, 0, 0);
}

// =====================================================================================================
// Candidate tree: node i at depth m >= 1 takes the rank_i-th candidate of head m; the root takes the
// token the target just sampled; position = committed length + depth.
// =====================================================================================================
__global__ void k_tree_build(const int32_t *depth, const int32_t *rank, int T, int K, int topk,
                             const int32_t *root_tok, const int32_t *topk_idx, const int32_t *kv_len, int32_t *tree_tok,
                             int32_t *tree_pos) {
  const int b = blockIdx.x, i = threadIdx.x;
  if (i >= T) return;
  const int m = depth[i];
  const int tok = (m == 0) ? root_tok[b] : topk_idx[((size_t)b * K + (m - 1)) * topk + rank[i]];
  tree_tok[(size_t)b * T + i] = tok;
  tree_pos[(size_t)b * T + i] = kv_len[b] + m;
}

hipError_t launch_tree_build(hipStream_t st, const int32_t *depth, const int32_t *rank, int T, int B, int K, int topk,
                             const int32_t *root_tok, const int32_t *topk_idx, const int32_t *kv_len, int32_t *tree_tok,
                             int32_t *tree_pos) {
  hipLaunchKernelGGL(k_tree_build, dim3(B), dim3(AMPH_MAX_TREE), 0, st, depth, rank, T, K, topk, root_tok, topk_idx,
                     kv_len, tree_tok, tree_pos);
  return hipGetLastError();
}

// =====================================================================================================
// Greedy acceptance.  Thread i checks its whole ancestor chain (at most K hops): node i is accepted
// iff every node j on the chain carries the target's argmax at parent(j).  The deepest accepted node
// wins (lowest id among equals); thread 0 writes the path by walking up from it.
// =====================================================================================================
__global__ __launch_bounds__(AMPH_MAX_TREE) void k_accept(const int32_t *parent, const int32_t *depth, int T, int K,
                                                          const int32_t *tree_tok, const int32_t *tgt, int32_t *accept_len,
                                                          int32_t *accept_path, int32_t *next_tok, int32_t *best_node) {
  __shared__ int s_key[AMPH_MAX_TREE / WAVE];
  const int b = blockIdx.x, i = threadIdx.x;
  const int32_t *tok = tree_tok + (size_t)b * T;
  const int32_t *tg = tgt + (size_t)b * T;
  int key = -1;
  if (i < T) {
    bool ok = true;
    int j = i;
    for (int hop = 0; hop < AMPH_MAX_HEADS_K && j > 0; ++hop) {
      const int p = parent[j];
      if (tok[j] != tg[p]) { ok = false; break; }
      j = p;
    }
    if (ok) key = depth[i] * 256 + (255 - i);
  }
  #pragma unroll
  for (int off = 32; off >= 1; off >>= 1) key = max(key, __shfl_xor(key, off, WAVE));
  if ((i & 63) == 0) s_key[i >> 6] = key;
  __syncthreads();
  if (i == 0) {
    int best_key = s_key[0];
    for (int w = 1; w < AMPH_MAX_TREE / WAVE; ++w) best_key = max(best_key, s_key[w]);
    const int a = best_key >> 8, best = 255 - (best_key & 255);     // the root always qualifies
    accept_len[b] = a;
    best_node[b] = best;
    next_tok[b] = tg[best];
    for (int dd = 0; dd <= K; ++dd) accept_path[(size_t)b * (K + 1) + dd] = -1;
    int j = best;
    for (int dd = a; dd >= 0 && j >= 0; --dd) { accept_path[(size_t)b * (K + 1) + dd] = j; j = parent[j]; }
  }
}

hipError_t launch_accept(hipStream_t st, const int32_t *parent, const int32_t *depth, int T, int B, int K,
                         const int32_t *tree_tok, const int32_t *tgt, int32_t *accept_len, int32_t *accept_path,
                         int32_t *next_tok, int32_t *best_node) {
  hipLaunchKernelGGL(k_accept, dim3(B), dim3(AMPH_MAX_TREE), 0, st, parent, depth, T, K, tree_tok, tgt, accept_len,
                     accept_path, next_tok, best_node);
  return hipGetLastError();
}

// =====================================================================================================
// Row-wise RMSNorm for the target path: xn = x / rms(x) * g, stored as T for the matrix cores.
// With tok != NULL the row is first gathered from the embedding table (and kept in x as float32).
// =====================================================================================================
template <typename T>
__global__ __launch_bounds__(256) void k_rmsnorm_rows(float *x, const T *embed, const int32_t *tok, int vocab, const T *g,
                                                      int d, float eps, T *xn, float *hidden_out, uint32_t *dev_status) {
  __shared__ float red[4];
  const int row = blockIdx.x;
  float *xr = x + (size_t)row * d;
  if (tok) {
    int t = tok[row];
    if (t < 0 || t >= vocab) { if (threadIdx.x == 0) atomicOr(dev_status, 4u); t = 0; }
    const T *er = embed + (size_t)t * d;
    for (int k = threadIdx.x; k < d; k += 256) xr[k] = Elem<T>::to_f32(er[k]);
  }
  float ss = 0.f;
  for (int k = threadIdx.x; k < d; k += 256) { const float v = xr[k]; ss = fmaf(v, v, ss); }   // own writes: visible
  const float rs = rsqrtf(block_sum_256(ss, red) / (float)d + eps);
  for (int k = threadIdx.x; k < d; k += 256) {
    const float v = xr[k] * rs * Elem<T>::to_f32(g[k]);
    xn[(size_t)row * d + k] = Elem<T>::from_f32(v);
    if (hidden_out) hidden_out[(size_t)row * d + k] = v;
  }
}

template <typename T>
hipError_t launch_rmsnorm_rows(hipStream_t st, float *x, const void *embed, const int32_t *tok, int vocab,
                               const void *g, int rows, int d, float eps, void *xn, float *hidden_out,
                               uint32_t *dev_status) {
  hipLaunchKernelGGL((k_rmsnorm_rows<T>), dim3(rows), dim3(256), 0, st, x, (const T *)embed, tok, vocab, (const T *)g, d,
                     eps, (T *)xn, hidden_out, dev_status);
  return hipGetLastError();
}
template hipError_t launch_rmsnorm_rows<float>(hipStream_t, float *, const void *, const int32_t *, int, const void *,
                                               int, int, float, void *, float *, uint32_t *);
template hipError_t launch_rmsnorm_rows<bf16_t>(hipStream_t, float *, const void *, const int32_t *, int, const void *,
                                                int, int, float, void *, float *, uint32_t *);

}  // namespace amph
