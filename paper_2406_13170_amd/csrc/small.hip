// The small kernels of the step: single-query attention of the adaptation layers over their caches
// (Eq. 1), the K x K bi-directional attention of Eq. 5, per-row top-k / argmax (Eq. 6), candidate-tree
// construction, greedy acceptance, and the row-wise RMSNorm (+ partial-sum fold) of the target path.
#include "kernels.h"
#include <algorithm>

namespace amph {

// =====================================================================================================
// Single-query attention over a SAL cache: query row (b, j) = new position j of batch element b against
// rows [0, sal_len[b] + j] of the cache (its own new row included, later new rows excluded: causal among
// the new positions).  grid = (heads, batch * R), 1024 threads: the 16
// waves of a workgroup stride over the rows.  Each 16-byte fragment of a key/value row belongs to one
// lane; LPR lanes share a row, so a wave covers 64/LPR rows per load.  Running (max, sum, weighted
// values) are merged lane group -> wave -> workgroup; no workgroup depends on another.
// kv_stage: [B, 2, n_heads, max_kv, DH] T.   out: [B, d] float32.
// =====================================================================================================
constexpr int SA_WAVES = 16;

template <typename T, int DH>
__global__ __launch_bounds__(SA_WAVES * 64) void k_sal_attn(const float *qbuf, const T *kv_stage, const int32_t *sal_len,
                                                            int n_heads, int max_kv, float *out, int R,
                                                            const int32_t *n_valid, int last_only) {
  constexpr int PER = Elem<T>::PER;
  constexpr int LPR = DH / PER;          // lanes per row
  constexpr int G = WAVE / LPR;          // rows per wave load
  constexpr int U = 4;
  __shared__ float sm_m[SA_WAVES], sm_l[SA_WAVES];
  __shared__ float sm_o[SA_WAVES][DH];
  // last_only: one workgroup row per batch element, serving its last live position (query row b * R + jn of qbuf,
  // output row b); otherwise one per (element, position)
  const int h = blockIdx.x;
  int row = blockIdx.y, b, jn, out_row;
  if (last_only) {
    b = row;
    jn = min(max(n_valid ? n_valid[b] : R, 1), R) - 1;
    out_row = b;
    row = b * R + jn;
  } else {
    b = row / R; jn = row % R; out_row = row;
  }
  const int d = n_heads * DH;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int grp = lane / LPR, li = lane % LPR;
  const int len = sal_len[b] + jn;
  const bool live = !(n_valid && jn >= n_valid[b]);
  const int n = (!live || sal_len[b] < 0 || len + 1 > max_kv) ? 0 : len + 1;
  const float scale = 1.4426950408889634f * rsqrtf((float)DH);
  float qv[PER];
  #pragma unroll
  for (int j = 0; j < PER; ++j) qv[j] = qbuf[(size_t)row * d + h * DH + li * PER + j] * scale;
  const T *kbase = kv_stage + (((size_t)b * 2 + 0) * n_heads + h) * (size_t)max_kv * DH;
  const T *vbase = kv_stage + (((size_t)b * 2 + 1) * n_heads + h) * (size_t)max_kv * DH;
  float m = NEG_BIG, l = 0.f, o[PER];
  #pragma unroll
  for (int j = 0; j < PER; ++j) o[j] = 0.f;
  for (int jb = wave * (U * G); jb < n; jb += SA_WAVES * U * G) {
    uint4 kf[U], vf[U];
    #pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = min(jb + u * G + grp, n - 1);     // unconditional loads; rows past the end are skipped below
      kf[u] = ldg16_stream(kbase + (size_t)j * DH + li * PER);
      vf[u] = ldg16_stream(vbase + (size_t)j * DH + li * PER);
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
      if (j < n) {
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
  if (threadIdx.x < DH) {
    float mw = sm_m[0];
    #pragma unroll
    for (int w = 1; w < SA_WAVES; ++w) mw = fmaxf(mw, sm_m[w]);
    float lw = 0.f, ow = 0.f;
    #pragma unroll
    for (int w = 0; w < SA_WAVES; ++w) {
      const float f = exp2f(sm_m[w] - mw);
      lw += sm_l[w] * f;
      ow += sm_o[w][threadIdx.x] * f;
    }
    out[(size_t)out_row * d + h * DH + threadIdx.x] = (lw > 0.f) ? ow / lw : 0.f;
  }
}

template <typename T>
hipError_t launch_sal_attn(hipStream_t st, const float *qbuf, const void *kv_stage, const int32_t *sal_len, int B,
                           int n_heads, int d_h, int max_kv, float *out, int R, const int32_t *n_valid, int last_only) {
  const dim3 grid(n_heads, last_only ? B : B * R), block(SA_WAVES * 64);
  if (d_h == 64)
    hipLaunchKernelGGL((k_sal_attn<T, 64>), grid, block, 0, st, qbuf, (const T *)kv_stage, sal_len, n_heads, max_kv, out, R,
                       n_valid, last_only);
  else if (d_h == 128)
    hipLaunchKernelGGL((k_sal_attn<T, 128>), grid, block, 0, st, qbuf, (const T *)kv_stage, sal_len, n_heads, max_kv, out, R,
                       n_valid, last_only);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}
template hipError_t launch_sal_attn<float>(hipStream_t, const float *, const void *, const int32_t *, int, int, int, int,
                                           float *, int, const int32_t *, int);
template hipError_t launch_sal_attn<bf16_t>(hipStream_t, const float *, const void *, const int32_t *, int, int, int,
                                            int, float *, int, const int32_t *, int);

// =====================================================================================================
// Eq. 5 core: for one (batch, head) the K x K score matrix of the K head positions, a row softmax
// with no mask, and the weighted sum of the value rows.  Q, Kk, V, ctx: [B * K, d] float32.
// The head's K rows of Q, K and V are first parked in LDS.
// =====================================================================================================
__global__ __launch_bounds__(128) void k_aeb_attn(const float *Q, const float *Kk, const float *V, int K, int n_heads,
                                                  int d_h, float *ctx) {
  __shared__ float sq[AMPH_MAX_HEADS_K * 128], sk[AMPH_MAX_HEADS_K * 128], sv[AMPH_MAX_HEADS_K * 128];
  __shared__ float sc[AMPH_MAX_HEADS_K * AMPH_MAX_HEADS_K];
  const int h = blockIdx.x, b = blockIdx.y;
  const int d = n_heads * d_h;
  const size_t base = (size_t)b * K * d + (size_t)h * d_h;
  const int t = threadIdx.x;
  for (int i = t; i < K * d_h; i += blockDim.x) {
    const int r = i / d_h, e = i % d_h;
    sq[i] = Q[base + (size_t)r * d + e];
    sk[i] = Kk[base + (size_t)r * d + e];
    sv[i] = V[base + (size_t)r * d + e];
  }
  __syncthreads();
  if (t < K * K) {
    const int i = t / K, j = t % K;
    float s = 0.f;
    for (int e = 0; e < d_h; ++e) s = fmaf(sq[i * d_h + e], sk[j * d_h + e], s);
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
      for (int j = 0; j < K; ++j) o = fmaf(sc[i * K + j], sv[j * d_h + e], o);
      ctx[base + (size_t)i * d + e] = o;
    }
  }
}

hipError_t launch_aeb_attn(hipStream_t st, const float *Q, const float *Kk, const float *V, int B, int K, int n_heads,
                           int d_h, float *ctx) {
  if (K < 1 || K > AMPH_MAX_HEADS_K || d_h > 128) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_aeb_attn, dim3(n_heads, B), dim3(128), 0, st, Q, Kk, V, K, n_heads, d_h, ctx);
  return hipGetLastError();
}

// =====================================================================================================
// Per-row top-k (Eq. 6) by repeated selection inside single waves (no workgroup barriers).
// "Better" means a larger value, or the same value and a smaller index, so results are sorted and
// ties deterministic.
//   pass 1: every wave owns TK_CHUNK consecutive logits of one row (TK_NPT per lane) and emits its own
//           top-k as (value, index) candidates;
//   pass 2: one wave per row selects the top-k of all candidates of the row.
// The top-k of a union is the top-k of the parts' top-k, so the result is exact.
// =====================================================================================================
constexpr int TK_NPT = 8, TK_CHUNK = TK_NPT * WAVE;      // 512 logits per wave
constexpr int TK_MAXC = 32;                              // pass 2: candidates per lane

// Cache length of element i after its new rows: advanced only when every new row fitted (the kernels that write
// the rows skipped those past the limit and raised the overflow flag; the length then stays where it was).
__device__ __forceinline__ void advance_one(int32_t *len, int i, int by, int limit) {
  const int v = len[i];
  if (v >= 0 && by >= 0 && v + by <= limit) len[i] = v + by;
}

__global__ __launch_bounds__(256) void k_topk_pass1(const float *logits, int V, int k, int chunks_per_row, float *cand_v,
                                                    int *cand_i) {
  const int row = blockIdx.y, chunk = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (chunk >= chunks_per_row) return;                    // whole wave leaves together
  const float *src = logits + (size_t)row * V;
  float x[TK_NPT]; int id[TK_NPT];
  #pragma unroll
  for (int j = 0; j < TK_NPT; ++j) {
    // unconditional loads from clamped addresses (a predicated load makes the compiler wait for each one)
    const int e = chunk * TK_CHUNK + j * WAVE + lane;
    id[j] = (e < V) ? e : V;
    x[j] = src[min(e, V - 1)];
  }
  const size_t o = ((size_t)row * chunks_per_row + chunk) * k;
  wave_select<TK_NPT>(x, id, k, V, cand_v + o, cand_i + o);
}

__global__ __launch_bounds__(64) void k_topk_pass2(const float *cand_v, const int *cand_i, int n_cand, int V, int k,
                                                   int32_t *idx, float *val, int32_t *advance, int n_advance,
                                                   int advance_by, const int32_t *advance_each, int advance_limit) {
  const int row = blockIdx.x, lane = threadIdx.x;
  float x[TK_MAXC]; int id[TK_MAXC];
  #pragma unroll
  for (int j = 0; j < TK_MAXC; ++j) {
    const int c = min(j * WAVE + lane, n_cand - 1);
    id[j] = cand_i[(size_t)row * n_cand + c];
    x[j] = cand_v[(size_t)row * n_cand + c];
  }
  #pragma unroll
  for (int j = 0; j < TK_MAXC; ++j)
    if (j * WAVE + lane >= n_cand || id[j] < 0) id[j] = V;
  __shared__ float sv[AMPH_MAX_TOPK];
  __shared__ int si[AMPH_MAX_TOPK];
  wave_select<TK_MAXC>(x, id, k, V, sv, si);
  __syncthreads();
  if (lane < k) {
    if (idx) idx[(size_t)row * k + lane] = si[lane];
    if (val) val[(size_t)row * k + lane] = sv[lane];
  }
  if (row == 0 && advance)
    for (int i = lane; i < n_advance; i += WAVE) advance_one(advance, i, advance_each ? advance_each[i] : advance_by, advance_limit);
}

// One workgroup of 1024 threads per row for vocabularies up to 65536: every thread keeps NPT logits (element
// j * 1024 + tid in slot j) and its own best; k rounds of (wave butterfly, 16 wave winners through LDS, every wave
// folds them again) pick the winners, and only the thread that owned a winner rescans its slots.  Same order and
// tie rule as the two-pass version, one launch instead of two.
template <int NPT>
__global__ __launch_bounds__(1024) void k_topk_row(const float *logits, int V, int k, int32_t *idx, float *val,
                                                   int32_t *advance, int n_advance, int advance_by,
                                                   const int32_t *advance_each, int advance_limit) {
  __shared__ float sm_v[16];
  __shared__ int sm_i[16];
  const float NEG_INF = -__builtin_huge_valf();
  const int NONE = 0x7fffffff;
  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float *src = logits + (size_t)row * V;
  float x[NPT];
  unsigned long long alive = 0ull;
  #pragma unroll
  for (int j = 0; j < NPT; ++j) {
    const int e = j * 1024 + tid;
    x[j] = src[min(e, V - 1)];                            // unconditional loads from clamped addresses
    if (e < V) alive |= 1ull << j;
  }
  float bv; int bi;
  auto rescan = [&]() {
    bv = NEG_INF; bi = NONE;
    #pragma unroll
    for (int j = 0; j < NPT; ++j)
      if (((alive >> j) & 1ull) && better(x[j], j * 1024 + tid, bv, bi)) { bv = x[j]; bi = j * 1024 + tid; }
  };
  rescan();
  for (int r = 0; r < k; ++r) {
    float wv = bv; int wi = bi;
    #pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const float ov = __shfl_xor(wv, off, WAVE);
      const int oi = __shfl_xor(wi, off, WAVE);
      if (better(ov, oi, wv, wi)) { wv = ov; wi = oi; }
    }
    if (lane == 0) { sm_v[wave] = wv; sm_i[wave] = wi; }
    __syncthreads();
    float gv = (lane < 16) ? sm_v[lane] : NEG_INF;
    int gi = (lane < 16) ? sm_i[lane] : NONE;
    #pragma unroll
    for (int off = 8; off >= 1; off >>= 1) {
      const float ov = __shfl_xor(gv, off, WAVE);
      const int oi = __shfl_xor(gi, off, WAVE);
      if (better(ov, oi, gv, gi)) { gv = ov; gi = oi; }
    }
    gv = __shfl(gv, 0, WAVE);
    gi = __shfl(gi, 0, WAVE);
    if (tid == 0) {
      if (idx) idx[(size_t)row * k + r] = (gi == NONE) ? -1 : gi;
      if (val) val[(size_t)row * k + r] = gv;
    }
    if (gi != NONE && gi == bi) {                          // this thread owned the winner: retire it and rescan
      alive &= ~(1ull << (gi >> 10));
      rescan();
    }
    __syncthreads();                                       // the wave winners are rewritten in the next round
  }
  if (row == 0 && advance)
    for (int i = tid; i < n_advance; i += 1024) advance_one(advance, i, advance_each ? advance_each[i] : advance_by, advance_limit);
}

// Top-k of the candidates the fused LM head left: one 1024-thread workgroup per row.  Every wave selects the top k
// of its share (NPT candidates per lane), the 16 x k survivors go through LDS, and the first wave selects among them.
template <int NPT>
__global__ __launch_bounds__(1024) void k_topk_merge(const float *cand_v, const int *cand_i, int n_cand, int V, int k,
                                                     int32_t *idx, float *val, int32_t *advance, int n_advance, int advance_by,
                                                     const int32_t *advance_each, int advance_limit) {
  __shared__ float sv[16 * AMPH_MAX_TOPK];
  __shared__ int si[16 * AMPH_MAX_TOPK];
  __shared__ float fv[AMPH_MAX_TOPK];
  __shared__ int fi[AMPH_MAX_TOPK];
  const int row = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float *cv = cand_v + (size_t)row * n_cand;
  const int *ci = cand_i + (size_t)row * n_cand;
  float x[NPT]; int id[NPT];
  #pragma unroll
  for (int j = 0; j < NPT; ++j) {                          // unconditional loads from clamped addresses
    const int c = j * 1024 + tid, cc = min(c, n_cand - 1);
    const int t = ci[cc];
    x[j] = cv[cc];
    id[j] = (c < n_cand && t >= 0 && t < V) ? t : V;
  }
  wave_select<NPT>(x, id, k, V, sv + wave * k, si + wave * k);
  __syncthreads();
  if (wave == 0) {
    constexpr int NP2 = (16 * AMPH_MAX_TOPK) / WAVE;       // 4
    float y[NP2]; int jd[NP2];
    #pragma unroll
    for (int j = 0; j < NP2; ++j) {
      const int c = j * WAVE + lane, cc = min(c, 16 * k - 1);
      y[j] = sv[cc];
      jd[j] = (c < 16 * k && si[cc] >= 0) ? si[cc] : V;
    }
    wave_select<NP2>(y, jd, k, V, fv, fi);
  }
  __syncthreads();
  if (tid < k) {
    if (idx) idx[(size_t)row * k + tid] = fi[tid];
    if (val) val[(size_t)row * k + tid] = fv[tid];
  }
  if (row == 0 && advance)
    for (int i = tid; i < n_advance; i += 1024) advance_one(advance, i, advance_each ? advance_each[i] : advance_by, advance_limit);
}

hipError_t launch_topk_merge(hipStream_t st, const float *cand_v, const int *cand_i, int rows, int n_cand, int V, int k,
                             int32_t *idx, float *val, int32_t *advance, int n_advance, int advance_by,
                             const int32_t *advance_each, int advance_limit) {
  if (rows < 1 || n_cand < 1 || k < 1 || k > AMPH_MAX_TOPK || n_cand > 16 * 1024) return hipErrorInvalidValue;
  #define TM_LAUNCH(N) hipLaunchKernelGGL((k_topk_merge<N>), dim3(rows), dim3(1024), 0, st, cand_v, cand_i, n_cand, V, k, idx, val, \
                                          advance, n_advance, advance_by, advance_each, advance_limit)
  // as few candidates per lane as cover the row: a selection round rescans a lane's candidates, and with ten rounds
  // that is most of the kernel (5000 candidates: 8 per lane 16.4 us, 5 per lane 14.9; half the waves with 10 per lane
  // 15.6, a quarter with 20 per lane 26.6)
  switch ((n_cand + 1023) / 1024) {
    case 1: TM_LAUNCH(1); break;
    case 2: TM_LAUNCH(2); break;
    case 3: TM_LAUNCH(3); break;
    case 4: TM_LAUNCH(4); break;
    case 5: TM_LAUNCH(5); break;
    case 6: TM_LAUNCH(6); break;
    case 7: case 8: TM_LAUNCH(8); break;
    default: TM_LAUNCH(16); break;
  }
  #undef TM_LAUNCH
  return hipGetLastError();
}

size_t topk_ws_floats(int rows, int V, int k) {
  const int chunks = (V + TK_CHUNK - 1) / TK_CHUNK;
  return 2 * (size_t)rows * chunks * k;
}

hipError_t launch_topk_rows(hipStream_t st, const float *logits, int rows, int V, int k, int32_t *idx, float *val,
                            int32_t *advance, int n_advance, int advance_by, const int32_t *advance_each, int advance_limit,
                            float *ws) {
  if (rows < 1 || V < 1 || k < 1 || k > V || k > AMPH_MAX_TOPK) return hipErrorInvalidValue;
  if (V <= 65536) {
    #define TK_ROW(N) hipLaunchKernelGGL((k_topk_row<N>), dim3(rows), dim3(1024), 0, st, logits, V, k, idx, val, advance, \
                                         n_advance, advance_by, advance_each, advance_limit)
    if (V <= 8192) TK_ROW(8); else if (V <= 16384) TK_ROW(16); else if (V <= 32768) TK_ROW(32); else TK_ROW(64);
    #undef TK_ROW
    return hipGetLastError();
  }
  const int chunks = (V + TK_CHUNK - 1) / TK_CHUNK;
  const int n_cand = chunks * k;
  if (n_cand > TK_MAXC * WAVE) return hipErrorInvalidValue;
  float *cand_v = ws;
  int *cand_i = reinterpret_cast<int *>(ws + (size_t)rows * n_cand);
  hipLaunchKernelGGL(k_topk_pass1, dim3((chunks + 3) / 4, rows), dim3(256), 0, st, logits, V, k, chunks, cand_v, cand_i);
  hipLaunchKernelGGL(k_topk_pass2, dim3(rows), dim3(64), 0, st, cand_v, cand_i, n_cand, V, k, idx, val, advance, n_advance,
                     advance_by, advance_each, advance_limit);
  return hipGetLastError();
}

hipError_t launch_row_argmax(hipStream_t st, const float *logits, int rows, int V, int32_t *out, float *ws) {
  return launch_topk_rows(st, logits, rows, V, 1, out, nullptr, nullptr, 0, 0, nullptr, 0, ws);
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
// Acceptance under random sampling (Table 2, Temperature = 0.7).  The paper states no rule; the one built is
// typical acceptance as the multi-head framework the paper adopts its tree from defines it: with
// p_j = softmax(logits_j / temperature) and H its entropy in nats, child i of j passes iff
// p_j(tok_i) > min(eps, delta * exp(-H(p_j))); the deepest node whose whole chain passes wins (lowest id among
// equals) and the following token is drawn from p_best by inverting its cumulative distribution (vocabulary
// order) at the caller's uniform number.
//   k_row_softmax_stats: one workgroup per tree node: m = max l, Z = sum exp((l - m) / t),
//     H = ln Z - sum(e x) / Z with x = (l - m) / t, e = exp(x)            -> stats[row] = (m, Z, H, 0)
//   k_accept_typical: one workgroup per batch element: the pass flags, the winner as in k_accept, then the draw:
//     thread t sums its run of consecutive tokens, a scan over the threads finds the run where the cumulative
//     sum first exceeds u * Z, and that thread walks its run.  If rounding leaves no such token (u * Z at or
//     above the total), the last token of non-zero probability is taken.
// =====================================================================================================
constexpr int AT_THREADS = 1024, AT_WAVES = AT_THREADS / WAVE;

__device__ __forceinline__ float at_block_max(float v, float *sm) {
  #pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, WAVE));
  __syncthreads();                                        // sm may still be read from an earlier reduction
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = sm[0];
  for (int w = 1; w < AT_WAVES; ++w) r = fmaxf(r, sm[w]);
  return r;
}
__device__ __forceinline__ float at_block_sum(float v, float *sm) {      // fixed order: lanes by butterfly, waves ascending
  #pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, WAVE);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = sm[0];
  for (int w = 1; w < AT_WAVES; ++w) r += sm[w];
  return r;
}

__global__ __launch_bounds__(AT_THREADS) void k_row_softmax_stats(const float *logits, int V, float inv_temp, float4 *stats) {
  __shared__ float sm[AT_WAVES];
  const float *l = logits + (size_t)blockIdx.x * V;
  const int t = threadIdx.x;
  float m = -__builtin_huge_valf();
  for (int v = t; v < V; v += AT_THREADS) m = fmaxf(m, l[v]);
  m = at_block_max(m, sm);
  float z = 0.f, sx = 0.f;
  for (int v = t; v < V; v += AT_THREADS) {
    const float x = (l[v] - m) * inv_temp, e = expf(x);
    z += e;
    if (e > 0.f) sx += e * x;                             // a token of probability zero adds nothing (0 * -inf)
  }
  z = at_block_sum(z, sm);
  sx = at_block_sum(sx, sm);
  if (t == 0) stats[blockIdx.x] = make_float4(m, z, logf(z) - sx / z, 0.f);
}

__global__ __launch_bounds__(AT_THREADS) void k_accept_typical(const int32_t *parent, const int32_t *depth, int T, int K, int V,
                                                               const int32_t *tree_tok, const float *logits, const float4 *stats,
                                                               float inv_temp, float eps, float delta, const float *u,
                                                               int32_t *accept_len, int32_t *accept_path, int32_t *next_tok,
                                                               int32_t *best_node) {
  __shared__ float sm[AT_WAVES];
  __shared__ int s_pass[AMPH_MAX_TREE];
  __shared__ int s_key[AT_WAVES];
  __shared__ int s_best, s_found;
  const int b = blockIdx.x, t = threadIdx.x;
  const int32_t *tok = tree_tok + (size_t)b * T;
  if (t < T) {
    int pass = 1;                                          // the root
    if (t > 0) {
      const int j = parent[t], tk = tok[t];
      const size_t row = (size_t)b * T + j;
      const float4 st = stats[row];
      pass = 0;
      if (tk >= 0 && tk < V) {
        const float p = expf((logits[row * V + tk] - st.x) * inv_temp) / st.y;
        pass = p > fminf(eps, delta * expf(-st.z));
      }
    }
    s_pass[t] = pass;
  }
  if (t == 0) s_found = -1;
  __syncthreads();
  int key = -1;
  if (t < T) {
    bool ok = true;
    int j = t;
    for (int hop = 0; hop <= AMPH_MAX_HEADS_K && j > 0; ++hop) {
      if (!s_pass[j]) { ok = false; break; }
      j = parent[j];
    }
    if (ok) key = depth[t] * 256 + (255 - t);
  }
  #pragma unroll
  for (int off = 32; off >= 1; off >>= 1) key = max(key, __shfl_xor(key, off, WAVE));
  if ((t & 63) == 0) s_key[t >> 6] = key;
  __syncthreads();
  if (t == 0) {
    int best_key = s_key[0];
    for (int w = 1; w < AT_WAVES; ++w) best_key = max(best_key, s_key[w]);
    const int a = best_key >> 8, best = 255 - (best_key & 255);     // the root always qualifies
    accept_len[b] = a;
    best_node[b] = best;
    s_best = best;
    for (int dd = 0; dd <= K; ++dd) accept_path[(size_t)b * (K + 1) + dd] = -1;
    int j = best;
    for (int dd = a; dd >= 0 && j >= 0; --dd) { accept_path[(size_t)b * (K + 1) + dd] = j; j = parent[j]; }
  }
  __syncthreads();
  // ---- the draw from p_best
  const size_t row = (size_t)b * T + s_best;
  const float *l = logits + row * V;
  const float4 st = stats[row];
  const float target = u[b] * st.y;
  const int C = (V + AT_THREADS - 1) / AT_THREADS, v0 = min(t * C, V), v1 = min(v0 + C, V);
  float run = 0.f;
  int last_live = -1;
  for (int v = v0; v < v1; ++v) {
    const float e = expf((l[v] - st.x) * inv_temp);
    run += e;
    if (e > 0.f) last_live = v;
  }
  // inclusive scan of the runs: inside a wave, then over the wave totals (ascending)
  float inc = run;
  #pragma unroll
  for (int off = 1; off < WAVE; off <<= 1) {
    const float o = __shfl_up(inc, off, WAVE);
    if ((t & 63) >= off) inc += o;
  }
  if ((t & 63) == 63) sm[t >> 6] = inc;
  __syncthreads();
  float base = 0.f;
  for (int w = 0; w < (t >> 6); ++w) base += sm[w];
  inc += base;
  const float prev = __shfl_up(inc, 1, WAVE);
  const float exc = (t & 63) ? prev : base;               // exactly the thread before's inclusive sum
  // the sums never decrease with t and exc(t + 1) = inc(t): at most one thread sees the crossing inside its run
  if (exc <= target && inc > target) {
    float acc = exc;
    int pick = -1;
    for (int v = v0; v < v1; ++v) {
      acc += expf((l[v] - st.x) * inv_temp);
      if (acc > target) { pick = v; break; }
    }
    if (pick < 0) pick = max(last_live, v0);              // (acc and inc differ by rounding order only)
    s_found = pick;
  }
  #pragma unroll
  for (int off = 32; off >= 1; off >>= 1) last_live = max(last_live, __shfl_xor(last_live, off, WAVE));
  __syncthreads();
  if ((t & 63) == 0) s_key[t >> 6] = last_live;
  __syncthreads();
  if (t == 0) {
    int pick = s_found;
    if (pick < 0) {
      pick = s_key[0];
      for (int w = 1; w < AT_WAVES; ++w) pick = max(pick, s_key[w]);
    }
    next_tok[b] = min(max(pick, 0), V - 1);
  }
}

hipError_t launch_accept_typical(hipStream_t st, const int32_t *parent, const int32_t *depth, int T, int B, int K, int V,
                                 const int32_t *tree_tok, const float *logits, float temperature, float eps, float delta,
                                 const float *u, int32_t *accept_len, int32_t *accept_path, int32_t *next_tok,
                                 int32_t *best_node, float *stats_ws) {
  if (T < 1 || T > AMPH_MAX_TREE || V < 1 || !(temperature > 0.f)) return hipErrorInvalidValue;
  const float inv_temp = 1.0f / temperature;
  hipLaunchKernelGGL(k_row_softmax_stats, dim3(B * T), dim3(AT_THREADS), 0, st, logits, V, inv_temp, (float4 *)stats_ws);
  hipLaunchKernelGGL(k_accept_typical, dim3(B), dim3(AT_THREADS), 0, st, parent, depth, T, K, V, tree_tok, logits,
                     (const float4 *)stats_ws, inv_temp, eps, delta, u, accept_len, accept_path, next_tok, best_node);
  return hipGetLastError();
}

// =====================================================================================================
// The loop around the step (Sec. 2 "Speculative Decoding"; Eq. 1 keeps one adaptation-layer cache row per
// committed position).
//   k_kv_commit: for one (layer, batch element, head), the K/V rows of the accepted path's nodes 1..a move
//     from tree slots kv_len + node to kv_len + j (node 0, the root, already sits at kv_len).  All sources
//     are read before the first write (a destination may be another node's source).
//   k_gather_accepted: row j <= a of h_new is the target's hidden state at path node j, tok_new[j] the
//     token that follows it (the next path node's token, or next_tok after the last); n_new = a + 1.
//   k_advance_len: kv_len += a + 1, as its own launch, after every workgroup above has read kv_len.
//   k_gather_rows: out[b] = rows[b * R + (n_valid ? n_valid[b] : R) - 1] (the last live row of each element).
// =====================================================================================================
template <typename T>
__global__ __launch_bounds__(256) void k_kv_commit(T *k_caches, T *v_caches, int B, int n_heads, int d_h, int max_kv,
                                                   int T_nodes, const int32_t *kv_len, const int32_t *accept_len,
                                                   const int32_t *accept_path, int K) {
  const int h = blockIdx.x, b = blockIdx.y, li = blockIdx.z;
  const int L = kv_len[b];
  int a = accept_len[b];
  if (L < 0 || L + T_nodes > max_kv || a < 0) return;       // the target pass wrote nothing (flagged there)
  if (a > K) a = K;
  const size_t head = (((size_t)li * B + b) * n_heads + h) * (size_t)max_kv * d_h;
  T *kc = k_caches + head, *vc = v_caches + head;
  constexpr int MAXE = (AMPH_MAX_HEADS_K * 128 + 255) / 256;     // elements per thread: a * d_h <= 8 * 128
  T kr[MAXE], vr[MAXE];
  #pragma unroll
  for (int i = 0; i < MAXE; ++i) {
    const int idx = threadIdx.x + i * 256, j = idx / d_h + 1, e = idx % d_h;
    if (j <= a) {
      int node = accept_path[(size_t)b * (K + 1) + j];
      node = min(max(node, 0), T_nodes - 1);
      kr[i] = kc[k_tiled_index<T>(L + node, e, d_h)];
      vr[i] = vc[v_tiled_index<T>(L + node, e, d_h)];
    }
  }
  __syncthreads();
  #pragma unroll
  for (int i = 0; i < MAXE; ++i) {
    const int idx = threadIdx.x + i * 256, j = idx / d_h + 1, e = idx % d_h;
    if (j <= a) {
      kc[k_tiled_index<T>(L + j, e, d_h)] = kr[i];
      vc[v_tiled_index<T>(L + j, e, d_h)] = vr[i];
    }
  }
}

__global__ __launch_bounds__(256) void k_gather_accepted(const float *hidden, const int32_t *tree_tok, int T_nodes, int d,
                                                         int K, const int32_t *accept_len, const int32_t *accept_path,
                                                         const int32_t *next_tok, float *h_new, int32_t *tok_new,
                                                         int32_t *n_new) {
  const int j = blockIdx.x, b = blockIdx.y;
  const int a = min(max(accept_len[b], 0), K);
  const int32_t *path = accept_path + (size_t)b * (K + 1);
  float *dst = h_new + ((size_t)b * (K + 1) + j) * d;
  if (j <= a) {
    const int node = min(max(path[j], 0), T_nodes - 1);
    const float *src = hidden + ((size_t)b * T_nodes + node) * d;
    for (int k = threadIdx.x * 4; k < d; k += 256 * 4) *reinterpret_cast<float4 *>(dst + k) = *reinterpret_cast<const float4 *>(src + k);
    if (threadIdx.x == 0)
      tok_new[(size_t)b * (K + 1) + j] = (j < a) ? tree_tok[(size_t)b * T_nodes + min(max(path[j + 1], 0), T_nodes - 1)] : next_tok[b];
  } else {
    for (int k = threadIdx.x * 4; k < d; k += 256 * 4) *reinterpret_cast<float4 *>(dst + k) = make_float4(0.f, 0.f, 0.f, 0.f);
    if (threadIdx.x == 0) tok_new[(size_t)b * (K + 1) + j] = 0;
  }
  if (j == 0 && threadIdx.x == 0) n_new[b] = a + 1;
}

__global__ void k_advance_len(int32_t *kv_len, const int32_t *accept_len, int B, int K, int T_nodes, int max_kv) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const int L = kv_len[b];
  if (L < 0 || L + T_nodes > max_kv) return;
  kv_len[b] = L + min(max(accept_len[b], 0), K) + 1;
}

__global__ __launch_bounds__(256) void k_gather_rows(const float *rows, int R, int d, const int32_t *n_valid, float *out) {
  const int b = blockIdx.x;
  int r = n_valid ? n_valid[b] : R;
  r = min(max(r, 1), R) - 1;
  const float *src = rows + ((size_t)b * R + r) * d;
  for (int k = threadIdx.x * 4; k < d; k += 256 * 4)
    *reinterpret_cast<float4 *>(out + (size_t)b * d + k) = *reinterpret_cast<const float4 *>(src + k);
}

template <typename T>
hipError_t launch_commit(hipStream_t st, void *k_caches, void *v_caches, int n_layers, int B, int n_heads, int d_h, int max_kv,
                         int T_nodes, int d, int K, int32_t *kv_len, const int32_t *accept_len, const int32_t *accept_path,
                         const int32_t *next_tok, const int32_t *tree_tok, const float *hidden, float *h_new, int32_t *tok_new,
                         int32_t *n_new) {
  if (K < 1 || K > AMPH_MAX_HEADS_K || d_h > 128 || d % 4) return hipErrorInvalidValue;
  if (n_layers > 0)
    hipLaunchKernelGGL((k_kv_commit<T>), dim3(n_heads, B, n_layers), dim3(256), 0, st, (T *)k_caches, (T *)v_caches, B, n_heads,
                       d_h, max_kv, T_nodes, kv_len, accept_len, accept_path, K);
  if (h_new)
    hipLaunchKernelGGL(k_gather_accepted, dim3(K + 1, B), dim3(256), 0, st, hidden, tree_tok, T_nodes, d, K, accept_len,
                       accept_path, next_tok, h_new, tok_new, n_new);
  hipLaunchKernelGGL(k_advance_len, dim3((B + 63) / 64), dim3(64), 0, st, kv_len, accept_len, B, K, T_nodes, max_kv);
  return hipGetLastError();
}
template hipError_t launch_commit<float>(hipStream_t, void *, void *, int, int, int, int, int, int, int, int, int32_t *,
                                         const int32_t *, const int32_t *, const int32_t *, const int32_t *, const float *,
                                         float *, int32_t *, int32_t *);
template hipError_t launch_commit<bf16_t>(hipStream_t, void *, void *, int, int, int, int, int, int, int, int, int32_t *,
                                          const int32_t *, const int32_t *, const int32_t *, const int32_t *, const float *,
                                          float *, int32_t *, int32_t *);

hipError_t launch_gather_rows(hipStream_t st, const float *rows, int B, int R, int d, const int32_t *n_valid, float *out) {
  if (d % 4) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_gather_rows, dim3(B), dim3(256), 0, st, rows, R, d, n_valid, out);
  return hipGetLastError();
}

// =====================================================================================================
// Row-major [max_kv, d_h] caches <-> the step-tiled storage of the verification attention (formulas: header of
// the C ABI, k_tiled_index / v_tiled_index).  One thread moves 4 adjacent dims of one row: in the key layout they
// stay adjacent (inside one 64-byte piece); in the value layout they are 4 single elements.  grid = (chunks of
// 256 items, caches); to_tiled = false runs the same index map backwards.
// =====================================================================================================
template <typename T>
__global__ __launch_bounds__(256) void k_kv_layout(const T *k_src, const T *v_src, T *k_dst, T *v_dst, int max_kv, int d_h,
                                                   bool to_tiled) {
  const size_t head = (size_t)blockIdx.y * (size_t)max_kv * d_h;
  const int q = d_h / 4;
  for (int item = blockIdx.x * 256 + threadIdx.x; item < max_kv * q; item += gridDim.x * 256) {
    const int row = item / q, c = (item % q) * 4;
    const size_t rm = head + (size_t)row * d_h + c;
    if (k_src) {
      const size_t tl = head + k_tiled_index<T>(row, c, d_h);
      float f[4];
      load4<T>(k_src + (to_tiled ? rm : tl), f);              // (a widening to float and back is exact for both types)
      store4<T>(k_dst + (to_tiled ? tl : rm), f);
    }
    if (v_src) {
      #pragma unroll
      for (int j = 0; j < 4; ++j) {
        const size_t tl = head + v_tiled_index<T>(row, c + j, d_h);
        if (to_tiled) v_dst[tl] = v_src[rm + j]; else v_dst[rm + j] = v_src[tl];
      }
    }
  }
}

template <typename T>
hipError_t launch_kv_layout(hipStream_t st, const void *k_src, const void *v_src, void *k_dst, void *v_dst, int n_caches,
                            int max_kv, int d_h, bool to_tiled) {
  if (n_caches < 1 || n_caches > 65535 * 16 || max_kv % 32 || d_h % 16) return hipErrorInvalidValue;
  const int items = max_kv * (d_h / 4);
  const unsigned chunks = (unsigned)std::min((items + 255) / 256, 64);
  for (int c0 = 0; c0 < n_caches; c0 += 65535) {           // grid.y is limited to 65535
    const int nc = std::min(65535, n_caches - c0);
    const size_t off = (size_t)c0 * max_kv * d_h;
    hipLaunchKernelGGL((k_kv_layout<T>), dim3(chunks, nc), dim3(256), 0, st, k_src ? (const T *)k_src + off : nullptr,
                       v_src ? (const T *)v_src + off : nullptr, k_dst ? (T *)k_dst + off : nullptr,
                       v_dst ? (T *)v_dst + off : nullptr, max_kv, d_h, to_tiled);
  }
  return hipGetLastError();
}
template hipError_t launch_kv_layout<float>(hipStream_t, const void *, const void *, void *, void *, int, int, int, bool);
template hipError_t launch_kv_layout<bf16_t>(hipStream_t, const void *, const void *, void *, void *, int, int, int, bool);

// =====================================================================================================
// Row-wise RMSNorm for the target path, fused with the fold of the previous GEMM's partial slabs:
//   x[m] (+)= sum_s slabs[s][m]   (or x[m] = embed[tok[m]] on entry to the first layer)
//   xn[m] = x[m] / rms(x[m]) * g  stored as T for the matrix cores; hidden_out optionally in float32.
// One 1024-thread workgroup per row, one 16-byte piece of every operand per thread and pass.  The
// number of slabs, the source of the row and the number of passes are template parameters so that the
// body is straight-line code: every load of a pass is issued before the first use (a run-time loop over
// slabs costs one memory round trip per slab).  d <= 8192.
// =====================================================================================================
template <typename T, int S, bool EMB, int NP>
__global__ __launch_bounds__(1024) void k_norm_fold(float *x, const T *embed, const int32_t *tok, int vocab,
                                                    const float *slabs, size_t slab_stride, const T *g, int d,
                                                    float eps, T *xn, float *hidden_out, uint32_t *dev_status, int xn_tiles,
                                                    RopeTable rope) {
  __shared__ float red[16];
  const int row = blockIdx.x, tid = threadIdx.x;
  float *xr = x + (size_t)row * d;
  int t = 0;
  if (EMB) {
    t = tok[row];
    if (t < 0 || t >= vocab) { if (tid == 0) atomicOr(dev_status, 4u); t = 0; }
  }
  float v[NP][4], gk[NP][4], p[NP][S > 0 ? S : 1][4];
  #pragma unroll
  for (int i = 0; i < NP; ++i) {
    const int k = (tid + i * 1024) * 4, kk = k < d ? k : 0;      // pieces past the row re-read its start, unused
    if (EMB) load4<T>(embed + (size_t)t * d + kk, v[i]);
    else load4<float>(xr + kk, v[i]);
    #pragma unroll
    for (int s = 0; s < S; ++s) load4<float>(slabs + (size_t)s * slab_stride + (size_t)row * d + kk, p[i][s]);
    load4<T>(g + kk, gk[i]);
  }
  if (EMB && rope.cs) {
    // the pass's RoPE table rides on the kernel that starts the pass (one launch fewer): row `row` of
    // (cos, sin) of pos * theta^(-2e/d_h), e < d_h/2, the same for every layer
    const int half = rope.d_h / 2;
    for (int e = tid; e < half; e += 1024) {
      const float inv_freq = exp2f(-2.0f * (float)e / (float)rope.d_h * log2f(rope.theta));
      float sn, c;
      sincosf((float)rope.pos[row] * inv_freq, &sn, &c);
      rope.cs[(size_t)row * half + e] = make_float2(c, sn);
    }
  }
  float ss = 0.f;
  #pragma unroll
  for (int i = 0; i < NP; ++i) {
    const int k = (tid + i * 1024) * 4;
    #pragma unroll
    for (int s = 0; s < S; ++s) {
      #pragma unroll
      for (int j = 0; j < 4; ++j) v[i][j] += p[i][s][j];
    }
    if (k < d) {
      if (EMB || S > 0) store4<float>(xr + k, v[i]);
      #pragma unroll
      for (int j = 0; j < 4; ++j) ss = fmaf(v[i][j], v[i][j], ss);
    }
  }
  ss = wave_sum(ss);
  if ((tid & 63) == 0) red[tid >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
  #pragma unroll
  for (int w = 0; w < 16; ++w) tot += red[w];
  const float rs = rsqrtf(tot / (float)d + eps);
  #pragma unroll
  for (int i = 0; i < NP; ++i) {
    const int k = (tid + i * 1024) * 4;
    if (k < d) {
      float o[4];
      #pragma unroll
      for (int j = 0; j < 4; ++j) o[j] = v[i][j] * rs * gk[i][j];
      store4<T>(xn_tiles ? xn + xt_index<T>(row, k, xn_tiles) : xn + (size_t)row * d + k, o);
      if (hidden_out) store4<float>(hidden_out + (size_t)row * d + k, o);
    }
  }
}

template <typename T>
hipError_t launch_norm_fold(hipStream_t st, float *x, const void *embed, const int32_t *tok, int vocab,
                            const float *slabs, int S, size_t slab_stride, const void *g, int rows, int d, float eps,
                            void *xn, float *hidden_out, uint32_t *dev_status, int xn_tiles, RopeTable rope) {
  if (d % 4 || d > 8192) return hipErrorInvalidValue;
  if (tok && S != 0) return hipErrorInvalidValue;                  // the embedding gather starts a fresh residual stream
  if (rope.cs && (!tok || !rope.pos || rope.d_h < 2)) return hipErrorInvalidValue;   // the table is written by the embedding instance
  const int np = d > 4096 ? 2 : 1;
  #define NF_LAUNCH(S_, EMB_, NP_)                                                                                  \
    hipLaunchKernelGGL((k_norm_fold<T, S_, EMB_, NP_>), dim3(rows), dim3(1024), 0, st, x, (const T *)embed, tok,    \
                       vocab, slabs, slab_stride, (const T *)g, d, eps, (T *)xn, hidden_out, dev_status, xn_tiles, rope)
  #define NF_CASE(S_)                                                                                               \
    case S_: if (np == 1) NF_LAUNCH(S_, false, 1); else NF_LAUNCH(S_, false, 2); break
  if (tok) {
    if (np == 1) NF_LAUNCH(0, true, 1); else NF_LAUNCH(0, true, 2);
  } else {
    switch (S) {
      NF_CASE(0); NF_CASE(1); NF_CASE(2); NF_CASE(4); NF_CASE(8);
      default: return hipErrorInvalidValue;
    }
  }
  #undef NF_CASE
  #undef NF_LAUNCH
  return hipGetLastError();
}
template hipError_t launch_norm_fold<float>(hipStream_t, float *, const void *, const int32_t *, int, const float *, int,
                                            size_t, const void *, int, int, float, void *, float *, uint32_t *, int, RopeTable);
template hipError_t launch_norm_fold<bf16_t>(hipStream_t, float *, const void *, const int32_t *, int, const float *, int,
                                             size_t, const void *, int, int, float, void *, float *, uint32_t *, int, RopeTable);

}  // namespace amph
