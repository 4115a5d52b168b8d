// Weight-streaming GEMV family for the draft path (Sec. 3.1 Eq. 1, Sec. 3.2 Eq. 2-6): M <= 8
// activation rows against a [N, Kd] weight matrix that is read exactly once from HBM.
//
// Shape of every kernel here: a 256-thread workgroup first parks the M activation rows in LDS as
// float32 (after the prologue: concat with the token embedding, or RMSNorm scaling), then each of
// its 4 waves walks over groups of R = 4 weight rows.  For a group the 64 lanes stride over the
// reduction axis in 16-byte fragments, keeping R x U fragments in flight, and multiply them with the
// LDS copy of x; a wave-wide butterfly sum finishes the R x M dot products and the epilogue (RoPE and
// cache write, residual add, SwiGLU, head MLP) is applied to them directly.  No matrix cores: with
// M <= 8 the contraction is a stream of dot products bound by HBM.
#include "kernels.h"
#include <algorithm>

namespace amph {

constexpr int GV_THREADS = 256;
constexpr int GV_R = 4;        // weight rows per wave step
constexpr int GV_U = 4;        // 16-byte fragments in flight per row

// LDS layout of x: for wave-chunk c (64 lanes x PER elements), quad q (4 floats), lane l:
//   xs[((m * nC + c) * NQ + q) * 256 + l * 4 + j]  holds x[m][c * CH + l * PER + q * 4 + j]
// so that a lane's float4 reads are contiguous across the wave.
template <typename T> struct XLayout {
  static constexpr int PER = Elem<T>::PER;
  static constexpr int NQ = PER / 4;
  static constexpr int CH = WAVE * PER;
  static __device__ __forceinline__ int index(int m, int nC, int k) {
    const int c = k / CH, r = k % CH, l = r / PER, e = r % PER;
    return ((m * nC + c) * NQ + e / 4) * 256 + l * 4 + (e % 4);
  }
};

// Request the GV_U fragments from chunk c0 on of each of the R rows.  Unconditional loads (a predicated load with a
// zero alternative makes the compiler wait for every load at the merge): lanes past the end re-read the row's
// first fragment; x is zero-padded there and weights are finite, so they add nothing.
template <typename T>
__device__ __forceinline__ void gemv_request(const T *const (&rows)[GV_R], int c0, int Kd, uint4 (&w)[GV_U][GV_R]) {
  constexpr int PER = Elem<T>::PER, CH = WAVE * PER;
  const int lane = threadIdx.x & 63;
  #pragma unroll
  for (int u = 0; u < GV_U; ++u) {
    const int k = (c0 + u) * CH + lane * PER;
    #pragma unroll
    for (int r = 0; r < GV_R; ++r) w[u][r] = ldg16_stream(rows[r] + (k < Kd ? k : 0));
  }
}

// acc[r][m] += the fragments of chunks c0 .. c0 + GV_U - 1 times the LDS copy of x
template <typename T, int M>
__device__ __forceinline__ void gemv_consume(const float *xs, int nC, int c0, const uint4 (&w)[GV_U][GV_R],
                                             float (&acc)[GV_R][M]) {
  constexpr int PER = Elem<T>::PER, NQ = PER / 4;
  const int lane = threadIdx.x & 63;
  const float4 *xs4 = reinterpret_cast<const float4 *>(xs);
  #pragma unroll
  for (int u = 0; u < GV_U; ++u) {
    if (c0 + u < nC) {
      float wf[GV_R][PER];
      #pragma unroll
      for (int r = 0; r < GV_R; ++r) Elem<T>::unpack(w[u][r], wf[r]);
      #pragma unroll
      for (int q = 0; q < NQ; ++q) {
        #pragma unroll
        for (int m = 0; m < M; ++m) {
          const float4 xv = xs4[((m * nC + c0 + u) * NQ + q) * 64 + lane];
          #pragma unroll
          for (int r = 0; r < GV_R; ++r) {
            acc[r][m] = fmaf(wf[r][q * 4 + 0], xv.x, acc[r][m]);
            acc[r][m] = fmaf(wf[r][q * 4 + 1], xv.y, acc[r][m]);
            acc[r][m] = fmaf(wf[r][q * 4 + 2], xv.z, acc[r][m]);
            acc[r][m] = fmaf(wf[r][q * 4 + 3], xv.w, acc[r][m]);
          }
        }
      }
    }
  }
}

// one of three pointers by index, as selects on the address bits (written as a conditional chain it may be turned
// into a table in scratch memory when it is evaluated in more than one place)
template <typename P> __device__ __forceinline__ P *pick3(int i, P *a, P *b, P *c) {
  const uintptr_t v = (i == 0 ? (uintptr_t)a : (uintptr_t)0) | (i == 1 ? (uintptr_t)b : (uintptr_t)0) | (i >= 2 ? (uintptr_t)c : (uintptr_t)0);
  return (P *)v;
}

// With five or more activation rows a batch of fragments takes about as long to multiply as to fetch, and the rows
// in LDS leave room for one workgroup per compute unit only, so nothing else would cover the fetch: those
// instantiations keep two batches per wave and always have the next one on its way, across row groups as well
// (measured with 5 rows at 7B shapes: gate/up 77.8 -> 62.7 us, the three SAL projections 45.2 -> 46.7, Wo / down
// 17.5 -> 16.5).  With fewer rows several workgroups share a compute unit and a second batch per wave gains nothing
// (1 row) or loses (4 rows: the LM head 52.9 -> 60.5 us).
template <int M> struct GvPipe { static constexpr bool on = (M >= 5); };

// The weight fragments a wave holds: one batch, or two when pipelined.  In the pipelined form w0 always holds (or
// awaits) the first batch of the group that is multiplied next.
template <typename T, bool PIPE> struct GvFrags {
  uint4 w0[GV_U][GV_R];
  uint4 w1[PIPE ? GV_U : 1][GV_R];
};

template <typename T, bool PIPE>
__device__ __forceinline__ void gemv_begin(const T *const (&rows)[GV_R], int Kd, GvFrags<T, PIPE> &f) {
  if (PIPE) gemv_request<T>(rows, 0, Kd, f.w0);
}

// Accumulate acc[r][m] += sum_k W_r[k] * x[m][k] over the whole reduction axis for this lane's slots.
// next: the rows of the group this wave multiplies after this one (any valid rows if there is none).
template <typename T, int M, bool PIPE>
__device__ __forceinline__ void gemv_rows(const T *const (&rows)[GV_R], const T *const (&next)[GV_R], const float *xs,
                                          int Kd, int nC, float (&acc)[GV_R][M], GvFrags<T, PIPE> &f) {
  if constexpr (PIPE) {
    // every request is unconditional (clamped inside the row), so the compiler can count the loads in flight: a
    // batch is waited for with the one requested after it still outstanding
    for (int c0 = 0; c0 < nC; c0 += 2 * GV_U) {
      gemv_request<T>(rows, c0 + GV_U, Kd, f.w1);
      gemv_consume<T, M>(xs, nC, c0, f.w0, acc);
      const bool more = c0 + 2 * GV_U < nC;
      const T *sel[GV_R];
      #pragma unroll
      for (int r = 0; r < GV_R; ++r) sel[r] = more ? rows[r] : next[r];
      gemv_request<T>(sel, more ? c0 + 2 * GV_U : 0, Kd, f.w0);
      gemv_consume<T, M>(xs, nC, c0 + GV_U, f.w1, acc);
    }
  } else {
    for (int c0 = 0; c0 < nC; c0 += GV_U) {
      gemv_request<T>(rows, c0, Kd, f.w0);
      gemv_consume<T, M>(xs, nC, c0, f.w0, acc);
    }
  }
  #pragma unroll
  for (int r = 0; r < GV_R; ++r)
    #pragma unroll
    for (int m = 0; m < M; ++m) acc[r][m] = wave_sum(acc[r][m]);
}

// After gemv_rows every lane holds all R x M sums, so the epilogues spread their outputs over the lanes (lane ->
// (row of the group, activation row)) instead of walking them on lane 0: the loads an epilogue needs (residual,
// positions) and its transcendental functions then run side by side.  acc_at picks a lane's sum by selects.
template <int M> __device__ __forceinline__ float acc_at(const float (&acc)[GV_R][M], int r, int m) {
  float v = 0.f;
  #pragma unroll
  for (int mm = 0; mm < M; ++mm)
    #pragma unroll
    for (int rr = 0; rr < GV_R; ++rr) v = (mm == m && rr == r) ? acc[rr][mm] : v;
  return v;
}

template <int M> __device__ __forceinline__ void zero_acc(float (&acc)[GV_R][M]) {
  #pragma unroll
  for (int r = 0; r < GV_R; ++r)
    #pragma unroll
    for (int m = 0; m < M; ++m) acc[r][m] = 0.f;
}

// ---- prologues: fill xs (and zero its padding), return per-row inverse RMS where asked ---------------
// float4 slot of the 4 consecutive elements starting at k (k % 4 == 0) of row m in the layout above
template <typename T> __device__ __forceinline__ int xs_quad(int m, int nC, int k) {
  constexpr int PER = XLayout<T>::PER, NQ = XLayout<T>::NQ, CH = XLayout<T>::CH;
  const int c = k / CH, r = k % CH;
  return ((m * nC + c) * NQ + (r % PER) / 4) * 64 + r / PER;
}

// Rows x[m][k] (float32, leading dimension ldx), optionally multiplied by g[k], into xs; rows
// m >= m_valid and the padding up to nC chunks become zero.  With NORM, ss[m] receives this thread's
// share of sum_k x[m][k]^2.  Every thread issues the 16-byte loads of several pieces of all M rows
// before it uses any of them; pieces out of range read the row's start and are replaced by zeros
// (a predicated load would make the compiler wait for each load on its own).
template <typename T, int M, bool NORM>
__device__ __forceinline__ void fill_xs(float *xs, const float *x, int ldx, const T *g, int m_valid, int Kd, int nC,
                                        float (&ss)[M]) {
  constexpr int UJ = (M >= 4) ? 2 : 4;
  const int nq = nC * XLayout<T>::CH / 4;
  float4 *xs4 = reinterpret_cast<float4 *>(xs);
  for (int j0 = threadIdx.x; j0 < nq; j0 += GV_THREADS * UJ) {
    float v[UJ][M][4], gk[UJ][4];
    #pragma unroll
    for (int u = 0; u < UJ; ++u) {
      const int k = (j0 + u * GV_THREADS) * 4, kk = (k < Kd) ? k : 0;
      if (NORM) load4<T>(g + kk, gk[u]);
      #pragma unroll
      for (int m = 0; m < M; ++m) load4<float>(x + (size_t)(m < m_valid ? m : 0) * ldx + kk, v[u][m]);
    }
    #pragma unroll
    for (int u = 0; u < UJ; ++u) {
      const int q = j0 + u * GV_THREADS, k = q * 4;
      if (q < nq) {
        #pragma unroll
        for (int m = 0; m < M; ++m) {
          const bool ok = k < Kd && m < m_valid;
          float4 o;
          o.x = ok ? v[u][m][0] : 0.f; o.y = ok ? v[u][m][1] : 0.f; o.z = ok ? v[u][m][2] : 0.f; o.w = ok ? v[u][m][3] : 0.f;
          if (NORM) {
            ss[m] = fmaf(o.x, o.x, fmaf(o.y, o.y, fmaf(o.z, o.z, fmaf(o.w, o.w, ss[m]))));
            o.x *= gk[u][0]; o.y *= gk[u][1]; o.z *= gk[u][2]; o.w *= gk[u][3];
          }
          xs4[xs_quad<T>(m, nC, k)] = o;
        }
      }
    }
  }
}

// plain float32 rows x[m][k], leading dimension ldx; rows m >= m_valid are zero.
template <typename T, int M>
__device__ __forceinline__ void load_x_plain(float *xs, const float *x, int ldx, int m_valid, int Kd, int nC) {
  float ss[M];
  fill_xs<T, M, false>(xs, x, ldx, (const T *)nullptr, m_valid, Kd, nC, ss);
}

// x[m][k] * g[k] with the row's 1/rms returned in rs[m] (applied by the caller to the dot products).
template <typename T, int M>
__device__ __forceinline__ void load_x_rmsnorm(float *xs, float *red, const float *x, int ldx, const T *g,
                                               int m_valid, int Kd, int nC, float eps, float (&rs)[M]) {
  float ss[M];
  #pragma unroll
  for (int m = 0; m < M; ++m) ss[m] = 0.f;
  fill_xs<T, M, true>(xs, x, ldx, g, m_valid, Kd, nC, ss);
  #pragma unroll
  for (int m = 0; m < M; ++m) {
    const float tot = block_sum_256(ss[m], red);
    rs[m] = rsqrtf(tot / (float)Kd + eps);
  }
}

// =====================================================================================================
// K1: x^s = fc^s([u ; e]) of Eq. 1, e = embed[tok] gathered on the fly.  out [M, d] float32.
// half < 0: the whole product.  half = 0 / 1: only the columns that meet u / e (out = / out +=), for row counts whose
// concatenated rows do not fit in LDS: two launches over half the columns each read the matrix once, where two
// launches over fewer rows would read it twice.
// =====================================================================================================
template <typename T, int M, bool PIPE>
__global__ __launch_bounds__(GV_THREADS) void k_fc_concat(const T *W, const float *u, const T *embed,
                                                          const int32_t *tok, int vocab, int d, int m_valid,
                                                          float *out, uint32_t *dev_status, int half) {
  extern __shared__ __align__(16) float smem[];
  constexpr int CH = XLayout<T>::CH;
  const int ldw = 2 * d, k_lo = (half == 1) ? d : 0;       // weight row length; first column of this launch
  const int Kd = (half < 0) ? 2 * d : d, nC = (Kd + CH - 1) / CH, Kp = nC * CH;
  float *xs = smem;
  {
    // [u ; e]: both halves are loaded for every piece (clamped addresses) and the right one is kept
    float4 *xs4 = reinterpret_cast<float4 *>(xs);
    const int nq = Kp / 4;
    int t[M]; bool tok_ok[M];
    #pragma unroll
    for (int m = 0; m < M; ++m) {
      t[m] = tok[m < m_valid ? m : 0];
      tok_ok[m] = t[m] >= 0 && t[m] < vocab;
      if (!tok_ok[m]) {
        if (m < m_valid && blockIdx.x == 0 && threadIdx.x == 0) atomicOr(dev_status, 4u);
        t[m] = 0;
      }
    }
    for (int j0 = threadIdx.x; j0 < nq; j0 += GV_THREADS * 2) {
      float vu[2][M][4], ve[2][M][4];
      #pragma unroll
      for (int q2 = 0; q2 < 2; ++q2) {
        const int k = (j0 + q2 * GV_THREADS) * 4, kg = k + k_lo;
        const int ku = (kg < d) ? kg : 0, ke = (kg >= d && k < Kd) ? kg - d : 0;
        #pragma unroll
        for (int m = 0; m < M; ++m) {
          load4<float>(u + (size_t)(m < m_valid ? m : 0) * d + ku, vu[q2][m]);
          load4<T>(embed + (size_t)t[m] * d + ke, ve[q2][m]);
        }
      }
      #pragma unroll
      for (int q2 = 0; q2 < 2; ++q2) {
        const int q = j0 + q2 * GV_THREADS, k = q * 4;
        if (q < nq) {
          #pragma unroll
          for (int m = 0; m < M; ++m) {
            const bool in_u = k + k_lo < d, ok = m < m_valid && k < Kd && (in_u || tok_ok[m]);
            float4 o;
            o.x = ok ? (in_u ? vu[q2][m][0] : ve[q2][m][0]) : 0.f;
            o.y = ok ? (in_u ? vu[q2][m][1] : ve[q2][m][1]) : 0.f;
            o.z = ok ? (in_u ? vu[q2][m][2] : ve[q2][m][2]) : 0.f;
            o.w = ok ? (in_u ? vu[q2][m][3] : ve[q2][m][3]) : 0.f;
            xs4[xs_quad<T>(m, nC, k)] = o;
          }
        }
      }
    }
  }
  __syncthreads();
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int G = (d + GV_R - 1) / GV_R;
  const int g_first = blockIdx.x * 4 + wave, g_step = gridDim.x * 4;
  auto set_rows = [&](int g, const T *(&rw)[GV_R]) {
    #pragma unroll
    for (int r = 0; r < GV_R; ++r) rw[r] = W + (size_t)min(g * GV_R + r, d - 1) * ldw + k_lo;
  };
  GvFrags<T, PIPE> fr;
  const T *rows[GV_R];
  set_rows(min(g_first, G - 1), rows);
  gemv_begin<T, PIPE>(rows, Kd, fr);
  for (int g = g_first; g < G; g += g_step) {
    const T *next[GV_R];
    set_rows(min(g + g_step, G - 1), next);
    float acc[GV_R][M];
    zero_acc<M>(acc);
    gemv_rows<T, M, PIPE>(rows, next, xs, Kd, nC, acc, fr);
    #pragma unroll
    for (int r = 0; r < GV_R; ++r) rows[r] = next[r];
    {
      const int r = lane & (GV_R - 1), m = lane / GV_R, n = g * GV_R + r;
      float v = acc_at<M>(acc, r, m);
      if (m < m_valid && n < d) {
        if (half == 1) v += out[(size_t)m * d + n];
        out[(size_t)m * d + n] = v;
      }
    }
  }
}

// =====================================================================================================
// K2: SAL q/k/v projections on RMSNorm(x) with RoPE; k and v go straight into the stage's cache, q
// (float32) to qbuf [M, d].  Row row0 + m of the call is new position j = row % R of batch element
// b = row / R: its RoPE position and cache row are sal_len[b] + j; positions j >= n_valid[b] (when
// n_valid is given) write nothing.  A wave step handles the two RoPE pairs (i, i + half),
// (i + 1, i + 1 + half) of one head.  kv_stage points at [B, 2, n_heads, max_kv, d_h] of this stage.
// =====================================================================================================
// weight rows of group g of the stacked q, k, v matrices (Gseg groups each): two RoPE pairs (i0, i0 + 1 and their
// partners half a head further on) of one head for q and k, four adjacent rows for v
struct SalGroup { int seg, i0, n0, n1, n2, n3; };
__device__ __forceinline__ SalGroup sal_group(int g, int Gseg, int d_h) {
  SalGroup o;
  o.seg = g / Gseg;
  const int gl = g % Gseg, half = d_h / 2;
  if (o.seg < 2) {
    const int gph = half / 2;                // groups per head
    o.i0 = (gl % gph) * 2;
    o.n0 = (gl / gph) * d_h + o.i0; o.n1 = o.n0 + 1; o.n2 = o.n0 + half; o.n3 = o.n2 + 1;
  } else {
    o.i0 = 0;
    o.n0 = gl * GV_R; o.n1 = o.n0 + 1; o.n2 = o.n0 + 2; o.n3 = o.n0 + 3;
  }
  return o;
}

template <typename T, int M, bool PIPE>
__global__ __launch_bounds__(GV_THREADS) void k_sal_qkv(const T *wq, const T *wk, const T *wv, const T *norm_w,
                                                        const float *x, int d, int n_heads, int d_h, int m_valid,
                                                        float eps, float theta, const int32_t *sal_len, int max_kv,
                                                        T *kv_stage, float *qbuf, uint32_t *dev_status, int row0, int R,
                                                        const int32_t *n_valid) {
  extern __shared__ __align__(16) float smem[];
  constexpr int CH = XLayout<T>::CH;
  const int Kd = d, nC = (Kd + CH - 1) / CH;
  float *xs = smem + 4;
  float rs[M];
  load_x_rmsnorm<T, M>(xs, smem, x, d, norm_w, m_valid, Kd, nC, eps, rs);
  __syncthreads();
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int Gseg = d / GV_R;                 // groups per matrix (d is a multiple of 4)
  const int G = 3 * Gseg;
  const int g_first = blockIdx.x * 4 + wave, g_step = gridDim.x * 4;
  auto set_rows = [&](int g, const T *(&rw)[GV_R]) {
    const SalGroup sg = sal_group(g, Gseg, d_h);
    const T *Wm = pick3(sg.seg, wq, wk, wv);
    rw[0] = Wm + (size_t)sg.n0 * Kd; rw[1] = Wm + (size_t)sg.n1 * Kd; rw[2] = Wm + (size_t)sg.n2 * Kd; rw[3] = Wm + (size_t)sg.n3 * Kd;
  };
  // epilogue role of this lane: activation row em, pair member ep (outputs ep and 2 + ep of a group); its position
  // in the cache is read once, here
  const int em = lane >> 1, ep = lane & 1;
  bool e_live = false, e_bad = false;
  int e_pos = 0, e_bb = 0;
  float e_rs = 0.f;
  if (em < M && em < m_valid) {
    e_bb = (row0 + em) / R;
    const int jn = (row0 + em) % R;
    const bool valid = !(n_valid && jn >= n_valid[e_bb]);
    const int sl = sal_len[e_bb];
    e_pos = sl + jn;
    e_bad = valid && (sl < 0 || e_pos + 1 > max_kv);
    e_live = valid && !e_bad;
    #pragma unroll
    for (int m = 0; m < M; ++m) if (m == em) e_rs = rs[m];
  }
  GvFrags<T, PIPE> fr;
  const T *rows[GV_R];
  set_rows(min(g_first, G - 1), rows);
  gemv_begin<T, PIPE>(rows, Kd, fr);
  for (int g = g_first; g < G; g += g_step) {
    const SalGroup sg = sal_group(g, Gseg, d_h);
    const int seg = sg.seg, i0 = sg.i0;
    const int n[GV_R] = {sg.n0, sg.n1, sg.n2, sg.n3};
    const T *next[GV_R];
    set_rows(min(g + g_step, G - 1), next);
    float acc[GV_R][M];
    zero_acc<M>(acc);
    gemv_rows<T, M, PIPE>(rows, next, xs, Kd, nC, acc, fr);
    #pragma unroll
    for (int r = 0; r < GV_R; ++r) rows[r] = next[r];
    if (g == 0 && e_bad && ep == 0) atomicOr(dev_status, 1u);
    if (e_live) {
      float ya = acc_at<M>(acc, ep, em) * e_rs, yb = acc_at<M>(acc, 2 + ep, em) * e_rs;
      if (seg < 2) {
        const float inv_freq = exp2f(-2.0f * (float)(i0 + ep) / (float)d_h * log2f(theta));
        float sn, cs;
        sincosf((float)e_pos * inv_freq, &sn, &cs);
        const float a = ya, b = yb;
        ya = a * cs - b * sn;
        yb = b * cs + a * sn;
      }
      const int na = ep ? n[1] : n[0], nb = ep ? n[3] : n[2];
      if (seg == 0) {
        qbuf[(size_t)em * d + na] = ya;
        qbuf[(size_t)em * d + nb] = yb;
      } else {
        // [B, 2, n_heads, max_kv, d_h]
        T *base = kv_stage + (((size_t)e_bb * 2 + (seg - 1)) * n_heads) * (size_t)max_kv * d_h + (size_t)e_pos * d_h;
        base[(size_t)(na / d_h) * max_kv * d_h + na % d_h] = Elem<T>::from_f32(ya);
        base[(size_t)(nb / d_h) * max_kv * d_h + nb % d_h] = Elem<T>::from_f32(yb);
      }
    }
  }
}

// =====================================================================================================
// K3: generic linear with up to three stacked matrices of `seg_rows` rows each (AEB q/k/v, Wo, W_down,
// LM head).  out_s[m][n] = (res ? res[m][n] : 0) + sum_k x[m][k] W_s[n][k].  x float32 [M, Kd].
// A launch may cover a slice of the reduction axis only (Kd = its length, ldw = the length of a weight row, the
// pointers already at the slice): with add_out it adds its sums to what out_s holds, so that consecutive launches
// over consecutive slices build the product of rows too wide to sit in LDS whole while reading the matrix once.
// =====================================================================================================
template <typename T, int M, bool PIPE>
__global__ __launch_bounds__(GV_THREADS) void k_linear(const T *w0, const T *w1, const T *w2, int n_seg, int seg_rows,
                                                       int Kd, const float *x, int ldx, int m_valid, const float *res,
                                                       float *o0, float *o1, float *o2, int ldo, int ldw, int add_out) {
  extern __shared__ __align__(16) float smem[];
  constexpr int CH = XLayout<T>::CH;
  const int nC = (Kd + CH - 1) / CH;
  float *xs = smem;
  load_x_plain<T, M>(xs, x, ldx, m_valid, Kd, nC);
  __syncthreads();
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int Gseg = (seg_rows + GV_R - 1) / GV_R;
  const int G = n_seg * Gseg;
  const int g_first = blockIdx.x * 4 + wave, g_step = gridDim.x * 4;
  auto set_rows = [&](int g, const T *(&rw)[GV_R]) {
    const int seg = g / Gseg, gl = g % Gseg;
    const T *Wm = pick3(seg, w0, w1, w2);
    #pragma unroll
    for (int r = 0; r < GV_R; ++r) rw[r] = Wm + (size_t)min(gl * GV_R + r, seg_rows - 1) * ldw;
  };
  GvFrags<T, PIPE> fr;
  const T *rows[GV_R];
  set_rows(min(g_first, G - 1), rows);
  gemv_begin<T, PIPE>(rows, Kd, fr);
  for (int g = g_first; g < G; g += g_step) {
    const int seg = g / Gseg, gl = g % Gseg;
    float *om = (seg == 0) ? o0 : (seg == 1) ? o1 : o2;
    const T *next[GV_R];
    set_rows(min(g + g_step, G - 1), next);
    float acc[GV_R][M];
    zero_acc<M>(acc);
    gemv_rows<T, M, PIPE>(rows, next, xs, Kd, nC, acc, fr);
    #pragma unroll
    for (int r = 0; r < GV_R; ++r) rows[r] = next[r];
    {
      const int r = lane & (GV_R - 1), m = lane / GV_R, n = gl * GV_R + r;
      float v = acc_at<M>(acc, r, m);
      if (m < m_valid && n < seg_rows) {
        if (res) v += res[(size_t)m * ldo + n];
        if (add_out) v += om[(size_t)m * ldo + n];
        om[(size_t)m * ldo + n] = v;
      }
    }
  }
}

// =====================================================================================================
// K4: SwiGLU front half: act[m][j] = SiLU(W_gate[j] . n) * (W_up[j] . n), n = RMSNorm(x).
// A wave step handles gate rows j, j+1 and up rows j, j+1.
// =====================================================================================================
template <typename T, int M, bool PIPE>
__global__ __launch_bounds__(GV_THREADS) void k_gate_up(const T *w_gate, const T *w_up, const T *norm_w, const float *x,
                                                        int d, int f, int m_valid, float eps, float *act) {
  extern __shared__ __align__(16) float smem[];
  constexpr int CH = XLayout<T>::CH;
  const int Kd = d, nC = (Kd + CH - 1) / CH;
  float *xs = smem + 4;
  float rs[M];
  load_x_rmsnorm<T, M>(xs, smem, x, d, norm_w, m_valid, Kd, nC, eps, rs);
  __syncthreads();
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int G = (f + 1) / 2;
  const int g_first = blockIdx.x * 4 + wave, g_step = gridDim.x * 4;
  auto set_rows = [&](int g, const T *(&rw)[GV_R]) {
    const int j0 = g * 2, j1 = min(j0 + 1, f - 1);
    rw[0] = w_gate + (size_t)j0 * Kd; rw[1] = w_gate + (size_t)j1 * Kd; rw[2] = w_up + (size_t)j0 * Kd; rw[3] = w_up + (size_t)j1 * Kd;
  };
  GvFrags<T, PIPE> fr;
  const T *rows[GV_R];
  set_rows(min(g_first, G - 1), rows);
  gemv_begin<T, PIPE>(rows, Kd, fr);
  for (int g = g_first; g < G; g += g_step) {
    const int j0 = g * 2;
    const T *next[GV_R];
    set_rows(min(g + g_step, G - 1), next);
    float acc[GV_R][M];
    zero_acc<M>(acc);
    gemv_rows<T, M, PIPE>(rows, next, xs, Kd, nC, acc, fr);
    #pragma unroll
    for (int r = 0; r < GV_R; ++r) rows[r] = next[r];
    {
      const int jj = lane & 1, m = lane >> 1;
      float rsm = 0.f;
      #pragma unroll
      for (int mm = 0; mm < M; ++mm) if (mm == m) rsm = rs[mm];
      const float gt = acc_at<M>(acc, jj, m) * rsm, up = acc_at<M>(acc, 2 + jj, m) * rsm;
      if (m < M && m < m_valid && j0 + jj < f) act[(size_t)m * f + j0 + jj] = silu_f(gt) * up;
    }
  }
}

// =====================================================================================================
// K5: head MLPs of Eq. 2-4.  For head k (0-based) the source is h1 when k < floor(K/2), else h2;
// Hp[b, k, n] = src[b][n] + SiLU(W_k[n] . src[b]) + PE[k][n].  Rows m are batch elements.
// Both sources sit in LDS; a workgroup handles groups of one head at a time.
// =====================================================================================================
template <typename T, int M, bool PIPE>
__global__ __launch_bounds__(GV_THREADS) void k_head_mlp(const T *w_mlp, const T *pe, const float *h1, const float *h2,
                                                         int d, int K, int m_valid, float *Hp, int k0, int nk) {
  // this launch serves heads k0 .. k0 + nk - 1; only the sources they read are staged (a launch over the heads of one
  // source needs half the LDS, which is what lets all rows of a wide model share one pass over the matrices)
  extern __shared__ __align__(16) float smem[];
  constexpr int CH = XLayout<T>::CH;
  const int Kd = d, nC = (Kd + CH - 1) / CH;
  const bool use1 = k0 < K / 2, use2 = k0 + nk > K / 2;
  float *xs1 = smem;
  float *xs2 = use1 ? smem + (size_t)M * nC * CH : smem;
  if (use1) load_x_plain<T, M>(xs1, h1, d, m_valid, Kd, nC);
  if (use2) load_x_plain<T, M>(xs2, h2, d, m_valid, Kd, nC);
  __syncthreads();
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int Gseg = (d + GV_R - 1) / GV_R;
  const int G = nk * Gseg;
  const int g_first = blockIdx.x * 4 + wave, g_step = gridDim.x * 4;
  auto set_rows = [&](int g, const T *(&rw)[GV_R]) {
    const int k = k0 + g / Gseg, gl = g % Gseg;
    const T *Wm = w_mlp + (size_t)k * d * d;
    #pragma unroll
    for (int r = 0; r < GV_R; ++r) rw[r] = Wm + (size_t)min(gl * GV_R + r, d - 1) * Kd;
  };
  GvFrags<T, PIPE> fr;
  const T *rows[GV_R];
  set_rows(min(g_first, G - 1), rows);
  gemv_begin<T, PIPE>(rows, Kd, fr);
  for (int g = g_first; g < G; g += g_step) {
    const int k = k0 + g / Gseg, gl = g % Gseg;
    const bool first = (k < K / 2);
    const float *xs = first ? xs1 : xs2;
    const float *src = first ? h1 : h2;
    const T *next[GV_R];
    set_rows(min(g + g_step, G - 1), next);
    float acc[GV_R][M];
    zero_acc<M>(acc);
    gemv_rows<T, M, PIPE>(rows, next, xs, Kd, nC, acc, fr);
    #pragma unroll
    for (int r = 0; r < GV_R; ++r) rows[r] = next[r];
    {
      const int r = lane & (GV_R - 1), m = lane / GV_R, n = gl * GV_R + r;
      const float v = acc_at<M>(acc, r, m);
      if (m < m_valid && n < d) {
        const float pek = pe ? Elem<T>::to_f32(pe[(size_t)k * d + n]) : 0.f;     // no position encoding: PE = 0
        Hp[((size_t)m * K + k) * d + n] = src[(size_t)m * d + n] + silu_f(v) + pek;
      }
    }
  }
}

// =====================================================================================================
// K6: the shared LM head of Eq. 6 with the top-k candidates taken in the epilogue.  A workgroup owns Gp
// consecutive row groups (4 * Gp vocabulary rows), keeps their logits of the M rows in LDS and, when its rows
// are done, each wave selects the top k of one activation row's 4 * Gp logits: the workgroup emits k (value,
// token) candidates per row instead of 4 * Gp logits, and k_topk_merge picks the row's top k from the n_wg * k
// candidates (the top k of a union is the top k of the parts' top k, so the result is exact).  The logits
// themselves go to global memory only if the caller wants them.
//   cand_v / cand_i: [M rows of this launch][n_wg][k]
// =====================================================================================================
constexpr int LMTK_NPT = 4;                      // logits per lane in the selection: a workgroup owns at most 256 rows

template <typename T, int M, bool PIPE>
__global__ __launch_bounds__(GV_THREADS) void k_lmhead_topk(const T *W, int V, int Kd, const float *x, int m_valid, int Gp,
                                                            int k, float *logits, float *cand_v, int *cand_i) {
  extern __shared__ __align__(16) float smem[];
  constexpr int CH = XLayout<T>::CH;
  const int nC = (Kd + CH - 1) / CH;
  float *xs = smem;
  const int RP = Gp * GV_R;                      // vocabulary rows of a workgroup
  float *lg = smem + (size_t)M * nC * CH;        // [M][RP]
  load_x_plain<T, M>(xs, x, Kd, m_valid, Kd, nC);
  __syncthreads();
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int G = (V + GV_R - 1) / GV_R;
  const int g0 = blockIdx.x * Gp, g1 = min(g0 + Gp, G);
  auto set_rows = [&](int g, const T *(&rw)[GV_R]) {
    #pragma unroll
    for (int r = 0; r < GV_R; ++r) rw[r] = W + (size_t)min(g * GV_R + r, V - 1) * Kd;
  };
  GvFrags<T, PIPE> fr;
  const T *rows[GV_R];
  set_rows(min(g0 + wave, G - 1), rows);
  gemv_begin<T, PIPE>(rows, Kd, fr);
  for (int g = g0 + wave; g < g1; g += 4) {
    const T *next[GV_R];
    set_rows(min(g + 4, G - 1), next);
    float acc[GV_R][M];
    zero_acc<M>(acc);
    gemv_rows<T, M, PIPE>(rows, next, xs, Kd, nC, acc, fr);
    #pragma unroll
    for (int r = 0; r < GV_R; ++r) rows[r] = next[r];
    {
      const int r = lane & (GV_R - 1), m = lane / GV_R, n = g * GV_R + r;
      const float v = acc_at<M>(acc, r, m);
      if (m < M) {
        lg[m * RP + (g - g0) * GV_R + r] = v;
        if (logits && n < V && m < m_valid) logits[(size_t)m * V + n] = v;
      }
    }
  }
  __syncthreads();
  const int n_live = min((g1 - g0) * GV_R, V - g0 * GV_R);       // this workgroup's rows inside the vocabulary
  for (int m = wave; m < m_valid; m += 4) {
    float xv[LMTK_NPT]; int id[LMTK_NPT];
    #pragma unroll
    for (int j = 0; j < LMTK_NPT; ++j) {
      const int e = j * WAVE + lane;
      id[j] = (e < n_live) ? g0 * GV_R + e : V;
      xv[j] = lg[m * RP + min(e, RP - 1)];
    }
    const size_t o = ((size_t)m * gridDim.x + blockIdx.x) * k;
    wave_select<LMTK_NPT>(xv, id, k, V, cand_v + o, cand_i + o);
  }
}

// ---- host launchers ---------------------------------------------------------------------------------
// Workgroups of a launch over `groups` row groups: one wave per group until the chip is full, i.e. at most as many
// workgroups as stay resident at once with `smem` bytes of LDS each (at most four per compute unit).  Beyond that
// the waves walk several groups each: a second round of workgroups would stage the activation rows again (with 80 KB
// of rows, four rounds read more activations than weights) and leave nothing to request ahead.
static inline int gv_grid(int groups, size_t smem) {
  int per_cu = (int)((160 * 1024) / (smem < 1 ? 1 : smem));
  per_cu = per_cu < 1 ? 1 : (per_cu > 4 ? 4 : per_cu);
  const int g = (groups + 3) / 4, cap = 256 * per_cu;
  return g < 1 ? 1 : (g > cap ? cap : g);
}
template <typename T> static inline size_t gv_xs_bytes(int M, int Kd) {
  constexpr int CH = XLayout<T>::CH;
  return (size_t)M * ((Kd + CH - 1) / CH) * CH * sizeof(float);
}

// Two batches of fragments per wave (see GvPipe): always from five rows on; for fewer rows where a compute unit gets
// a single workgroup, whose four waves would otherwise each wait out every round trip with nothing else to run:
// because the matrix has so few row groups, or because the rows of a wide model fill more than half the LDS.
static inline bool gv_pipe(int mm, int grid, size_t smem) {
  return mm >= 5 || grid <= 256 || 2 * smem > 160 * 1024;
}

// launch KERN<T, MM, pipelined or not> (MM, e, st from the enclosing launcher)
#define GV_LAUNCH(KERN, GRID, SM, ...)                                                                      \
  do {                                                                                                      \
    const int grid_ = (GRID);                                                                               \
    const size_t sm_ = (SM);                                                                                \
    if (gv_pipe(MM, grid_, sm_)) {                                                                          \
      e = gv_set_smem<T>(KERN<T, MM, true>, sm_);                                                           \
      if (e != hipSuccess) return e;                                                                        \
      hipLaunchKernelGGL((KERN<T, MM, true>), dim3(grid_), dim3(GV_THREADS), sm_, st, __VA_ARGS__);         \
    } else if constexpr (!GvPipe<MM>::on) {                                                                 \
      e = gv_set_smem<T>(KERN<T, MM, false>, sm_);                                                          \
      if (e != hipSuccess) return e;                                                                        \
      hipLaunchKernelGGL((KERN<T, MM, false>), dim3(grid_), dim3(GV_THREADS), sm_, st, __VA_ARGS__);        \
    }                                                                                                       \
  } while (0)

#define GV_DISPATCH_M(Mv, BODY)                                   \
  switch (Mv) {                                                    \
    case 1: { constexpr int MM = 1; BODY; } break;                 \
    case 2: { constexpr int MM = 2; BODY; } break;                 \
    case 3: case 4: { constexpr int MM = 4; BODY; } break;         \
    case 5: { constexpr int MM = 5; BODY; } break;                 \
    default: { constexpr int MM = 8; BODY; } break;                \
  }

template <typename T, typename Kern> static hipError_t gv_set_smem(Kern kern, size_t bytes) {
  if (bytes > 48 * 1024) return hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  return hipSuccess;
}

// Rows per launch: the activation rows of a launch sit in LDS as float32 and a wave keeps at most 8 rows of
// accumulators, so a call with more rows than that (catch-up positions of several sequences), or more than fit
// in LDS (wide models), is served in several launches over row ranges; every launch then streams the weights
// again.  Returns 0 if not even one row fits.
static inline int gv_rows_per_launch(int M, size_t bytes_per_row, size_t extra) {
  static const int sizes[] = {8, 5, 4, 2, 1};       // the instantiated row counts
  for (int mm : sizes)
    if (mm * bytes_per_row + extra <= GV_MAX_SMEM) return mm < M ? mm : M;
  return 0;
}

template <typename T>
hipError_t launch_fc_concat(hipStream_t st, const void *W, const float *u, const void *embed, const int32_t *tok,
                            int vocab, int d, int M, float *out, uint32_t *dev_status) {
  if (M < 1 || d % 8) return hipErrorInvalidValue;
  int mc = gv_rows_per_launch(M, gv_xs_bytes<T>(1, 2 * d), 0);
  // rows that fit only without their other half: two launches over d columns each
  const int mch = gv_rows_per_launch(M, gv_xs_bytes<T>(1, d), 0);
  const bool halves = mc < M && mch > mc;
  if (halves) mc = mch;
  if (mc < 1) return hipErrorInvalidValue;
  for (int m0 = 0; m0 < M; m0 += mc) {
    const int m = std::min(mc, M - m0);
    for (int half = halves ? 0 : -1; half < (halves ? 2 : 0); ++half) {
      hipError_t e = hipSuccess;
      GV_DISPATCH_M(m, {
        const size_t sm = gv_xs_bytes<T>(MM, halves ? d : 2 * d);
        GV_LAUNCH(k_fc_concat, gv_grid((d + 3) / 4, sm), sm, (const T *)W, u + (size_t)m0 * d, (const T *)embed, tok + m0, vocab, d, m,
                  out + (size_t)m0 * d, dev_status, half);
      });
    }
  }
  return hipGetLastError();
}

template <typename T>
hipError_t launch_sal_qkv(hipStream_t st, const amph_layer_w &lw, const float *x, int d, int n_heads, int d_h, int M,
                          float eps, float theta, const int32_t *sal_len, int max_kv, void *kv_stage, float *qbuf,
                          uint32_t *dev_status, int R, const int32_t *n_valid) {
  if (M < 1 || d % 8 || d_h % 4) return hipErrorInvalidValue;
  const int mc = gv_rows_per_launch(M, gv_xs_bytes<T>(1, d), 16);
  if (mc < 1) return hipErrorInvalidValue;
  for (int m0 = 0; m0 < M; m0 += mc) {
    const int m = std::min(mc, M - m0);
    hipError_t e = hipSuccess;
    GV_DISPATCH_M(m, {
      const size_t sm = gv_xs_bytes<T>(MM, d) + 16;
      GV_LAUNCH(k_sal_qkv, gv_grid(3 * d / 4, sm), sm, (const T *)lw.wq, (const T *)lw.wk, (const T *)lw.wv, (const T *)lw.rms1,
                x + (size_t)m0 * d, d, n_heads, d_h, m, eps, theta, sal_len, max_kv, (T *)kv_stage, qbuf + (size_t)m0 * d,
                dev_status, m0, R, n_valid);
    });
  }
  return hipGetLastError();
}

template <typename T>
hipError_t launch_linear(hipStream_t st, const void *w0, const void *w1, const void *w2, int n_seg, int seg_rows, int Kd,
                         const float *x, int ldx, int M, const float *res, float *o0, float *o1, float *o2, int ldo) {
  if (M < 1 || Kd % 8) return hipErrorInvalidValue;
  int mc = gv_rows_per_launch(M, gv_xs_bytes<T>(1, Kd), 0);
  // Rows too wide for all of them (up to 8) to sit in LDS whole: cut the reduction axis into ks slices instead of
  // the rows into more launches, each of which would read the matrix again.
  const int want = std::min(M, 8);
  int ks = 1;
  if (mc < want) {
    for (int c = 2; c <= 8; c *= 2)
      if (Kd % (8 * c) == 0 && gv_rows_per_launch(M, gv_xs_bytes<T>(1, Kd / c), 0) >= want) { ks = c; break; }
    if (ks > 1) mc = gv_rows_per_launch(M, gv_xs_bytes<T>(1, Kd / ks), 0);
  }
  if (mc < 1) return hipErrorInvalidValue;
  const int Kq = Kd / ks;
  for (int m0 = 0; m0 < M; m0 += mc) {
    const int m = std::min(mc, M - m0);
    const size_t oo = (size_t)m0 * ldo;
    for (int kq = 0; kq < ks; ++kq) {
      const size_t ko = (size_t)kq * Kq;
      hipError_t e = hipSuccess;
      GV_DISPATCH_M(m, {
        const size_t sm = gv_xs_bytes<T>(MM, Kq);
        GV_LAUNCH(k_linear, gv_grid(n_seg * ((seg_rows + 3) / 4), sm), sm, (const T *)w0 + ko, w1 ? (const T *)w1 + ko : nullptr,
                  w2 ? (const T *)w2 + ko : nullptr, n_seg, seg_rows, Kq, x + (size_t)m0 * ldx + ko, ldx, m,
                  (res && kq == 0) ? res + oo : nullptr, o0 + oo, o1 ? o1 + oo : nullptr, o2 ? o2 + oo : nullptr, ldo, Kd,
                  kq > 0 ? 1 : 0);
      });
    }
  }
  return hipGetLastError();
}

template <typename T>
hipError_t launch_gate_up(hipStream_t st, const amph_layer_w &lw, const float *x, int d, int f, int M, float eps,
                          float *act) {
  if (M < 1 || d % 8) return hipErrorInvalidValue;
  const int mc = gv_rows_per_launch(M, gv_xs_bytes<T>(1, d), 16);
  if (mc < 1) return hipErrorInvalidValue;
  for (int m0 = 0; m0 < M; m0 += mc) {
    const int m = std::min(mc, M - m0);
    hipError_t e = hipSuccess;
    GV_DISPATCH_M(m, {
      const size_t sm = gv_xs_bytes<T>(MM, d) + 16;
      GV_LAUNCH(k_gate_up, gv_grid((f + 1) / 2, sm), sm, (const T *)lw.w_gate, (const T *)lw.w_up, (const T *)lw.rms2,
                x + (size_t)m0 * d, d, f, m, eps, act + (size_t)m0 * f);
    });
  }
  return hipGetLastError();
}

template <typename T>
hipError_t launch_head_mlp(hipStream_t st, const void *w_mlp, const void *pe, const float *h1, const float *h2, int d,
                           int K, int M, float *Hp) {
  if (M < 1 || d % 8) return hipErrorInvalidValue;
  int mc = gv_rows_per_launch(M, 2 * gv_xs_bytes<T>(1, d), 0);
  // rows that fit only with one of the two sources staged: one launch for the heads of each source
  const int mch = gv_rows_per_launch(M, gv_xs_bytes<T>(1, d), 0);
  const bool by_source = mc < M && mch > mc && K / 2 > 0;
  if (by_source) mc = mch;
  if (mc < 1) return hipErrorInvalidValue;
  for (int m0 = 0; m0 < M; m0 += mc) {
    const int m = std::min(mc, M - m0);
    for (int part = 0; part < (by_source ? 2 : 1); ++part) {
      const int k0 = (by_source && part == 1) ? K / 2 : 0;
      const int nk = !by_source ? K : (part == 0 ? K / 2 : K - K / 2);
      hipError_t e = hipSuccess;
      GV_DISPATCH_M(m, {
        const size_t sm = (by_source ? 1 : 2) * gv_xs_bytes<T>(MM, d);
        GV_LAUNCH(k_head_mlp, gv_grid(nk * ((d + 3) / 4), sm), sm, (const T *)w_mlp, (const T *)pe, h1 + (size_t)m0 * d,
                  h2 + (size_t)m0 * d, d, K, m, Hp + (size_t)m0 * K * d, k0, nk);
      });
    }
  }
  return hipGetLastError();
}

// Workgroups of the fused LM head for one launch of m rows: as many as stay resident at once (the activation rows
// of a launch sit in LDS), at most LMTK_MAX_WG, each owning at most 64 * LMTK_NPT vocabulary rows.
template <typename T> static inline void lmtk_shape(int V, int Kd, int m, int *n_wg, int *Gp) {
  const int G = (V + GV_R - 1) / GV_R;
  const size_t sm = gv_xs_bytes<T>(m, Kd);
  int per_cu = (int)((160 * 1024) / (sm + 4096));
  per_cu = per_cu < 1 ? 1 : (per_cu > 4 ? 4 : per_cu);
  int want = std::min(std::min(G, 256 * per_cu), LMTK_MAX_WG);
  int gp = (G + want - 1) / want;
  *Gp = gp;
  *n_wg = (G + gp - 1) / gp;
}

template <typename T>
hipError_t launch_lmhead_cands(hipStream_t st, const void *W, int V, int Kd, const float *x, int M, int k, float *logits,
                               float *ws, int *n_cand) {
  if (M < 1 || Kd % 8 || k < 1 || k > AMPH_MAX_TOPK || k > V) return hipErrorInvalidValue;
  const int mc = gv_rows_per_launch(M, gv_xs_bytes<T>(1, Kd), 8 * 64 * LMTK_NPT * sizeof(float));
  if (mc < 1) return hipErrorInvalidValue;
  // every launch uses the shape of a full launch of mc rows, so that all rows have the same number of candidates
  int n_wg = 0, Gp = 0;
  lmtk_shape<T>(V, Kd, mc > 4 ? 8 : mc, &n_wg, &Gp);
  if (Gp * GV_R > 64 * LMTK_NPT) return hipErrorInvalidValue;
  float *cand_v = ws;
  int *cand_i = reinterpret_cast<int *>(ws + (size_t)M * n_wg * k);
  for (int m0 = 0; m0 < M; m0 += mc) {
    const int m = std::min(mc, M - m0);
    hipError_t e = hipSuccess;
    GV_DISPATCH_M(m, {
      const size_t sm = gv_xs_bytes<T>(MM, Kd) + (size_t)MM * Gp * GV_R * sizeof(float);
      GV_LAUNCH(k_lmhead_topk, n_wg, sm, (const T *)W, V, Kd, x + (size_t)m0 * Kd, m, Gp, k,
                logits ? logits + (size_t)m0 * V : nullptr, cand_v + (size_t)m0 * n_wg * k, cand_i + (size_t)m0 * n_wg * k);
    });
  }
  *n_cand = n_wg * k;
  return hipGetLastError();
}

size_t lmtk_ws_floats(int rows, int k) { return 2 * (size_t)rows * LMTK_MAX_WG * k; }

#define INSTANTIATE(T)                                                                                                   \
  template hipError_t launch_fc_concat<T>(hipStream_t, const void *, const float *, const void *, const int32_t *, int, \
                                          int, int, float *, uint32_t *);                                               \
  template hipError_t launch_sal_qkv<T>(hipStream_t, const amph_layer_w &, const float *, int, int, int, int, float,    \
                                        float, const int32_t *, int, void *, float *, uint32_t *, int,                  \
                                        const int32_t *);                                                               \
  template hipError_t launch_linear<T>(hipStream_t, const void *, const void *, const void *, int, int, int,            \
                                       const float *, int, int, const float *, float *, float *, float *, int);         \
  template hipError_t launch_gate_up<T>(hipStream_t, const amph_layer_w &, const float *, int, int, int, float, float *); \
  template hipError_t launch_head_mlp<T>(hipStream_t, const void *, const void *, const float *, const float *, int,    \
                                         int, int, float *);                                                            \
  template hipError_t launch_lmhead_cands<T>(hipStream_t, const void *, int, int, const float *, int, int, float *,     \
                                             float *, int *);
INSTANTIATE(float)
INSTANTIATE(bf16_t)

}  // namespace amph
