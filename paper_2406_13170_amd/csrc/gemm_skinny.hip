// Skinny GEMM for the target's forward pass over the tree tokens (Sec. 2 "Tree Attention"): M = B*T
// activation rows (64 per block) against [N, Kd] weights that stream from HBM once, on the matrix
// cores.
//
// A 256-thread workgroup owns a 64 (tokens) x 64 (weight rows) output tile and a slice of the
// reduction axis.  Each wave keeps 16 weight rows: its A fragments are 16-byte loads straight from
// global memory (lane = row, 16 contiguous bytes of that row), prefetched one chunk ahead in
// registers.  The activations of the chunk (64 rows x 256 bytes) are staged through a padded,
// double-buffered LDS tile and read back as B fragments, so every weight byte is fetched once and
// multiplied against all 64 tokens.  Partial tiles of a split reduction axis are summed in a fixed
// order by the last workgroup to arrive (bit-reproducible, no float atomics), which then runs the
// fused epilogue: residual add, RoPE + KV-cache write, SwiGLU, or per-row argmax.
#include "kernels.h"

namespace amph {

constexpr int GM_BM = 64, GM_BN = 64;
constexpr int GM_CHUNK_B = 256;                 // bytes of one activation row per chunk
constexpr int GM_PITCH = GM_CHUNK_B + 16;       // LDS row pitch (bytes): rows shift by 4 banks
constexpr int GM_STEPS = GM_CHUNK_B / 64;       // matrix-core steps per chunk (64 bytes of k each)
constexpr int GM_CT_PITCH = GM_BN + 4;          // floats
constexpr int GM_LDS_BYTES = 2 * GM_BM * GM_PITCH;
static_assert(GM_LDS_BYTES >= GM_BM * GM_CT_PITCH * 4, "output tile must fit in the staging buffers");

// weight row (within its matrix) and matrix index of tile row r
struct RowMap { int seg; int n; bool valid; };

template <int EPI>
__device__ __forceinline__ RowMap map_row(const GemmArgs &a, int tile, int r) {
  RowMap o;
  if (EPI == EPI_QKV_ROPE) {
    const int d = a.n_heads * a.d_h, tps = d / GM_BN;
    o.seg = tile / tps;
    const int tl = tile % tps;
    if (o.seg < 2) {
      const int half = a.d_h / 2, tph = a.d_h / GM_BN;
      const int head = tl / tph, p = tl % tph;
      o.n = head * a.d_h + p * 32 + (r & 31) + ((r >= 32) ? half : 0);
    } else {
      o.n = tl * GM_BN + r;
    }
    o.valid = true;
  } else if (EPI == EPI_SWIGLU) {
    o.seg = (r >= 32) ? 1 : 0;
    o.n = tile * 32 + (r & 31);
    o.valid = o.n < a.seg_rows;
  } else {
    o.seg = 0;
    o.n = tile * GM_BN + r;
    o.valid = o.n < a.seg_rows;
  }
  return o;
}

template <typename T, int EPI>
__global__ __launch_bounds__(256) void k_gemm_skinny(const GemmArgs a, int tiles) {
  __shared__ __align__(16) unsigned char lds[GM_LDS_BYTES];
  __shared__ int s_flag;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 4, r16 = lane & 15;
  const int S = a.split_k;
  const int tile = blockIdx.x / S, split = blockIdx.x % S, mblock = blockIdx.y;
  const int m_base = mblock * GM_BM;
  const int row_bytes = a.Kd * (int)sizeof(T);
  const int total_steps = row_bytes / 64;
  const int s0 = (int)((long long)total_steps * split / S), s1 = (int)((long long)total_steps * (split + 1) / S);
  const int nch = (s1 - s0 + GM_STEPS - 1) / GM_STEPS;

  const RowMap rm = map_row<EPI>(a, tile, wave * 16 + r16);
  const void *wm = (rm.seg == 0) ? a.w0 : (rm.seg == 1) ? a.w1 : a.w2;
  const unsigned char *wrow = (const unsigned char *)wm + (size_t)(rm.valid ? rm.n : 0) * row_bytes + g * 16;
  const unsigned char *xg = (const unsigned char *)a.x;
  const int x_row0 = tid >> 4, x_col = (tid & 15) * 16;

  uint4 a_cur[GM_STEPS], a_nxt[GM_STEPS], xr[4];
  auto load_chunk = [&](int c, uint4 (&af)[GM_STEPS]) {
    #pragma unroll
    for (int s = 0; s < GM_STEPS; ++s) {
      const int st = s0 + c * GM_STEPS + s;
      if (rm.valid && st < s1) af[s] = ldg16(wrow + (size_t)st * 64);
      else af[s] = make_uint4(0u, 0u, 0u, 0u);
    }
    const int byte = (s0 + c * GM_STEPS) * 64 + x_col;
    #pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int mg = m_base + x_row0 + 16 * j;
      if (mg < a.M && byte < s1 * 64) xr[j] = ldg16(xg + (size_t)mg * row_bytes + byte);
      else xr[j] = make_uint4(0u, 0u, 0u, 0u);
    }
  };

  f32x4 acc[4];
  #pragma unroll
  for (int mb = 0; mb < 4; ++mb) acc[mb] = (f32x4){0.f, 0.f, 0.f, 0.f};

  if (nch > 0) load_chunk(0, a_cur);
  for (int c = 0; c < nch; ++c) {
    unsigned char *buf = lds + (c & 1) * (GM_BM * GM_PITCH);
    #pragma unroll
    for (int j = 0; j < 4; ++j) *reinterpret_cast<uint4 *>(buf + (x_row0 + 16 * j) * GM_PITCH + x_col) = xr[j];
    __syncthreads();
    if (c + 1 < nch) load_chunk(c + 1, a_nxt);
    #pragma unroll
    for (int s = 0; s < GM_STEPS; ++s) {
      #pragma unroll
      for (int mb = 0; mb < 4; ++mb) {
        const uint4 bfrag = *reinterpret_cast<const uint4 *>(buf + (mb * 16 + r16) * GM_PITCH + s * 64 + g * 16);
        acc[mb] = mma16<T>(a_cur[s], bfrag, acc[mb]);
      }
    }
    #pragma unroll
    for (int s = 0; s < GM_STEPS; ++s) a_cur[s] = a_nxt[s];
  }
  __syncthreads();                                   // everyone is done with the staging buffers

  // accumulators -> Ct[m][r] (float32): lane holds rows r = wave*16 + g*4 .. +4 of column m
  float *Ct = reinterpret_cast<float *>(lds);
  #pragma unroll
  for (int mb = 0; mb < 4; ++mb)
    *reinterpret_cast<f32x4 *>(Ct + (mb * 16 + r16) * GM_CT_PITCH + wave * 16 + g * 4) = acc[mb];
  __syncthreads();

  if (S > 1) {
    float *part = a.partials + ((size_t)(mblock * tiles + tile) * S) * (GM_BM * GM_BN);
    float *mine = part + (size_t)split * (GM_BM * GM_BN);
    #pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int i4 = tid + it * 256, m = i4 >> 4, n4 = (i4 & 15) * 4;
      *reinterpret_cast<f32x4 *>(mine + m * GM_BN + n4) = *reinterpret_cast<const f32x4 *>(Ct + m * GM_CT_PITCH + n4);
    }
    if (!arrive_and_is_last(a.counters + mblock * tiles + tile, (unsigned)S, &s_flag)) return;
    #pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int i4 = tid + it * 256, m = i4 >> 4, n4 = (i4 & 15) * 4;
      f32x4 sum = *reinterpret_cast<const f32x4 *>(part + m * GM_BN + n4);
      for (int sp = 1; sp < S; ++sp)
        sum += *reinterpret_cast<const f32x4 *>(part + (size_t)sp * (GM_BM * GM_BN) + m * GM_BN + n4);
      *reinterpret_cast<f32x4 *>(Ct + m * GM_CT_PITCH + n4) = sum;
    }
    __syncthreads();
  }

  // ---------------------------------------------------------------------------------- epilogues
  if (EPI == EPI_STORE || EPI == EPI_RESIDUAL) {
    const int N = a.seg_rows;
    for (int idx = tid; idx < GM_BM * GM_BN; idx += 256) {
      const int m = idx >> 6, r = idx & 63, mg = m_base + m, n = tile * GM_BN + r;
      if (mg < a.M && n < N) {
        float v = Ct[m * GM_CT_PITCH + r];
        float *dst = a.out + (size_t)mg * N + n;
        if (EPI == EPI_RESIDUAL) v += *dst;
        *dst = v;
      }
    }
  } else if (EPI == EPI_SWIGLU) {
    const int f = a.seg_rows;
    T *act = (T *)a.act;
    for (int idx = tid; idx < GM_BM * 32; idx += 256) {
      const int m = idx >> 5, r = idx & 31, mg = m_base + m, j = tile * 32 + r;
      if (mg < a.M && j < f)
        act[(size_t)mg * f + j] = Elem<T>::from_f32(silu_f(Ct[m * GM_CT_PITCH + r]) * Ct[m * GM_CT_PITCH + r + 32]);
    }
  } else if (EPI == EPI_QKV_ROPE) {
    const int d_h = a.d_h, d = a.n_heads * d_h, tps = d / GM_BN;
    const int seg = tile / tps, tl = tile % tps;
    if (seg < 2) {
      const int half = d_h / 2, tph = d_h / GM_BN;
      const int head = tl / tph, p = tl % tph;
      const float l2t = log2f(a.theta);
      for (int idx = tid; idx < GM_BM * 32; idx += 256) {
        const int m = idx >> 5, r = idx & 31, mg = m_base + m;
        if (mg >= a.M) continue;
        const int e = p * 32 + r;
        const float inv_freq = exp2f(-2.0f * (float)e / (float)d_h * l2t);
        float sn, cs;
        sincosf((float)a.tree_pos[mg] * inv_freq, &sn, &cs);
        const float x1 = Ct[m * GM_CT_PITCH + r], x2 = Ct[m * GM_CT_PITCH + r + 32];
        const float y1 = x1 * cs - x2 * sn, y2 = x2 * cs + x1 * sn;
        if (seg == 0) {
          T *q = (T *)a.q_out + (size_t)mg * d + head * d_h + e;
          q[0] = Elem<T>::from_f32(y1);
          q[half] = Elem<T>::from_f32(y2);
        } else {
          const int b = mg / a.T_nodes, node = mg % a.T_nodes, L = a.kv_len[b];
          if (L < 0 || L + a.T_nodes > a.max_kv) {
            if (r == 0 && node == 0) atomicOr(a.dev_status, 2u);
            continue;
          }
          T *kc = (T *)a.k_cache + (((size_t)b * a.n_heads + head) * a.max_kv + (L + node)) * d_h + e;
          kc[0] = Elem<T>::from_f32(y1);
          kc[half] = Elem<T>::from_f32(y2);
        }
      }
    } else {
      // values: dimension-major cache, consecutive threads -> consecutive tree rows
      for (int idx = tid; idx < GM_BM * GM_BN; idx += 256) {
        const int r = idx >> 6, m = idx & 63, mg = m_base + m;
        if (mg >= a.M) continue;
        const int n = tl * GM_BN + r, head = n / d_h, e = n % d_h;
        const int b = mg / a.T_nodes, node = mg % a.T_nodes, L = a.kv_len[b];
        if (L < 0 || L + a.T_nodes > a.max_kv) continue;
        T *vc = (T *)a.v_cache + (((size_t)b * a.n_heads + head) * d_h + e) * a.max_kv + (L + node);
        *vc = Elem<T>::from_f32(Ct[m * GM_CT_PITCH + r]);
      }
    }
  } else if (EPI == EPI_ARGMAX) {
    const int N = a.seg_rows;
    if (a.logits) {
      for (int idx = tid; idx < GM_BM * GM_BN; idx += 256) {
        const int m = idx >> 6, r = idx & 63, mg = m_base + m, n = tile * GM_BN + r;
        if (mg < a.M && n < N) a.logits[(size_t)mg * N + n] = Ct[m * GM_CT_PITCH + r];
      }
    }
    {   // 4 threads per token row, 16 columns each, then a 4-lane butterfly (ties -> lower column)
      const int m = tid >> 2, part = tid & 3, mg = m_base + m;
      float bv = -__builtin_huge_valf(); int bi = 0x7fffffff;
      for (int r = part * 16; r < part * 16 + 16; ++r) {
        const int n = tile * GM_BN + r;
        const float v = Ct[m * GM_CT_PITCH + r];
        if (n < N && (v > bv || (v == bv && n < bi))) { bv = v; bi = n; }
      }
      #pragma unroll
      for (int off = 1; off <= 2; off <<= 1) {
        const float ov = __shfl_xor(bv, off, WAVE);
        const int oi = __shfl_xor(bi, off, WAVE);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
      }
      if (part == 0 && mg < a.M) {
        a.amax_val[(size_t)tile * a.M + mg] = bv;
        a.amax_idx[(size_t)tile * a.M + mg] = bi;
      }
    }
    // the last tile of this block of rows folds the per-tile winners
    if (!arrive_and_is_last(a.counters + 8192 + mblock, (unsigned)tiles, &s_flag)) return;
    {
      const int m = tid >> 2, part = tid & 3, mg = m_base + m;
      float bv = -__builtin_huge_valf(); int bi = 0x7fffffff;
      if (mg < a.M) {
        for (int t = part; t < tiles; t += 4) {
          const float v = a.amax_val[(size_t)t * a.M + mg];
          const int i = a.amax_idx[(size_t)t * a.M + mg];
          if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
        }
      }
      #pragma unroll
      for (int off = 1; off <= 2; off <<= 1) {
        const float ov = __shfl_xor(bv, off, WAVE);
        const int oi = __shfl_xor(bi, off, WAVE);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
      }
      if (part == 0 && mg < a.M) a.tgt[mg] = bi;
    }
  }
}

int gemm_tiles_n(int epi, int n_seg, int seg_rows, int d_h) {
  (void)d_h;
  if (epi == EPI_QKV_ROPE) return 3 * (seg_rows / GM_BN);
  if (epi == EPI_SWIGLU) return (seg_rows + 31) / 32;
  (void)n_seg;
  return (seg_rows + GM_BN - 1) / GM_BN;
}

int gemm_auto_split(int tiles, int Kd, int elem_bytes) {
  const int total_steps = Kd * elem_bytes / 64;
  int s = 1;
  while (s < 8 && tiles * s < 256 && total_steps / (s * 2) >= 16) s *= 2;
  return s;
}

template <typename T>
hipError_t launch_gemm(hipStream_t st, int epi, const GemmArgs &a) {
  if (a.M < 1 || a.Kd < 1 || (a.Kd * (int)sizeof(T)) % 64) return hipErrorInvalidValue;
  if (a.split_k != 1 && a.split_k != 2 && a.split_k != 4 && a.split_k != 8) return hipErrorInvalidValue;
  const int tiles = gemm_tiles_n(epi, a.n_seg, a.seg_rows, a.d_h);
  const int mblocks = (a.M + GM_BM - 1) / GM_BM;
  if (tiles * mblocks > 8192 || mblocks > 64) return hipErrorInvalidValue;
  if (a.split_k > 1 && (size_t)tiles * mblocks * a.split_k * (GM_BM * GM_BN) > a.partials_cap) return hipErrorInvalidValue;
  if (epi == EPI_QKV_ROPE && (a.d_h % 64 || (a.n_heads * a.d_h) % GM_BN)) return hipErrorInvalidValue;
  const dim3 grid(tiles * a.split_k, mblocks), block(256);
  switch (epi) {
    case EPI_STORE: hipLaunchKernelGGL((k_gemm_skinny<T, EPI_STORE>), grid, block, 0, st, a, tiles); break;
    case EPI_RESIDUAL: hipLaunchKernelGGL((k_gemm_skinny<T, EPI_RESIDUAL>), grid, block, 0, st, a, tiles); break;
    case EPI_QKV_ROPE: hipLaunchKernelGGL((k_gemm_skinny<T, EPI_QKV_ROPE>), grid, block, 0, st, a, tiles); break;
    case EPI_SWIGLU: hipLaunchKernelGGL((k_gemm_skinny<T, EPI_SWIGLU>), grid, block, 0, st, a, tiles); break;
    case EPI_ARGMAX: hipLaunchKernelGGL((k_gemm_skinny<T, EPI_ARGMAX>), grid, block, 0, st, a, tiles); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
template hipError_t launch_gemm<float>(hipStream_t, int, const GemmArgs &);
template hipError_t launch_gemm<bf16_t>(hipStream_t, int, const GemmArgs &);

}  // namespace amph
