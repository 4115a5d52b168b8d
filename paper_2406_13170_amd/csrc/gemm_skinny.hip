// Skinny GEMM for the target's forward pass over the tree tokens (Sec. 2 "Tree Attention"): M = B*T
// activation rows (64 per block) against [N, Kd] weights that stream from HBM once, on the matrix
// cores.
//
// A 256-thread workgroup owns a 64 (tokens) x 64 (weight rows) output tile and a slice of the
// reduction axis.  Each wave keeps 16 weight rows: its A fragments are 16-byte loads straight from
// global memory (lane = row, 16 contiguous bytes of that row), prefetched three 512-byte chunks (8
// fragments each) ahead in a register ring, enough to cover HBM latency with one or two workgroups per CU.  The activations of the chunk (64 rows x 512 bytes) are staged
// through a padded, double-buffered LDS tile and read back as B fragments, so every weight byte is
// fetched once and multiplied against all 64 tokens.
//
// No workgroup ever communicates with another inside the kernel (a device-scope fence per workgroup
// costs far more than the kernel on this chip): a split reduction axis writes one partial slab per
// split, which the consumer (the RMSNorm kernel of the next sub-layer, or k_sum_slabs) adds up in a
// fixed order; per-tile argmax candidates are folded by k_argmax_fold.  Fused epilogues: RoPE from a
// precomputed table + KV-cache write, SwiGLU, per-tile row argmax.
#include "kernels.h"

namespace amph {

constexpr int GM_BM = 64, GM_BN = 64;
constexpr int GM_CHUNK_B = 512;                 // bytes of one activation row per chunk
constexpr int GM_PITCH = GM_CHUNK_B + 16;       // LDS row pitch (bytes): rows shift by 4 banks
constexpr int GM_STEPS = GM_CHUNK_B / 64;       // matrix-core steps per chunk (64 bytes of k each)
constexpr int GM_NST = 4;                       // register ring of weight chunks (even)
constexpr int GM_XL = GM_BM * GM_CHUNK_B / 16 / 256;   // 16-byte activation loads per thread per chunk
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
__global__ __launch_bounds__(256, 2) void k_gemm_skinny(const GemmArgs a, int tiles) {
  __shared__ __align__(16) unsigned char lds[GM_LDS_BYTES];
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
  if (nch <= 0) return;                                // cannot happen: every split owns at least one step
  const unsigned char *xg = (const unsigned char *)a.x;
  const int x_row0 = tid >> 5, x_col = (tid & 31) * 16;      // 32 lanes cover one 512-byte row piece

  // Software pipeline.  Weight fragments come from HBM: they are requested GM_NST-1 chunks ahead into a
  // register ring.  Activation pieces come from L2: requested two chunks ahead into registers, written to
  // the LDS buffer of the next chunk after the current chunk's math, one barrier per chunk.  Within an
  // iteration the activation loads are issued before the weight loads, so waiting for them (loads
  // complete in order) never waits for the younger, slower weight loads.
  uint4 aw[GM_NST][GM_STEPS], xr[2][GM_XL];
  auto load_w = [&](int c, uint4 (&af)[GM_STEPS]) {
    #pragma unroll
    for (int s = 0; s < GM_STEPS; ++s) {
      // Unconditional load (a predicated load with a zero alternative makes the compiler wait for every
      // load at the merge).  Steps past the slice re-read its last step: harmless, because the activation
      // tile is zero there and weights are finite; rows past N re-read row 0 and are never stored.
      const int st = min(s0 + c * GM_STEPS + s, s1 - 1);
      af[s] = ldg16(wrow + (size_t)st * 64);
    }
  };
  auto load_x = [&](int c, uint4 (&xf)[GM_XL]) {
    const int byte = (s0 + c * GM_STEPS) * 64 + x_col;
    const bool in_k = byte < s1 * 64;
    #pragma unroll
    for (int j = 0; j < GM_XL; ++j) {
      const int mg = m_base + x_row0 + 8 * j;
      const bool ok = in_k && mg < a.M;                 // out-of-range pieces read the tensor's first bytes ...
      xf[j] = ldg16(xg + (ok ? (size_t)mg * row_bytes + byte : (size_t)0));
    }
  };
  auto store_x = [&](int bufi, int c, const uint4 (&xf)[GM_XL]) {
    unsigned char *buf = lds + bufi * (GM_BM * GM_PITCH);
    const bool in_k = (s0 + c * GM_STEPS) * 64 + x_col < s1 * 64;
    #pragma unroll
    for (int j = 0; j < GM_XL; ++j) {
      const bool ok = in_k && (m_base + x_row0 + 8 * j) < a.M;   // ... and are replaced by zeros here
      *reinterpret_cast<uint4 *>(buf + (x_row0 + 8 * j) * GM_PITCH + x_col) = ok ? xf[j] : make_uint4(0u, 0u, 0u, 0u);
    }
  };

  f32x4 acc[4];
  #pragma unroll
  for (int mb = 0; mb < 4; ++mb) acc[mb] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // The chunk loop runs to a multiple of GM_NST with no conditional inside: chunks past the slice load
  // clamped addresses and stage zeros, so every iteration issues the same number of loads and the
  // compiler can count outstanding loads exactly instead of draining them at every join.
  const int nch4 = (nch + GM_NST - 1) / GM_NST * GM_NST;
  load_x(0, xr[0]);
  load_w(0, aw[0]);
  load_x(1, xr[1]);
  #pragma unroll
  for (int u = 1; u < GM_NST - 1; ++u) load_w(u, aw[u]);
  store_x(0, 0, xr[0]);
  __syncthreads();
  for (int c = 0; c < nch4; c += GM_NST) {
    #pragma unroll
    for (int u = 0; u < GM_NST; ++u) {
      const int cc = c + u;
      load_x(cc + 2, xr[u & 1]);                        // slot of chunk cc: already in LDS
      load_w(cc + GM_NST - 1, aw[(u + GM_NST - 1) % GM_NST]);
      const unsigned char *buf = lds + (u & 1) * (GM_BM * GM_PITCH);
      #pragma unroll
      for (int s = 0; s < GM_STEPS; ++s) {
        #pragma unroll
        for (int mb = 0; mb < 4; ++mb) {
          const uint4 bfrag = *reinterpret_cast<const uint4 *>(buf + (mb * 16 + r16) * GM_PITCH + s * 64 + g * 16);
          acc[mb] = mma16<T>(aw[u][s], bfrag, acc[mb]);
        }
      }
      store_x((u + 1) & 1, cc + 1, xr[(u + 1) & 1]);
      __syncthreads();
    }
  }

  // accumulators -> Ct[m][r] (float32): lane holds rows r = wave*16 + g*4 .. +4 of column m
  float *Ct = reinterpret_cast<float *>(lds);
  #pragma unroll
  for (int mb = 0; mb < 4; ++mb)
    *reinterpret_cast<f32x4 *>(Ct + (mb * 16 + r16) * GM_CT_PITCH + wave * 16 + g * 4) = acc[mb];
  __syncthreads();

  // ---------------------------------------------------------------------------------- epilogues
  if (EPI == EPI_STORE) {
    // out is [split_k][M][N]: slab `split` receives this workgroup's partial sums
    const int N = a.seg_rows;
    float *slab = a.out + (size_t)split * a.M * N;
    for (int idx = tid; idx < GM_BM * GM_BN; idx += 256) {
      const int m = idx >> 6, r = idx & 63, mg = m_base + m, n = tile * GM_BN + r;
      if (mg < a.M && n < N) slab[(size_t)mg * N + n] = Ct[m * GM_CT_PITCH + r];
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
      for (int idx = tid; idx < GM_BM * 32; idx += 256) {
        const int m = idx >> 5, r = idx & 31, mg = m_base + m;
        if (mg >= a.M) continue;
        const int e = p * 32 + r;
        const float2 cs = a.rope_cs[(size_t)mg * half + e];          // (cos, sin) of tree_pos[mg] * theta^(-2e/d_h)
        const float x1 = Ct[m * GM_CT_PITCH + r], x2 = Ct[m * GM_CT_PITCH + r + 32];
        const float y1 = x1 * cs.x - x2 * cs.y, y2 = x2 * cs.x + x1 * cs.y;
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
    // 4 threads per token row, 16 columns each, then a 4-lane butterfly (ties -> lower column)
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
}

// tgt[m] = index of the best of the per-tile winners (ties -> lower index); one wave per row
__global__ __launch_bounds__(64) void k_argmax_fold(const float *amax_val, const int32_t *amax_idx, int tiles, int M,
                                                    int32_t *tgt) {
  const int mg = blockIdx.x, lane = threadIdx.x;
  float bv = -__builtin_huge_valf(); int bi = 0x7fffffff;
  for (int t = lane; t < tiles; t += WAVE) {
    const float v = amax_val[(size_t)t * M + mg];
    const int i = amax_idx[(size_t)t * M + mg];
    if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
  }
  #pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const float ov = __shfl_xor(bv, off, WAVE);
    const int oi = __shfl_xor(bi, off, WAVE);
    if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
  }
  if (lane == 0) tgt[mg] = bi;
}

// out[i] = sum_s slabs[s][i], s ascending
__global__ __launch_bounds__(256) void k_sum_slabs(const float *slabs, int S, size_t n, float *out) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    float v = slabs[i];
    for (int s = 1; s < S; ++s) v += slabs[(size_t)s * n + i];
    out[i] = v;
  }
}

// (cos, sin) of pos[m] * theta^(-2e/d_h) for e < d_h/2: the same table serves every layer of a pass
__global__ void k_rope_table(const int32_t *pos, int M, int d_h, float theta, float2 *cs) {
  const int half = d_h / 2;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= M * half) return;
  const int m = i / half, e = i % half;
  const float inv_freq = exp2f(-2.0f * (float)e / (float)d_h * log2f(theta));
  float sn, c;
  sincosf((float)pos[m] * inv_freq, &sn, &c);
  cs[i] = make_float2(c, sn);
}

hipError_t launch_rope_table(hipStream_t st, const int32_t *pos, int M, int d_h, float theta, float2 *cs) {
  const int n = M * (d_h / 2);
  hipLaunchKernelGGL(k_rope_table, dim3((n + 255) / 256), dim3(256), 0, st, pos, M, d_h, theta, cs);
  return hipGetLastError();
}

hipError_t launch_sum_slabs(hipStream_t st, const float *slabs, int S, size_t n, float *out) {
  int blocks = (int)((n + 255) / 256);
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(k_sum_slabs, dim3(blocks), dim3(256), 0, st, slabs, S, n, out);
  return hipGetLastError();
}

hipError_t launch_argmax_fold(hipStream_t st, const float *amax_val, const int32_t *amax_idx, int tiles, int M,
                              int32_t *tgt) {
  hipLaunchKernelGGL(k_argmax_fold, dim3(M), dim3(64), 0, st, amax_val, amax_idx, tiles, M, tgt);
  return hipGetLastError();
}

int gemm_tiles_n(int epi, int n_seg, int seg_rows, int d_h) {
  (void)d_h; (void)n_seg;
  if (epi == EPI_QKV_ROPE) return 3 * (seg_rows / GM_BN);
  if (epi == EPI_SWIGLU) return (seg_rows + 31) / 32;
  return (seg_rows + GM_BN - 1) / GM_BN;
}

// Split the reduction axis only where the output alone gives too few workgroups for the chip.
int gemm_auto_split(int tiles, int Kd, int elem_bytes) {
  const int total_steps = Kd * elem_bytes / 64;
  int s = 1;
  while (s < 8 && tiles * s < 192 && total_steps / (s * 2) >= 16) s *= 2;
  return s;
}

template <typename T>
hipError_t launch_gemm(hipStream_t st, int epi, const GemmArgs &a) {
  if (a.M < 1 || a.Kd < 1 || (a.Kd * (int)sizeof(T)) % 64) return hipErrorInvalidValue;
  if (a.split_k != 1 && a.split_k != 2 && a.split_k != 4 && a.split_k != 8) return hipErrorInvalidValue;
  if (epi != EPI_STORE && a.split_k != 1) return hipErrorInvalidValue;     // fused epilogues need complete sums
  const int tiles = gemm_tiles_n(epi, a.n_seg, a.seg_rows, a.d_h);
  const int mblocks = (a.M + GM_BM - 1) / GM_BM;
  if (mblocks > 65535) return hipErrorInvalidValue;
  if (epi == EPI_QKV_ROPE && (a.d_h % 64 || (a.n_heads * a.d_h) % GM_BN || !a.rope_cs)) return hipErrorInvalidValue;
  const dim3 grid(tiles * a.split_k, mblocks), block(256);
  switch (epi) {
    case EPI_STORE: hipLaunchKernelGGL((k_gemm_skinny<T, EPI_STORE>), grid, block, 0, st, a, tiles); break;
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
