// Shared device helpers for the gfx950 kernels: 16-byte fragments of float / bfloat16, the matrix-core
// step on such fragments, and wave / block reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace amph {

typedef __bf16 bf16_t;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int WAVE = 64;
constexpr float NEG_BIG = -1.0e30f;   // finite stand-in for -inf in running maxima

// ---- element traits: PER = elements in one 16-byte fragment ------------------------------------
template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int PER = 4;
  static __device__ __forceinline__ void unpack(const uint4 &v, float *f) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  }
  static __device__ __forceinline__ float to_f32(float v) { return v; }
  static __device__ __forceinline__ float from_f32(float v) { return v; }
};
template <> struct Elem<bf16_t> {
  static constexpr int PER = 8;
  static __device__ __forceinline__ void unpack(const uint4 &v, float *f) {
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
  }
  static __device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
  static __device__ __forceinline__ bf16_t from_f32(float v) { return (bf16_t)v; }   // RNE
};

// pack PER floats into one 16-byte fragment of T (RNE for bf16)
template <typename T> __device__ __forceinline__ uint4 pack16(const float *f);
template <> __device__ __forceinline__ uint4 pack16<float>(const float *f) {
  return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
}
template <> __device__ __forceinline__ uint4 pack16<bf16_t>(const float *f) {
  union { bf16x8 v; uint4 u; } c;
  #pragma unroll
  for (int i = 0; i < 8; ++i) c.v[i] = (bf16_t)f[i];
  return c.u;
}

__device__ __forceinline__ uint4 ldg16(const void *p) { return *reinterpret_cast<const uint4 *>(p); }
// the same load marked non-temporal: data that is read once (a weight stream) should not push reused data out of L2
__device__ __forceinline__ uint4 ldg16_stream(const void *p) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void stg16(void *p, const uint4 &v) { *reinterpret_cast<uint4 *>(p) = v; }

// 4 consecutive elements of T <-> float[4]
template <typename T> __device__ __forceinline__ void load4(const T *p, float *f);
template <> __device__ __forceinline__ void load4<float>(const float *p, float *f) {
  const float4 v = *reinterpret_cast<const float4 *>(p);
  f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
}
template <> __device__ __forceinline__ void load4<bf16_t>(const bf16_t *p, float *f) {
  const uint2 v = *reinterpret_cast<const uint2 *>(p);
  f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
  f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
}
template <typename T> __device__ __forceinline__ void store4(T *p, const float *f);
template <> __device__ __forceinline__ void store4<float>(float *p, const float *f) {
  *reinterpret_cast<float4 *>(p) = make_float4(f[0], f[1], f[2], f[3]);
}
template <> __device__ __forceinline__ void store4<bf16_t>(bf16_t *p, const float *f) {
  typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
  bf16x4 v;
  #pragma unroll
  for (int i = 0; i < 4; ++i) v[i] = (bf16_t)f[i];
  *reinterpret_cast<bf16x4 *>(p) = v;
}

// ---- matrix-core step on 16-byte fragments --------------------------------------------------------
// D[16 x 16] += A[16 x KS] * B[KS x 16] with KS = 4 * PER.  Lane l holds for A: row l%16, contraction
// slots (l/16)*PER .. +PER; for B: column l%16, the same slots; for D: column l%16, rows (l/16)*4..+4.
// bf16: one 16x16x32 instruction.  float: four 16x16x4 instructions, the j-th using element j of
// every lane's fragment (any one-to-one slot assignment is valid as long as A and B agree).
template <typename T> __device__ __forceinline__ f32x4 mma16(const uint4 &a, const uint4 &b, f32x4 acc);
template <> __device__ __forceinline__ f32x4 mma16<bf16_t>(const uint4 &a, const uint4 &b, f32x4 acc) {
  union { uint4 u; bf16x8 v; } ca, cb;
  ca.u = a; cb.u = b;
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(ca.v, cb.v, acc, 0, 0, 0);
}
template <> __device__ __forceinline__ f32x4 mma16<float>(const uint4 &a, const uint4 &b, f32x4 acc) {
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
  return acc;
}

// acc[32 x 32] += A[32 rows x 32 bytes of k] * B[32 columns x 32 bytes of k]: lane (half = lane / 32, r = lane % 32)
// holds the 16 bytes at half * 16 of row (column) r; afterwards lane (half, r) holds column r, rows
// (i / 4) * 8 + half * 4 + (i % 4) in acc[i].  On this chip the 32 x 32 bf16 instruction runs at twice the
// rate of the 16 x 16 one (measured: 2.3 against 1.3 PFLOP/s with every SIMD busy).
typedef float f32x16 __attribute__((ext_vector_type(16)));
template <typename T> __device__ __forceinline__ f32x16 mma32(const uint4 &a, const uint4 &b, f32x16 acc);
template <> __device__ __forceinline__ f32x16 mma32<bf16_t>(const uint4 &a, const uint4 &b, f32x16 acc) {
  union { uint4 u; bf16x8 v; } ca, cb;
  ca.u = a; cb.u = b;
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(ca.v, cb.v, acc, 0, 0, 0);
}
template <> __device__ __forceinline__ f32x16 mma32<float>(const uint4 &a, const uint4 &b, f32x16 acc) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
  return acc;
}

// Element index of (row, dim) in the step-tiled K and V caches of one head (layout: header of the C ABI).
template <typename T> __device__ __forceinline__ size_t k_tiled_index(int row, int c, int d_h) {
  constexpr int PER = Elem<T>::PER, KSTEP = 4 * PER, PIECE = 64 / (int)sizeof(T);   // elements in 64 bytes
  const int s = row / KSTEP, kk = row % KSTEP, t = (kk % PER) / 4, i = (kk / PER) * 4 + (kk & 3);
  return ((size_t)(s * (PER / 4) + t) * (d_h / PIECE) + c / PIECE) * (16 * PIECE) + i * PIECE + c % PIECE;
}
template <typename T> __device__ __forceinline__ size_t v_tiled_index(int row, int c, int d_h) {
  constexpr int PER = Elem<T>::PER, KSTEP = 4 * PER, PIECE = 64 / (int)sizeof(T);
  return ((size_t)(row / KSTEP) * (d_h / 16) + c / 16) * (16 * PIECE) + (c % 16) * PIECE + row % KSTEP;
}

// Element index of (row m, element k) in the fragment-tiled activation layout the wide GEMM reads: 32 rows x 32 bytes
// of k per KB, lane-linear (lane = half * 32 + m % 32 holds the 16 bytes at half * 16).  4 elements starting at a
// multiple of 4 stay inside one 16-byte piece.
template <typename T> __device__ __forceinline__ size_t xt_index(int m, int k, int m32_tiles) {
  const int kb = k * (int)sizeof(T);
  const size_t byte = ((size_t)(kb >> 5) * m32_tiles + (m >> 5)) * 1024 + (size_t)((((kb >> 4) & 1) * 32 + (m & 31)) << 4) + (kb & 15);
  return byte / sizeof(T);
}

// ---- wave-level reductions ---------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
  #pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, WAVE);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
  #pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, WAVE));
  return v;
}

// sum over a whole 256-thread block; every thread gets the result.  red must hold 4 floats.
__device__ __forceinline__ float block_sum_256(float v, float *red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

// ---- selection inside one wave (top-k of Eq. 6) ---------------------------------------------------------
// "Better" means a larger value, or the same value and a smaller index, so results are sorted and ties deterministic.
__device__ __forceinline__ bool better(float v1, int i1, float v2, int i2) {
  return (v1 > v2) || (v1 == v2 && i1 < i2);
}

// The best (value, index) pair of the wave, in every lane.  Six data-parallel-primitive steps instead of a
// butterfly of cross-lane permutes through the LDS crossbar (twelve dependent permutes cost about 1400 clocks per
// selection round, which made a ten-round top-k the longest part of its kernel): inside each row of 16 lanes
// the pair is folded with its neighbour at distance 1, 2, then its mirror inside 8 and inside 16 lanes (after which
// every lane of a row holds the row's best); lane 15 of rows 0 and 2 is then broadcast into rows 1 and 3, lane 31
// into rows 2 and 3, so lane 63 ends with the wave's best, which a lane read hands to everybody.  A lane that a
// step does not write keeps its own pair, which never beats itself.  All 64 lanes must be active.
__device__ __forceinline__ void wave_best(float &v, int &i) {
  #define AMPH_DPP_STEP(CTRL, ROWS)                                                                              \
    {                                                                                                            \
      const int ovb = __builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, ROWS, 0xf, false); \
      const int oi = __builtin_amdgcn_update_dpp(i, i, CTRL, ROWS, 0xf, false);                                  \
      const float ov = __int_as_float(ovb);                                                                      \
      if (better(ov, oi, v, i)) { v = ov; i = oi; }                                                              \
    }
  AMPH_DPP_STEP(0xb1, 0xf)       // quad_perm [1, 0, 3, 2]
  AMPH_DPP_STEP(0x4e, 0xf)       // quad_perm [2, 3, 0, 1]
  AMPH_DPP_STEP(0x141, 0xf)      // row_half_mirror
  AMPH_DPP_STEP(0x140, 0xf)      // row_mirror
  AMPH_DPP_STEP(0x142, 0xa)      // row_bcast:15 into rows 1 and 3
  AMPH_DPP_STEP(0x143, 0xc)      // row_bcast:31 into rows 2 and 3
  #undef AMPH_DPP_STEP
  v = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
  i = __builtin_amdgcn_readlane(i, 63);
}

// Select k times from NPT per-lane (value, index) pairs spread over a wave.  Lane 0 writes the results.
template <int NPT>
__device__ __forceinline__ void wave_select(float (&x)[NPT], int (&id)[NPT], int k, int none, float *out_v, int *out_i) {
  const float NEG_INF = -__builtin_huge_valf();
  const int lane = threadIdx.x & 63;
  float bv = NEG_INF; int bi = none, bj = -1;
  #pragma unroll
  for (int j = 0; j < NPT; ++j)
    if (id[j] != none && better(x[j], id[j], bv, bi)) { bv = x[j]; bi = id[j]; bj = j; }
  for (int r = 0; r < k; ++r) {
    float wv = bv; int wi = bi;
    wave_best(wv, wi);
    if (lane == 0) { out_v[r] = wv; out_i[r] = (wi == none) ? -1 : wi; }
    if (wi != none && wi == bi) {              // this lane owned the winner: retire it and rescan
      bv = NEG_INF; bi = none;
      const int gone = bj; bj = -1;
      #pragma unroll
      for (int j = 0; j < NPT; ++j) {
        if (j == gone) id[j] = none;
        if (id[j] != none && better(x[j], id[j], bv, bi)) { bv = x[j]; bi = id[j]; bj = j; }
      }
    }
  }
}

}  // namespace amph
