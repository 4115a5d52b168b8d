// Tree-masked verification attention (Sec. 2 "Tree Attention"; Appendix "Draft Tree"): T tree
// queries of one head against the committed cache rows [0, L) and the tree's own rows [L, L+T),
// where query i sees tree row j only if node j is i or an ancestor of i.
//
// Everything runs on the matrix cores with operands taken straight from global memory:
//   S^T[key, q] = K[key, :] . Q[q, :]      A = 16 keys x 64 bytes of K rows, B = 16 queries of Q
//   O^T[d, q]  += V^T[d, keys] . P^T[keys, q]   A = 16 dims x the step's keys of V
// Both caches are stored step-tiled (layout in the header of the C ABI): each A fragment is one
// contiguous 1 KB piece, in the order the loop below asks for them.
// The 16 keys fed to one S^T tile are chosen so that the accumulator a lane ends up with (4 keys of
// its lane group per tile) is exactly the contraction-slot layout the second product expects from
// its B operand, so P never leaves registers.  A wave owns whole key steps (32 keys in bf16, 16 in
// float) for up to 32 queries; the four waves of a workgroup take different steps and merge their
// running (max, sum, O) through LDS; workgroups that split the keys of one head merge through global
// memory: a second small kernel (k_verify_fold) folds them in a fixed order, so no workgroup ever
// waits for or signals another.
#include "kernels.h"

namespace amph {

// 2^x through the hardware instruction alone: arguments here are <= 0 (or hugely negative for masked keys), so
// the library version's rescue of results below the normal range (four more instructions per call) buys nothing.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <typename T, int DH, int NQB>
struct VA {
  static constexpr int PER = Elem<T>::PER;
  static constexpr int KSTEP = 4 * PER;            // keys per step
  static constexpr int NT = KSTEP / 16;            // S^T tiles per step
  static constexpr int DSTEPS = DH / (4 * PER);    // 64-byte pieces of a K/Q row
  static constexpr int DB = DH / 16;               // 16-row blocks of O^T
  static constexpr int NQ = NQB * 16;              // queries per workgroup
  static constexpr int OPITCH = DH + 4;            // floats
  static constexpr int PART = NQ * DH + 2 * NQ;    // floats of one partial: O, then m, then l
};

template <typename T, int DH, int NQB>
__global__ __launch_bounds__(256) void k_verify_attn(const VerifyArgs a, int n_qg) {
  using C = VA<T, DH, NQB>;
  constexpr int PER = C::PER, KSTEP = C::KSTEP, NT = C::NT, DSTEPS = C::DSTEPS, DB = C::DB, NQ = C::NQ;
  __shared__ __align__(16) float sm_o[4][NQ][C::OPITCH];
  __shared__ float sm_m[4][NQ], sm_l[4][NQ];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 4, r16 = lane & 15;
  const int S = gridDim.x, split = blockIdx.x, h = blockIdx.y;
  const int b = blockIdx.z / n_qg, qg = blockIdx.z % n_qg;
  const int Tn = a.T, n_h = a.n_heads, max_kv = a.max_kv;
  int L = a.kv_len[b];
  const bool bad = (L < 0 || L + Tn > max_kv);
  if (bad) {                                         // whole workgroup leaves; nobody else waits for it
    if (tid == 0 && split == 0 && h == 0) atomicOr(a.dev_status, 2u);
    return;
  }
  const int n_keys = L + Tn;
  const int n_steps = (n_keys + KSTEP - 1) / KSTEP;
  const int st0 = (int)((long long)n_steps * split / S), st1 = (int)((long long)n_steps * (split + 1) / S);
  const float scale = 1.4426950408889634f * rsqrtf((float)DH);
  const float NEG_INF = -__builtin_huge_valf();

  const unsigned char *Kb = (const unsigned char *)((const T *)a.k_cache + ((size_t)b * n_h + h) * (size_t)max_kv * DH) + r16 * 64 + g * 16;
  const unsigned char *Vb = (const unsigned char *)((const T *)a.v_cache + ((size_t)b * n_h + h) * (size_t)DH * max_kv) + r16 * 64 + g * 16;
  const int q_base = qg * NQ;

  // queries as B fragments: lane = query r16 of block qb, 16 bytes of dims per 64-byte piece
  uint4 Qf[NQB][DSTEPS];
  uint64_t mk_lo[NQB], mk_hi[NQB];
  #pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int qi = q_base + qb * 16 + r16;
    #pragma unroll
    for (int ds = 0; ds < DSTEPS; ++ds) {      // padding queries re-read query 0; their rows are never stored
      const int qs = (qi < Tn) ? qi : 0;
      Qf[qb][ds] = ldg16((const T *)a.q + (((size_t)b * Tn + qs) * n_h + h) * DH + ds * (4 * PER) + g * PER);
    }
    mk_lo[qb] = (qi < Tn) ? a.mask_bits[(size_t)qi * 2] : 0ull;
    mk_hi[qb] = (qi < Tn) ? a.mask_bits[(size_t)qi * 2 + 1] : 0ull;
  }

  f32x4 O[NQB][DB];
  float m_run[NQB], l_run[NQB];
  #pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    m_run[qb] = NEG_BIG; l_run[qb] = 0.f;
    #pragma unroll
    for (int db = 0; db < DB; ++db) O[qb][db] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }

  // A wave's key steps are processed in groups of GS.  Pass 1 of a group computes all its scores (S^T tiles) and
  // keeps them in registers; the running maximum then moves once per group, so the accumulators are rescaled once
  // per group (never on the first one) instead of once per step, and one cross-lane maximum serves the whole group.
  // Pass 2 turns the scores into probabilities and adds V^T P^T.  K fragments are requested one step ahead, V
  // fragments one step ahead within pass 2 (two register sets each); every load is unconditional: steps past
  // the wave's last one re-read it and contribute nothing.
  constexpr int GS = 4;
  auto load_k = [&](int st, uint4 (&Kf)[NT][DSTEPS]) {
    // fragment (t, ds) of the step holds keys st*KSTEP + (i>>2)*(4*NT) + t*4 + (i&3) at slot i = lane & 15, so
    // that the S^T accumulators come out in the contraction-slot order of the second product
    #pragma unroll
    for (int t = 0; t < NT; ++t) {
      #pragma unroll
      for (int ds = 0; ds < DSTEPS; ++ds) Kf[t][ds] = ldg16(Kb + ((size_t)(st * NT + t) * DSTEPS + ds) * 1024);
    }
  };
  auto load_v = [&](int st, uint4 (&Vf)[DB]) {
    #pragma unroll
    for (int db = 0; db < DB; ++db) Vf[db] = ldg16(Vb + ((size_t)st * DB + db) * 1024);
  };
  // scores of one step for every query block of the wave, scaled, masked where the tree or the end of the cache says so
  auto scores = [&](int st, const uint4 (&Kf)[NT][DSTEPS], float (&sv)[NQB][PER], float (&mx)[NQB]) {
    const int key0 = st * KSTEP;
    const bool tail = (key0 + KSTEP > L);            // this step touches tree rows or rows past the end
    #pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      // lane gets keys key0 + g*PER + (t*4 + i), query r16
      #pragma unroll
      for (int t = 0; t < NT; ++t) {
        f32x4 sacc = (f32x4){0.f, 0.f, 0.f, 0.f};
        #pragma unroll
        for (int ds = 0; ds < DSTEPS; ++ds) sacc = mma16<T>(Kf[t][ds], Qf[qb][ds], sacc);
        #pragma unroll
        for (int i = 0; i < 4; ++i) sv[qb][t * 4 + i] = sacc[i] * scale;
      }
      if (tail) {
        const int qi = q_base + qb * 16 + r16;
        #pragma unroll
        for (int j = 0; j < PER; ++j) {
          const int key = key0 + g * PER + j;
          bool vis = key < L;
          if (!vis && key < n_keys) {
            const int bit = key - L;
            vis = ((bit < 64 ? (mk_lo[qb] >> bit) : (mk_hi[qb] >> (bit - 64))) & 1ull) != 0ull;
          }
          if (!vis || qi >= Tn) sv[qb][j] = NEG_INF;
        }
      }
      #pragma unroll
      for (int j = 0; j < PER; ++j) mx[qb] = fmaxf(mx[qb], sv[qb][j]);
    }
  };
  // probabilities of one step against the group's maximum, and O^T += V^T P^T
  auto accumulate = [&](int st, uint4 (&Vf)[DB], const float (&sv)[NQB][PER]) {
    const int key0 = st * KSTEP;
    if (key0 + KSTEP > n_keys) {
      // rows past L+T may hold anything (even NaN): zero their values so that 0 * V stays 0
      #pragma unroll
      for (int db = 0; db < DB; ++db) {
        float vv[PER];
        Elem<T>::unpack(Vf[db], vv);
        #pragma unroll
        for (int j = 0; j < PER; ++j) if (key0 + g * PER + j >= n_keys) vv[j] = 0.f;
        Vf[db] = pack16<T>(vv);
      }
    }
    #pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      float pv[PER], ls = 0.f;
      #pragma unroll
      for (int j = 0; j < PER; ++j) { pv[j] = fast_exp2(sv[qb][j] - m_run[qb]); ls += pv[j]; }
      l_run[qb] += ls;
      const uint4 Pf = pack16<T>(pv);
      #pragma unroll
      for (int db = 0; db < DB; ++db) O[qb][db] = mma16<T>(Vf[db], Pf, O[qb][db]);
    }
  };

  const int n_w = (st1 - (st0 + wave) + 3) / 4;        // key steps of this wave: st0 + wave, + 4, ...
  if (n_w > 0) {
    const int first = st0 + wave;
    auto step_of = [&](int i) { return first + 4 * min(i, n_w - 1); };
    uint4 KA[NT][DSTEPS], KB_[NT][DSTEPS], VA_[DB], VB_[DB];
    load_k(step_of(0), KA);
    for (int i0 = 0; i0 < n_w; i0 += GS) {
      float sv[GS][NQB][PER], mx[NQB];
      #pragma unroll
      for (int qb = 0; qb < NQB; ++qb) mx[qb] = NEG_INF;
      // ---- pass 1 (GS is even: step s of a group always finds its K fragments in the same register set)
      #pragma unroll
      for (int s = 0; s < GS; ++s) {
        if (s & 1) load_k(step_of(i0 + s + 1), KA); else load_k(step_of(i0 + s + 1), KB_);
        if (s == GS - 1) load_v(step_of(i0), VA_);
        if (i0 + s < n_w) {
          if (s & 1) scores(step_of(i0 + s), KB_, sv[s], mx); else scores(step_of(i0 + s), KA, sv[s], mx);
        }
      }
      // ---- the group's maximum per query; rescale what earlier groups accumulated
      #pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        float m2 = fmaxf(mx[qb], __shfl_xor(mx[qb], 16, WAVE));
        m2 = fmaxf(m2, __shfl_xor(m2, 32, WAVE));
        const float mn = fmaxf(m_run[qb], m2);
        if (i0 > 0) {
          const float corr = fast_exp2(m_run[qb] - mn);
          l_run[qb] *= corr;
          #pragma unroll
          for (int db = 0; db < DB; ++db) O[qb][db] *= corr;
        }
        m_run[qb] = mn;
      }
      // ---- pass 2
      #pragma unroll
      for (int s = 0; s < GS; ++s) {
        if (s + 1 < GS) { if (s & 1) load_v(step_of(i0 + s + 1), VA_); else load_v(step_of(i0 + s + 1), VB_); }
        if (i0 + s < n_w) {
          if (s & 1) accumulate(step_of(i0 + s), VB_, sv[s]); else accumulate(step_of(i0 + s), VA_, sv[s]);
        }
      }
    }
  }

  // ---- lane groups hold partial sums of l for the same query: fold them
  #pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    l_run[qb] += __shfl_xor(l_run[qb], 16, WAVE);
    l_run[qb] += __shfl_xor(l_run[qb], 32, WAVE);
  }

  // ---- waves -> workgroup through LDS
  #pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    if (g == 0) { sm_m[wave][qb * 16 + r16] = m_run[qb]; sm_l[wave][qb * 16 + r16] = l_run[qb]; }
    #pragma unroll
    for (int db = 0; db < DB; ++db)
      *reinterpret_cast<f32x4 *>(&sm_o[wave][qb * 16 + r16][db * 16 + g * 4]) = O[qb][db];
  }
  __syncthreads();

  float *part = a.partials + (((size_t)(b * n_qg + qg) * n_h + h) * S + split) * C::PART;
  T *outp = (T *)a.out;
  // thread handles 4 consecutive dims of one query per iteration
  for (int idx = tid; idx < NQ * (DH / 4); idx += 256) {
    const int q = idx / (DH / 4), d4 = (idx % (DH / 4)) * 4;
    const float mw = fmaxf(fmaxf(sm_m[0][q], sm_m[1][q]), fmaxf(sm_m[2][q], sm_m[3][q]));
    f32x4 o = (f32x4){0.f, 0.f, 0.f, 0.f};
    float l = 0.f;
    #pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float f = fast_exp2(sm_m[w][q] - mw);
      o += *reinterpret_cast<const f32x4 *>(&sm_o[w][q][d4]) * f;
      l += sm_l[w][q] * f;
    }
    const int qi = q_base + q;
    if (S == 1) {
      if (qi < Tn) {
        const float inv = (l > 0.f) ? 1.0f / l : 0.f;
        T *dst = outp + (((size_t)b * Tn + qi) * n_h + h) * DH + d4;
        #pragma unroll
        for (int i = 0; i < 4; ++i) dst[i] = Elem<T>::from_f32(o[i] * inv);
      }
    } else {
      *reinterpret_cast<f32x4 *>(part + (size_t)q * DH + d4) = o;
      if (d4 == 0) { part[NQ * DH + q] = mw; part[NQ * DH + NQ + q] = l; }
    }
  }
}

// Fold the S key-split partials of one (batch, query group, head): out = sum_s O_s 2^(m_s - m) / sum_s l_s 2^(m_s - m),
// s ascending.  grid = (heads, B * query groups), 256 threads, 4 dims of one query per thread and iteration.
template <typename T, int DH>
__global__ __launch_bounds__(256) void k_verify_fold(const VerifyArgs a, int n_qg, int nqb, int S) {
  constexpr int QW = 256 / (DH / 4);                    // queries per workgroup: one float4 of one query per thread
  const int NQ = nqb * 16, PART = NQ * DH + 2 * NQ;
  const int h = blockIdx.x, b = blockIdx.y / n_qg, qg = blockIdx.y % n_qg, tid = threadIdx.x;
  const int Tn = a.T, n_h = a.n_heads;
  const int L = a.kv_len[b];
  if (L < 0 || L + Tn > a.max_kv) return;               // the main kernel wrote nothing for this element
  const int q = blockIdx.z * QW + tid / (DH / 4), d4 = (tid % (DH / 4)) * 4;
  const int qi = qg * NQ + q;
  if (q >= NQ || qi >= Tn) return;
  const float *p0 = a.partials + ((size_t)(b * n_qg + qg) * n_h + h) * S * PART;
  float mt = NEG_BIG;
  for (int s = 0; s < S; ++s) mt = fmaxf(mt, p0[(size_t)s * PART + NQ * DH + q]);
  f32x4 o = (f32x4){0.f, 0.f, 0.f, 0.f};
  float l = 0.f;
  for (int s = 0; s < S; ++s) {
    const float *ps = p0 + (size_t)s * PART;
    const float f = exp2f(ps[NQ * DH + q] - mt);
    o += *reinterpret_cast<const f32x4 *>(ps + (size_t)q * DH + d4) * f;
    l += ps[NQ * DH + NQ + q] * f;
  }
  const float inv = (l > 0.f) ? 1.0f / l : 0.f;
  float r[4] = {o[0] * inv, o[1] * inv, o[2] * inv, o[3] * inv};
  T *dst = (T *)a.out + (((size_t)b * Tn + qi) * n_h + h) * DH + d4;
  #pragma unroll
  for (int i = 0; i < 4; ++i) dst[i] = Elem<T>::from_f32(r[i]);
}

// queries per workgroup: as few 16-query blocks per wave as cover T in ceil(T/64) groups
// Queries per workgroup: at most two 16-query blocks per wave.  Larger blocks per wave would save K/V
// re-reads (they come from L2) but need more registers than leave room for a second set of K/V fragments.
constexpr int VA_MAX_QB = 2;
static inline void va_groups(int T, int *nqb, int *n_qg) {
  const int blocks = (T + 15) / 16;
  *n_qg = (blocks + VA_MAX_QB - 1) / VA_MAX_QB;
  *nqb = (blocks + *n_qg - 1) / *n_qg;
}

int verify_splits(int B, int T, int n_heads, int max_kv, int elem_bytes) {
  int nqb, n_qg;
  va_groups(T, &nqb, &n_qg);
  const int kstep = 4 * (16 / elem_bytes);
  const int max_steps = max_kv / kstep;
  int s = 256 / (B * n_qg * n_heads);
  const int cap = (max_steps + 3) / 4;        // at least one step per wave
  if (s > cap) s = cap;
  if (s > 32) s = 32;
  return s < 1 ? 1 : s;
}

size_t verify_ws_floats(int B, int T, int n_heads, int d_h, int max_kv, int elem_bytes) {
  int nqb, n_qg;
  va_groups(T, &nqb, &n_qg);
  const size_t part = (size_t)nqb * 16 * d_h + 2 * nqb * 16;
  return (size_t)B * n_qg * n_heads * verify_splits(B, T, n_heads, max_kv, elem_bytes) * part;
}

template <typename T, int DH>
static hipError_t launch_va_dh(hipStream_t st, const VerifyArgs &a) {
  int nqb, n_qg;
  va_groups(a.T, &nqb, &n_qg);
  const int S = verify_splits(a.B, a.T, a.n_heads, a.max_kv, (int)sizeof(T));
  const dim3 grid(S, a.n_heads, a.B * n_qg), block(256);
  switch (nqb) {
    case 1: hipLaunchKernelGGL((k_verify_attn<T, DH, 1>), grid, block, 0, st, a, n_qg); break;
    case 2: hipLaunchKernelGGL((k_verify_attn<T, DH, 2>), grid, block, 0, st, a, n_qg); break;
    default: return hipErrorInvalidValue;
  }
  if (S > 1) {
    constexpr int QW = 256 / (DH / 4);
    hipLaunchKernelGGL((k_verify_fold<T, DH>), dim3(a.n_heads, a.B * n_qg, (nqb * 16 + QW - 1) / QW), block, 0, st, a, n_qg, nqb, S);
  }
  return hipGetLastError();
}

template <typename T>
hipError_t launch_verify_attn(hipStream_t st, const VerifyArgs &a) {
  if (a.T < 1 || a.T > AMPH_MAX_TREE || a.max_kv % 32) return hipErrorInvalidValue;
  if (verify_ws_floats(a.B, a.T, a.n_heads, a.d_h, a.max_kv, (int)sizeof(T)) > a.partials_cap) return hipErrorInvalidValue;
  if (a.d_h == 64) return launch_va_dh<T, 64>(st, a);
  if (a.d_h == 128) return launch_va_dh<T, 128>(st, a);
  return hipErrorInvalidValue;
}
template hipError_t launch_verify_attn<float>(hipStream_t, const VerifyArgs &);
template hipError_t launch_verify_attn<bf16_t>(hipStream_t, const VerifyArgs &);

}  // namespace amph
