// Tree-masked verification attention (Sec. 2 "Tree Attention"; Appendix "Draft Tree"): T tree
// queries of one head against the committed cache rows [0, L) and the tree's own rows [L, L+T),
// where query i sees tree row j only if node j is i or an ancestor of i.
//
// Everything runs on the matrix cores:
//   S^T[key, q] = K[key, :] . Q[q, :]      A = 16 keys x 64 bytes of K rows, B = 16 queries of Q
//   O^T[d, q]  += V^T[d, keys] . P^T[keys, q]   A = 16 dims x the step's keys of V
// Both caches are stored step-tiled (layout in the header of the C ABI): each A fragment is one
// contiguous 1 KB piece and the fragments of one key step (32 keys in bf16, 16 in float) are adjacent.
// The 16 keys fed to one S^T tile are chosen so that the accumulator a lane ends up with (4 keys of
// its lane group per tile) is exactly the contraction-slot layout the second product expects from
// its B operand, so P never leaves registers.
//
// Two kernels share this arithmetic and differ in how the fragments reach the matrix cores:
//
// k_verify_attn_regs (short key ranges: few steps per wave, fixed costs dominate).  Operands go from
// global memory straight to registers.  A wave owns whole key steps for up to 32 queries; the four waves of a
// workgroup take different steps and merge their running (max, sum, O) through LDS.
//
// k_verify_attn_ring (long key ranges: one workgroup streams all keys of a (batch element, head)).  Two loader
// waves stream the fragments from global memory straight into a ring of LDS stages without passing through
// registers; each math wave owns 16 queries (up to eight waves) for the whole range, reads the fragments of its
// key steps from LDS (lane-linear, free of bank conflicts) and keeps its running (max, sum, O) in registers: the
// keys are read once per workgroup instead of once per 32 queries.  One barrier per stage hands a landed stage to
// the math waves and a consumed one back to the loaders.  On long walks two groups of math waves share every
// query block (a stage then holds one key step for each group) and merge their states through LDS once at the
// end.  Measured at 52 heads, T = 96, batch 4, L = 4096: 89 us against 167 us; at 32 heads, T = 64,
// batch 1, L = 1024: 17.0 us against 15.4 us, hence the other kernel there.
//
// Workgroups that split the keys of one head merge through global memory: a second small kernel
// (k_verify_fold) folds them in a fixed order, so no workgroup ever waits for or signals another.
#include "kernels.h"

namespace amph {

// 2^x through the hardware instruction alone: arguments here are <= 0 (or hugely negative for masked keys), so
// the library version's rescue of results below the normal range (four more instructions per call) buys nothing.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// =====================================================================================================
// operands through registers
// =====================================================================================================
template <typename T, int DH, int NQB>
struct VAR {
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
__global__ __launch_bounds__(256) void k_verify_attn_regs(const VerifyArgs a, int n_qg) {
  using C = VAR<T, DH, NQB>;
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
  // (32-bit: key steps x splits stay far below 2^31; a 64-bit division costs a few hundred instructions up front)
  const int st0 = (int)((unsigned)(n_steps * split) / (unsigned)S), st1 = (int)((unsigned)(n_steps * (split + 1)) / (unsigned)S);
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
        T *dst = a.out_tiles ? outp + xt_index<T>(b * Tn + qi, h * DH + d4, a.out_tiles)
                             : outp + (((size_t)b * Tn + qi) * n_h + h) * DH + d4;
        #pragma unroll
        for (int i = 0; i < 4; ++i) dst[i] = Elem<T>::from_f32(o[i] * inv);
      }
    } else {
      *reinterpret_cast<f32x4 *>(part + (size_t)q * DH + d4) = o;
      if (d4 == 0) { part[NQ * DH + q] = mw; part[NQ * DH + NQ + q] = l; }
    }
  }
}

// =====================================================================================================
// operands through an LDS ring
// =====================================================================================================
template <typename T, int DH, int KG = 1>
struct VA {
  static constexpr int PER = Elem<T>::PER;
  static constexpr int KSTEP = 4 * PER;            // keys per step
  static constexpr int NT = KSTEP / 16;            // S^T tiles per step
  static constexpr int DSTEPS = DH / (4 * PER);    // 64-byte pieces of a K/Q row
  static constexpr int DB = DH / 16;               // 16-row blocks of O^T
  static constexpr int FK = NT * DSTEPS;           // K fragments of a step
  static constexpr int FR = FK + DB;               // fragments (KB) of a step: its K, then its V
  static constexpr int STEPB = FR * 1024;          // bytes of a step
  static constexpr int NS = KG;                    // key steps per ring stage: one per key group of math waves
  static constexpr int STAGE = NS * STEPB;
  static constexpr int NL = 2;                     // loader waves
  static constexpr int PERL = NS * FR / NL;        // loads per loader wave and stage
  static constexpr int R = 4;                      // stages in the ring (8 measured no faster)
  static_assert(FK % NL == 0 && FR % NL == 0, "a loader wave's j-th fragment must be K or V for both waves alike");
  static_assert(PERL * (R - 2) <= 63, "outstanding loads of a loader wave must fit the hardware counter");
};
constexpr int VA_MAX_MATH = 8;                     // math waves per workgroup: 16 queries each covers the largest tree

// Waits until at most N vector-memory operations of this wave are outstanding (they complete in order).
template <int N> __device__ __forceinline__ void wait_vm() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0f70);
}
// at most k whole stages of this loader wave's loads may still be in flight
template <int PERL> __device__ __forceinline__ void wait_stages(int k) {
  switch (k) {
    case 0: wait_vm<0>(); break;
    case 1: wait_vm<PERL>(); break;
    default: wait_vm<2 * PERL>(); break;
  }
}
template <int N> struct IntTag { static constexpr int value = N; };

// grid = (key splits, heads, batch); block = (math waves + 2 loader waves) * 64; dynamic LDS = R stages.
// KG = 2: two groups of math waves share every query block, one taking the even key steps and one the odd ones
// (a stage holds one step for each), and merge their running states through LDS at the end; this doubles the
// waves that hide each other's exponentials and LDS reads when one workgroup walks a long cache on its own.
template <typename T, int DH, int NQB, int KG>
__global__ __launch_bounds__(KG == 2 ? 1024 : (VA_MAX_MATH + 2) * 64) void k_verify_attn_ring(const VerifyArgs a) {
  using C = VA<T, DH, KG>;
  constexpr int PER = C::PER, KSTEP = C::KSTEP, NT = C::NT, DSTEPS = C::DSTEPS, DB = C::DB, FK = C::FK, FR = C::FR;
  constexpr int STEPB = C::STEPB, NS = C::NS, STAGE = C::STAGE, NL = C::NL, PERL = C::PERL, R = C::R;
  extern __shared__ __align__(16) unsigned char sm_ring[];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 4, r16 = lane & 15;
  const int nm = (int)(blockDim.x >> 6) - NL;        // math waves: KG key groups of nmq waves
  const int nmq = nm / KG;
  const int S = gridDim.x, split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int Tn = a.T, n_h = a.n_heads, max_kv = a.max_kv;
  const int L = a.kv_len[b];
  if (L < 0 || L + Tn > max_kv) {                    // whole workgroup leaves before any barrier; nobody else waits for it
    if (tid == 0 && split == 0 && h == 0) atomicOr(a.dev_status, 2u);
    return;
  }
  const int n_keys = L + Tn;
  const int n_steps = (n_keys + KSTEP - 1) / KSTEP;
  // (32-bit: key steps x splits stay far below 2^31; a 64-bit division costs a few hundred instructions up front)
  const int st0 = (int)((unsigned)(n_steps * split) / (unsigned)S), st1 = (int)((unsigned)(n_steps * (split + 1)) / (unsigned)S);
  const int n = st1 - st0;                           // key steps of this workgroup; may be 0
  const int n_stages = (n + NS - 1) / NS;            // ring stages: NS steps each, the last one possibly ragged
  const size_t head_bytes = ((size_t)b * n_h + h) * (size_t)max_kv * DH * sizeof(T);

  if (wave >= nm) {
    // ---------------- loader wave: fragments w, w + 2, ... of every step of every stage ----------------
    // A lane fetches the 16 bytes its counterpart in a math wave feeds to the matrix core (row r16 of the
    // fragment, piece g); they land in LDS at lane * 16, where the math lane reads them back.  A ragged last
    // stage loads its last step again (never used), so every stage counts the same number of loads.
    const int w = wave - nm;
    const unsigned char *Kg = (const unsigned char *)a.k_cache + head_bytes + r16 * 64 + g * 16;
    const unsigned char *Vg = (const unsigned char *)a.v_cache + head_bytes + r16 * 64 + g * 16;
    auto issue = [&](int p) {
      #pragma unroll
      for (int s = 0; s < NS; ++s) {
        const int rel = (p * NS + s < n) ? p * NS + s : n - 1;
        const size_t st = (size_t)(st0 + rel);
        unsigned char *lp = sm_ring + (p % R) * STAGE + s * STEPB;
        #pragma unroll
        for (int j = 0; j < FR / NL; ++j) {
          const int f = w + j * NL;
          const unsigned char *src = (j * NL < FK) ? Kg + (st * FK + f) * 1024 : Vg + (st * DB + (f - FK)) * 1024;
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                           (__attribute__((address_space(3))) void *)(lp + f * 1024), 16, 0, 0);
        }
      }
    };
    const int pro = n_stages < R - 1 ? n_stages : R - 1;
    for (int p = 0; p < pro; ++p) issue(p);
    for (int p = 0; p < n_stages; ++p) {
      const int newest = (p + R - 2 < n_stages - 1) ? p + R - 2 : n_stages - 1;    // newest stage issued so far
      wait_stages<PERL>(newest - p);                 // stage p has landed
      __builtin_amdgcn_s_barrier();                  // math waves may read stage p; they are done with stage p - 1
      if (p + R - 1 < n_stages) issue(p + R - 1);    // into the slot of stage p - 1
    }
    if (KG == 2) {                                   // the two barriers of the key groups' merge
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_s_barrier();
    }
    return;
  }

  // ---------------- math wave: queries [q0, q0 + 16 * NQB) against all stages ----------------
  const float scale = 1.4426950408889634f * rsqrtf((float)DH);
  const float NEG_INF = -__builtin_huge_valf();
  const int kg = wave / nmq;                         // this wave's key group: step kg of every stage
  const int q0 = (wave - kg * nmq) * NQB * 16;

  // queries as B fragments: lane = query r16 of block qb, 16 bytes of dims per 64-byte piece
  uint4 Qf[NQB][DSTEPS];
  uint64_t mk_lo[NQB], mk_hi[NQB];
  #pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int qi = q0 + qb * 16 + r16;
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

  // NSL consecutive key steps (first key key0) whose fragments start at sb: their scores together, one move of the
  // running maximum, then their probabilities and values.  Independent steps give the matrix cores and the LDS
  // reads something to overlap with the exponentials.
  auto process = [&](auto tag, const unsigned char *sb, int key0) {
    constexpr int NSL = decltype(tag)::value;
    // ---- scores: fragment (t, ds) holds keys step0 + (slot >> 2) * (4 * NT) + t * 4 + (slot & 3) at slot = lane & 15,
    // so the S^T accumulators come out in the contraction-slot order of the second product:
    // the lane gets keys step0 + g * PER + (t * 4 + c), query r16
    f32x4 sacc[NSL][NQB][NT];
    #pragma unroll
    for (int s = 0; s < NSL; ++s)
      #pragma unroll
      for (int qb = 0; qb < NQB; ++qb)
        #pragma unroll
        for (int t = 0; t < NT; ++t) sacc[s][qb][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    #pragma unroll
    for (int s = 0; s < NSL; ++s)
      #pragma unroll
      for (int t = 0; t < NT; ++t)
        #pragma unroll
        for (int ds = 0; ds < DSTEPS; ++ds) {
          const uint4 Kf = *reinterpret_cast<const uint4 *>(sb + s * STEPB + (t * DSTEPS + ds) * 1024);
          #pragma unroll
          for (int qb = 0; qb < NQB; ++qb) sacc[s][qb][t] = mma16<T>(Kf, Qf[qb][ds], sacc[s][qb][t]);
        }
    float sv[NSL][NQB][PER], mn[NQB];
    bool grow = false;
    #pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      float mx = NEG_INF;
      #pragma unroll
      for (int s = 0; s < NSL; ++s) {
        #pragma unroll
        for (int t = 0; t < NT; ++t)
          #pragma unroll
          for (int c = 0; c < 4; ++c) sv[s][qb][t * 4 + c] = sacc[s][qb][t][c] * scale;
        const int k0 = key0 + s * KSTEP;
        if (k0 + KSTEP > L) {                          // this step touches tree rows or rows past the end
          const int qi = q0 + qb * 16 + r16;
          #pragma unroll
          for (int j = 0; j < PER; ++j) {
            const int key = k0 + g * PER + j;
            bool vis = key < L;
            if (!vis && key < n_keys) {
              const int bit = key - L;
              vis = ((bit < 64 ? (mk_lo[qb] >> bit) : (mk_hi[qb] >> (bit - 64))) & 1ull) != 0ull;
            }
            if (!vis || qi >= Tn) sv[s][qb][j] = NEG_INF;
          }
        }
        #pragma unroll
        for (int j = 0; j < PER; ++j) mx = fmaxf(mx, sv[s][qb][j]);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 16, WAVE));
      mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE));
      mn[qb] = fmaxf(m_run[qb], mx);
      grow |= (mn[qb] > m_run[qb]);
    }
    // ---- the running maximum rarely moves after the first steps: rescale only when some query's did
    if (__any(grow)) {
      #pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        const float corr = fast_exp2(m_run[qb] - mn[qb]);
        l_run[qb] *= corr;
        #pragma unroll
        for (int db = 0; db < DB; ++db) O[qb][db] *= corr;
        m_run[qb] = mn[qb];
      }
    }
    // ---- probabilities, and O^T += V^T P^T
    uint4 Pf[NSL][NQB];
    #pragma unroll
    for (int s = 0; s < NSL; ++s)
      #pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        float pv[PER], ls = 0.f;
        #pragma unroll
        for (int j = 0; j < PER; ++j) { pv[j] = fast_exp2(sv[s][qb][j] - m_run[qb]); ls += pv[j]; }
        l_run[qb] += ls;
        Pf[s][qb] = pack16<T>(pv);
      }
    #pragma unroll
    for (int s = 0; s < NSL; ++s) {
      const int k0 = key0 + s * KSTEP;
      const bool ragged = (k0 + KSTEP > n_keys);
      #pragma unroll
      for (int db = 0; db < DB; ++db) {
        uint4 Vf = *reinterpret_cast<const uint4 *>(sb + s * STEPB + (FK + db) * 1024);
        if (ragged) {
          // rows past L+T may hold anything (even NaN): zero their values so that 0 * V stays 0
          float vv[PER];
          Elem<T>::unpack(Vf, vv);
          #pragma unroll
          for (int j = 0; j < PER; ++j) if (k0 + g * PER + j >= n_keys) vv[j] = 0.f;
          Vf = pack16<T>(vv);
        }
        #pragma unroll
        for (int qb = 0; qb < NQB; ++qb) O[qb][db] = mma16<T>(Vf, Pf[s][qb], O[qb][db]);
      }
    }
  };

  for (int p = 0; p < n_stages; ++p) {
    __syncthreads();                                   // stage p is in LDS (pairs with the loaders' barrier)
    const unsigned char *sb = sm_ring + (p % R) * STAGE + lane * 16;
    if (p * KG + kg < n) process(IntTag<1>{}, sb + kg * STEPB, (st0 + p * KG + kg) * KSTEP);   // a ragged last stage has one live step
  }

  if (KG == 2) {
    static_assert(KG == 1 || 7 * NQB * (DB * 256 + 128) * 4 <= R * STAGE, "merge area of seven query waves must fit the ring");
    // ---- the second key group hands its state over through LDS (the ring is free once everyone has passed the
    // first barrier), the first one merges it into its own and writes the result
    float *mo = reinterpret_cast<float *>(sm_ring) + (size_t)(wave - kg * nmq) * NQB * (DB * 256 + 128);
    __syncthreads();
    if (kg == 1) {
      #pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        #pragma unroll
        for (int db = 0; db < DB; ++db) *reinterpret_cast<f32x4 *>(mo + (qb * DB + db) * 256 + lane * 4) = O[qb][db];
        mo[NQB * DB * 256 + qb * 128 + lane] = m_run[qb];
        mo[NQB * DB * 256 + qb * 128 + 64 + lane] = l_run[qb];
      }
    }
    __syncthreads();
    if (kg == 1) return;
    #pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const float m1 = mo[NQB * DB * 256 + qb * 128 + lane], l1 = mo[NQB * DB * 256 + qb * 128 + 64 + lane];
      const float mn = fmaxf(m_run[qb], m1);
      const float c0 = fast_exp2(m_run[qb] - mn), c1 = fast_exp2(m1 - mn);
      #pragma unroll
      for (int db = 0; db < DB; ++db)
        O[qb][db] = O[qb][db] * c0 + *reinterpret_cast<const f32x4 *>(mo + (qb * DB + db) * 256 + lane * 4) * c1;
      l_run[qb] = l_run[qb] * c0 + l1 * c1;
      m_run[qb] = mn;
    }
  }

  // ---- lane groups hold partial sums of l for the same query: fold them; then the lane writes dims
  // db * 16 + g * 4 .. + 3 of query r16 of each of its blocks
  const int NQ = nmq * NQB * 16;                       // query rows of a partial
  float *part = a.partials + ((((size_t)b * n_h + h) * S + split) * (size_t)(NQ * DH + 2 * NQ));
  #pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    float l = l_run[qb];
    l += __shfl_xor(l, 16, WAVE);
    l += __shfl_xor(l, 32, WAVE);
    const int q = q0 + qb * 16 + r16;
    if (S == 1) {
      if (q < Tn) {
        const float inv = (l > 0.f) ? 1.0f / l : 0.f;
        #pragma unroll
        for (int db = 0; db < DB; ++db) {
          const float r[4] = {O[qb][db][0] * inv, O[qb][db][1] * inv, O[qb][db][2] * inv, O[qb][db][3] * inv};
          T *dst = a.out_tiles ? (T *)a.out + xt_index<T>(b * Tn + q, h * DH + db * 16 + g * 4, a.out_tiles)
                               : (T *)a.out + (((size_t)b * Tn + q) * n_h + h) * DH + db * 16 + g * 4;
          store4<T>(dst, r);
        }
      }
    } else {
      #pragma unroll
      for (int db = 0; db < DB; ++db) *reinterpret_cast<f32x4 *>(part + (size_t)q * DH + db * 16 + g * 4) = O[qb][db];
      if (g == 0) { part[NQ * DH + q] = m_run[qb]; part[NQ * DH + NQ + q] = l; }
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
  const int q = blockIdx.z * QW + tid / (DH / 4), d4 = (tid % (DH / 4)) * 4;
  const int qi = qg * NQ + q;
  const bool dead = (q >= NQ || qi >= Tn);
  const int qc = dead ? 0 : q;                          // (dead threads read query 0's partials and store nothing)
  const float *p0 = a.partials + ((size_t)(b * n_qg + qg) * n_h + h) * S * PART;
  // The kernel is a chain of memory round trips and little else, so everything a thread needs is requested before
  // anything is looked at: the committed length and, four splits at a time, each split's maximum, sum and four
  // dims (splits past the last re-read it and are left out).  The splits are merged in ascending order.
  const int L = a.kv_len[b];
  constexpr int FU = 4;
  float mt = NEG_BIG, l = 0.f;
  f32x4 o = (f32x4){0.f, 0.f, 0.f, 0.f};
  for (int s0 = 0; s0 < S; s0 += FU) {
    float ms[FU], ls[FU];
    f32x4 os[FU];
    #pragma unroll
    for (int u = 0; u < FU; ++u) {
      const float *ps = p0 + (size_t)min(s0 + u, S - 1) * PART;
      ms[u] = ps[NQ * DH + qc];
      ls[u] = ps[NQ * DH + NQ + qc];
      os[u] = *reinterpret_cast<const f32x4 *>(ps + (size_t)qc * DH + d4);
    }
    float mb = mt;
    #pragma unroll
    for (int u = 0; u < FU; ++u) if (s0 + u < S) mb = fmaxf(mb, ms[u]);
    const float f0 = exp2f(mt - mb);
    o *= f0; l *= f0;
    #pragma unroll
    for (int u = 0; u < FU; ++u) {
      if (s0 + u < S) {
        const float f = exp2f(ms[u] - mb);
        o += os[u] * f;
        l += ls[u] * f;
      }
    }
    mt = mb;
  }
  if (L < 0 || L + Tn > a.max_kv) return;               // the main kernel wrote nothing for this element
  if (dead) return;
  const float inv = (l > 0.f) ? 1.0f / l : 0.f;
  float r[4] = {o[0] * inv, o[1] * inv, o[2] * inv, o[3] * inv};
  T *dst = a.out_tiles ? (T *)a.out + xt_index<T>(b * Tn + qi, h * DH + d4, a.out_tiles)
                       : (T *)a.out + (((size_t)b * Tn + qi) * n_h + h) * DH + d4;
  #pragma unroll
  for (int i = 0; i < 4; ++i) dst[i] = Elem<T>::from_f32(r[i]);
}

// =====================================================================================================
// launch plan
// =====================================================================================================
struct VaPlan {
  bool ring;        // which kernel
  int S;            // key splits
  int nqb;          // 16-query blocks per wave
  int groups;       // regs: query groups (workgroups per head and split); ring: 1
  int nm;           // ring: math waves per key group
  int kg;           // ring: key groups of math waves (1 or 2)
  int nq;           // query rows of one partial
};
constexpr int VA_MAX_QB = 2;       // regs: more blocks per wave would leave no room for a second set of K/V fragments

// force: -1 chooses by shape, 0 = registers, 1 = LDS ring
static VaPlan va_plan(int B, int T, int n_heads, int max_kv, int elem_bytes, int force) {
  VaPlan p{};
  const int kstep = 4 * (16 / elem_bytes);
  const int max_steps = max_kv / kstep;
  // regs: at most two blocks per wave, as few query groups as cover T; enough splits for every compute unit,
  // at least one step per wave
  const int blocks = (T + 15) / 16;
  const int n_qg = (blocks + VA_MAX_QB - 1) / VA_MAX_QB;
  int s = 256 / (B * n_qg * n_heads);
  const int cap = (max_steps + 3) / 4;
  if (s > cap) s = cap;
  if (s > 32) s = 32;
  if (s < 1) s = 1;
  // ring: when a workgroup walks a whole head anyway (no room for key splits) and the walk is long, or when the
  // register kernel would need more workgroups than there are compute units (measured: 32 heads, T = 64, L = 1024:
  // batch 1 15.4 us regs / 17.3 ring, batch 4 21.1 / 23.2, batch 8 40.6 / 31.0; 40 heads, L = 2048, batch 4: 57.8 / 46.4)
  const bool ring = (force < 0) ? ((B * n_qg * n_heads > 256) || (s == 1 && max_steps >= 64)) : (force == 1);
  p.ring = ring;
  if (ring) {
    p.nqb = 1;                                         // 16 queries per math wave cover the largest tree
    p.nm = (T + 16 * p.nqb - 1) / (16 * p.nqb);
    p.groups = 1;
    int sr = 256 / (B * n_heads);                      // never more workgroups than compute units: a second round costs more
    if (sr > max_steps / 2) sr = max_steps / 2;
    if (sr > 32) sr = 32;
    p.S = sr < 1 ? 1 : sr;
    p.nq = p.nm * p.nqb * 16;
    // two key groups pay when a workgroup walks many steps (measured, ring kernel alone, one / two groups:
    // 52 heads, T = 96, L = 4096: batch 4 109.3 / 89.4 us, batch 1 37.3 / 33.4; 40 heads, T = 64, L = 2048, batch 4:
    // 47.5 / 35.4; 32 heads, T = 64, L = 4096: batch 8 102.2 / 96.7, batch 1 (16 steps per workgroup) 25.7 / 26.5)
    const bool fits = p.nqb == 1 && (2 * p.nm + 2) * 64 <= 1024;
    p.kg = (fits && (p.S == 1 || max_steps / p.S >= 32)) ? 2 : 1;
  } else {
    p.groups = n_qg;
    p.nqb = (blocks + n_qg - 1) / n_qg;
    p.S = s;
    p.nm = 4;
    p.nq = p.nqb * 16;
  }
  return p;
}

// floats of key-split partials a plan writes: none without key splits (the kernels then write the output directly)
static size_t va_plan_floats(const VaPlan &p, int B, int n_heads, int d_h) {
  if (p.S <= 1) return 0;
  return (size_t)B * p.groups * n_heads * p.S * ((size_t)p.nq * d_h + 2 * p.nq);
}

size_t verify_partials_floats(int B, int T, int n_heads, int d_h, int max_kv, int elem_bytes, int kernel) {
  return va_plan_floats(va_plan(B, T, n_heads, max_kv, elem_bytes, kernel), B, n_heads, d_h);
}

// partial results of the larger of the two kernels' plans: the choice may be overridden per call
size_t verify_ws_floats(int B, int T, int n_heads, int d_h, int max_kv, int elem_bytes) {
  const size_t a = va_plan_floats(va_plan(B, T, n_heads, max_kv, elem_bytes, 0), B, n_heads, d_h);
  const size_t b = va_plan_floats(va_plan(B, T, n_heads, max_kv, elem_bytes, 1), B, n_heads, d_h);
  return a > b ? a : b;
}

template <typename T, int DH, int NQB, int KG>
static hipError_t launch_va_ring(hipStream_t st, const VerifyArgs &a, const VaPlan &p) {
  using C = VA<T, DH, KG>;
  constexpr size_t smem = (size_t)C::R * C::STAGE;
  static bool attr_set = false;                       // once per instantiation and process
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void *)k_verify_attn_ring<T, DH, NQB, KG>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((k_verify_attn_ring<T, DH, NQB, KG>), dim3(p.S, a.n_heads, a.B), dim3((p.nm * KG + C::NL) * 64), smem, st, a);
  return hipGetLastError();
}

template <typename T, int DH>
static hipError_t launch_va_dh(hipStream_t st, const VerifyArgs &a) {
  const VaPlan p = va_plan(a.B, a.T, a.n_heads, a.max_kv, (int)sizeof(T), a.kernel);
  if (p.nqb < 1 || p.nqb > 2) return hipErrorInvalidValue;
  if (va_plan_floats(p, a.B, a.n_heads, DH) > a.partials_cap) return hipErrorInvalidValue;
  if (p.ring) {
    if (p.nm < 1 || p.nm > VA_MAX_MATH) return hipErrorInvalidValue;
    if (p.nqb != 1 || (p.kg == 2 && (2 * p.nm + 2) * 64 > 1024)) return hipErrorInvalidValue;
    hipError_t e = (p.kg == 2) ? launch_va_ring<T, DH, 1, 2>(st, a, p) : launch_va_ring<T, DH, 1, 1>(st, a, p);
    if (e != hipSuccess) return e;
  } else {
    const dim3 grid(p.S, a.n_heads, a.B * p.groups), block(256);
    if (p.nqb == 1) hipLaunchKernelGGL((k_verify_attn_regs<T, DH, 1>), grid, block, 0, st, a, p.groups);
    else hipLaunchKernelGGL((k_verify_attn_regs<T, DH, 2>), grid, block, 0, st, a, p.groups);
  }
  if (p.S > 1) {
    constexpr int QW = 256 / (DH / 4);
    hipLaunchKernelGGL((k_verify_fold<T, DH>), dim3(a.n_heads, a.B * p.groups, (p.nq + QW - 1) / QW), dim3(256), 0, st, a, p.groups,
                       p.nq / 16, p.S);
  }
  return hipGetLastError();
}

template <typename T>
hipError_t launch_verify_attn(hipStream_t st, const VerifyArgs &a) {
  if (a.T < 1 || a.T > AMPH_MAX_TREE || a.max_kv % 32 || a.kernel < -1 || a.kernel > 1 || a.out_tiles < 0) return hipErrorInvalidValue;
  if (a.d_h == 64) return launch_va_dh<T, 64>(st, a);
  if (a.d_h == 128) return launch_va_dh<T, 128>(st, a);
  return hipErrorInvalidValue;
}
template hipError_t launch_verify_attn<float>(hipStream_t, const VerifyArgs &);
template hipError_t launch_verify_attn<bf16_t>(hipStream_t, const VerifyArgs &);

}  // namespace amph
