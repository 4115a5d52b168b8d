// GEMMs of the target's forward pass over the tree tokens (Sec. 2 "Tree Attention"): M = B*T activation rows
// against [N, Kd] weights that stream from HBM once, on the matrix cores.  Two kernels: the skinny one
// (described first; up to two blocks of 64 rows) and the wide one (further down; three blocks or more).
//
// The unit of work is a ROW BLOCK: 16 weight rows that one wave keeps as matrix-core A fragments and
// whose outputs need nothing from any other block:
//   * plain / LM head: rows 16b .. 16b+15;
//   * q and k: 8 rows of a head and their 8 RoPE partners (i, i + d_h/2); v: 16 consecutive rows
//     (blocks numbered q, then k, then v);
//   * gate/up: rows 8b .. 8b+7 of W_gate and the same rows of W_up.
// A workgroup owns nb consecutive blocks (a 64 x 16*nb output tile) and a slice of the reduction axis,
// and its waves have two roles:
//   * nb math waves, one block each.  Their A fragments are 16-byte loads straight from global memory,
//     requested one 512-byte chunk (8 fragments) ahead; B fragments come from LDS.  They issue nothing
//     else, so waiting for a chunk of weights never waits for anything younger.
//   * 4 loader waves, which bring the activations of each chunk (64 rows x 512 bytes, L2 hits) into a
//     padded, double-buffered LDS tile one chunk ahead.
// One barrier per chunk joins the two.  nb (2..12) and the split of the reduction axis are chosen per
// shape by gemm_plan: every workgroup reads the whole activation slice from L2, so that traffic is
// (64 / tile height) times the weight bytes and measurably slows the weight stream; taller tiles cut
// it as far as filling the 256 CUs in whole rounds allows.
//
// Weight layouts.  Row-major [N, Kd] works, but a matrix-core A fragment is 16 rows x 64 bytes, so
// every wave load touches 16 half cache lines; the vector L1 handles such loads at about a quarter of
// the rate of a contiguous 1 KB load and the weight stream then stalls on the CU side, not on HBM
// (measured: 41 us against 33 us for the gate/up shape).  The tiled layout (k_pack_weights, run once
// per matrix) stores every fragment as one contiguous 1 KB piece, block-major:
//   tiled[(block * (Kd * sizeof(T) / 64) + step) * 1024 + r * 64 + byte]  =  W[row(block, r)][step * 64 + byte]
// with rows past N stored as zeros.
//
// No workgroup ever communicates with another inside the kernel (a device-scope fence per workgroup
// costs far more than the kernel on this chip): a split reduction axis writes one partial slab per
// split, which the consumer (the RMSNorm kernel of the next sub-layer, or k_sum_slabs) adds up in a
// fixed order; per-tile argmax candidates are folded by k_argmax_fold.  Fused epilogues: RoPE from a
// precomputed table + KV-cache write, SwiGLU, per-tile row argmax.
#include "kernels.h"
#include <hip/hip_ext.h>
#include <algorithm>

namespace amph {

constexpr int GM_BM = 64;
constexpr int GM_CHUNK_B = 512;                 // bytes of one activation row per chunk
constexpr int GM_PITCH = GM_CHUNK_B + 16;       // LDS row pitch (bytes): rows shift by 4 banks
constexpr int GM_STEPS = GM_CHUNK_B / 64;       // matrix-core steps per chunk (64 bytes of k each)
constexpr int GM_STAGE = GM_BM * GM_PITCH;      // one activation stage
constexpr int GM_LDS_BYTES = 2 * GM_STAGE;
constexpr int GM_NLW = 4;                       // loader waves
constexpr int GM_XROWS = GM_BM / GM_NLW, GM_XL = GM_XROWS / 2;   // activation rows / 16-byte loads per loader lane per chunk
constexpr int GM_MIN_NB = 2, GM_MAX_NB = 12;    // math waves (= row blocks) per workgroup
static_assert(GM_LDS_BYTES >= GM_BM * (16 * GM_MAX_NB + 4) * 4, "output tile must fit in the staging buffers");
static_assert(64 * (GM_MAX_NB + GM_NLW) <= 1024, "workgroup size");

// number of row blocks of a GEMM
__host__ __device__ inline int gemm_blocks(int epi, int seg_rows) {
  if (epi == EPI_QKV_ROPE) return 3 * (seg_rows / 16);
  if (epi == EPI_SWIGLU) return (seg_rows + 7) / 8;
  return (seg_rows + 15) / 16;
}

// weight row (within its matrix) and matrix index of row r16 of block b
struct RowMap { int seg; int n; bool valid; };

template <int EPI>
__device__ __forceinline__ RowMap map_block(const GemmArgs &a, int b, int r16) {
  RowMap o;
  if (EPI == EPI_QKV_ROPE) {
    const int d = a.n_heads * a.d_h, bps = d / 16, bph = a.d_h / 16;
    o.valid = true;
    o.seg = b / bps;
    const int bl = b % bps;
    if (o.seg < 2) o.n = (bl / bph) * a.d_h + (bl % bph) * 8 + (r16 & 7) + ((r16 >= 8) ? a.d_h / 2 : 0);
    else o.n = bl * 16 + r16;
  } else if (EPI == EPI_SWIGLU) {
    o.seg = (r16 >= 8) ? 1 : 0;
    o.n = b * 8 + (r16 & 7);
    o.valid = o.n < a.seg_rows;
  } else {
    o.seg = 0;
    o.n = b * 16 + r16;
    o.valid = o.n < a.seg_rows;
  }
  return o;
}

// Epilogue of one 64-row block of a workgroup's output tile: Ct[m][r] (float32, pitch CT_PITCH) holds rows
// m_base .. m_base + 63 of the activations against the tile's nb row blocks (BN = 16 * nb columns).  Every thread
// of the workgroup (NT of them) takes part.
template <typename T, int EPI>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs &a, const float *Ct, int CT_PITCH, int tile, int nb, int m_base,
                                              int split, int nblk, int tid, int NT, int rows = GM_BM) {   // rows of Ct that are live
  const int BN = 16 * nb;
  if (EPI == EPI_STORE) {
    // out is [split_k][M][N]: slab `split` receives this workgroup's partial sums
    const int N = a.seg_rows;
    float *slab = a.out + (size_t)split * a.M * N;
    const int Q = BN / 4;                                   // 4 adjacent columns per thread (one by one in a ragged last tile)
    for (int idx = tid; idx < rows * Q; idx += NT) {
      const int m = idx / Q, r = (idx % Q) * 4, mg = m_base + m, n = tile * BN + r;
      if (mg >= a.M || n >= N) continue;
      const f32x4 v = *reinterpret_cast<const f32x4 *>(Ct + m * CT_PITCH + r);
      float *dst = slab + (size_t)mg * N + n;
      if (n + 4 <= N && (N & 3) == 0) {
        *reinterpret_cast<f32x4 *>(dst) = v;
      } else {
        for (int c = 0; c < 4 && n + c < N; ++c) dst[c] = v[c];
      }
    }
  } else if (EPI == EPI_SWIGLU) {
    // block w of the tile: columns 0..7 = gate rows, 8..15 = the same rows of up
    const int f = a.seg_rows, H = 8 * nb;
    T *act = (T *)a.act;
    // one (token, block) per thread: 8 adjacent outputs leave as one piece (element by element in a ragged last block)
    for (int idx = tid; idx < rows * nb; idx += NT) {
      const int m = idx / nb, w = idx % nb, mg = m_base + m, j0 = tile * H + w * 8;
      if (mg >= a.M || j0 >= f) continue;
      const float *crow = Ct + m * CT_PITCH + w * 16;
      float y[8];
      #pragma unroll
      for (int j = 0; j < 8; ++j) y[j] = silu_f(crow[j]) * crow[8 + j];
      T *dst = act + (size_t)mg * f + j0;
      if (a.act_tiles) {                                   // tiled for the wide GEMM that follows (f is a multiple of 16)
        store4<T>(act + xt_index<T>(mg, j0, a.act_tiles), y);
        store4<T>(act + xt_index<T>(mg, j0 + 4, a.act_tiles), y + 4);
      } else if (j0 + 8 <= f && (f & 7) == 0) {
        store4<T>(dst, y); store4<T>(dst + 4, y + 4);
      } else {
        for (int j = 0; j < 8 && j0 + j < f; ++j) dst[j] = Elem<T>::from_f32(y[j]);
      }
    }
  } else if (EPI == EPI_QKV_ROPE) {
    // d_h is a power of two (checked at launch): heads and dims come from shifts; the segment of a block (q, k or v:
    // bps blocks each) from two comparisons instead of a division by a run-time value
    const int d_h = a.d_h, d = a.n_heads * d_h, bps = d >> 4, bph = d_h >> 4, bsh = __ffs(bph) - 1, half = d_h >> 1;
    auto seg_of = [&](int b) { return (b >= 2 * bps) ? 2 : (b >= bps) ? 1 : 0; };
    // q and k blocks: one (block, token) per thread = 8 rotation pairs.  Everything the item needs from global
    // memory (64 bytes of the cos/sin table, the committed length) is requested first, for up to QK_U items of the
    // thread at once: a wave of the wide kernel walks several items, and stores in between would keep the next item's
    // loads from starting early.  The 8 + 8 results leave as 16-byte pieces: dims e0 .. e0+7 (and their partners at
    // + d_h/2) are adjacent in q and inside a fragment of the tiled K cache.
    constexpr int QK_U = 3;
    for (int base = tid; base < nb * rows; base += QK_U * NT) {
      float4 tab[QK_U][4];
      int Lb[QK_U];
      #pragma unroll
      for (int u = 0; u < QK_U; ++u) {
        const int idx = base + u * NT, w = idx / rows, m = idx % rows, b = tile * nb + w, mg = m_base + m;
        const bool live = idx < nb * rows && b < nblk && mg < a.M && seg_of(b) < 2;
        const int e0 = ((b - seg_of(b) * bps) & (bph - 1)) * 8;
        // (unconditional loads from clamped addresses: dead items read the table's first entry and element 0's length)
        const float4 *csp = reinterpret_cast<const float4 *>(a.rope_cs + (live ? (size_t)mg * half + e0 : (size_t)0));
        #pragma unroll
        for (int k = 0; k < 4; ++k) tab[u][k] = csp[k];
        Lb[u] = a.kv_len[live ? mg / a.T_nodes : 0];
      }
      #pragma unroll
      for (int u = 0; u < QK_U; ++u) {
        const int idx = base + u * NT, w = idx / rows, m = idx % rows, b = tile * nb + w, mg = m_base + m;
        if (idx >= nb * rows || b >= nblk || mg >= a.M) continue;
        const int seg = seg_of(b), bl = b - seg * bps;
        if (seg >= 2) continue;
        const int head = bl >> bsh, e0 = (bl & (bph - 1)) * 8;
        const float4 c01 = tab[u][0], c23 = tab[u][1], c45 = tab[u][2], c67 = tab[u][3];
        const float cs[8] = {c01.x, c01.z, c23.x, c23.z, c45.x, c45.z, c67.x, c67.z};
        const float sn[8] = {c01.y, c01.w, c23.y, c23.w, c45.y, c45.w, c67.y, c67.w};
        const float *crow = Ct + m * CT_PITCH + w * 16;
        float y1[8], y2[8];
        #pragma unroll
        for (int j = 0; j < 8; ++j) {
          const float x1 = crow[j], x2 = crow[8 + j];
          y1[j] = x1 * cs[j] - x2 * sn[j];
          y2[j] = x2 * cs[j] + x1 * sn[j];
        }
        T *dst1, *dst2;
        if (seg == 0) {
          dst1 = (T *)a.q_out + (size_t)mg * d + head * d_h + e0;
          dst2 = dst1 + half;
        } else {
          const int bb = mg / a.T_nodes, node = mg % a.T_nodes, L = Lb[u];
          if (L < 0 || L + a.T_nodes > a.max_kv) {
            if (node == 0 && e0 == 0) atomicOr(a.dev_status, 2u);
            continue;
          }
          T *kc = (T *)a.k_cache + ((size_t)bb * a.n_heads + head) * (size_t)a.max_kv * d_h;
          dst1 = kc + k_tiled_index<T>(L + node, e0, d_h);
          dst2 = kc + k_tiled_index<T>(L + node, e0 + half, d_h);
        }
        store4<T>(dst1, y1); store4<T>(dst1 + 4, y1 + 4);
        store4<T>(dst2, y2); store4<T>(dst2 + 4, y2 + 4);
      }
    }
    // v blocks: 8 * rows items per row block (8 dims x the live tokens).  rows (32 or 64) divides the number of
    // threads, so a thread keeps its token through the loop: its committed length is read once, ahead of the stores,
    // and consecutive threads write consecutive tree rows, which are adjacent inside a step-tiled piece.
    {
      const int m = tid % rows, mg = m_base + m;
      const bool row_ok = mg < a.M;
      const int bb = row_ok ? mg / a.T_nodes : 0, node = row_ok ? mg % a.T_nodes : 0;
      const int L = a.kv_len[bb];
      if (row_ok && L >= 0 && L + a.T_nodes <= a.max_kv) {
        for (int q = tid / rows; q < nb * 8; q += NT / rows) {
          const int w = q >> 3, j = q & 7, b = tile * nb + w;
          if (b >= nblk) continue;
          const int seg = seg_of(b), bl = b - seg * bps;
          if (seg < 2) continue;
          #pragma unroll
          for (int hh = 0; hh < 2; ++hh) {
            const int head = bl >> bsh, e = ((bl & (bph - 1)) << 4) + j + 8 * hh;
            T *vc = (T *)a.v_cache + ((size_t)bb * a.n_heads + head) * (size_t)a.max_kv * d_h;
            vc[v_tiled_index<T>(L + node, e, d_h)] = Elem<T>::from_f32(Ct[m * CT_PITCH + w * 16 + j + 8 * hh]);
          }
        }
      }
    }
  } else if (EPI == EPI_ARGMAX) {
    const int N = a.seg_rows;
    if (a.logits) {
      for (int idx = tid; idx < rows * BN; idx += NT) {
        const int m = idx / BN, r = idx % BN, mg = m_base + m, n = tile * BN + r;
        if (mg < a.M && n < N) a.logits[(size_t)mg * N + n] = Ct[m * CT_PITCH + r];
      }
    }
    // 4 threads per token row, BN/4 columns each, then a 4-lane butterfly (ties -> lower column)
    for (int t4 = tid; t4 < 4 * rows; t4 += NT) {         // NT and 4 * rows are multiples of 64: the 4 lanes of a row stay in one wave
      const int m = t4 >> 2, part = t4 & 3, mg = m_base + m;
      float bv = -__builtin_huge_valf(); int bi = 0x7fffffff;
      for (int r = part * (BN / 4); r < (part + 1) * (BN / 4); ++r) {
        const int n = tile * BN + r;
        const float v = Ct[m * CT_PITCH + r];
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
}

template <typename T, int EPI, bool TILED>
__global__ __launch_bounds__(64 * (GM_MAX_NB + GM_NLW)) void k_gemm_skinny(const GemmArgs a, int tiles) {
  __shared__ __align__(16) unsigned char lds[GM_LDS_BYTES];
  const int nb = a.nb, BN = 16 * nb, NT = 64 * (nb + GM_NLW), CT_PITCH = BN + 4;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 4, r16 = lane & 15;
  const int S = a.split_k;
  // Workgroup index -> (unit = tile and split, block of 64 activation rows).  With more than one row block
  // the workgroups that stream the SAME weights get indices 8 apart: they are dispatched together and
  // land on the same XCD, so the weights come from HBM once and from that XCD's L2 for the others.
  const int mblocks = (a.M + GM_BM - 1) / GM_BM;
  const int id = blockIdx.x, unit = (id / 8 / mblocks) * 8 + (id & 7), mblock = (id / 8) % mblocks;
  if (unit >= tiles * S) return;                          // padding of the last group of 8 units (whole workgroup)
  const int tile = unit / S, split = unit % S;
  const int m_base = mblock * GM_BM;
  const int row_bytes = a.Kd * (int)sizeof(T);
  const int total_steps = row_bytes / 64;
  const int ssh = __ffs(S) - 1;                           // S is 1, 2, 4 or 8
  const int s0 = (total_steps * split) >> ssh, s1 = (total_steps * (split + 1)) >> ssh;
  const int nch = (s1 - s0 + GM_STEPS - 1) / GM_STEPS;
  const int nblk = gemm_blocks(EPI, a.seg_rows);
  // Both roles run the same number of iterations (a multiple of two, the depth of every ring) with
  // no conditional inside: chunks past the slice load clamped addresses and stage zeros, so the
  // compiler can count outstanding loads exactly instead of draining them at every join.
  const int nch2 = (nch + 1) & ~1;

  f32x4 acc[4];
  #pragma unroll
  for (int mb = 0; mb < 4; ++mb) acc[mb] = (f32x4){0.f, 0.f, 0.f, 0.f};

  if (wave < nb) {
    // ------------------------------------------------------------------------------- math wave
    // A block past the end (last tile only) re-reads the last block; its results are never stored.
    const int blk = min(tile * nb + wave, nblk - 1);
    const unsigned char *wrow;
    if (TILED) {
      // the block's fragments lie one after another: step st is the 1 KB at st * 1024, this lane's 16 bytes at
      // (r16 * 64 + g * 16) inside it
      wrow = (const unsigned char *)a.wt + (size_t)blk * total_steps * 1024 + r16 * 64 + g * 16;
    } else {
      const RowMap rm = map_block<EPI>(a, blk, r16);
      const void *wm = (rm.seg == 0) ? a.w0 : (rm.seg == 1) ? a.w1 : a.w2;
      wrow = (const unsigned char *)wm + (size_t)(rm.valid ? rm.n : 0) * row_bytes + g * 16;
    }
    uint4 aw[2][GM_STEPS];
    auto load_w = [&](int c, uint4 (&af)[GM_STEPS]) {
      #pragma unroll
      for (int s = 0; s < GM_STEPS; ++s) {
        // Unconditional load (a predicated load with a zero alternative makes the compiler wait for every
        // load at the merge).  Steps past the slice re-read its last step: harmless, because the activation
        // tile is zero there and weights are finite; rows past N re-read row 0 and are never stored.
        const int st = min(s0 + c * GM_STEPS + s, s1 - 1);
        af[s] = ldg16_stream(wrow + (size_t)st * (TILED ? 1024 : 64));
      }
    };
    load_w(0, aw[0]);
    __syncthreads();
    for (int c = 0; c < nch2; c += 2) {
      #pragma unroll
      for (int u = 0; u < 2; ++u) {
        load_w(c + u + 1, aw[u ^ 1]);
        const unsigned char *buf = lds + u * GM_STAGE;
        #pragma unroll
        for (int s = 0; s < GM_STEPS; ++s) {
          #pragma unroll
          for (int mb = 0; mb < 4; ++mb) {
            const uint4 bfrag = *reinterpret_cast<const uint4 *>(buf + (mb * 16 + r16) * GM_PITCH + s * 64 + g * 16);
            acc[mb] = mma16<T>(aw[u][s], bfrag, acc[mb]);
          }
        }
        __syncthreads();
      }
    }
  } else {
    // ----------------------------------------------------------------------------- loader wave
    // 32 lanes cover one 512-byte row piece, a wave instruction two rows; chunk c+1 is written to its
    // stage while the math waves work on chunk c, and chunk c+2 is already on its way from L2.
    const unsigned char *xg = (const unsigned char *)a.x;
    const int x_row0 = (wave - nb) * GM_XROWS + (lane >> 5), x_col = (lane & 31) * 16;
    uint4 xr[2][GM_XL];
    auto load_x = [&](int c, uint4 (&xf)[GM_XL]) {
      const int byte = (s0 + c * GM_STEPS) * 64 + x_col;
      const bool in_k = byte < s1 * 64;
      #pragma unroll
      for (int j = 0; j < GM_XL; ++j) {
        const int mg = m_base + x_row0 + 2 * j;
        const bool ok = in_k && mg < a.M;                 // out-of-range pieces read the tensor's first bytes ...
        xf[j] = ldg16(xg + (ok ? (size_t)mg * row_bytes + byte : (size_t)0));
      }
    };
    auto store_x = [&](int stage, int c, const uint4 (&xf)[GM_XL]) {
      unsigned char *buf = lds + stage * GM_STAGE;
      const bool in_k = (s0 + c * GM_STEPS) * 64 + x_col < s1 * 64;
      #pragma unroll
      for (int j = 0; j < GM_XL; ++j) {
        const bool ok = in_k && (m_base + x_row0 + 2 * j) < a.M;   // ... and are replaced by zeros here
        *reinterpret_cast<uint4 *>(buf + (x_row0 + 2 * j) * GM_PITCH + x_col) = ok ? xf[j] : make_uint4(0u, 0u, 0u, 0u);
      }
    };
    load_x(0, xr[0]);
    load_x(1, xr[1]);
    store_x(0, 0, xr[0]);
    __syncthreads();
    for (int c = 0; c < nch2; c += 2) {
      #pragma unroll
      for (int u = 0; u < 2; ++u) {
        load_x(c + u + 2, xr[u]);                         // slot of chunk c+u: already in LDS
        store_x(u ^ 1, c + u + 1, xr[u ^ 1]);
        __syncthreads();
      }
    }
  }

  // Partial slabs need no regrouping: a math lane holds 4 adjacent outputs (weight rows wave*16 + g*4 .. +3) of
  // activation row mb*16 + r16, which are 16 adjacent bytes of out[split][m][n].
  if (EPI == EPI_STORE && (a.seg_rows & 3) == 0) {
    if (wave < nb) {
      const int N = a.seg_rows, n0 = tile * BN + wave * 16 + g * 4;
      float *slab = a.out + (size_t)split * a.M * N + n0;
      #pragma unroll
      for (int mb = 0; mb < 4; ++mb) {
        const int mg = m_base + mb * 16 + r16;
        if (mg < a.M && n0 < N) *reinterpret_cast<f32x4 *>(slab + (size_t)mg * N) = acc[mb];
      }
    }
    return;
  }
  // SwiGLU needs no regrouping either: lane groups 0, 1 hold the block's 8 gate rows, groups 2, 3 the same rows of
  // W_up, 32 lanes further on; after one exchange a lane of group 0 or 1 owns 4 adjacent outputs of its token.
  if (EPI == EPI_SWIGLU && (a.seg_rows & 3) == 0) {
    if (wave < nb) {
      const int f = a.seg_rows, j0 = tile * 8 * nb + wave * 8 + g * 4;
      T *act = (T *)a.act;
      #pragma unroll
      for (int mb = 0; mb < 4; ++mb) {
        float y[4];
        #pragma unroll
        for (int c = 0; c < 4; ++c) {
          const float up = __shfl_down(acc[mb][c], 32, WAVE);
          y[c] = silu_f(acc[mb][c]) * up;
        }
        const int mg = m_base + mb * 16 + r16;
        if (g < 2 && mg < a.M && j0 < f) store4<T>(act + (size_t)mg * f + j0, y);
      }
    }
    return;
  }
  // accumulators -> Ct[m][r] (float32): a math lane holds rows r = wave*16 + g*4 .. +4 of column m.
  // The last barrier of the loop has passed, so nobody reads the stages any more; the one write still
  // outstanding (the loaders' zero chunk nch2) went to stage nch2 % 2 before that barrier.
  float *Ct = reinterpret_cast<float *>(lds);
  if (wave < nb) {
    #pragma unroll
    for (int mb = 0; mb < 4; ++mb)
      *reinterpret_cast<f32x4 *>(Ct + (mb * 16 + r16) * CT_PITCH + wave * 16 + g * 4) = acc[mb];
  }
  __syncthreads();

  gemm_epilogue<T, EPI>(a, Ct, CT_PITCH, tile, nb, m_base, split, nblk, tid, NT);
}

// =====================================================================================================
// Wide GEMM: 128 or more activation rows (batches of trees).  The skinny kernel above re-reads the weights
// from L2 once per block of 64 rows, every math wave re-reads the whole activation chunk from LDS, and its
// 16 x 16 matrix-core instruction runs at half the rate of the 32 x 32 one: with several blocks of rows L2, LDS
// and the matrix cores, not HBM, set the pace.  Here a workgroup owns a group of up to 16 tiles of 32 activation
// rows (all rows, up to 512; more rows form several groups) against NB weight row blocks, and the roles of the
// operands are swapped:
//   * the weights are the shared operand: two loader waves stream the workgroup's NB blocks from HBM straight
//     into a ring of LDS stages (global-to-LDS loads, 8 steps of 64 bytes of k per stage), so they cross L2 once;
//   * each math wave owns 2 (or 3) of the group's tiles against all NB blocks, taken in pairs (32 weight rows): per
//     step and half-step it reads one weight fragment per pair from LDS and one activation fragment per tile from
//     global memory (L2 hits, requested 2 or 4 steps ahead into registers) and issues one matrix-core instruction
//     of 32 x 32 per pair and tile; one barrier per 8 steps.  Up to 8 tiles there is one math wave per SIMD (2
//     adjacent tiles each); from 9 tiles on two per SIMD, wave w owning tiles w and w + 8.
// A 32 x 32 instruction takes, per lane (half, r), 16 bytes of row r: the bytes [half * 16, half * 16 + 16) of
// 32 bytes of k.  The weight fragments in LDS are the 16-row x 64-byte ones of the tiled layout, piece (g, r16)
// at (g * 16 + r16) * 16: lane (half, r) of half-step h reads piece (2h + half, r % 16) of block r / 16 of the
// pair, 16 lanes per 256 contiguous bytes.  The activations must be tiled to match (a fragment gathered from
// row-major rows is the slow many-half-lines load): k_tile_rows rewrites [M, Kd] as
// xt[(q * m32_tiles + tile) * 1024 + lane * 16], q = index of 32 bytes of k, lane = half * 32 + row % 32, rows
// past M as zeros (a few microseconds).
// =====================================================================================================
constexpr int GW_STEPS = 8;        // steps (64 bytes of k) per weight stage
constexpr int GW_R = 3;            // weight stages in the LDS ring
constexpr int GW_NL = 2;           // loader waves
constexpr int GW_MAX_NP = 3;       // pairs of weight row blocks per workgroup
constexpr int GW_MAX_NW = 8;       // math waves per workgroup with 2 tiles of 32 activation rows each (two waves per SIMD)
constexpr int GW_MAX_NW3 = 4;      // ... with 3 tiles each: one wave per SIMD (three tiles of accumulators need 222 registers)
constexpr int GW_MAX_TW = 3;
constexpr int GW_XD = 4;           // steps of activations requested ahead
constexpr int GW_MIN_MBLOCKS = 3;  // blocks of 64 activation rows from which the wide kernel is used
constexpr int GW_AUX_NT = 2;       // cache-policy bits of the global-to-LDS load: non-temporal (the weights are read once)
static_assert(GW_STEPS % GW_XD == 0, "the activation ring is indexed statically inside a stage");

template <int N> struct GwTag { static constexpr int value = N; };
template <int N> __device__ __forceinline__ void gw_wait_vm() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0f70);
}

template <typename T>
__global__ __launch_bounds__(256) void k_tile_rows(const unsigned char *x, int M, int row_bytes, int m32_tiles, unsigned char *xt) {
  const int qn = row_bytes / 32;
  const size_t pieces = (size_t)qn * m32_tiles * 64;
  for (size_t p = (size_t)blockIdx.x * 256 + threadIdx.x; p < pieces; p += (size_t)gridDim.x * 256) {
    const int lane = (int)(p & 63), half = lane >> 5, r32 = lane & 31;
    const size_t frag = p >> 6;
    const int mt = (int)(frag % m32_tiles), q = (int)(frag / m32_tiles);
    const int m = mt * 32 + r32;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (m < M) v = ldg16(x + (size_t)m * row_bytes + (size_t)q * 32 + half * 16);
    stg16(xt + p * 16, v);
  }
}

template <typename T, int EPI, int NP, int TW, int NWMAX>      // NWMAX = 4: one math wave per SIMD (256 registers each); 8: two (168)
__global__ __launch_bounds__(64 * (NWMAX + GW_NL)) void k_gemm_wide(const GemmArgs a, int tiles, int mgroups, int m32_tiles, int gt) {
  extern __shared__ __align__(16) unsigned char gw_lds[];
  constexpr int NB = 2 * NP, STAGE = NB * GW_STEPS * 1024, PERL = NB * GW_STEPS / GW_NL;
  static_assert(GW_R == 3 && PERL * (GW_R - 2) <= 63, "loader wave's outstanding loads");
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int NT = blockDim.x, nw = (NT >> 6) - GW_NL;       // math waves
  const int S = a.split_k;
  const int id = blockIdx.x, unit = (id / 8 / mgroups) * 8 + (id & 7), mgroup = (id / 8) % mgroups;
  if (unit >= tiles * S) return;                          // padding of the last group of 8 units (whole workgroup)
  const int tile = unit / S, split = unit % S;
  constexpr int XD = (TW == 3 || NWMAX == 8) ? 2 : GW_XD; // steps of activations requested ahead (registers)
  static_assert(GW_STEPS % XD == 0, "the activation ring is indexed statically inside a stage");
  // Tiles of this group: gt of them from g0 on.  One wave per SIMD (NWMAX = 4): wave w owns the TW adjacent tiles
  // from w * TW on.  Two waves per SIMD (NWMAX = 8): wave w owns tiles w and w + nw, so that with fewer than 2 * nw
  // tiles the waves left with one tile are the upper half, which share their SIMDs with the lower half.
  const int g0 = mgroup * gt;
  auto tile_of = [&](int t) { return g0 + (NWMAX == 8 ? wave + t * nw : wave * TW + t); };
  auto live = [&](int t) { const int x = tile_of(t); return x < g0 + gt && x < m32_tiles; };
  const int total_steps = a.Kd * (int)sizeof(T) / 64;
  const int ssh = __ffs(S) - 1;                           // S is 1, 2, 4 or 8
  const int s0 = (total_steps * split) >> ssh, s1 = (total_steps * (split + 1)) >> ssh;
  const int n = s1 - s0;
  const int P = (n + GW_STEPS - 1) / GW_STEPS;             // weight stages
  const int nblk = gemm_blocks(EPI, a.seg_rows);

  f32x16 acc[NP][TW];
  #pragma unroll
  for (int p = 0; p < NP; ++p)
    #pragma unroll
    for (int t = 0; t < TW; ++t)
      #pragma unroll
      for (int i = 0; i < 16; ++i) acc[p][t][i] = 0.f;

  if (wave >= nw) {
    // ---------------------------------------------------------------------------- loader wave
    // Loader l takes steps l * HS .. + HS - 1 of every block of a stage (fragment f = block * GW_STEPS + step lies at
    // f * 1024 of the stage).  Lane (g, r16) fetches piece g of row r16, which lands at (g * 16 + r16) * 16 of the
    // fragment's KB in LDS.  Those HS fragments are adjacent both in memory and in LDS, so they share one address and
    // one LDS base and differ in the instruction's immediate offset (applied to both sides): a load costs the wave one
    // instruction instead of a dozen.  That matters because the loader shares its SIMD's issue port with a math wave
    // whose matrix-core instructions keep it busy (measured before: 233 clocks per load, the weight ring the
    // bottleneck).  A ragged last stage takes the general path: steps past the slice re-read its last step and are
    // never used.
    constexpr int HS = GW_STEPS / GW_NL;
    static_assert(GW_STEPS % GW_NL == 0 && HS == 4, "four immediate offsets per block, written out below");
    const int l = wave - nw, g = lane >> 4, r16 = lane & 15;
    const unsigned char *wbase = (const unsigned char *)a.wt + r16 * 64 + g * 16;
    const unsigned char *bsrc[NB];
    #pragma unroll
    for (int b = 0; b < NB; ++b) bsrc[b] = wbase + ((size_t)min(tile * NB + b, nblk - 1) * total_steps + s0 + l * HS) * 1024;
    auto issue = [&](int p) {
      unsigned char *lp = gw_lds + (p % GW_R) * STAGE;
      if ((p + 1) * GW_STEPS <= n) {                       // a whole stage (wave-uniform)
        #pragma unroll
        for (int b = 0; b < NB; ++b) {
          const unsigned char *src = bsrc[b] + (size_t)p * (GW_STEPS * 1024);
          unsigned char *dst = lp + (b * GW_STEPS + l * HS) * 1024;
          const auto *gs = (const __attribute__((address_space(1))) void *)src;
          auto *ld = (__attribute__((address_space(3))) void *)dst;
          __builtin_amdgcn_global_load_lds(gs, ld, 16, 0, GW_AUX_NT);       // (the offset must be a literal)
          __builtin_amdgcn_global_load_lds(gs, ld, 16, 1024, GW_AUX_NT);
          __builtin_amdgcn_global_load_lds(gs, ld, 16, 2048, GW_AUX_NT);
          __builtin_amdgcn_global_load_lds(gs, ld, 16, 3072, GW_AUX_NT);
        }
      } else {
        #pragma unroll
        for (int j = 0; j < PERL; ++j) {
          const int b = j / HS, s = l * HS + j % HS, f = b * GW_STEPS + s;
          const int blk = min(tile * NB + b, nblk - 1);
          const int st = min(s0 + p * GW_STEPS + s, s1 - 1);
          const unsigned char *src = wbase + ((size_t)blk * total_steps + st) * 1024;
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                           (__attribute__((address_space(3))) void *)(lp + f * 1024), 16, 0, GW_AUX_NT);
        }
      }
    };
    const int pro = P < GW_R - 1 ? P : GW_R - 1;
    for (int p = 0; p < pro; ++p) issue(p);
    for (int p = 0; p < P; ++p) {
      if (p + 1 < P) gw_wait_vm<PERL>(); else gw_wait_vm<0>();   // stage p has landed (one younger stage may be in flight)
      __builtin_amdgcn_s_barrier();                        // math waves may read stage p; they are done with stage p - 1
      if (p + GW_R - 1 < P) issue(p + GW_R - 1);           // into the slot of stage p - 1
    }
  } else {
    // ------------------------------------------------------------------------------ math wave
    // activation tiles TW * wave .. + TW - 1 of the group (32 rows each); the 2 * TW fragments of a step (two halves
    // of the step's 64 bytes for every tile) are requested XD steps ahead
    const int half = lane >> 5, r32 = lane & 31;
    const unsigned char *xb = (const unsigned char *)a.xt + lane * 16;
    uint4 xq[XD][2][TW];
    auto load_x = [&](int i, uint4 (&xf)[2][TW]) {
      const int st = s0 + max(min(i, n - 1), 0);           // unconditional: steps past the slice re-read the last one
      #pragma unroll
      for (int h = 0; h < 2; ++h)
        #pragma unroll
        for (int t = 0; t < TW; ++t) {
          const int mt = min(tile_of(t), m32_tiles - 1);   // tiles past the end (last wave) re-read the last tile; never stored
          xf[h][t] = ldg16(xb + ((size_t)(2 * st + h) * m32_tiles + mt) * 1024);
        }
    };
    // weight piece of this lane inside a pair's two fragments of a step, for half-step h: + h * 512
    const int woff = (r32 >> 4) * (GW_STEPS * 1024) + (half * 16 + (r32 & 15)) * 16;
    #pragma unroll
    for (int i = 0; i < XD; ++i) load_x(i, xq[i]);
    // NTL = tiles this wave multiplies: TW, or 1 for a wave of the two-per-SIMD layout whose second tile does not exist
    auto run = [&](auto tag) {
      constexpr int NTL = decltype(tag)::value;
      for (int p = 0; p < P; ++p) {
        // Stage p is in LDS (pairs with the loaders' barrier).  A bare barrier: __syncthreads() would also wait for this
        // wave's outstanding activation loads (the fence it carries counts them since the kernel contains global-to-LDS
        // loads) and drain the prefetch ring at every stage.  The "memory" clobber keeps the LDS reads below it; the
        // reads of stage p - 1 are complete because the matrix-core instructions that used them have been issued.
        asm volatile("s_barrier" ::: "memory");
        const unsigned char *sb = gw_lds + (p % GW_R) * STAGE + woff;
        #pragma unroll
        for (int s = 0; s < GW_STEPS; ++s) {
          const int i = p * GW_STEPS + s;
          if (i < n) {                                     // wave-uniform
            #pragma unroll
            for (int h = 0; h < 2; ++h)
              #pragma unroll
              for (int pr = 0; pr < NP; ++pr) {
                const uint4 wf = *reinterpret_cast<const uint4 *>(sb + (2 * pr * GW_STEPS + s) * 1024 + h * 512);
                #pragma unroll
                for (int t = 0; t < NTL; ++t) acc[pr][t] = mma32<T>(wf, xq[s % XD][h][t], acc[pr][t]);
              }
          }
          load_x(i + XD, xq[s % XD]);
        }
      }
    };
    if (NWMAX == 8 && !live(1)) run(GwTag<1>{}); else run(GwTag<TW>{});
  }

  // ---- epilogues: every math wave handles its own activation rows through its own Ct region in LDS (the ring is
  // free by now), one tile of 32 rows at a time, the 64 lanes playing the workgroup of the shared epilogue code.
  // Lane (half, r32) holds activation row t * 32 + r32 and weight rows (i / 4) * 8 + half * 4 + (i % 4) of each pair.
  const int CT_PITCH = 16 * NB + 4;
  __syncthreads();                                         // every wave has left the ring
  if (wave < nw && live(0)) {                              // whole waves
    float *Ct = reinterpret_cast<float *>(gw_lds) + (size_t)wave * 32 * CT_PITCH;
    const int half = lane >> 5, r32 = lane & 31;
    #pragma unroll
    for (int t = 0; t < TW; ++t) {
      if (!live(t)) break;                                 // (wave-uniform)
      if (t > 0) {                                         // the lanes are done reading the tile before
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      }
      #pragma unroll
      for (int pr = 0; pr < NP; ++pr)
        #pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const f32x4 v = {acc[pr][t][4 * q4], acc[pr][t][4 * q4 + 1], acc[pr][t][4 * q4 + 2], acc[pr][t][4 * q4 + 3]};
          *reinterpret_cast<f32x4 *>(Ct + r32 * CT_PITCH + pr * 32 + q4 * 8 + half * 4) = v;
        }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // the wave's LDS writes before its lanes read each other's
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      gemm_epilogue<T, EPI>(a, Ct, CT_PITCH, tile, NB, tile_of(t) * 32, split, nblk, lane, WAVE, 32);
    }
  }
}

// Row-major -> tiled (see the layout above).  One thread per 16-byte piece of the tiled buffer.
template <typename T, int EPI>
__global__ __launch_bounds__(256) void k_pack_weights(const GemmArgs a, unsigned char *dst) {
  const int total_steps = a.Kd * (int)sizeof(T) / 64;
  const size_t pieces = (size_t)gemm_blocks(EPI, a.seg_rows) * total_steps * 64;   // 64 pieces of 16 bytes per fragment
  for (size_t p = (size_t)blockIdx.x * 256 + threadIdx.x; p < pieces; p += (size_t)gridDim.x * 256) {
    const int g = (int)(p & 3), r16 = (int)((p >> 2) & 15);
    const size_t frag = p >> 6;
    const int st = (int)(frag % total_steps);
    const int blk = (int)(frag / total_steps);
    const RowMap rm = map_block<EPI>(a, blk, r16);
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (rm.valid) {
      const void *wm = (rm.seg == 0) ? a.w0 : (rm.seg == 1) ? a.w1 : a.w2;
      v = ldg16((const unsigned char *)wm + ((size_t)rm.n * a.Kd * sizeof(T) + (size_t)st * 64 + g * 16));
    }
    stg16(dst + p * 16, v);
  }
}

size_t gemm_tiled_bytes(int epi, int seg_rows, int Kd, int elem_bytes) {
  return (size_t)gemm_blocks(epi, seg_rows) * 16 * (size_t)Kd * elem_bytes;
}

template <typename T>
hipError_t launch_pack_weights(hipStream_t st, int epi, const GemmArgs &a, void *dst) {
  if (a.Kd < 1 || (a.Kd * (int)sizeof(T)) % 64) return hipErrorInvalidValue;
  if (epi == EPI_QKV_ROPE && (a.d_h % 16 || a.seg_rows != a.n_heads * a.d_h)) return hipErrorInvalidValue;
  const size_t pieces = gemm_tiled_bytes(epi, a.seg_rows, a.Kd, (int)sizeof(T)) / 16;
  const int blocks = (int)std::min<size_t>((pieces + 255) / 256, 65536);
  unsigned char *d8 = (unsigned char *)dst;
  switch (epi) {
    case EPI_STORE: hipLaunchKernelGGL((k_pack_weights<T, EPI_STORE>), dim3(blocks), dim3(256), 0, st, a, d8); break;
    case EPI_QKV_ROPE: hipLaunchKernelGGL((k_pack_weights<T, EPI_QKV_ROPE>), dim3(blocks), dim3(256), 0, st, a, d8); break;
    case EPI_SWIGLU: hipLaunchKernelGGL((k_pack_weights<T, EPI_SWIGLU>), dim3(blocks), dim3(256), 0, st, a, d8); break;
    case EPI_ARGMAX: hipLaunchKernelGGL((k_pack_weights<T, EPI_ARGMAX>), dim3(blocks), dim3(256), 0, st, a, d8); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
template hipError_t launch_pack_weights<float>(hipStream_t, int, const GemmArgs &, void *);
template hipError_t launch_pack_weights<bf16_t>(hipStream_t, int, const GemmArgs &, void *);

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

// Tile height and reduction split for one GEMM.  Model, in units of one weight fragment: a workgroup's
// time is its steps times (nb fragments + 2 for its share of the activation chunk); the kernel's time
// is that times the number of rounds the grid needs on 256 CUs; every split beyond the first costs the
// write and the later read of one more float32 slab.  The two constants are fitted to measurements of
// the 7B shapes (Wo: 4 blocks x 4 splits beats 2 x 2 and 8 x 8; down: 4 x 4 beats 8 x 8).
GemmPlan gemm_plan(int epi, int seg_rows, int Kd, int elem_bytes, int M, int split_req, bool tiled) {
  GemmPlan best{};
  const int blocks = gemm_blocks(epi, seg_rows);
  const int total_steps = Kd * elem_bytes / 64;
  const int mblocks = (M + GM_BM - 1) / GM_BM;
  const bool fused = epi != EPI_STORE;
  const double slab_units = fused ? 0.0 : (double)M * seg_rows * 1.0e-4 + 2.0;   // per extra split
  double best_cost = 1e300;
  best.blocks = blocks;
  // measured at 7B shapes, ms per step skinny / wide: 2 blocks of 64 rows 5.60 / 6.49, 3 blocks 7.37 / 7.02, 4 blocks
  // 8.23 / 7.86, 6 blocks 12.44 / 11.07, 8 blocks 14.46 / 12.40; 33B shapes, 6 blocks: 59.1 / 47.4
  best.wide = gemm_is_wide(M, tiled);
  if (best.wide) {
    // A workgroup owns a group of tiles of 32 activation rows against nb weight row blocks.  Inside a group the
    // tiles are dealt to math waves so that the four SIMDs carry the same matrix-core load: 2 tiles per wave, or 3
    // per wave for 9 to 12 tiles (one wave per SIMD; six waves of two tiles kept two SIMDs twice as busy as the
    // others), up to 8 waves of 2.  Two ways to form the groups are priced: as few groups as possible (up to 16
    // tiles: the weights cross LDS once) or groups of at most 8 tiles (twice the workgroups: pays when the weight
    // matrix has too few row blocks to fill the chip).  A workgroup's time goes with its steps, its nb + 2
    // fragments per step and the tiles its busiest SIMD carries; ties go to the fewer groups.
    const int mt = (M + 31) / 32;
    // candidates (the later one wins ties): groups of at most 8 tiles, one wave of 2 tiles per SIMD; as few groups as
    // possible with 3 tiles per wave (9 to 12 tiles a group); the same with two waves per SIMD (9 to 16 tiles)
    for (int cand = 0; cand < 3; ++cand) {
      const int max_tiles = cand == 0 ? 8 : cand == 1 ? 12 : 16;
      const int mg = (mt + max_tiles - 1) / max_tiles;
      const int gt = (mt + mg - 1) / mg;                                // tiles per group
      if (cand > 0 && gt <= 8) continue;                                // nothing new
      const int tw = cand == 1 ? 3 : 2;
      const int nw = cand == 2 ? GW_MAX_NW : (gt + tw - 1) / tw;
      // tiles on the busiest SIMD; two waves on a SIMD cover part of each other's waits (measured: 23.5 against
      // 25.7 us per tile and SIMD for gate/up at 7B shapes)
      const double simd_tiles = cand == 2 ? 0.92 * ((gt + 3) / 4) : (double)((nw + 3) / 4) * tw;
      for (int s = 1; s <= 8; s *= 2) {
        if (split_req > 0 && s != split_req) continue;
        if (split_req == 0 && (fused ? s > 1 : (s > 1 && total_steps / s < 2 * GW_STEPS))) continue;
        for (int nb = 2; nb <= 2 * GW_MAX_NP; nb += 2) {      // blocks are taken in pairs
          if (nb > std::max(blocks, 2)) break;
          const int tiles = (blocks + nb - 1) / nb;
          const long wgs = (long)tiles * s * mg;
          const long rounds = (wgs + 255) / 256;
          const double cost = (double)rounds * ((total_steps + s - 1) / s) * (nb + 2) * (simd_tiles / 2) + slab_units * (s - 1);
          if (cost <= best_cost) {
            best_cost = cost; best.nb = nb; best.split = s; best.tiles = tiles;
            best.mgroups = mg; best.nw = nw; best.tw = tw; best.gt = gt;
          }
        }
      }
    }
    return best;
  }
  best.mgroups = mblocks;
  best.nw = 1;
  best.tw = 2;
  best.gt = 2;
  for (int s = 1; s <= 8; s *= 2) {
    if (split_req > 0 && s != split_req) continue;
    if (split_req == 0 && (fused ? s > 1 : (s > 1 && total_steps / s < 2 * GM_STEPS))) continue;
    for (int nb = GM_MIN_NB; nb <= GM_MAX_NB; ++nb) {
      if (nb > std::max(blocks, GM_MIN_NB)) break;
      const int tiles = (blocks + nb - 1) / nb;
      const long wgs = (long)tiles * s * mblocks;
      const long rounds = (wgs + 255) / 256;
      const double cost = (double)rounds * ((total_steps + s - 1) / s) * (nb + 2) + slab_units * (s - 1);
      if (cost <= best_cost) { best_cost = cost; best.nb = nb; best.split = s; best.tiles = tiles; }
    }
  }
  return best;
}

bool gemm_is_wide(int M, bool tiled) { return tiled && (M + GM_BM - 1) / GM_BM >= GW_MIN_MBLOCKS; }

size_t gemm_xt_bytes(int M, int Kd, int elem_bytes) { return (size_t)((M + 31) / 32) * 32 * (size_t)Kd * elem_bytes; }

template <typename T, int EPI, int NP, int TW, int NWMAX>
static hipError_t launch_wide_np(hipStream_t st, const GemmArgs &a, const GemmPlan &pl, int m32_tiles, dim3 grid, dim3 block,
                                 hipEvent_t ev_start, hipEvent_t ev_stop) {
  // the weight ring, or (afterwards, in the same memory) one float32 output tile of 64 rows per math wave
  constexpr size_t ring = (size_t)GW_R * 2 * NP * GW_STEPS * 1024, ct_wave = (size_t)32 * (32 * NP + 4) * 4;
  constexpr size_t smem_max = ring > NWMAX * ct_wave ? ring : NWMAX * ct_wave;
  static_assert(smem_max <= 160 * 1024, "LDS of one workgroup");
  const size_t smem = std::max(ring, (size_t)pl.nw * ct_wave);
  static bool attr_set = false;                           // once per instantiation and process
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void *)k_gemm_wide<T, EPI, NP, TW, NWMAX>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_max);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  if (ev_start && ev_stop)
    hipExtLaunchKernelGGL((k_gemm_wide<T, EPI, NP, TW, NWMAX>), grid, block, smem, st, ev_start, ev_stop, 0, a, pl.tiles, pl.mgroups, m32_tiles, pl.gt);
  else
    hipLaunchKernelGGL((k_gemm_wide<T, EPI, NP, TW, NWMAX>), grid, block, smem, st, a, pl.tiles, pl.mgroups, m32_tiles, pl.gt);
  return hipGetLastError();
}

template <typename T, int EPI>
static hipError_t launch_wide(hipStream_t st, const GemmArgs &a, const GemmPlan &pl, hipEvent_t ev_start, hipEvent_t ev_stop) {
  if (!a.wt || !a.xt || pl.nw < 1 || pl.nw > (pl.tw == 3 ? GW_MAX_NW3 : GW_MAX_NW) || pl.tw < 2 || pl.tw > GW_MAX_TW || pl.nb < 2 ||
      pl.nb > 2 * GW_MAX_NP || pl.nb % 2)
    return hipErrorInvalidValue;
  if ((long long)pl.mgroups * pl.gt * 32 < a.M || pl.gt > pl.nw * pl.tw) return hipErrorInvalidValue;   // groups cover every row, waves every tile
  const int m32_tiles = (a.M + 31) / 32, row_bytes = a.Kd * (int)sizeof(T);
  const size_t pieces = (size_t)(row_bytes / 32) * m32_tiles * 64;
  GemmArgs aw = a;
  if (a.x_tiled) aw.xt = const_cast<void *>(a.x);         // the producer of x wrote it tiled
  else hipLaunchKernelGGL((k_tile_rows<T>), dim3((unsigned)std::min<size_t>((pieces + 255) / 256, 4096)), dim3(256), 0, st,
                          (const unsigned char *)a.x, a.M, row_bytes, m32_tiles, (unsigned char *)a.xt);
  const long long wgs = (long long)((pl.tiles * a.split_k + 7) / 8) * pl.mgroups * 8;
  if (wgs > 0x7fffffffLL) return hipErrorInvalidValue;
  const dim3 grid((unsigned)wgs), block(64 * (pl.nw + GW_NL));
  #define GW_LAUNCH(NP_)                                                                                            \
    return pl.tw == 3 ? launch_wide_np<T, EPI, NP_, 3, 4>(st, aw, pl, m32_tiles, grid, block, ev_start, ev_stop)   \
         : pl.nw > 4  ? launch_wide_np<T, EPI, NP_, 2, 8>(st, aw, pl, m32_tiles, grid, block, ev_start, ev_stop)   \
                      : launch_wide_np<T, EPI, NP_, 2, 4>(st, aw, pl, m32_tiles, grid, block, ev_start, ev_stop)
  switch (pl.nb / 2) {
    case 1: GW_LAUNCH(1);
    case 2: GW_LAUNCH(2);
    default: GW_LAUNCH(3);
  }
  #undef GW_LAUNCH
}

template <typename T>
hipError_t launch_gemm(hipStream_t st, int epi, const GemmArgs &a_in, hipEvent_t ev_start, hipEvent_t ev_stop) {
  GemmArgs a = a_in;
  if (a.M < 1 || a.Kd < 1 || (a.Kd * (int)sizeof(T)) % 64) return hipErrorInvalidValue;
  if (a.split_k != 1 && a.split_k != 2 && a.split_k != 4 && a.split_k != 8) return hipErrorInvalidValue;
  if (epi != EPI_STORE && a.split_k != 1) return hipErrorInvalidValue;     // fused epilogues need complete sums
  if (epi == EPI_QKV_ROPE && (a.d_h < 16 || (a.d_h & (a.d_h - 1)) || a.seg_rows != a.n_heads * a.d_h || !a.rope_cs)) return hipErrorInvalidValue;
  const GemmPlan pl = gemm_plan(epi, a.seg_rows, a.Kd, (int)sizeof(T), a.M, a.split_k, a.wt != nullptr && a.xt != nullptr);
  a.nb = pl.nb;
  if (!pl.wide && (a.x_tiled || a.act_tiles)) return hipErrorInvalidValue;   // only the wide kernel knows the tiled activations
  if (pl.wide) {
    switch (epi) {
      case EPI_STORE: return launch_wide<T, EPI_STORE>(st, a, pl, ev_start, ev_stop);
      case EPI_QKV_ROPE: return launch_wide<T, EPI_QKV_ROPE>(st, a, pl, ev_start, ev_stop);
      case EPI_SWIGLU: return launch_wide<T, EPI_SWIGLU>(st, a, pl, ev_start, ev_stop);
      case EPI_ARGMAX: return launch_wide<T, EPI_ARGMAX>(st, a, pl, ev_start, ev_stop);
      default: return hipErrorInvalidValue;
    }
  }
  const int tiles = pl.tiles;
  const int mblocks = (a.M + GM_BM - 1) / GM_BM;
  const long long wgs = (long long)((tiles * a.split_k + 7) / 8) * mblocks * 8;     // see the index mapping in the kernel
  if (wgs > 0x7fffffffLL) return hipErrorInvalidValue;
  const dim3 grid((unsigned)wgs), block(64 * (a.nb + GM_NLW));
  // With a pair of events the launch itself carries them: they take the kernel's own begin and end time stamps,
  // so reading them costs the stream nothing and includes nothing but the kernel.
  #define GM_LAUNCH(E)                                                                                           \
    if (ev_start && ev_stop) {                                                                                   \
      if (a.wt) hipExtLaunchKernelGGL((k_gemm_skinny<T, E, true>), grid, block, 0, st, ev_start, ev_stop, 0, a, tiles);  \
      else hipExtLaunchKernelGGL((k_gemm_skinny<T, E, false>), grid, block, 0, st, ev_start, ev_stop, 0, a, tiles);      \
    } else if (a.wt) hipLaunchKernelGGL((k_gemm_skinny<T, E, true>), grid, block, 0, st, a, tiles);              \
    else hipLaunchKernelGGL((k_gemm_skinny<T, E, false>), grid, block, 0, st, a, tiles)
  switch (epi) {
    case EPI_STORE: GM_LAUNCH(EPI_STORE); break;
    case EPI_QKV_ROPE: GM_LAUNCH(EPI_QKV_ROPE); break;
    case EPI_SWIGLU: GM_LAUNCH(EPI_SWIGLU); break;
    case EPI_ARGMAX: GM_LAUNCH(EPI_ARGMAX); break;
    default: return hipErrorInvalidValue;
  }
  #undef GM_LAUNCH
  return hipGetLastError();
}
template hipError_t launch_gemm<float>(hipStream_t, int, const GemmArgs &, hipEvent_t, hipEvent_t);
template hipError_t launch_gemm<bf16_t>(hipStream_t, int, const GemmArgs &, hipEvent_t, hipEvent_t);

}  // namespace amph
