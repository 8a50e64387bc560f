// bf16 prompt phase on the gfx950 matrix cores.
//
//  attn_fwd   masked attention rows (Section 1; Section 3.1 Eq.3 of the paper): for a block
//             of query rows, K/V tiles of 64 keys stream through LDS, S^T = K Q^T and
//             O^T = V^T P^T run on v_mfma_f32_32x32x16_bf16 with an online softmax.
//             Writes O (optional) and the base-2 log-sum-exp of every row.
//  col_scores forgotten accumulated score of every key (Section 3.3 Eq.5):
//             S_j = sum_{i>=j} alpha^(n-1-i) * P[i, j].  A block of key columns stays in
//             registers, Q tiles stream through LDS, the logit tile is recomputed on the
//             matrix cores, exp2(s - lse_i + (n-1-i) log2 alpha) is formed per element (the
//             forgetting weight is folded into the exponent) and summed down the tile's
//             rows.  The n x n probability matrix is never written.
//
// Both kernels compute the TRANSPOSED logit tile (keys = M, queries = N).  In the 32x32
// accumulator layout a lane then owns one query (column l%32) and 16 keys
// (rows 8*(i/4) + 4*(l/32) + i%4, i = 0..15), so
//   - row statistics of the softmax are per-lane scalars (one exchange with lane^32),
//   - P^T is already in the B-operand layout of the second product (no LDS round trip),
//   - the column sums of col_scores accumulate per lane and are reduced across lanes once.
#include <math.h>

#include "a2sf_dev.h"
#include "a2sf_internal.h"

namespace a2sf {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kTile = 64;  // keys (attn_fwd) or query rows (col_scores) per LDS tile
constexpr float kLazyRescale = 8.0f;  // log2 units
constexpr int kPrefetch = 4;  // LDS fragment reads in flight ahead of their matrix op
constexpr int kFwdNB = 1;     // 32-row query blocks per wave in attn_fwd_bf16_kernel / attn_fwd128_kernel
constexpr int kFwdOcc = 2;    // workgroups per compute unit the register budget of attn_fwd_bf16_kernel is sized for

__device__ __forceinline__ f32x16 mfma_bf16(const uint4& a, const uint4& b, const f32x16& c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ---- LDS layouts ----------------------------------------------------------------------
// Row tile [64][D] bf16 in 16-byte chunks, chunk index XOR-swizzled by the row so that the
// 16 lanes of a quarter-wave reading one chunk column of 16 consecutive rows hit 16
// different bank groups, and the 16 lanes writing one row do too.
template <int D>
__device__ __forceinline__ int row_tile_unit(int row, int chunk) {
  constexpr int CPR = D / 8;
  const int swz = (CPR == 16) ? (row & 15) : ((row >> 1) & 7);
  return row * CPR + (chunk ^ swz);
}
// Transposed V tile [D][64 keys] bf16, 128 bytes per d-row = 8 chunks of 8 keys.  Inside
// each group of 16 keys the keys are stored in the order the matrix-core operand wants:
// key kappa sits at 8*((kappa>>2)&1) + (kappa&3) + 4*(kappa>>3).
__device__ __forceinline__ int vt_swizzle(int d) { return ((d >> 1) ^ (d >> 4)) & 7; }

template <int D>
struct Stage {
  static constexpr int CPR = D / 8;
  static constexpr int KU = kTile * CPR / kThreads;        // K units (16 B) per thread
  static constexpr int VTASKS = 16 * CPR;                  // (key quad, d chunk) tasks
  uint4 kreg[KU];
  uint4 vreg[4];

  template <bool WITH_V>
  __device__ __forceinline__ void load(const bf16_t* __restrict__ Kg, const bf16_t* __restrict__ Vg,
                                       int row0, int n) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int u = 0; u < KU; ++u) {
      const int unit = tid + u * kThreads;
      int r = row0 + unit / CPR;
      r = r < n ? r : n - 1;
      kreg[u] = load16(Kg + (size_t)r * D + (unit % CPR) * 8);
    }
    if (WITH_V && tid < VTASKS) {
      const int dc = tid % CPR, kq = tid / CPR;
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        int r = row0 + 4 * kq + rr;
        r = r < n ? r : n - 1;
        vreg[rr] = load16(Vg + (size_t)r * D + dc * 8);
      }
    }
  }
  template <bool WITH_V>
  __device__ __forceinline__ void store(uint4* ks, char* vt) const {
    const int tid = threadIdx.x;
#pragma unroll
    for (int u = 0; u < KU; ++u) {
      const int unit = tid + u * kThreads;
      ks[row_tile_unit<D>(unit / CPR, unit % CPR)] = kreg[u];
    }
    if (WITH_V && tid < VTASKS) {
      const int dc = tid % CPR, kq = tid / CPR;
      const int chunk = 2 * (kq >> 2) + (kq & 1), half = (kq & 3) >> 1;
      const uint32_t* x0 = reinterpret_cast<const uint32_t*>(&vreg[0]);
      const uint32_t* x1 = reinterpret_cast<const uint32_t*>(&vreg[1]);
      const uint32_t* x2 = reinterpret_cast<const uint32_t*>(&vreg[2]);
      const uint32_t* x3 = reinterpret_cast<const uint32_t*>(&vreg[3]);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int w = i >> 1, d = dc * 8 + i;
        uint2 out;
        if (i & 1) {
          out.x = (x0[w] >> 16) | (x1[w] & 0xFFFF0000u);
          out.y = (x2[w] >> 16) | (x3[w] & 0xFFFF0000u);
        } else {
          out.x = (x0[w] & 0xFFFFu) | (x1[w] << 16);
          out.y = (x2[w] & 0xFFFFu) | (x3[w] << 16);
        }
        *reinterpret_cast<uint2*>(vt + d * 128 + ((chunk ^ vt_swizzle(d)) << 4) + half * 8) = out;
      }
    }
  }
};

// Workgroup id -> flat work id such that each of the 8 accelerator dies (which receive
// consecutive workgroup ids round-robin) works on a contiguous range of work ids, i.e. on
// whole heads whose K/V stay in that die's L2.
__device__ __forceinline__ long long xcd_contiguous_id(long long total) {
  const long long per = (total + 7) / 8;
  return (long long)(blockIdx.x % 8) * per + blockIdx.x / 8;
}

// ---------------------------------------------------------------------------------------
// Geometry as in AttnRect: n = rc.m query rows per head; row i sees keys 0 .. off + i of the nk =
// off + n keys of its head (the prompt phase: off = 0, the keys are the rows' own).
template <int D, int NB, bool WITH_O>
__global__ __launch_bounds__(kThreads, kFwdOcc) void attn_fwd_bf16_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    bf16_t* __restrict__ O, float* __restrict__ LSE2, AttnRect rc, int G, int nqb, float scale_log2e) {
  constexpr int BM = kWaves * 32 * NB;
  constexpr int CPR = D / 8;
  constexpr int KK = D / 16;   // k-steps of the first product
  constexpr int DB = D / 32;   // 32-wide blocks of the head dimension
  __shared__ uint4 ks[2][kTile * CPR];
  __shared__ __attribute__((aligned(16))) char vt[WITH_O ? 2 : 1][WITH_O ? D * 128 : 16];

  const long long total = (long long)G * nqb;
  const long long vid = xcd_contiguous_id(total);
  if (vid >= total) return;
  const int g = (int)(vid / nqb);
  const int qb = nqb - 1 - (int)(vid % nqb);  // longest rows first

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: branches on it are scalar
  const int l32 = lane & 31, h = lane >> 5;
  const int n = rc.m;
  const int gk = g / rc.kv_group;  // the K/V head this query head reads
  const int off = rc.off_heads ? rc.off_heads[gk] : 0;
  const int row0 = qb * BM;
  if (off < 0) {  // a head the caller's precondition excludes: its rows are flagged with NaN
    if (WITH_O)
      for (int e = tid; e < min(BM, n - row0) * D; e += kThreads)
        O[((size_t)g * n + row0) * D + e] = (bf16_t)0x7FC0;
    return;
  }
  const int nk = off + n;  // keys of this head
  const bf16_t* Qg = Q + (size_t)g * n * D;
  const bf16_t* Kg = K + (size_t)gk * rc.kv_stride * D;
  const bf16_t* Vg = V + (size_t)gk * rc.kv_stride * D;
  const int wrow0 = row0 + wave * 32 * NB;  // first query row of this wave

  // Q fragments (B operand): lane (query l32, half h) holds Q[query][16kk + 8h .. +7]
  uint4 qf[NB][KK];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    int r = wrow0 + nb * 32 + l32;
    r = r < n ? r : n - 1;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[nb][kk] = load16(Qg + (size_t)r * D + kk * 16 + h * 8);
  }

  f32x16 oacc[NB][DB];
  float m[NB], lsum[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    m[nb] = -INFINITY;
    lsum[nb] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[nb][db][i] = 0.f;
  }

  const int last_key = off + min(n, row0 + BM) - 1;  // newest key the block's rows see
  const int ntiles = last_key / kTile + 1;
  Stage<D> stg;
  stg.template load<WITH_O>(Kg, Vg, 0, nk);
  stg.template store<WITH_O>(ks[0], vt[0]);
  __syncthreads();

  for (int t = 0; t < ntiles; ++t) {
    const int buf = t & 1;
    if (t + 1 < ntiles) stg.template load<WITH_O>(Kg, Vg, (t + 1) * kTile, nk);
    const int key0 = t * kTile;
    if (key0 <= off + wrow0 + 32 * NB - 1) {  // some key of the tile is visible to this wave
      // ---- S^T = K Q^T
      f32x16 sacc[NB][2];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) sacc[nb][kb][i] = 0.f;
      {
        // fragment i = (kk, kb): the two key blocks alternate so that consecutive matrix
        // instructions never depend on each other; LDS reads run kPrefetch fragments ahead.
        constexpr int NF = 2 * KK;
        uint4 fr[NF];
        auto kfrag = [&](int i) {
          return ks[buf][row_tile_unit<D>((i & 1) * 32 + l32, 2 * (i >> 1) + h)];
        };
#pragma unroll
        for (int i = 0; i < kPrefetch && i < NF; ++i) fr[i] = kfrag(i);
#pragma unroll
        for (int i = 0; i < NF; ++i) {
          if (i + kPrefetch < NF) fr[i + kPrefetch] = kfrag(i + kPrefetch);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
            sacc[nb][i & 1] = mfma_bf16(fr[i], qf[nb][i >> 1], sacc[nb][i & 1]);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // one LDS read
          __builtin_amdgcn_sched_group_barrier(0x008, NB, 0); // then this step's matrix ops
        }
      }
      const bool diag = key0 + kTile - 1 > off + wrow0;  // tile reaches past the wave's first row
      uint4 pf[NB][2][2];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const int qrow = off + wrow0 + nb * 32 + l32;   // newest key this lane's row sees
        if (diag) {
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int key = key0 + kb * 32 + 8 * (i >> 2) + 4 * h + (i & 3);
              if (key > qrow) sacc[nb][kb][i] = -INFINITY;
            }
        }
        float mx = sacc[nb][0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[nb][kb][i]);
        mx = across_rows(mx, OpMax(), false, true);
        // The running maximum only has to bound the exponents, not equal the true maximum:
        // it is raised (and the accumulators rescaled) only when some row of the wave
        // exceeds it by more than 2^kLazyRescale, so probabilities stay below that factor
        // and the rescale, which costs a multiply per accumulator register, becomes rare.
        // (Rows past the end of a ragged block can be fully masked: keep m finite.)
        const float mxs = fmaxf(mx * scale_log2e, -1e30f);
        if (__any(mxs > m[nb] + kLazyRescale)) {
          const float m_new = fmaxf(m[nb], mxs);
          const float corr = fast_exp2(m[nb] - m_new);
          lsum[nb] *= corr;
          if (WITH_O) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
              for (int i = 0; i < 16; ++i) oacc[nb][db][i] *= corr;
          }
          m[nb] = m_new;
        }
        float rs = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          float p[16];
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            p[i] = fast_exp2(fmaf(sacc[nb][kb][i], scale_log2e, -m[nb]));
            rs += p[i];
          }
          if (WITH_O) {
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
              uint4 w;
              w.x = pack_bf16(p[8 * tt + 0], p[8 * tt + 1]);
              w.y = pack_bf16(p[8 * tt + 2], p[8 * tt + 3]);
              w.z = pack_bf16(p[8 * tt + 4], p[8 * tt + 5]);
              w.w = pack_bf16(p[8 * tt + 6], p[8 * tt + 7]);
              pf[nb][kb][tt] = w;
            }
          }
        }
        lsum[nb] += rs;
      }
      // ---- O^T += V^T P^T
      if (WITH_O) {
        // fragment i = (kb, tt, db): the head-dimension block is the fastest index, so that
        // consecutive matrix instructions go to different accumulators (a dependent
        // back-to-back pair costs 48 instead of 32 cycles).
        constexpr int NF = DB * 4;
        uint4 fr[NF];
        auto vfrag = [&](int i) {
          const int d = (i % DB) * 32 + l32;
          return *reinterpret_cast<const uint4*>(vt[buf] + d * 128 + ((((i / DB) * 2 + h) ^ vt_swizzle(d)) << 4));
        };
#pragma unroll
        for (int i = 0; i < kPrefetch && i < NF; ++i) fr[i] = vfrag(i);
#pragma unroll
        for (int i = 0; i < NF; ++i) {
          if (i + kPrefetch < NF) fr[i + kPrefetch] = vfrag(i + kPrefetch);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
            oacc[nb][i % DB] = mfma_bf16(fr[i], pf[nb][(i / DB) >> 1][(i / DB) & 1], oacc[nb][i % DB]);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, NB, 0);
        }
      }
    }
    if (t + 1 < ntiles) stg.template store<WITH_O>(ks[buf ^ 1], vt[WITH_O ? (buf ^ 1) : 0]);
    __syncthreads();
  }

  // ---- epilogue
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int qrow = wrow0 + nb * 32 + l32;
    const float l = across_rows(lsum[nb], OpAdd(), false, true);
    if (qrow < n) {
      if (h == 0) LSE2[(size_t)g * n + qrow] = m[nb] + log2f(l);
      if (WITH_O) {
        const float inv = 1.0f / l;
        bf16_t* orow = O + ((size_t)g * n + qrow) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            uint2 w;
            w.x = pack_bf16(oacc[nb][db][4 * i4 + 0] * inv, oacc[nb][db][4 * i4 + 1] * inv);
            w.y = pack_bf16(oacc[nb][db][4 * i4 + 2] * inv, oacc[nb][db][4 * i4 + 3] * inv);
            *reinterpret_cast<uint2*>(orow + db * 32 + 8 * i4 + 4 * h) = w;
          }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// d = 128 variant built on two gfx950 features:
//  * K and V tiles go from global memory straight into LDS (global_load_lds, 16 bytes per
//    lane, a wave fills 1 KB = 4 rows per instruction; lane l's data lands at base + 16 l,
//    so the swizzle is applied by choosing which global chunk each lane fetches).  No
//    staging registers, no LDS store instructions.
//  * V stays row-major [key][d] in LDS; the V^T operand of O^T = V^T P^T is read with
//    ds_read_b64_tr_b16, which transposes 4x4 blocks of 16-bit elements across the 16
//    lanes of a group: output lane i, element r  <-  source lane 4r + i/4, element i%4.
//    Source lane (r, q) therefore points at V[key_r][d0 + 4q ..+3] and output lane i
//    receives V[key_0..3][d0 + i]: exactly the 4 consecutive keys of one half operand.
// Same mathematics and operand conventions as attn_fwd_bf16_kernel above.
typedef short v4i16_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) char lds_char;

__device__ __forceinline__ uint2 lds_read_tr16(const lds_char* p) {
  v4i16_t r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) v4i16_t*)p);
  return __builtin_bit_cast(uint2, r);
}
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 lds_read16(const lds_char* p) {
  const u32x4_t r = *reinterpret_cast<const __attribute__((address_space(3))) u32x4_t*>(p);
  return make_uint4(r.x, r.y, r.z, r.w);
}

typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void lds_write8(lds_char* p, const uint2& v) {
  const u32x2_t x = {v.x, v.y};
  *reinterpret_cast<__attribute__((address_space(3))) u32x2_t*>(p) = x;
}

constexpr int kTileBytes = kTile * 256;  // one 64-row tile of 128 bf16

// Chunk swizzles (16-byte chunks of a 256-byte row; the LDS has 64 four-byte banks).  K is
// read 16 rows x one chunk column per 16 lanes: XOR with the row spreads them over all 16
// chunk positions.  V is read by 32 lanes as 4 rows x 4 chunk columns x 2 halves: XOR with
// 4*(row%4) sends the four rows to disjoint groups of four chunk positions.  Both measure
// zero LDS bank conflicts (SQ_LDS_BANK_CONFLICT).
__device__ __forceinline__ int k_swizzle(int row) { return row & 15; }
__device__ __forceinline__ int v_swizzle(int row) { return (row & 3) << 2; }

template <bool V_LAYOUT>
__device__ __forceinline__ void dma_tile(const bf16_t* __restrict__ Mg, int row0, int n,
                                         lds_char* tile) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int rr = lane >> 4, pc = lane & 15;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int lrow = (u * 4 + wave) * 4 + rr;
    const int c = pc ^ (V_LAYOUT ? v_swizzle(lrow) : k_swizzle(lrow));
    int r = row0 + lrow;
    r = r < n ? r : n - 1;
    __builtin_amdgcn_global_load_lds((const void*)(Mg + (size_t)r * 128 + c * 8),
                                     (__attribute__((address_space(3))) void*)(tile + (u * 4 + wave) * 1024),
                                     16, 0, 0);
  }
}

// dma_tile for a tile that straddles two sources: rows below `off` are rows of A, rows from
// `off` on are rows 0 .. of B (n rows in all).
template <bool V_LAYOUT>
__device__ __forceinline__ void dma_tile2(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                          int off, int row0, int n, lds_char* tile) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int rr = lane >> 4, pc = lane & 15;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int lrow = (u * 4 + wave) * 4 + rr;
    const int c = pc ^ (V_LAYOUT ? v_swizzle(lrow) : k_swizzle(lrow));
    int r = row0 + lrow;
    r = r < n ? r : n - 1;
    const bf16_t* src = r < off ? A + (size_t)r * 128 : B + (size_t)(r - off) * 128;
    __builtin_amdgcn_global_load_lds((const void*)(src + c * 8),
                                     (__attribute__((address_space(3))) void*)(tile + (u * 4 + wave) * 1024),
                                     16, 0, 0);
  }
}

// Same as dma_tile for a tile that lies completely inside the matrix: the per-lane byte
// offsets `loff` (row-in-tile and swizzled chunk) are loop invariants, the tile base is
// wave-uniform, so a tile costs four load instructions and no address arithmetic per lane.
template <bool V_LAYOUT>
__device__ __forceinline__ void dma_offsets(int (&loff)[4]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int rr = lane >> 4, pc = lane & 15;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int lrow = (u * 4 + wave) * 4 + rr;
    loff[u] = lrow * 256 + ((pc ^ (V_LAYOUT ? v_swizzle(lrow) : k_swizzle(lrow))) << 4);
  }
}
__device__ __forceinline__ void dma_full_tile(const bf16_t* __restrict__ Mg, int row0,
                                              const int (&loff)[4], lds_char* tile) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const char* base = reinterpret_cast<const char*>(Mg) + (size_t)row0 * 256;
#pragma unroll
  for (int u = 0; u < 4; ++u)
    __builtin_amdgcn_global_load_lds((const void*)(base + loff[u]),
                                     (__attribute__((address_space(3))) void*)(tile + (u * 4 + wave) * 1024),
                                     16, 0, 0);
}

constexpr int kScoreOnlyNB = 1;   // 32-row query blocks per wave when no outputs are wanted
constexpr int kScoreOnlyOcc = 4;  // workgroups per compute unit then (32 KB of LDS each: K tiles only)

template <bool WITH_O, int NB>
__global__ __launch_bounds__(kThreads, !WITH_O ? kScoreOnlyOcc : (NB == 1 ? 2 : 1)) void attn_fwd128_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    bf16_t* __restrict__ O, float* __restrict__ LSE2, AttnRect rc, int G, int nqb, float scale_log2e) {
  constexpr int D = 128, BM = kWaves * 32 * NB, KK = D / 16, DB = D / 32;
  // [stage][K tile | V tile]; without outputs there are no V tiles.  A deeper ring (tiles
  // fetched three steps ahead) was measured for that pass and is slower: it costs occupancy.
  constexpr int kBuf = (WITH_O ? 2 : 1) * kTileBytes;
  constexpr int RING = 2;                        // tiles are fetched RING - 1 steps ahead
  constexpr int kLoadsPerTile = WITH_O ? 8 : 4;  // direct-to-LDS loads a wave issues per fetch
  static_assert((RING - 2) * kLoadsPerTile <= 15, "pending loads must fit the wait count used below");
  __shared__ __attribute__((aligned(1024))) char smem[RING * kBuf];
  lds_char* const lds = (lds_char*)smem;

  const long long total = (long long)G * nqb;
  const long long vid = xcd_contiguous_id(total);
  if (vid >= total) return;
  const int g = (int)(vid / nqb);
  // longest rows first; without outputs the launch covers only the nqb row blocks from the one
  // that holds rc.first_row on
  const int qb = (WITH_O ? 0 : rc.first_row / BM) + nqb - 1 - (int)(vid % nqb);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: branches on it are scalar
  const int l32 = lane & 31, h = lane >> 5;
  const int n = rc.m;
  const int gk = g / rc.kv_group;  // the K/V head this query head reads
  const int off = rc.off_heads ? rc.off_heads[gk] : 0;  // older tokens in front of the rows' own
  const int row0 = qb * BM;
  if (off < 0) {  // a head the caller's precondition excludes: its rows are flagged with NaN
    if (WITH_O)
      for (int e = tid; e < min(BM, n - row0) * D; e += kThreads)
        O[((size_t)g * n + row0) * D + e] = (bf16_t)0x7FC0;
    return;
  }
  const int nk = off + n;  // keys of this head
  const bf16_t* Qg = Q + (size_t)g * n * D;
  const bf16_t* Kg = K + (size_t)gk * rc.kv_stride * D;
  const bf16_t* Vg = V + (size_t)gk * rc.kv_stride * D;
  // second source (keys off .. off+n-1), or null
  const bf16_t* K2g = rc.k2 ? (const bf16_t*)rc.k2 + (size_t)gk * n * D : nullptr;
  const bf16_t* V2g = rc.k2 ? (const bf16_t*)rc.v2 + (size_t)gk * n * D : nullptr;
  const int wrow0 = row0 + wave * 32 * NB;  // first query row of this wave

  // Q fragments (B operand): lane (query l32, half h) holds Q[query][16kk + 8h .. +7]
  uint4 qf[NB][KK];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    int r = wrow0 + nb * 32 + l32;
    r = r < n ? r : n - 1;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[nb][kk] = load16(Qg + (size_t)r * D + kk * 16 + h * 8);
  }
  // per-lane LDS byte offsets inside a K / V tile
  int koff[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) koff[kk] = l32 * 256 + (((2 * kk + h) ^ k_swizzle(l32)) << 4);
  int voff[DB];
  {
    const int i = lane & 15, r = i >> 2, qd = i & 3, gq = (lane >> 4) & 1;
    const int cl = 2 * gq + (qd >> 1), vs = v_swizzle(4 * h + r);  // key = 8*x + 4h + r
#pragma unroll
    for (int db = 0; db < DB; ++db)
      voff[db] = (4 * h + r) * 256 + ((((4 * db + cl) ^ vs)) << 4) + (qd & 1) * 8;
  }

  f32x16 oacc[NB][DB];
  float m[NB], lsum[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    m[nb] = -INFINITY;
    lsum[nb] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[nb][db][i] = 0.f;
  }

  const int last_key = off + min(n, row0 + BM) - 1;  // newest key the block's rows see
  const int ntiles = last_key / kTile + 1;
  int k_loff[4], v_loff[4];
  dma_offsets<false>(k_loff);
  dma_offsets<true>(v_loff);
  auto fetch = [&](int t, lds_char* buf) {  // K tile t and V tile t into buf | buf + 16 KB
    if (K2g && (t + 1) * kTile > off) {       // the tile holds rows of the second source
      if (t * kTile >= off && (t + 1) * kTile <= nk) {
        dma_full_tile(K2g, t * kTile - off, k_loff, buf);
        if (WITH_O) dma_full_tile(V2g, t * kTile - off, v_loff, buf + kTileBytes);
      } else {
        dma_tile2<false>(Kg, K2g, off, t * kTile, nk, buf);
        if (WITH_O) dma_tile2<true>(Vg, V2g, off, t * kTile, nk, buf + kTileBytes);
      }
      return;
    }
    if ((t + 1) * kTile <= nk) {
      dma_full_tile(Kg, t * kTile, k_loff, buf);
      if (WITH_O) dma_full_tile(Vg, t * kTile, v_loff, buf + kTileBytes);
    } else {
      dma_tile<false>(Kg, t * kTile, nk, buf);
      if (WITH_O) dma_tile<true>(Vg, t * kTile, nk, buf + kTileBytes);
    }
  };
  // a wave's loads complete in order: tile t has landed once at most the loads of the tiles
  // fetched after it are outstanding
  // `later` = tiles fetched after the one that is needed (at most RING - 2)
  auto wait_all_but = [&](int later) {
    if (later >= 2 && RING > 2) __builtin_amdgcn_s_waitcnt(0x0f70 | (2 * kLoadsPerTile));
    else if (later == 1 && RING > 2) __builtin_amdgcn_s_waitcnt(0x0f70 | kLoadsPerTile);
    else __builtin_amdgcn_s_waitcnt(0x0f70);
  };
#pragma unroll
  for (int i = 0; i < RING - 1; ++i)
    if (i < ntiles) fetch(i, lds + i * kBuf);
  wait_all_but(min(RING - 2, ntiles - 1));  // tile 0; tiles 1 .. RING-2 may still be on their way
  __syncthreads();

  auto tile_step = [&](int t, const lds_char* kt, const lds_char* vt_) {
    const int key0 = t * kTile;
    if (key0 > off + wrow0 + 32 * NB - 1) return;  // no key of the tile is visible to this wave
    f32x16 sacc[NB][2];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[nb][kb][i] = 0.f;
    {
      constexpr int NF = 2 * KK;  // fragment i = (kk, kb)
      uint4 fr[NF];
#pragma unroll
      for (int i = 0; i < kPrefetch; ++i) fr[i] = lds_read16(kt + (i & 1) * 32 * 256 + koff[i >> 1]);
#pragma unroll
      for (int i = 0; i < NF; ++i) {
        if (i + kPrefetch < NF)
          fr[i + kPrefetch] = lds_read16(kt + ((i + kPrefetch) & 1) * 32 * 256 + koff[(i + kPrefetch) >> 1]);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) sacc[nb][i & 1] = mfma_bf16(fr[i], qf[nb][i >> 1], sacc[nb][i & 1]);
      }
      // keep that order: kPrefetch reads up front, then one new read per fragment's matrix ops
      __builtin_amdgcn_sched_group_barrier(0x100, kPrefetch, 0);
#pragma unroll
      for (int i = 0; i < NF; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, NB, 0);
        if (i + kPrefetch < NF) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
    }
    const bool diag = key0 + kTile - 1 > off + wrow0;  // tile reaches past the wave's first row
    uint4 pf[NB][2][2];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      if (diag) {  // causal mask
        const int newest = off + wrow0 + nb * 32 + l32;  // newest key this lane's row sees
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int key = key0 + kb * 32 + 8 * (i >> 2) + 4 * h + (i & 3);
            if (key > newest) sacc[nb][kb][i] = -INFINITY;
          }
      }
      if constexpr (!WITH_O) {
        // Statistics only.  The exponentials are taken against the running maximum as it is,
        // without looking for the tile's own: floating point keeps their relative precision
        // whatever their size, so the maximum has to move only when a sum leaves the range
        // (>= 2^30, or not a number: the first tile, whose running maximum is -inf).
        float rs = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) rs += fast_exp2(fmaf(sacc[nb][kb][i], scale_log2e, -m[nb]));
        if (__any(!(rs < 1073741824.f))) {
          float mx = sacc[nb][0][0];
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[nb][kb][i]);
          mx = across_rows(mx, OpMax(), false, true);
          const float m_new = fmaxf(m[nb], fmaxf(mx * scale_log2e, -1e30f));
          lsum[nb] *= fast_exp2(m[nb] - m_new);  // 0 on the first tile
          m[nb] = m_new;
          rs = 0.f;
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) rs += fast_exp2(fmaf(sacc[nb][kb][i], scale_log2e, -m_new));
        }
        lsum[nb] += rs;
        continue;
      }
      float mx = sacc[nb][0][0];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[nb][kb][i]);
      mx = across_rows(mx, OpMax(), false, true);
      const float mxs = fmaxf(mx * scale_log2e, -1e30f);
      if (__any(mxs > m[nb] + kLazyRescale)) {  // see attn_fwd_bf16_kernel
        const float m_new = fmaxf(m[nb], mxs);
        const float corr = fast_exp2(m[nb] - m_new);
        lsum[nb] *= corr;
        if (WITH_O) {
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[nb][db][i] *= corr;
        }
        m[nb] = m_new;
      }
      float rs = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        float p[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          p[i] = fast_exp2(fmaf(sacc[nb][kb][i], scale_log2e, -m[nb]));
          rs += p[i];
        }
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
          pf[nb][kb][tt] = make_uint4(pack_bf16(p[8 * tt + 0], p[8 * tt + 1]), pack_bf16(p[8 * tt + 2], p[8 * tt + 3]),
                                      pack_bf16(p[8 * tt + 4], p[8 * tt + 5]), pack_bf16(p[8 * tt + 6], p[8 * tt + 7]));
      }
      lsum[nb] += rs;
    }
    if (WITH_O) {
      constexpr int NF = DB * 4;  // fragment i = (kb, tt, db), db fastest
      uint2 lo[NF], hi[NF];
      auto vread = [&](int i, uint2& a, uint2& b) {
        const lds_char* p = vt_ + ((i / DB) * 16) * 256 + voff[i % DB];
        a = lds_read_tr16(p);
        b = lds_read_tr16(p + 8 * 256);
      };
#pragma unroll
      for (int i = 0; i < kPrefetch; ++i) vread(i, lo[i], hi[i]);
#pragma unroll
      for (int i = 0; i < NF; ++i) {
        if (i + kPrefetch < NF) vread(i + kPrefetch, lo[i + kPrefetch], hi[i + kPrefetch]);
        const uint4 a = make_uint4(lo[i].x, lo[i].y, hi[i].x, hi[i].y);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          oacc[nb][i % DB] = mfma_bf16(a, pf[nb][(i / DB) >> 1][(i / DB) & 1], oacc[nb][i % DB]);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 2 * kPrefetch, 0);
#pragma unroll
      for (int i = 0; i < NF; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, NB, 0);
        if (i + kPrefetch < NF) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      }
    }
  };

  for (int t0 = 0; t0 < ntiles; t0 += RING) {
    // tile t in stage t % RING: unrolled over the ring, all LDS offsets are immediates
#pragma unroll
    for (int b = 0; b < RING; ++b) {
      const int t = t0 + b;
      if (t >= ntiles) break;
      // the stage of tile t - 1 is free: every wave passed the barrier that ended its step
      if (t + RING - 1 < ntiles) fetch(t + RING - 1, lds + ((b + RING - 1) % RING) * kBuf);
      tile_step(t, lds + b * kBuf, lds + b * kBuf + kTileBytes);
      // tile t + 1 for every wave of the workgroup
      wait_all_but(min(RING - 2, ntiles - 2 - t));
      __syncthreads();
    }
  }

  // ---- epilogue.  The accumulator layout gives a lane 4 consecutive d of one row at a time:
  // written straight to memory that is 32 rows x 16 bytes per instruction.  Instead each wave
  // transposes its 32 x 128 output block through its own 8 KB strip of LDS (free after the
  // loop's last barrier; 16-byte chunks XOR-swizzled by the row) and stores whole 256-byte
  // rows, 4 rows per instruction.
  lds_char* const ostrip = lds + wave * 8192;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int qrow = wrow0 + nb * 32 + l32;
    const float l = across_rows(lsum[nb], OpAdd(), false, true);
    if (qrow < n && h == 0) LSE2[(size_t)g * n + qrow] = m[nb] + log2f(l);
    if (WITH_O) {
      const float inv = 1.0f / l;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          uint2 w;
          w.x = pack_bf16(oacc[nb][db][4 * i4 + 0] * inv, oacc[nb][db][4 * i4 + 1] * inv);
          w.y = pack_bf16(oacc[nb][db][4 * i4 + 2] * inv, oacc[nb][db][4 * i4 + 3] * inv);
          // row l32, elements 32db + 8*i4 + 4h .. +3  ->  chunk 4db + i4, half h
          lds_write8(ostrip + l32 * 256 + (((4 * db + i4) ^ (l32 & 15)) << 4) + 8 * h, w);
        }
      __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
      __builtin_amdgcn_wave_barrier();
      const int rr = lane >> 4, c = lane & 15;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int r = 4 * u + rr;
        const uint4 v = lds_read16(ostrip + r * 256 + ((c ^ (r & 15)) << 4));
        const int orow = wrow0 + nb * 32 + r;
        if (orow < n) store16(O + ((size_t)g * n + orow) * D + c * 8, v);
      }
      __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
      __builtin_amdgcn_wave_barrier();
    }
  }
}

// ---------------------------------------------------------------------------------------
// d = 128 with two 32-row query blocks per wave (64 rows per wave, 256 per workgroup) and one
// wave per SIMD.  Same operand conventions, LDS tile layouts and mathematics as
// attn_fwd128_kernel; the instruction stream (register map, phase schedule, hazards) is
// written by gen_attn_fwd128x2.py, whose header describes it.  This wrapper derives the
// per-lane offsets and per-wave pointers and hands them to that stream.  Requires
// n % 256 == 0 and an output pointer.
#include "attn_fwd128x2_body.inc"

constexpr int kX2Rows = 256;             // query rows per workgroup and block
constexpr int kX2RingBytes = 4 * 32768;  // four stages of one K tile + one V tile
constexpr int kX2LdsBytes = kX2RingBytes + 4 * 8192;  // + one 8 KB output strip per wave
constexpr int kX2MinRows = 2048;
constexpr int kX2MinRowsPersistent = 512;
constexpr int kX2Slots = 32;             // persistent launch: workgroups per XCD (one per CU)

// rounds == 1: one workgroup per (head, 256-row block), ids mapped as in the other kernels.
// rounds > 1 (persistent launch, 8 * kX2Slots workgroups, nqb a power of two): the workgroup
// in slot r of XCD x works on ids x * (total / 8) + r + 32 j, j = 0 .. rounds - 1; the K/V tile
// stream runs on from one block into the next and a block's Q rows are loaded during the last
// tile of the block before, so a block starts with its first tiles already in LDS.
__global__ __launch_bounds__(kThreads, 1) void attn_fwd128x2_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    bf16_t* __restrict__ O, float* __restrict__ LSE2, int n, int nqb, int id_base, int ids,
    int rounds, int kv_shift, unsigned kv_magic, float scale_log2e) {
  // query head g reads the keys and values of K/V head g / r (grouped-query heads) =
  // mulhi(g, kv_magic) + (g >> kv_shift): r a power of two: kv_magic = 0, kv_shift = log2 r;
  // otherwise kv_shift = 31 and kv_magic = floor(2^32 / r) + 1
  __shared__ __attribute__((aligned(1024))) char smem[kX2LdsBytes];
  // this launch covers the ids id_base .. id_base + ids - 1; id = head * nqb + block position
  int vid0;
  if (rounds > 1) {
    vid0 = id_base + (int)(blockIdx.x % 8) * (ids / 8) + (int)(blockIdx.x / 8);
  } else {
    const long long vid = xcd_contiguous_id(ids);
    if (vid >= ids) return;
    vid0 = id_base + (int)vid;
  }
  const int g0 = vid0 / nqb;
  const int qb0 = nqb - 1 - vid0 % nqb;  // longest rows first
  const int lgnqb = 31 - __builtin_clz(nqb), nqbm1 = nqb - 1;  // used from the second round on

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int l32 = lane & 31, h = lane >> 5;
  const unsigned lds0 = (unsigned)(size_t)smem;  // LDS byte address of the stage ring

  // K fragment (16 d-chunk 2kk+h of key row l32): row base and the kk-independent swizzle term
  const unsigned krow = lds0 + l32 * 256, hx16 = (unsigned)((h ^ k_swizzle(l32)) << 4);
  // V fragment (see attn_fwd128_kernel): source lane (r, qd) of group gq, key rows 4h + r
  const int i16 = lane & 15, r4 = i16 >> 2, qd = i16 & 3, gq = (lane >> 4) & 1;
  const unsigned clvs16 = (unsigned)(((2 * gq + (qd >> 1)) ^ v_swizzle(r4)) << 4);
  const unsigned vrow = lds0 + kTileBytes + (4 * h + r4) * 256 + (qd & 1) * 8;
  // DMA: this wave fills rows 16u + 4 wave + rr of a tile, lane (rr, pc) the chunk slot pc
  const int rr = lane >> 4, pc = lane & 15, lrow = 4 * wave + rr;
  const unsigned kl0 = (unsigned)(lrow * 256 + ((pc ^ k_swizzle(lrow)) << 4));
  const unsigned vl0 = (unsigned)(lrow * 256 + ((pc ^ v_swizzle(lrow)) << 4));
  const unsigned qoff = (unsigned)(l32 * 256 + h * 16);
  const int lv = l32 - 4 * h;
  const unsigned l32x4 = l32 * 4, lanex16 = lane * 16;
  // epilogue: a wave's 32 x 128 output blocks go, one after the other, through its own 8 KB
  // strip of LDS above the ring
  const unsigned strip = lds0 + kX2RingBytes + wave * 8192;
  const unsigned strip_w = strip + l32 * 256 + 8 * h, x16 = (unsigned)((l32 & 15) << 4);
  const unsigned strip_r = strip + rr * 256, crr16 = (unsigned)((pc ^ rr) << 4);

  // Rows: a 256-row block is cut into eight 32-row blocks; wave w owns blocks w ("block 0")
  // and 7 - w ("block 1"), so that every wave has the same number of key tiles to go through
  // although the rows further down see more keys.
  const int w32a = 32 * wave, w32b = 32 * (7 - wave), wodd = wave & 1;
  const unsigned wave_lds = lds0 + wave * 1024;
  const unsigned long long qa = (unsigned long long)Q, ka = (unsigned long long)K,
                           va = (unsigned long long)V, oa = (unsigned long long)O,
                           la = (unsigned long long)LSE2;

  asm volatile(A2SF_FWD128X2_ASM
               :
               : [hx16] "v"(hx16), [krow] "v"(krow), [clvs16] "v"(clvs16), [vrow] "v"(vrow),
                 [kl0] "v"(kl0), [vl0] "v"(vl0), [qoff] "v"(qoff), [lv] "v"(lv),
                 [l32x4] "v"(l32x4), [lanex16] "v"(lanex16), [strip_w] "v"(strip_w),
                 [x16] "v"(x16), [crr16] "v"(crr16), [strip_r] "v"(strip_r),
                 [qlo] "s"((unsigned)qa), [qhi] "s"((unsigned)(qa >> 32)),
                 [klo] "s"((unsigned)ka), [khi] "s"((unsigned)(ka >> 32)),
                 [vlo] "s"((unsigned)va), [vhi] "s"((unsigned)(va >> 32)),
                 [olo] "s"((unsigned)oa), [ohi] "s"((unsigned)(oa >> 32)),
                 [llo] "s"((unsigned)la), [lhi] "s"((unsigned)(la >> 32)),
                 [n] "s"(n), [g0] "s"(g0), [qb0] "s"(qb0), [vid0] "s"(vid0), [rounds] "s"(rounds),
                 [lgnqb] "s"(lgnqb), [nqbm1] "s"(nqbm1), [w32a] "s"(w32a), [w32b] "s"(w32b),
                 [wodd] "s"(wodd), [wave_lds] "s"(wave_lds), [kvs] "s"(kv_shift), [kvm] "s"(kv_magic),
                 [scale] "s"(scale_log2e)
               : A2SF_FWD128X2_CLOBBERS);
}

// ---------------------------------------------------------------------------------------
// Geometry as in AttnRect (n = rc.m rows, keys 0 .. off + n - 1, row i sees keys <= off + i).
// accumulate: the column sums are added to decay * S[] (a chunk: the cached tokens' older scores
// decayed by alpha^m) instead of replacing it.
template <int D>
__global__ __launch_bounds__(kThreads) void col_scores_bf16_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const float* __restrict__ LSE2,
    float* __restrict__ S, AttnRect rc, int s_stride, bool accumulate, float decay, int G, int ncb,
    int first_row, float log2_alpha, const float* __restrict__ alpha_heads, float scale_log2e) {
  constexpr int BC = kWaves * 32;  // key columns per workgroup
  constexpr int CPR = D / 8;
  constexpr int KK = D / 16;
  __shared__ uint4 qs[2][kTile * CPR];

  const long long total = (long long)G * ncb;
  const long long vid = xcd_contiguous_id(total);
  if (vid >= total) return;
  const int g = (int)(vid / ncb);
  const int cb = (int)(vid % ncb);  // column block 0 has the most rows: first
  const int n = rc.m;
  const int off = rc.off_heads ? rc.off_heads[g] : 0;
  const int nk = off + n;  // keys of this head
  const int c0 = cb * BC;
  if (off < 0 || c0 >= nk) return;
  head_window(alpha_heads, g, n, first_row, log2_alpha);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: branches on it are scalar
  const int l32 = lane & 31, h = lane >> 5;
  const bf16_t* Kg = K + (size_t)g * rc.kv_stride * D;
  const int wc0 = c0 + wave * 32;  // first key of this wave

  // K fragments (A operand): lane (key l32, half h) holds K[key][16kk + 8h .. +7]
  uint4 kf[KK];
  {
    int r = wc0 + l32;
    r = r < nk ? r : nk - 1;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) kf[kk] = load16(Kg + (size_t)r * D + kk * 16 + h * 8);
  }
  float acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;

  const int t_begin = max(max(c0 - off, first_row), 0) / kTile;   // first row tile that sees a key of the block
  const int t_end = (n + kTile - 1) / kTile;
  for (int hq = 0; hq < rc.kv_group; ++hq) {  // the query heads that share this K/V head
    const bf16_t* Qg = Q + ((size_t)g * rc.kv_group + hq) * n * D;
    const float* lse = LSE2 + ((size_t)g * rc.kv_group + hq) * n;
    Stage<D> stg;
    stg.template load<false>(Qg, nullptr, t_begin * kTile, n);
    __syncthreads();  // the previous query head's last tile has been read by every wave
    stg.template store<false>(qs[0], nullptr);
    __syncthreads();

    for (int t = t_begin; t < t_end; ++t) {
      const int buf = (t - t_begin) & 1;
      const int row0 = t * kTile;
      // the rows' log-sum-exp values are requested before the matrix ops that they follow (and
      // before the next tile's loads, so that waiting for them does not wait for those)
      float lse_r[2];
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) lse_r[qb] = lse[min(row0 + qb * 32 + l32, n - 1)];
      if (t + 1 < t_end) stg.template load<false>(Qg, nullptr, (t + 1) * kTile, n);
      if (off + row0 + kTile - 1 >= wc0) {  // some row of the tile sees a key of this wave
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          f32x16 sacc;
#pragma unroll
          for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
          for (int kk = 0; kk < KK; ++kk) {
            const uint4 b = qs[buf][row_tile_unit<D>(qb * 32 + l32, 2 * kk + h)];
            sacc = mfma_bf16(kf[kk], b, sacc);
          }
          const int r = row0 + qb * 32 + l32;
          // exponent offset of row r: -lse_r + (n-1-r) log2(alpha); rows past the end, and rows
          // whose weight is exactly 0 in fp32 (before first_row), add nothing
          const float bias = (r < n && r >= first_row)
                                 ? lse_r[qb] - (float)(n - 1 - r) * log2_alpha : INFINITY;
          const bool diag = off + row0 + qb * 32 < wc0 + 31;  // block reaches above the diagonal
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int key = wc0 + 8 * (i >> 2) + 4 * h + (i & 3);
            float p = fast_exp2(fmaf(sacc[i], scale_log2e, -bias));
            if (diag && key > off + r) p = 0.f;
            acc[i] += p;
          }
        }
      }
      if (t + 1 < t_end) stg.template store<false>(qs[buf ^ 1], nullptr);
      __syncthreads();
    }
  }
  // sum over the 32 queries (lanes with the same half)
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    acc[i] = group_sum<32>(acc[i]);
  }
  if (l32 == 0) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int key = wc0 + 8 * (i >> 2) + 4 * h + (i & 3);
      if (key < nk) {
        float* out = S + (size_t)g * s_stride + key;
        *out = accumulate ? fmaf(decay, *out, acc[i]) : acc[i];
      }
    }
  }
}

// attn_fwd_bf16_kernel for any head size and geometry
template <int D>
void launch_fwd_rect(const void* q, const void* k, const void* v, int G, const AttnRect& rc, void* o,
                     float* lse2, hipStream_t st) {
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)D);
  const int GQ = G * rc.kv_group;  // query heads
  if constexpr (D == 128) {
    // direct-to-LDS tiles and transposing LDS reads; without outputs one row block per wave
    const int nb = o ? 1 : kScoreOnlyNB;
    const int bm = kWaves * 32 * nb;
    const int nqb = (rc.m + bm - 1) / bm - (o ? 0 : rc.first_row / bm);  // row blocks to compute
    const long long total = (long long)GQ * nqb;
    const unsigned grid = (unsigned)(((total + 7) / 8) * 8);
    if (o)
      hipLaunchKernelGGL((attn_fwd128_kernel<true, 1>), dim3(grid), dim3(kThreads), 0, st,
                         (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)o, lse2, rc, GQ,
                         nqb, scale_log2e);
    else
      hipLaunchKernelGGL((attn_fwd128_kernel<false, kScoreOnlyNB>), dim3(grid), dim3(kThreads), 0, st,
                         (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)nullptr, lse2,
                         rc, GQ, nqb, scale_log2e);
    return;
  }
  constexpr int NB = kFwdNB;
  constexpr int BM = kWaves * 32 * NB;
  const int nqb = (rc.m + BM - 1) / BM;
  const long long total = (long long)GQ * nqb;
  const unsigned grid = (unsigned)(((total + 7) / 8) * 8);
  if (o)
    hipLaunchKernelGGL((attn_fwd_bf16_kernel<D, NB, true>), dim3(grid), dim3(kThreads), 0, st,
                       (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)o, lse2, rc, GQ,
                       nqb, scale_log2e);
  else
    hipLaunchKernelGGL((attn_fwd_bf16_kernel<D, NB, false>), dim3(grid), dim3(kThreads), 0, st,
                       (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)nullptr, lse2,
                       rc, GQ, nqb, scale_log2e);
}

// Square geometry (a whole prompt): G K/V heads, kv_group query heads each.
template <int D>
void launch_fwd(const void* q, const void* k, const void* v, int G_kv, int n, void* o, float* lse2,
                hipStream_t st, int kv_group = 1, int first_row = 0) {
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)D);
  const int G = G_kv * kv_group;  // query heads
  int kv_shift = 0;
  unsigned kv_magic = 0;
  while ((1 << kv_shift) < kv_group) ++kv_shift;
  if ((1 << kv_shift) != kv_group) {   // not a power of two: divide by multiplication
    kv_shift = 31;
    kv_magic = (unsigned)((1ull << 32) / (unsigned)kv_group) + 1u;
  }
  if constexpr (D == 128) {
    // Two query blocks per wave pay off once a workgroup streams enough key tiles to amortise
    // the start and end of a row block: from n = 2048 with one workgroup per block, from
    // n = 512 in the persistent form, which overlaps them with the neighbouring blocks.
    if (o && n % kX2Rows == 0 && (long long)G * n < (1ll << 31)) {
      const int nqb2 = n / kX2Rows;
      const long long items = (long long)G * nqb2;
      // persistent form: needs the id arithmetic of its later rounds to be shifts and an even
      // number of full rounds (two rounds together cost every workgroup the same)
      const bool persistent = (nqb2 & (nqb2 - 1)) == 0 && nqb2 <= kX2Slots &&
                              items >= 2 * 8 * kX2Slots && items < (1ll << 31);
      if (n >= kX2MinRows || (persistent && n >= kX2MinRowsPersistent)) {
        auto launch = [&](int id_base, int ids, int rounds) {
          const unsigned grid2 = rounds > 1 ? 8 * kX2Slots : (unsigned)(((ids + 7) / 8) * 8);
          hipLaunchKernelGGL(attn_fwd128x2_kernel, dim3(grid2), dim3(kThreads), 0, st,
                             (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)o, lse2, n,
                             nqb2, id_base, ids, rounds, kv_shift, kv_magic, scale_log2e);
        };
        // persistent part: an even number of full rounds; what is left over goes one workgroup
        // per row block
        const int chunk = 2 * 8 * kX2Slots;
        const int main_ids = persistent ? (int)(items / chunk) * chunk : 0;
        if (main_ids) launch(0, main_ids, main_ids / (8 * kX2Slots));
        if (items > main_ids) launch(main_ids, (int)(items - main_ids), 1);
        return;
      }
    }
    // Without outputs the pass is bound by the vector ALU as much as by the matrix cores
    // (fma + exp + add per logit against 1/16 matrix op): one 32-row block per wave at four
    // workgroups per compute unit overlaps the two better than two blocks per wave at two
    // (16384 heads of n = 2048: 11.1 ms against 12.75).
    AttnRect rc{n, n, nullptr, kv_group};
    rc.first_row = o ? 0 : first_row;
    launch_fwd_rect<D>(q, k, v, G_kv, rc, o, lse2, st);
  } else {
    launch_fwd_rect<D>(q, k, v, G_kv, AttnRect{n, n, nullptr, kv_group}, o, lse2, st);
  }
}

// ---------------------------------------------------------------------------------------
// col_scores for a short row window (alpha well below 1), d = 128.  Only rows >= first_row
// contribute (see first_contributing_row), at most kTailTiles tiles of 64 rows.  One
// workgroup per head (with few heads: per share of a head's keys) stages those Q rows in LDS
// once (direct global-to-LDS loads) and then walks over its key blocks: a wave keeps 32 keys
// as A fragments in registers (the next block's fragments are fetched while the current block
// is computed), recomputes the logit tiles against the staged Q rows, applies
// exp2(s - lse_i + (n-1-i) log2 alpha) and sums down the rows.  K is read exactly once, Q's
// window once per workgroup.
constexpr int kTailTiles = 4;
constexpr int kTailKB = 2;  // 32-key blocks per wave and step

// Row window for a relative tolerance on the scores (Section 3.3: the forgetting factor makes
// old rows' contributions go to 0).  All rows before n - W together add at most
// alpha^W / (1 - alpha) to any S_j (probabilities are <= 1), while S_j >= P[n-1, j]; so for a
// group of keys whose smallest P[n-1, j] is p_min every S_j of the group is exact to a
// relative `tol` once  alpha^W <= tol (1 - alpha) p_min.  p_min is read off the newest row,
// which a wave processes first; zmin is log2 of the probabilities a lane saw there.
struct RowWindow {
  bool on;
  float tl2, inv_l2a;
  __device__ RowWindow(float tol, float log2_alpha) {
    on = tol > 0.f && log2_alpha < 0.f;
    tl2 = on ? log2f(tol * (1.f - exp2f(log2_alpha))) : 0.f;
    inv_l2a = on ? 1.f / log2_alpha : 0.f;
  }
  // first row a wave has to process; zmin as held by the lanes `lane_last` and `lane_last + 32`
  // (the two halves of the newest row)
  __device__ __forceinline__ int first_row(int n, float zmin, int lane_last) const {
    const float z0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(zmin), lane_last));
    const float z1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(zmin), lane_last + 32));
    const float need = (tl2 + fminf(z0, z1)) * inv_l2a;   // rows needed (both factors negative)
    return need >= (float)n ? 0 : n - ((int)need + 2);
  }
};

__global__ __launch_bounds__(kThreads, 2) void col_scores_tail128_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const float* __restrict__ LSE2,
    float* __restrict__ S, AttnRect rc, int s_stride, bool accumulate, float decay, int first_row,
    float log2_alpha, const float* __restrict__ alpha_heads, float scale_log2e, float tol, int ksplit) {
  constexpr int D = 128, KK = D / 16, BC = kWaves * 32;
  __shared__ __attribute__((aligned(1024))) char smem[kTailTiles * kTileBytes];
  __shared__ __attribute__((aligned(16))) float strip[kWaves][32 * kTailKB];   // a wave's scores of one step
  lds_char* const qs = (lds_char*)smem;

  // ksplit workgroups share a head's keys (few heads with long prompts: one workgroup per head
  // would leave most of the chip idle); each stages the row window for itself
  const int g = blockIdx.x / ksplit, kpart = blockIdx.x % ksplit;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: branches on it are scalar
  const int l32 = lane & 31, h = lane >> 5;
  // n query rows; row i sees keys 0 .. off + i of the head's nk = off + n keys (the prompt
  // phase: off = 0; a chunk of a prompt: off = tokens cached before it)
  const int n = rc.m;
  const int off = rc.off_heads ? rc.off_heads[g] : 0;
  if (off < 0) return;  // a head the caller's precondition excludes
  const int nk = off + n;
  constexpr int STEP = BC * kTailKB;  // keys per workgroup step
  const int kspan = ((nk + ksplit * STEP - 1) / (ksplit * STEP)) * STEP;  // keys per workgroup
  const int c_begin = kpart * kspan, c_end = min(nk, c_begin + kspan);
  if (c_begin >= nk) return;
  const bf16_t* Qg = Q + (size_t)g * n * D;
  const bf16_t* Kg = K + (size_t)g * rc.kv_stride * D;
  const bf16_t* K2g = rc.k2 ? (const bf16_t*)rc.k2 + (size_t)g * n * D : nullptr;  // keys off .. from here
  const float* lse = LSE2 + (size_t)g * n;
  float* Sg = S + (size_t)g * s_stride;

  const int r_lo = (first_row / kTile) * kTile;          // first staged row (sized by the host)
  head_window(alpha_heads, g, n, first_row, log2_alpha);  // this head's own window inside it
  const int ntile = (n - r_lo + kTile - 1) / kTile;      // <= kTailTiles (checked by the host)
#pragma unroll
  for (int tt = 0; tt < kTailTiles; ++tt)
    if (tt < ntile) dma_tile<false>(Qg, r_lo + tt * kTile, n, qs + tt * kTileBytes);

  int qoff[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) qoff[kk] = l32 * 256 + (((2 * kk + h) ^ k_swizzle(l32)) << 4);
  // exponent offset of this lane's row in each 32-row block: lse_i - (n-1-i) log2 alpha;
  // +inf (probability 0) for rows past the end or before the window
  // (all loads issued before the first is used: the address is clamped, not the load skipped)
  float bias[2 * kTailTiles];
#pragma unroll
  for (int rb = 0; rb < 2 * kTailTiles; ++rb) bias[rb] = lse[min(r_lo + rb * 32 + l32, n - 1)];
#pragma unroll
  for (int rb = 0; rb < 2 * kTailTiles; ++rb) {
    const int r = r_lo + rb * 32 + l32;
    bias[rb] = (r < n && r >= first_row) ? bias[rb] - (float)(n - 1 - r) * log2_alpha : INFINITY;
  }
  // A wave owns kTailKB blocks of 32 keys at a time: every Q fragment read from LDS feeds
  // kTailKB matrix ops (one LDS kilobyte per matrix op is more than the LDS delivers).
  auto load_keys = [&](int c0, uint4 (&kf)[kTailKB][KK]) {
#pragma unroll
    for (int b = 0; b < kTailKB; ++b) {
      int r = c0 + (wave * kTailKB + b) * 32 + l32;
      r = r < nk ? r : nk - 1;
      const bf16_t* row = (K2g && r >= off) ? K2g + (size_t)(r - off) * D : Kg + (size_t)r * D;
#pragma unroll
      // (plain loads: a lane takes 32 bytes of its key's row per instruction, so every 128-byte
      // line is shared by four instructions and has to stay in the cache between them)
      for (int kk = 0; kk < KK; ++kk) kf[b][kk] = load16(row + kk * 16 + h * 8);
    }
  };
  uint4 kf[kTailKB][KK];
  load_keys(c_begin, kf);
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();

  const RowWindow win(tol, log2_alpha);
  const int rb_last = (n - 1 - r_lo) >> 5;   // the row block that holds the newest row
  const int lane_last = (n - 1 - r_lo) & 31;
  for (int c0 = c_begin; c0 < c_end; c0 += STEP) {
    const int wc0 = c0 + wave * kTailKB * 32;  // first key of this wave in this step
    int lim = max(wc0 - off, first_row);       // rows before `lim` add nothing to this wave's keys
    bool pending = c0 + STEP < c_end;          // the next step's keys still have to be fetched
    float acc[kTailKB][16];
#pragma unroll
    for (int b = 0; b < kTailKB; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;
    // newest rows first: the block of the last row tells how far back this wave has to go
#pragma unroll
    for (int rb = 2 * kTailTiles - 1; rb >= 0; --rb) {
      const int rr0 = r_lo + rb * 32;
      if (rb <= rb_last && rr0 + 31 >= lim) {  // wave-uniform
        f32x16 sacc[kTailKB];
#pragma unroll
        for (int b = 0; b < kTailKB; ++b)
#pragma unroll
          for (int i = 0; i < 16; ++i) sacc[b][i] = 0.f;
        const lds_char* qt = qs + rb * 32 * 256;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          const uint4 qf = lds_read16(qt + qoff[kk]);
#pragma unroll
          for (int b = 0; b < kTailKB; ++b) sacc[b] = mfma_bf16(kf[b][kk], qf, sacc[b]);
        }
        // last use of kf is behind us once no older row block follows
        if (pending && rb != rb_last && (rb == 0 || rr0 - 1 < lim)) {
          load_keys(c0 + STEP, kf);
          pending = false;
        }
        const int r = rr0 + l32;
        if (win.on && rb == rb_last) {   // log2 of the newest row's smallest probability, per lane
          float zmin = INFINITY;
#pragma unroll
          for (int b = 0; b < kTailKB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) zmin = fminf(zmin, fmaf(sacc[b][i], scale_log2e, -bias[rb]));
          lim = max(lim, win.first_row(n, zmin, lane_last));
        }
#pragma unroll
        for (int b = 0; b < kTailKB; ++b) {
          const int bk0 = wc0 + b * 32;
          if (bk0 + 31 > off + rr0) {  // block touches the diagonal: keys above the row contribute 0
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int key = bk0 + 8 * (i >> 2) + 4 * h + (i & 3);
              const float p = fast_exp2(fmaf(sacc[b][i], scale_log2e, -bias[rb]));
              acc[b][i] += key > off + r ? 0.f : p;
            }
          } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[b][i] += fast_exp2(fmaf(sacc[b][i], scale_log2e, -bias[rb]));
          }
        }
      }
    }
    if (pending) load_keys(c0 + STEP, kf);
    // sum over the 32 rows held by the lanes of one half; the wave's 32 * kTailKB scores go
    // through its LDS strip so that they leave as whole 16-byte pieces of one contiguous run
    // (two lanes hold them all, four consecutive keys per register quad)
#pragma unroll
    for (int b = 0; b < kTailKB; ++b) {
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[b][i] = group_sum<32>(acc[b][i]);
      if (l32 == 0) {
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4)   // keys b*32 + 8*i4 + 4h .. +3
          *reinterpret_cast<float4*>(&strip[wave][b * 32 + 8 * i4 + 4 * h]) =
              make_float4(acc[b][4 * i4], acc[b][4 * i4 + 1], acc[b][4 * i4 + 2], acc[b][4 * i4 + 3]);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __builtin_amdgcn_wave_barrier();
    if (lane < 8 * kTailKB) {
      const int key = wc0 + 4 * lane;
      float4 v = *reinterpret_cast<const float4*>(&strip[wave][4 * lane]);
      float* out = Sg + key;
      // `accumulate`: on top of `decay` times the older score (a chunk: alpha^n)
      if (key + 3 < nk && (reinterpret_cast<size_t>(out) & 15) == 0) {
        if (accumulate) {
          const float4 old = *reinterpret_cast<const float4*>(out);
          v = make_float4(fmaf(decay, old.x, v.x), fmaf(decay, old.y, v.y), fmaf(decay, old.z, v.z),
                          fmaf(decay, old.w, v.w));
        }
        *reinterpret_cast<float4*>(out) = v;
      } else {
        const float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (key + e < nk) out[e] = accumulate ? fmaf(decay, out[e], vv[e]) : vv[e];
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __builtin_amdgcn_wave_barrier();   // the strip is rewritten in the next step
  }
}

// ---------------------------------------------------------------------------------------
// col_scores for a long row window (alpha close to 1), d = 128: the streaming form of
// col_scores_tail128_kernel.  A workgroup owns 256 key columns (a wave two blocks of 32 keys,
// their K fragments resident in registers for the whole kernel) and walks down the rows that
// see them; Q tiles of 64 rows arrive by direct global-to-LDS loads in a ring of four stages,
// three tiles ahead of the one being used.  One barrier per tile publishes the tile that has
// landed and frees the stage of the previous one for the next fetch.
constexpr int kStreamStages = 4;
constexpr int kStreamKB = 2;  // 32-key blocks per wave

__global__ __launch_bounds__(kThreads, 2) void col_scores_stream128_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const float* __restrict__ LSE2,
    float* __restrict__ S, int n, int G, int ncb, int first_row, float log2_alpha,
    const float* __restrict__ alpha_heads, float scale_log2e, float tol) {
  constexpr int D = 128, KK = D / 16, BC = kWaves * 32 * kStreamKB;
  // Q tiles, then per wave and stage the 64 log-sum-exp values of the tile's rows
  __shared__ __attribute__((aligned(1024))) char smem[kStreamStages * kTileBytes + kWaves * kStreamStages * 256];
  __shared__ int wave_lim[kWaves];
  lds_char* const qs = (lds_char*)smem;

  const long long total = (long long)G * ncb;
  const long long vid = xcd_contiguous_id(total);
  if (vid >= total) return;
  const int g = (int)(vid / ncb);
  const int cb = (int)(vid % ncb);  // column block 0 has the most rows: first
  head_window(alpha_heads, g, n, first_row, log2_alpha);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: branches on it are scalar
  const int l32 = lane & 31, h = lane >> 5;
  const bf16_t* Qg = Q + (size_t)g * n * D;
  const bf16_t* Kg = K + (size_t)g * n * D;
  const float* lse = LSE2 + (size_t)g * n;
  const int c0 = cb * BC;
  const int wc0 = c0 + wave * 32 * kStreamKB;  // first key of this wave

  // Tiles are walked from the newest rows down: with a tolerance the newest row tells how far
  // back the workgroup has to go (RowWindow), and without one the order does not matter.
  const int t_last = (n + kTile - 1) / kTile - 1;
  int t_first = max(c0, first_row) / kTile;      // oldest tile any wave of the workgroup needs
  lds_char* const lse_s = qs + kStreamStages * kTileBytes +
                          __builtin_amdgcn_readfirstlane(wave) * (kStreamStages * 256);
  // Q tile t into its ring stage (every wave a quarter of the rows) and the rows' log-sum-exp
  // values into the wave's own strip of that stage: five loads per wave, always issued (a tile
  // below the window is clamped onto tile t_first and never used), so that the wait counts in
  // the loop are the same for every tile
  auto fetch = [&](int t) {
    const int stage = (t_last - t) % kStreamStages;
    const int tt = max(t, 0);
    dma_tile<false>(Qg, tt * kTile, n, qs + stage * kTileBytes);
    __builtin_amdgcn_global_load_lds((const void*)(lse + min(tt * kTile + lane, n - 1)),
                                     (__attribute__((address_space(3))) void*)(lse_s + stage * 256),
                                     4, 0, 0);
  };
  fetch(t_last);
  fetch(t_last - 1);
  fetch(t_last - 2);

  // K fragments (A operand): lane (key l32, half h) holds K[key][16kk + 8h .. +7]
  uint4 kf[kStreamKB][KK];
#pragma unroll
  for (int b = 0; b < kStreamKB; ++b) {
    int r = wc0 + b * 32 + l32;
    r = r < n ? r : n - 1;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) kf[b][kk] = load16(Kg + (size_t)r * D + kk * 16 + h * 8);
  }
  int qoff[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) qoff[kk] = l32 * 256 + (((2 * kk + h) ^ k_swizzle(l32)) << 4);
  float acc[kStreamKB][16];
#pragma unroll
  for (int b = 0; b < kStreamKB; ++b)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;

  const RowWindow win(tol, log2_alpha);
  int lim = max(wc0, first_row);   // rows before `lim` add nothing to this wave's keys
  for (int t = t_last; t >= t_first; --t) {
    // tile t has landed: of this wave's fetches only those of tiles t-1 and t-2 (five loads
    // each) may still be under way
    __builtin_amdgcn_s_waitcnt(0x0f70 | 10);  // vmcnt(10)
    __syncthreads();
    fetch(t - 3);  // into the stage of tile t+1, which every wave has left
    const int row0 = t * kTile;
    if (row0 + kTile - 1 >= lim) {  // some row of the tile counts for a key of this wave
      const int stage = (t_last - t) % kStreamStages;
      const lds_char* qt = qs + stage * kTileBytes;
      const __attribute__((address_space(3))) float* lse_t =
          (const __attribute__((address_space(3))) float*)(lse_s + stage * 256);
      float zmin[2] = {INFINITY, INFINITY};
#pragma unroll
      for (int qb = 1; qb >= 0; --qb) {
        f32x16 sacc[kStreamKB];
#pragma unroll
        for (int b = 0; b < kStreamKB; ++b)
#pragma unroll
          for (int i = 0; i < 16; ++i) sacc[b][i] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          const uint4 qf = lds_read16(qt + qb * 32 * 256 + qoff[kk]);
#pragma unroll
          for (int b = 0; b < kStreamKB; ++b) sacc[b] = mfma_bf16(kf[b][kk], qf, sacc[b]);
        }
        const int r = row0 + qb * 32 + l32;
        // exponent offset of row r: lse_r - (n-1-r) log2(alpha); rows past the end, and rows
        // whose weight is exactly 0 in fp32 (before first_row), add nothing
        const float bias = (r < n && r >= first_row)
                               ? lse_t[qb * 32 + l32] - (float)(n - 1 - r) * log2_alpha : INFINITY;
        if (win.on && t == t_last) {   // log2 of the newest row's smallest probability, per lane
          float zm = INFINITY;
#pragma unroll
          for (int b = 0; b < kStreamKB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) zm = fminf(zm, fmaf(sacc[b][i], scale_log2e, -bias));
          zmin[qb] = zm;
        }
#pragma unroll
        for (int b = 0; b < kStreamKB; ++b) {
          const int bk0 = wc0 + b * 32;
          if (bk0 + 31 > row0 + qb * 32) {  // block reaches above the diagonal
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int key = bk0 + 8 * (i >> 2) + 4 * h + (i & 3);
              const float p = fast_exp2(fmaf(sacc[b][i], scale_log2e, -bias));
              acc[b][i] += key > r ? 0.f : p;
            }
          } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[b][i] += fast_exp2(fmaf(sacc[b][i], scale_log2e, -bias));
          }
        }
      }
      if (win.on && t == t_last) {
        const int rl = n - 1 - row0;   // the newest row inside this tile
        lim = max(lim, win.first_row(n, rl >= 32 ? zmin[1] : zmin[0], rl & 31));
      }
    }
    if (win.on && t == t_last) {   // the workgroup stops at the oldest tile one of its waves needs
      if (lane == 0) wave_lim[wave] = lim;
      __syncthreads();
      const int wl = min(min(wave_lim[0], wave_lim[1]), min(wave_lim[2], wave_lim[3]));
      t_first = max(t_first, wl / kTile);
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0f70);  // tiles fetched ahead of the last one used: let them land
  // sum over the 32 rows held by the lanes of one half
#pragma unroll
  for (int b = 0; b < kStreamKB; ++b) {
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[b][i] = group_sum<32>(acc[b][i]);
    if (l32 == 0) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = wc0 + b * 32 + 8 * (i >> 2) + 4 * h + (i & 3);
        if (key < n) S[(size_t)g * n + key] = acc[b][i];
      }
    }
  }
}

// Workgroups per head of col_scores_tail128_kernel: with fewer heads than the chip takes
// workgroups (two per compute unit), a head's keys are shared out, in steps of 256 keys.
inline int tail_key_split(int G, int keys_per_head) {
  const int steps = (keys_per_head + kWaves * 32 * kTailKB - 1) / (kWaves * 32 * kTailKB);
  const int want = (512 + G - 1) / G;
  return want < 1 ? 1 : (want > steps ? steps : want);
}

// col_scores_bf16_kernel for any head size and geometry
template <int D>
void launch_cols_rect(const void* q, const void* k, const float* lse2, int G, const AttnRect& rc,
                      int keys_per_head, float alpha, const float* alpha_heads, float* scores,
                      int s_stride, bool accumulate, float decay, hipStream_t st) {
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)D);
  float l2a;
  const int first = first_contributing_row(rc.m, alpha, &l2a);
  if constexpr (D == 128) {
    // a row window of at most four tiles: staged once per head, every key streamed once
    if (bf16_two_source_ok(D, rc, alpha)) {  // (also the only score kernel that reads a second key source)
      const int ks = tail_key_split(G, keys_per_head);
      hipLaunchKernelGGL(col_scores_tail128_kernel, dim3(G * ks), dim3(kThreads), 0, st, (const bf16_t*)q,
                         (const bf16_t*)k, lse2, scores, rc, s_stride, accumulate, decay, first, l2a,
                         alpha_heads, scale_log2e, 0.f, ks);
      return;
    }
  }
  const int ncb = (keys_per_head + kWaves * 32 - 1) / (kWaves * 32);
  const long long total = (long long)G * ncb;
  const unsigned grid = (unsigned)(((total + 7) / 8) * 8);
  hipLaunchKernelGGL((col_scores_bf16_kernel<D>), dim3(grid), dim3(kThreads), 0, st, (const bf16_t*)q,
                     (const bf16_t*)k, lse2, scores, rc, s_stride, accumulate, decay, G, ncb, first, l2a,
                     alpha_heads, scale_log2e);
}

template <int D>
void launch_cols(const void* q, const void* k, const float* lse2, int G, int n, float alpha,
                 const float* alpha_heads, float tol, float* scores, hipStream_t st) {
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)D);
  float l2a;
  const int first = first_contributing_row(n, alpha, &l2a);
  if constexpr (D == 128) {
    if (n - (first / kTile) * kTile <= kTailTiles * kTile) {
      const int ks = tail_key_split(G, n);
      hipLaunchKernelGGL(col_scores_tail128_kernel, dim3(G * ks), dim3(kThreads), 0, st, (const bf16_t*)q,
                         (const bf16_t*)k, lse2, scores, AttnRect{n, n, nullptr}, n, false, 0.f, first, l2a,
                         alpha_heads, scale_log2e, tol, ks);
      return;
    }
    constexpr int BC = kWaves * 32 * kStreamKB;
    const int ncb = (n + BC - 1) / BC;
    const unsigned grid = (unsigned)((((long long)G * ncb + 7) / 8) * 8);
    hipLaunchKernelGGL(col_scores_stream128_kernel, dim3(grid), dim3(kThreads), 0, st,
                       (const bf16_t*)q, (const bf16_t*)k, lse2, scores, n, G, ncb, first, l2a,
                       alpha_heads, scale_log2e, tol);
  } else {
    launch_cols_rect<D>(q, k, lse2, G, AttnRect{n, n, nullptr}, n, alpha, alpha_heads, scores, n, false,
                        0.f, st);
  }
}

}  // namespace

bool bf16_two_source_ok(int d, const AttnRect& rc, float alpha) {
  if (d != 128 || rc.kv_group != 1) return false;
  float l2a;
  const int first = first_contributing_row(rc.m, alpha, &l2a);
  return rc.m - (first / kTile) * kTile <= kTailTiles * kTile;  // the staged-window score kernel
}

void launch_attn_bf16(const void* q, const void* k, const void* v, int G, const AttnRect& rc, int d,
                      void* o, float* lse2, hipStream_t st) {
  // a whole prompt (every head's keys are its own rows): the kernels chosen for the prompt phase
  const bool square = !rc.off_heads && !rc.k2 && rc.kv_stride == rc.m;
  if (d == 64) launch_fwd_rect<64>(q, k, v, G, rc, o, lse2, st);
  else if (square) launch_fwd<128>(q, k, v, G, rc.m, o, lse2, st, rc.kv_group, rc.first_row);
  else launch_fwd_rect<128>(q, k, v, G, rc, o, lse2, st);
}

void launch_colscores_bf16(const void* q, const void* k, const float* lse2, int G,
                           const AttnRect& rc, int keys_per_head, int d, float alpha, float* scores,
                           int s_stride, bool accumulate, float decay, hipStream_t st) {
  if (d == 64)
    launch_cols_rect<64>(q, k, lse2, G, rc, keys_per_head, alpha, nullptr, scores, s_stride, accumulate, decay, st);
  else
    launch_cols_rect<128>(q, k, lse2, G, rc, keys_per_head, alpha, nullptr, scores, s_stride, accumulate, decay, st);
}

void launch_prefill_bf16(const void* q, const void* k, const void* v, int G, int n, int d,
                         void* o, float* lse2, hipStream_t st, int first_row) {
  if (d == 64) launch_fwd<64>(q, k, v, G, n, o, lse2, st);
  else launch_fwd<128>(q, k, v, G, n, o, lse2, st, 1, first_row);
}

int bf16_first_lse_row(int n, int d, float alpha_max) {
  if (d != 128) return 0;
  float l2a;
  // every score kernel walks the row tiles from the one that holds the first contributing row
  // on (col_scores_tail128_kernel stages them, the others start their tile loop there; a tile
  // they fetch below it is never used)
  return (first_contributing_row(n, alpha_max, &l2a) / kTile) * kTile;
}

void launch_scores_bf16(const void* q, const void* k, const float* lse2, int G, int n, int d,
                        float alpha, const float* alpha_heads, float tol, float* scores,
                        hipStream_t st) {
  if (d == 64) launch_cols<64>(q, k, lse2, G, n, alpha, alpha_heads, tol, scores, st);
  else launch_cols<128>(q, k, lse2, G, n, alpha, alpha_heads, tol, scores, st);
}

}  // namespace a2sf
