// Fused generation step: attention of one query over the retained tokens, the forgetting
// update S <- alpha*S + a (abstract and Section 3.3 of the paper) and eviction of the
// lowest-score token (Section 2.2, Section 3.1), one head per workgroup.
//
// The step is bound by the stream of cached K and V rows (Section 1: loading the KV cache
// is the memory-bandwidth bottleneck), so there is no matrix-core work here: every lane
// loads 16 bytes of a row, rows are spread over the lanes of the four waves, the logits
// and probabilities of the head live in LDS and the softmax maximum / sum go through
// wavefront shuffles.  Bytes read per head: 2*L*d*e (K and V once) + 8*L (scores).
//
// Eviction without row moves: the new token's K/V row is not written at the end of the
// cache but straight into the slot of the evicted token, so a steady-state step writes two
// rows per head.  "Recent" is decided by stored position, not by slot order.
//
// With few heads (G small) the tokens of a head are split over several workgroups
// (partial kernel writes logits, per-split max / sum / unnormalised output) and a combine
// kernel per head finishes the softmax, the score update and the eviction.  With many heads and
// short caches a single wave works on a head (decode_wave_kernel), and with several times more
// heads than the chip holds waves a wave works through several heads and holds their small
// writes back in LDS (decode_wave_loop_kernel).
//
// Grouped-query heads (R query heads share a K/V head, beyond the paper) have the same three
// forms; there a loaded row serves R logits or R output rows, the arithmetic per byte grows
// with R, and for bf16 rows of 128 elements with R >= 3 both products go to the 4x4 matrix
// instructions, whose blocks four query heads fill exactly (decode_gqa_*).
#include <math.h>

#include <algorithm>
#include <type_traits>

#include "a2sf_dev.h"
#include "a2sf_internal.h"

namespace a2sf {
namespace {

template <typename T, int D>
struct RowGeom {
  static constexpr int EPL = Elem<T>::kPerLane;   // elements per lane
  static constexpr int LPR = D / EPL;             // lanes per row
  static constexpr int RPW = kWave / LPR;         // rows per wave-wide load
};

struct StepSmem {
  unsigned long long red64[8];
  float redf[8];
  int redi[8];
  int victim;
};

// The threads that cooperate on one head: a whole workgroup, or a single wave.
struct BlockGroup {
  static constexpr int kSize = kThreads, kNW = kWaves;
  __device__ static __forceinline__ int tid() { return threadIdx.x; }
  __device__ static __forceinline__ int wave() { return threadIdx.x >> 6; }
  __device__ static __forceinline__ void sync() { __syncthreads(); }
  __device__ static __forceinline__ float max(float v, StepSmem& sm) { return block_max(v, sm.redf); }
  __device__ static __forceinline__ float sum(float v, StepSmem& sm) { return block_sum(v, sm.redf); }
  __device__ static __forceinline__ int sum_i(int v, StepSmem& sm) { return block_sum_i(v, sm.redi); }
  __device__ static __forceinline__ unsigned long long min_u64(unsigned long long v, StepSmem& sm) {
    return block_min_u64(v, sm.red64);
  }
};
struct WaveGroup {
  static constexpr int kSize = kWave, kNW = 1;
  __device__ static __forceinline__ int tid() { return threadIdx.x & 63; }
  __device__ static __forceinline__ int wave() { return 0; }
  // LDS and global accesses of one wave, made visible to its other lanes
  __device__ static __forceinline__ void sync() {
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __builtin_amdgcn_wave_barrier();
  }
  __device__ static __forceinline__ float max(float v, StepSmem&) { return wave_max(v); }
  __device__ static __forceinline__ float sum(float v, StepSmem&) { return wave_sum(v); }
  __device__ static __forceinline__ int sum_i(int v, StepSmem&) { return wave_sum_i(v); }
  __device__ static __forceinline__ unsigned long long min_u64(unsigned long long v, StepSmem&) {
    return wave_min_u64(v);
  }
};

// logits z[r] (log2 units) of rows [row_begin, row_end) into LDS z[r - z_base].
// U = 16-byte loads in flight per lane; STREAM = the cache rows carry the non-temporal hint.
template <typename Grp, int U, bool STREAM, typename T, int D>
__device__ __forceinline__ void sweep_k(const T* __restrict__ Kg, const T* __restrict__ knew,
                                        int n_old, int row_begin, int row_end,
                                        const float* qv, float* z, int z_base) {
  using Gm = RowGeom<T, D>;
  constexpr int ROWS_PER_ITER = Grp::kNW * Gm::RPW * U;
  const int lane = threadIdx.x & 63, wave = Grp::wave();
  const int sub = lane % Gm::LPR, rgrp = lane / Gm::LPR;
  for (int base = row_begin; base < row_end; base += ROWS_PER_ITER) {
    uint4 x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int r = base + (u * Grp::kNW + wave) * Gm::RPW + rgrp;
      const T* p = (r == n_old) ? knew : Kg + (size_t)(r < row_end ? r : row_begin) * D;
      x[u] = load16_as<STREAM>(p + sub * Gm::EPL);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int r = base + (u * Grp::kNW + wave) * Gm::RPW + rgrp;
      float f[Gm::EPL];
      Elem<T>::unpack(x[u], f);
      float dot = 0.f;
#pragma unroll
      for (int e = 0; e < Gm::EPL; ++e) dot = fmaf(qv[e], f[e], dot);
      dot = group_sum<Gm::LPR>(dot);
      if (sub == 0 && r < row_end) z[r - z_base] = dot;
    }
  }
}

// sum of the per-row-group partial outputs of a wave: valid in the lanes with rgrp == 0
template <typename T, int D>
__device__ __forceinline__ void v_fold_row_groups(float* acc) {
  using Gm = RowGeom<T, D>;
#pragma unroll
  for (int e = 0; e < Gm::EPL; ++e) {
    if (Gm::LPR <= 8) acc[e] += dpp_move<0x128>(acc[e]);  // row_ror:8
    acc[e] = across_rows(acc[e], OpAdd(), Gm::LPR <= 16, true);
  }
}

// acc[e] = sum_r w[r] * V[r][sub*EPL + e] over this wave's share of rows [row_begin, row_end),
// summed over the row groups of the wave: valid in the lanes with rgrp == 0.
template <typename Grp, int U, bool STREAM, typename T, int D>
__device__ __forceinline__ void sweep_v(const T* __restrict__ Vg, const T* __restrict__ vnew,
                                        int n_old, int row_begin, int row_end, const float* w,
                                        int w_base, float* acc) {
  using Gm = RowGeom<T, D>;
  constexpr int ROWS_PER_ITER = Grp::kNW * Gm::RPW * U;
  const int lane = threadIdx.x & 63, wave = Grp::wave();
  const int sub = lane % Gm::LPR, rgrp = lane / Gm::LPR;
#pragma unroll
  for (int e = 0; e < Gm::EPL; ++e) acc[e] = 0.f;
  for (int base = row_begin; base < row_end; base += ROWS_PER_ITER) {
    uint4 x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int r = base + (u * Grp::kNW + wave) * Gm::RPW + rgrp;
      const T* p = (r == n_old) ? vnew : Vg + (size_t)(r < row_end ? r : row_begin) * D;
      x[u] = load16_as<STREAM>(p + sub * Gm::EPL);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int r = base + (u * Grp::kNW + wave) * Gm::RPW + rgrp;
      const float wr = r < row_end ? w[r - w_base] : 0.f;
      float f[Gm::EPL];
      Elem<T>::unpack(x[u], f);
#pragma unroll
      for (int e = 0; e < Gm::EPL; ++e) acc[e] = fmaf(wr, f[e], acc[e]);
    }
  }
  v_fold_row_groups<T, D>(acc);
}

// Workgroup-wide sum of the per-wave partial outputs; result in part[0][0..D).
template <typename T, int D>
__device__ __forceinline__ void reduce_output(const float* acc, float (*part)[128]) {
  using Gm = RowGeom<T, D>;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % Gm::LPR, rgrp = lane / Gm::LPR;
  __syncthreads();
  if (rgrp == 0) {
#pragma unroll
    for (int e = 0; e < Gm::EPL; ++e) part[wave][sub * Gm::EPL + e] = acc[e];
  }
  __syncthreads();
  if (threadIdx.x < D) {
    const int c = threadIdx.x;
    part[0][c] = (part[0][c] + part[1][c]) + (part[2][c] + part[3][c]);
  }
  __syncthreads();
}

// K and V row `src` -> row `dst` (pointers to the rows), by the first lanes of the group.
template <typename Grp, typename T, int D>
__device__ __forceinline__ void copy_kv_row(T* kdst, const T* ksrc, T* vdst, const T* vsrc) {
  using Gm = RowGeom<T, D>;
  const int t = Grp::tid();
  if (t < Gm::LPR) store16(kdst + t * Gm::EPL, load16(ksrc + t * Gm::EPL));
  else if (t < 2 * Gm::LPR)
    store16(vdst + (t - Gm::LPR) * Gm::EPL, load16(vsrc + (t - Gm::LPR) * Gm::EPL));
}

// A head whose stored length breaks the call's precondition (0 <= len, len + 1 <= capacity) is
// left untouched; its output row is filled with NaN so that the caller can see it.
template <typename T, int D>
__device__ __forceinline__ void flag_bad_head(T* og, int tid, int nthreads) {
  for (int c = tid; c < D; c += nthreads) Elem<T>::store(og + c, __int_as_float(0x7FC00000));
}

// Stable eviction of slot v by one wave: rows v+1 .. n_old-1 of X move down one slot and the
// new token's row goes to slot n_old-1 (slot order, i.e. ascending position, is kept).  In
// place: a batch's source rows (dst + 1) are all requested before its stores, a store only
// writes rows below every source still outstanding, and the next batch reads beyond everything
// written so far.
template <typename T, int D, int U>
__device__ __forceinline__ void shift_rows_down(T* Xg, const T* xnew, int v, int n_old) {
  using Gm = RowGeom<T, D>;
  const int lane = threadIdx.x & 63;
  const int sub = lane % Gm::LPR, rgrp = lane / Gm::LPR;
  for (int base = v; base < n_old; base += Gm::RPW * U) {
    uint4 x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int src = base + u * Gm::RPW + rgrp + 1;
      const T* p = (src == n_old) ? xnew : Xg + (size_t)(src < n_old ? src : v) * D;
      x[u] = load16(p + sub * Gm::EPL);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int dst = base + u * Gm::RPW + rgrp;
      if (dst < n_old) store16(Xg + (size_t)dst * D + sub * Gm::EPL, x[u]);
    }
  }
}

__device__ __forceinline__ unsigned long long evict_key(float score, int pos) {
  // smallest key = lowest score; among equal scores the highest position
  return ((unsigned long long)ordered_key(score) << 32) | (unsigned)(0x7FFFFFFF - pos);
}

// General eviction (several tokens at once, or a cache whose newest positions have gaps).
// On entry a[0..L) in LDS holds the UPDATED scores of the L = n_old+1 tokens; slot n_old is
// the new token, not yet stored.  Makes the new token physical, marks the `recent` largest
// positions, then evicts one token at a time, moving the last live row into the hole.
template <typename Grp, typename T, int D>
__device__ void evict_general(float* a, int n_old, int excess, T* Kg, T* Vg, float* Sg,
                              int32_t* Pg, int32_t* len_g, const T* knew, const T* vnew,
                              int t_pos, int recent, StepSmem& sm) {
  const int tid = Grp::tid();
  const int L = n_old + 1;
  for (int j = tid; j < L; j += Grp::kSize) Sg[j] = a[j];
  if (tid == 0) Pg[n_old] = t_pos;
  copy_kv_row<Grp, T, D>(Kg + (size_t)n_old * D, knew, Vg + (size_t)n_old * D, vnew);
  __threadfence_block();
  Grp::sync();
  // protected tokens get score +inf in LDS (their real score is already in Sg)
  for (int j = tid; j < L; j += Grp::kSize) {
    const int pj = Pg[j];
    int newer = 0;
    for (int i = 0; i < L; ++i) newer += Pg[i] > pj;
    if (newer < recent) a[j] = INFINITY;
  }
  Grp::sync();
  int live = L;
  for (int it = 0; it < excess; ++it) {
    unsigned long long b = ~0ull;
    for (int j = tid; j < live; j += Grp::kSize) {
      const unsigned long long key = evict_key(a[j], Pg[j]);
      b = key < b ? key : b;
    }
    if (tid == 0) sm.victim = live - 1;
    Grp::sync();
    const unsigned long long win = Grp::min_u64(b, sm);
    for (int j = tid; j < live; j += Grp::kSize)
      if (evict_key(a[j], Pg[j]) == win) sm.victim = j;
    Grp::sync();
    const int v = sm.victim, last = live - 1;
    if (v != last) {
      copy_kv_row<Grp, T, D>(Kg + (size_t)v * D, Kg + (size_t)last * D, Vg + (size_t)v * D,
                             Vg + (size_t)last * D);
      if (tid == Grp::kSize - 1) { Sg[v] = Sg[last]; Pg[v] = Pg[last]; a[v] = a[last]; }
    }
    --live;
    __threadfence_block();
    Grp::sync();
  }
  if (tid == 0) *len_g = live;
}

// The first slots a thread handles in update_and_evict (slot tid + b * kThreads): their old
// scores and positions, and one more value per slot for the caller's probability function.
// A kernel can request them long before the update needs them.
constexpr int kSlotBatch = 8;
struct SlotBatch {
  float s[kSlotBatch], aux[kSlotBatch];
  int p[kSlotBatch];
};
template <typename AuxFn>
__device__ __forceinline__ void load_slot_batch(SlotBatch& sb, AuxFn aux, const float* Sg,
                                                const int32_t* Pg, int j0, int n_old, int t_pos) {
#pragma unroll
  for (int b = 0; b < kSlotBatch; ++b) {
    const int j = j0 + b * kThreads;
    sb.s[b] = j < n_old ? Sg[j] : 0.f;
    sb.p[b] = j < n_old ? Pg[j] : t_pos;
    sb.aux[b] = j <= n_old ? aux(j) : 0.f;
  }
}

// Score update and eviction of one head by a whole workgroup.  prob(j, aux(j)) returns the
// probability of slot j (slot n_old = the new token, not yet stored in the cache); the
// updated scores are left in LDS a[0..L).  All 256 threads call this.  One pass reads the
// scores and positions (independent loads, eight per thread issued together; PRE: the first
// eight were loaded by the caller into `first`), one pass writes the scores.
template <typename T, int D, bool PRE, typename AuxFn, typename ProbFn>
__device__ void update_and_evict(AuxFn aux, ProbFn prob, const SlotBatch& first, float* a, int n_old,
                                 T* Kg, T* Vg, float* Sg, int32_t* Pg, int32_t* len_g,
                                 const T* knew, const T* vnew, int t_pos, float alpha, int select,
                                 int recent, bool evict_here, StepSmem& sm) {
  using Grp = BlockGroup;
  const int tid = threadIdx.x;
  const int L = n_old + 1;
  const int excess = evict_here ? L - (select + recent) : 0;

  // Recent window by position: in a cache that always kept its newest `recent` tokens the
  // window is exactly pos > t_pos - recent.  Verified by counting; otherwise rank by position.
  const int thr = t_pos - recent;
  int cnt = 0, best_slot = n_old;
  unsigned long long best = ~0ull;
  for (int j0 = tid; j0 < L; j0 += kThreads * kSlotBatch) {
    SlotBatch sb;
    if (PRE && j0 == tid) sb = first;
    else load_slot_batch(sb, aux, Sg, Pg, j0, n_old, t_pos);
#pragma unroll
    for (int b = 0; b < kSlotBatch; ++b) {
      const int j = j0 + b * kThreads;
      if (j < L) {
        const float s = fmaf(alpha, sb.s[b], prob(j, sb.aux[b]));  // the forgetting update
        a[j] = s;
        if (sb.p[b] > thr) {
          ++cnt;
        } else {
          const unsigned long long key = evict_key(s, sb.p[b]);
          if (key < best) { best = key; best_slot = j; }
        }
      }
    }
  }
  __syncthreads();

  if (excess <= 0) {  // room left: plain append
#pragma unroll 4
    for (int j = tid; j < L; j += kThreads) Sg[j] = a[j];
    if (tid == 0) { Pg[n_old] = t_pos; *len_g = L; }
    copy_kv_row<Grp, T, D>(Kg + (size_t)n_old * D, knew, Vg + (size_t)n_old * D, vnew);
    return;
  }
  cnt = block_sum_i(cnt, sm.redi);

  if (excess == 1 && cnt == recent) {
    // ---- steady state: one eviction, no row moves
    if (tid == 0) sm.victim = n_old;  // overwritten below by the owner of the minimum
    const unsigned long long win = block_min_u64(best, sm.red64);
    if (best == win && best != ~0ull) sm.victim = best_slot;  // keys are unique (positions are)
    __syncthreads();
    const int v = sm.victim;
    const float s_tok = a[n_old];
#pragma unroll 4
    for (int j = tid; j < n_old; j += kThreads) Sg[j] = (j == v) ? s_tok : a[j];
    if (v != n_old) {
      if (tid == kThreads - 1) Pg[v] = t_pos;
      copy_kv_row<Grp, T, D>(Kg + (size_t)v * D, knew, Vg + (size_t)v * D, vnew);
    }
    return;  // len stays n_old (= select + recent)
  }
  evict_general<Grp, T, D>(a, n_old, excess, Kg, Vg, Sg, Pg, len_g, knew, vnew, t_pos, recent, sm);
}

template <typename T, int D>
__device__ __forceinline__ void load_query(const T* qg, float scale_log2e, float* qv) {
  using Gm = RowGeom<T, D>;
  const int sub = (threadIdx.x & 63) % Gm::LPR;
  Elem<T>::unpack(load16(qg + sub * Gm::EPL), qv);
#pragma unroll
  for (int e = 0; e < Gm::EPL; ++e) qv[e] *= scale_log2e;
}

// What a kernel does when the step overfills the budget.
constexpr int kEvictNone = 0;   // nothing: the token is appended (selection / compaction kernels follow)
constexpr int kEvictInSlot = 1; // fast mode: the new token's rows go into the evicted slot
constexpr int kEvictShift = 2;  // stable mode, one-wave-per-head kernel: the slots behind the victim move down

constexpr int kBlockUnroll = 8;  // loads in flight per lane, workgroup-per-head kernels
constexpr int kWaveUnroll = 8;   // loads in flight per lane, wave-per-head kernel

// ---- one workgroup per head ---------------------------------------------------------
template <typename T, int D, bool STREAM>
__global__ __launch_bounds__(kThreads) void decode_fused_kernel(
    const T* __restrict__ q, const T* __restrict__ k_new, const T* __restrict__ v_new, int t_pos,
    T* K, T* V, float* S, int32_t* P, int32_t* len, int capacity, float alpha,
    const float* __restrict__ alpha_heads, int select, int recent, int evict_here,
    T* __restrict__ o, float scale_log2e) {
  extern __shared__ float a[];  // [capacity]
  __shared__ StepSmem sm;
  __shared__ float part[kWaves][128];
  const int g = blockIdx.x, tid = threadIdx.x;
  if (alpha_heads) alpha = alpha_heads[g];
  const int n_old = len[g];
  if (n_old < 0 || n_old >= capacity) { flag_bad_head<T, D>(o + (size_t)g * D, tid, kThreads); return; }
  const int L = n_old + 1;
  T* Kg = K + (size_t)g * capacity * D;
  T* Vg = V + (size_t)g * capacity * D;
  const T* knew = k_new + (size_t)g * D;
  const T* vnew = v_new + (size_t)g * D;

  // old scores and positions of the first slots: requested now, used after the V sweep
  const auto no_aux = [](int) { return 0.f; };
  float* Sg = S + (size_t)g * capacity;
  int32_t* Pg = P + (size_t)g * capacity;
  SlotBatch first;
  load_slot_batch(first, no_aux, Sg, Pg, tid, n_old, t_pos);

  float qv[RowGeom<T, D>::EPL];
  load_query<T, D>(q + (size_t)g * D, scale_log2e, qv);
  sweep_k<BlockGroup, kBlockUnroll, STREAM, T, D>(Kg, knew, n_old, 0, L, qv, a, 0);
  __syncthreads();

  float mx = -INFINITY;
  for (int j = tid; j < L; j += kThreads) mx = fmaxf(mx, a[j]);
  mx = block_max(mx, sm.redf);
  float sum = 0.f;
  for (int j = tid; j < L; j += kThreads) {
    const float p = exp2f(a[j] - mx);
    a[j] = p;
    sum += p;
  }
  sum = block_sum(sum, sm.redf);
  const float inv = 1.0f / sum;
  for (int j = tid; j < L; j += kThreads) a[j] *= inv;
  __syncthreads();

  float acc[RowGeom<T, D>::EPL];
  sweep_v<BlockGroup, kBlockUnroll, STREAM, T, D>(Vg, vnew, n_old, 0, L, a, 0, acc);
  reduce_output<T, D>(acc, part);
  if (tid < D) Elem<T>::store(o + (size_t)g * D + tid, part[0][tid]);

  update_and_evict<T, D, true>(no_aux, [&](int j, float) { return a[j]; }, first, a, n_old, Kg, Vg, Sg,
                               Pg, len + g, knew, vnew, t_pos, alpha, select, recent, evict_here != 0,
                               sm);
}

// ---- grouped-query heads on the 4x4 matrix instructions --------------------------------
// bf16, d = 128, R = 4 or 8 query heads per K/V head.  The wave-per-head kernel above spends
// ~20 vector instructions per row and query head on the logits (eight multiply-adds, a lane
// reduction, a masked LDS write) and eight per row and head on the output; with R >= 4 that
// arithmetic, not the row stream, sets its time.  Here both products go to the matrix pipe as
// sixteen independent 4x4 blocks per instruction, which fits four query heads exactly:
//   logits   v_mfma_f32_4x4x4_16B_bf16: block b = lane / 4 takes the 8 elements 8b .. 8b+7 of
//            4 K rows (lane 4b+i: row i, one 16-byte load = two k-steps) against the same
//            elements of the 4 queries (lane 4b+j: head j); register v of lane 4b+j then holds
//            the partial dot product of row v with head j over chunk b, and the 16 chunks are
//            summed across lanes: two halving steps that swap lane halves / odd and even rows
//            of 16 lanes between two registers (so the register count halves with each add),
//            then two rotations inside the rows of 16 lanes;
//   outputs  v_mfma_f32_4x4x1_16B_f32, an outer product per block: lane 4b+i brings the
//            probability of head i for the V row of its row group, lane 4b+j element e of its 16
//            bytes of that row; register i of lane 4b+j accumulates o[head i][8*(lane%16)+e] --
//            the layout the vector form ends in, so the fold over row groups is shared.
// Lane layouts of both instructions and of the two swaps were checked on the device against
// a host computation before this was written.
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef short bf16x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16x4_t as_bf16x4(uint32_t lo, uint32_t hi) {
  const u32x2_t t = {lo, hi};
  return __builtin_bit_cast(bf16x4_t, t);
}
// a, b -> sum over the lane pairs (l, l ^ 32): lanes < 32 get a's, lanes >= 32 get b's
__device__ __forceinline__ float fold_halves(float a, float b) {
  const u32x2_t r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// a, b -> sum over the lane pairs (l, l ^ 16): even rows of 16 lanes get a's, odd rows b's
// (of the half of the wave they are in)
__device__ __forceinline__ float fold_rows(float a, float b) {
  const u32x2_t r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// One round of a sweep in the matrix forms: load u of a lane is 16 bytes (`piece`) of row
// base + 4u + row0.  Rounds that end before the newest row take the plain addresses; the
// last ones redirect the newest row to the call's input and the rows past it to row 0
// (loaded, never used).
template <int U, bool STREAM>
__device__ __forceinline__ void gqa_request_rows(const bf16_t* rows, const bf16_t* newest, int base,
                                                 int row0, int piece, int n_old, uint4 (&x)[U]) {
  constexpr int D = 128;
  if (base + 4 * U <= n_old) {
    const bf16_t* p = rows + (size_t)(base + row0) * D + piece;
#pragma unroll
    for (int u = 0; u < U; ++u) x[u] = load16_as<STREAM>(p + (size_t)u * 4 * D);
  } else {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = base + 4 * u + row0;
      const bf16_t* p = (row == n_old) ? newest : rows + (size_t)(row < n_old ? row : 0) * D;
      x[u] = load16_as<STREAM>(p + piece);
    }
  }
}

// Logits of the 4U K rows of a round (x as requested with row0 = lane % 4, piece = 8 * (lane / 4))
// against four query heads (qb: elements 8 * (lane / 4) .. + 7 of head lane % 4).  The sum over
// the 16 blocks takes two registers and leaves one in its first two steps: the row of 16 lanes
// rho then holds, in w[c][v], K row 4 * (c + (U / 4) * rho) + v of the round, for head lane % 4
// (the same value in the four lanes of the row that share lane % 4).
template <int U>
__device__ __forceinline__ void gqa_block_logits(const uint4 (&x)[U], const uint4& qb, float scale,
                                                 float (&w)[U / 4][4]) {
  static_assert(U % 4 == 0, "the block sum halves the registers twice");
  constexpr int C = U / 4;
  f32x4_t dot[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
    dot[u] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(as_bf16x4(x[u].x, x[u].y), as_bf16x4(qb.x, qb.y), zero, 0, 0, 0);
    dot[u] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(as_bf16x4(x[u].z, x[u].w), as_bf16x4(qb.z, qb.w), dot[u], 0, 0, 0);
  }
#pragma unroll
  for (int c = 0; c < C; ++c)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const float a = fold_halves(dot[c][v], dot[c + 2 * C][v]);
      const float b = fold_halves(dot[c + C][v], dot[c + 3 * C][v]);
      float t = fold_rows(a, b);
      t += dpp_move<0x124>(t);  // row_ror:4
      t += dpp_move<0x128>(t);  // row_ror:8
      w[c][v] = t * scale;
    }
}

// acc[e][i] += pa * (element e of this lane's 16 bytes of a V row): lane 4b+i brings head i's
// probability of the row, register i of lane 4b+j gets o[head i][8 * (lane % 16) + e]
__device__ __forceinline__ void gqa_outer_products(const uint4& xu, float pa, f32x4_t (&acc)[8]) {
  float f[8];
  Elem<bf16_t>::unpack(xu, f);
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = __builtin_amdgcn_mfma_f32_4x4x1f32(pa, f[e], acc[e], 0, 0, 0);
}

// ---- grouped-query heads: one workgroup per K/V head, R query heads ---------------------
// The K and V rows of the head are streamed once and serve all R queries (R logits per row in
// the K sweep, R output accumulators in the V sweep); every query head has its own softmax.
// The score update adds the SUM of the R probability rows (a token is kept or evicted for the
// whole group, as Eq.1 of the paper sums over heads that share one pruning decision).
template <typename T, int D, int R, bool STREAM>
__global__ __launch_bounds__(kThreads) void decode_gqa_kernel(
    const T* __restrict__ q, const T* __restrict__ k_new, const T* __restrict__ v_new, int t_pos,
    T* K, T* V, float* S, int32_t* P, int32_t* len, int capacity, float alpha, int select,
    int recent, int evict_here, T* __restrict__ o, float scale_log2e) {
  using Gm = RowGeom<T, D>;
  constexpr int U = kBlockUnroll;
  constexpr int ROWS_PER_ITER = kWaves * Gm::RPW * U;
  extern __shared__ float a[];  // [R][capacity]: logits, then probabilities, of each query head
  __shared__ StepSmem sm;
  __shared__ float part[kWaves][128];
  const int g = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int sub = lane % Gm::LPR, rgrp = lane / Gm::LPR;
  const int n_old = len[g];
  if (n_old < 0 || n_old >= capacity) {
    for (int r = 0; r < R; ++r) flag_bad_head<T, D>(o + ((size_t)g * R + r) * D, tid, kThreads);
    return;
  }
  const int L = n_old + 1;
  T* Kg = K + (size_t)g * capacity * D;
  T* Vg = V + (size_t)g * capacity * D;
  const T* knew = k_new + (size_t)g * D;
  const T* vnew = v_new + (size_t)g * D;

  // old scores and positions of the first slots: requested now, used after the V sweep
  const auto no_aux = [](int) { return 0.f; };
  float* Sg = S + (size_t)g * capacity;
  int32_t* Pg = P + (size_t)g * capacity;
  SlotBatch first;
  load_slot_batch(first, no_aux, Sg, Pg, tid, n_old, t_pos);

  // bf16, d = 128, four or eight query heads: both products on the 4x4 matrix instructions (see
  // above; with R >= 4 the vector form is bound by its arithmetic: 640 K/V heads x 2001 slots,
  // R = 8: 228 us per step against 107 us of the same cache with ungrouped heads).  A wave takes
  // 4 * UM consecutive rows of every round of 4 * UM * kWaves.
  constexpr bool kMatrix = std::is_same<T, bf16_t>::value && D == 128 && R >= 3;   // (R = 2: the vector form is faster here, 108 against 114 us at 640 K/V heads x 2001 slots)
  constexpr int UM = 8, HB = (R + 3) / 4, MROWS = 4 * UM;   // a last block of fewer than four heads idles its other columns
  const int blk = lane >> 2, jl = lane & 3;  // matrix block, row / head inside it

  if constexpr (kMatrix) {
    uint4 qb[HB > 0 ? HB : 1];  // elements 8*blk .. 8*blk+7 of query head 4h + jl
#pragma unroll
    for (int h = 0; h < HB; ++h)
      qb[h] = load16(reinterpret_cast<const bf16_t*>(q) + ((size_t)g * R + min(4 * h + jl, R - 1)) * D + 8 * blk);
    for (int base = wave * MROWS; base < L; base += kWaves * MROWS) {
      uint4 x[UM];
      gqa_request_rows<UM, STREAM>(reinterpret_cast<const bf16_t*>(Kg), reinterpret_cast<const bf16_t*>(knew),
                                   base, jl, 8 * blk, n_old, x);
#pragma unroll
      for (int h = 0; h < HB; ++h) {
        float w[UM / 4][4];
        gqa_block_logits<UM>(x, qb[h], scale_log2e, w);
        if (sub < 4) {
#pragma unroll
          for (int c = 0; c < UM / 4; ++c)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const int row = base + UM * rgrp + 4 * c + v;
              if (row < L && 4 * h + jl < R) a[(4 * h + jl) * capacity + row] = w[c][v];
            }
        }
      }
    }
  } else {
    float qv[R][Gm::EPL];
#pragma unroll
    for (int r = 0; r < R; ++r) load_query<T, D>(q + ((size_t)g * R + r) * D, scale_log2e, qv[r]);

    // ---- K sweep: R logits per row
    for (int base = 0; base < L; base += ROWS_PER_ITER) {
      uint4 x[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int row = base + (u * kWaves + wave) * Gm::RPW + rgrp;
        const T* p = (row == n_old) ? knew : Kg + (size_t)(row < L ? row : 0) * D;
        x[u] = load16_as<STREAM>(p + sub * Gm::EPL);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int row = base + (u * kWaves + wave) * Gm::RPW + rgrp;
        float f[Gm::EPL];
        Elem<T>::unpack(x[u], f);
#pragma unroll
        for (int r = 0; r < R; ++r) {
          float dot = 0.f;
#pragma unroll
          for (int e = 0; e < Gm::EPL; ++e) dot = fmaf(qv[r][e], f[e], dot);
          dot = group_sum<Gm::LPR>(dot);
          if (sub == 0 && row < L) a[r * capacity + row] = dot;
        }
      }
    }
  }
  __syncthreads();

  // ---- R softmaxes
#pragma unroll 1
  for (int r = 0; r < R; ++r) {
    float* ar = a + r * capacity;
    float mx = -INFINITY;
    for (int j = tid; j < L; j += kThreads) mx = fmaxf(mx, ar[j]);
    mx = block_max(mx, sm.redf);
    float sum = 0.f;
    for (int j = tid; j < L; j += kThreads) {
      const float p = exp2f(ar[j] - mx);
      ar[j] = p;
      sum += p;
    }
    sum = block_sum(sum, sm.redf);
    const float inv = 1.0f / sum;
    for (int j = tid; j < L; j += kThreads) ar[j] *= inv;
  }
  __syncthreads();

  // ---- V sweep: R output rows
  if constexpr (kMatrix) {
    f32x4_t macc[HB > 0 ? HB : 1][8];  // macc[h][e][i] = o[head 4h+i][8*sub + e], this lane's row group
#pragma unroll
    for (int h = 0; h < HB; ++h)
#pragma unroll
      for (int e = 0; e < 8; ++e) macc[h][e] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    for (int base = wave * MROWS; base < L; base += kWaves * MROWS) {
      uint4 x[UM];
      gqa_request_rows<UM, STREAM>(reinterpret_cast<const bf16_t*>(Vg), reinterpret_cast<const bf16_t*>(vnew),
                                   base, rgrp, 8 * sub, n_old, x);
      float pa[UM][HB > 0 ? HB : 1];  // probability of head 4h + jl for the row of load u
#pragma unroll
      for (int u = 0; u < UM; ++u) {
        const int row = base + 4 * u + rgrp;
#pragma unroll
        for (int h = 0; h < HB; ++h) pa[u][h] = (row < L && 4 * h + jl < R) ? a[(4 * h + jl) * capacity + row] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < UM; ++u)
#pragma unroll
        for (int h = 0; h < HB; ++h) gqa_outer_products(x[u], pa[u][h], macc[h]);
    }
#pragma unroll
    for (int h = 0; h < HB; ++h)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (4 * h + i >= R) continue;
        float out[Gm::EPL];
#pragma unroll
        for (int e = 0; e < Gm::EPL; ++e) out[e] = macc[h][e < 8 ? e : 0][i];
        v_fold_row_groups<T, D>(out);
        reduce_output<T, D>(out, part);
        if (tid < D) Elem<T>::store(o + ((size_t)g * R + 4 * h + i) * D + tid, part[0][tid]);
      }
  } else {
    float acc[R][Gm::EPL];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int e = 0; e < Gm::EPL; ++e) acc[r][e] = 0.f;
    for (int base = 0; base < L; base += ROWS_PER_ITER) {
      uint4 x[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int row = base + (u * kWaves + wave) * Gm::RPW + rgrp;
        const T* p = (row == n_old) ? vnew : Vg + (size_t)(row < L ? row : 0) * D;
        x[u] = load16_as<STREAM>(p + sub * Gm::EPL);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int row = base + (u * kWaves + wave) * Gm::RPW + rgrp;
        float f[Gm::EPL];
        Elem<T>::unpack(x[u], f);
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const float wr = row < L ? a[r * capacity + row] : 0.f;
#pragma unroll
          for (int e = 0; e < Gm::EPL; ++e) acc[r][e] = fmaf(wr, f[e], acc[r][e]);
        }
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      v_fold_row_groups<T, D>(acc[r]);
      reduce_output<T, D>(acc[r], part);
      if (tid < D) Elem<T>::store(o + ((size_t)g * R + r) * D + tid, part[0][tid]);
    }
  }

  // ---- S <- alpha*S + sum of the R probability rows, eviction as for a single head
  update_and_evict<T, D, true>(
      no_aux,
      [&](int j, float) {
        float p = 0.f;
#pragma unroll
        for (int r = 0; r < R; ++r) p += a[r * capacity + j];
        return p;
      },
      first, a, n_old, Kg, Vg, Sg, Pg, len + g, knew, vnew, t_pos, alpha, select, recent,
      evict_here != 0, sm);
}

// Tail of a one-wave-per-head step: S <- alpha*S + prob on the head's slots held in registers
// (slot j = lane + 64k; slot n_old is the new token), then the eviction.  z = the wave's LDS
// strip of at least n_old + 1 floats (used by the rare general path).
// What a head's step has to write, held back in LDS (decode_wave_loop_kernel): the score row, the
// output row, and where the new token's rows go.
struct HeldStep {
  static constexpr int kOutFloats = 128;  // room for an output row of up to 512 bytes
  static constexpr int kMeta = 4;         // head, slot of the new token's rows (-1: none), scores to write, new length (-1: unchanged)
  template <int NJ>
  static constexpr int floats() { return NJ * 64 + kOutFloats + kMeta; }
};

template <typename T, int D, int NJ, bool HOLD = false>
__device__ __forceinline__ void wave_update_and_evict(const float (&s_old)[NJ], const float (&prob)[NJ],
                                                      const int (&pos)[NJ], float* z, int n_old, T* Kg,
                                                      T* Vg, float* Sg, int32_t* Pg, int32_t* len_g,
                                                      const T* knew, const T* vnew, int t_pos,
                                                      float alpha, int select, int recent,
                                                      bool evict_here, StepSmem& sm,
                                                      float* held = nullptr) {
  using Grp = WaveGroup;
  const int lane = threadIdx.x & 63;
  const int L = n_old + 1;
  // HOLD: the score row goes to held[0 .. ), the rest of the step's writes are described by
  // held[NJ*64 + kOutFloats + 1 ..] = (slot of the new rows, scores to write, new length)
  int* meta = HOLD ? reinterpret_cast<int*>(held + NJ * 64 + HeldStep::kOutFloats) : nullptr;
  float s_new[NJ];
#pragma unroll
  for (int k = 0; k < NJ; ++k) s_new[k] = fmaf(alpha, s_old[k], prob[k]);
  const int excess = evict_here ? L - (select + recent) : 0;
  if (excess <= 0) {  // room left: the new token takes slot n_old, nothing leaves
    if constexpr (HOLD) {
#pragma unroll
      for (int k = 0; k < NJ; ++k) held[lane + 64 * k] = s_new[k];
      if (lane == 0) { meta[1] = n_old; meta[2] = L; meta[3] = L; }
      return;
    }
#pragma unroll
    for (int k = 0; k < NJ; ++k) {
      const int j = lane + 64 * k;
      if (j < L) Sg[j] = s_new[k];
    }
    if (lane == 0) { Pg[n_old] = t_pos; *len_g = L; }
    copy_kv_row<Grp, T, D>(Kg + (size_t)n_old * D, knew, Vg + (size_t)n_old * D, vnew);
    return;
  }
  const int thr = t_pos - recent;
  int cnt = 0;
  unsigned long long best = ~0ull;
#pragma unroll
  for (int k = 0; k < NJ; ++k) {
    const int j = lane + 64 * k;
    if (j < L) {
      if (pos[k] > thr) {
        ++cnt;
      } else {
        const unsigned long long key = evict_key(s_new[k], pos[k]);
        best = key < best ? key : best;
      }
    }
  }
  cnt = wave_sum_i(cnt);
  if (excess == 1 && cnt == recent) {
    const unsigned long long win = wave_min_u64(best);
    int v = -1;
#pragma unroll
    for (int k = 0; k < NJ; ++k) {
      const int j = lane + 64 * k;
      if (j < L && pos[k] <= thr && evict_key(s_new[k], pos[k]) == win) v = j;
    }
    v = wave_max_i(v);
    if (v < 0) v = n_old;  // cannot happen for valid input: drop the new token rather than write out of range
    // the new token's updated score (= its probability) sits with lane n_old%64, slot n_old/64
    float s_tok = 0.f;
#pragma unroll
    for (int k = 0; k < NJ; ++k)
      if (k == n_old / 64) s_tok = s_new[k];
    s_tok = wave_broadcast(s_tok, n_old & 63);
    if constexpr (HOLD) {
#pragma unroll
      for (int k = 0; k < NJ; ++k) {
        const int j = lane + 64 * k;
        held[j] = (j == v) ? s_tok : s_new[k];
      }
      if (lane == 0) { meta[1] = v != n_old ? v : -1; meta[2] = n_old; meta[3] = -1; }
      return;
    }
    // one contiguous store of the scores; the victim's slot receives the new token's
#pragma unroll
    for (int k = 0; k < NJ; ++k) {
      const int j = lane + 64 * k;
      if (j < n_old) Sg[j] = (j == v) ? s_tok : s_new[k];
    }
    if (v != n_old) {
      if (lane == 63) Pg[v] = t_pos;
      copy_kv_row<Grp, T, D>(Kg + (size_t)v * D, knew, Vg + (size_t)v * D, vnew);
    }
    // len stays n_old (= select + recent): nothing to write
    return;
  }
  // rare: several evictions or gaps in the newest positions (written at once, also under HOLD)
  if constexpr (HOLD) {
    if (lane == 0) { meta[1] = -1; meta[2] = 0; meta[3] = -1; }
  }
#pragma unroll
  for (int k = 0; k < NJ; ++k) {
    const int j = lane + 64 * k;
    if (j < L) z[j] = s_new[k];
  }
  Grp::sync();
  evict_general<Grp, T, D>(z, n_old, excess, Kg, Vg, Sg, Pg, len_g, knew, vnew, t_pos, recent, sm);
}

// ---- one wave per head ----------------------------------------------------------------
// For many heads with short caches (capacity <= 64*NJ).  No workgroup barrier anywhere: a
// wave streams its head's K rows, keeps logits / probabilities in its own LDS strip, the
// scores and positions of its head in registers (slot j = lane + 64k), and finishes the
// softmax, the score update and the single eviction with wave shuffles only, so the four
// heads of a workgroup never wait for each other and loads of different heads overlap.
template <typename T, int D, int NJ, bool STABLE>
__global__ __launch_bounds__(kThreads) void decode_wave_kernel(
    const T* __restrict__ q, const T* __restrict__ k_new, const T* __restrict__ v_new, int t_pos,
    T* K, T* V, float* S, int32_t* P, int32_t* len, int G, int capacity, float alpha,
    const float* __restrict__ alpha_heads, int select, int recent, int evict_here,
    T* __restrict__ o, float scale_log2e) {
  using Gm = RowGeom<T, D>;
  using Grp = WaveGroup;
  __shared__ float zs[kWaves][NJ * 64];
  // scores and positions, for the slot shift of the stable mode
  __shared__ float szs[STABLE ? kWaves : 1][STABLE ? NJ * 64 : 1];
  __shared__ int pzs[STABLE ? kWaves : 1][STABLE ? NJ * 64 : 1];
  __shared__ StepSmem sms[kWaves];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = blockIdx.x * kWaves + wave;
  if (g >= G) return;
  const int n_old = len[g];
  if (n_old < 0 || n_old >= capacity) {
    flag_bad_head<T, D>(o + (size_t)g * D, lane, kWave);
    return;
  }
  const int L = n_old + 1;
  if (alpha_heads) alpha = alpha_heads[g];
  float* z = zs[wave];
  StepSmem& sm = sms[wave];
  T* Kg = K + (size_t)g * capacity * D;
  T* Vg = V + (size_t)g * capacity * D;
  float* Sg = S + (size_t)g * capacity;
  int32_t* Pg = P + (size_t)g * capacity;
  const T* knew = k_new + (size_t)g * D;
  const T* vnew = v_new + (size_t)g * D;
  const int sub = lane % Gm::LPR, rgrp = lane / Gm::LPR;

  // bookkeeping of the head, fetched up front so that it is in registers when needed
  float s_old[NJ];
  int pos[NJ];
#pragma unroll
  for (int k = 0; k < NJ; ++k) {
    const int j = lane + 64 * k;
    s_old[k] = j < n_old ? Sg[j] : 0.f;
    pos[k] = j < n_old ? Pg[j] : t_pos;
  }
  float qv[Gm::EPL];
  load_query<T, D>(q + (size_t)g * D, scale_log2e, qv);
  sweep_k<Grp, kWaveUnroll, true, T, D>(Kg, knew, n_old, 0, L, qv, z, 0);
  Grp::sync();

  float zr[NJ];
  float mx = -INFINITY;
#pragma unroll
  for (int k = 0; k < NJ; ++k) {
    const int j = lane + 64 * k;
    zr[k] = j < L ? z[j] : -INFINITY;
    mx = fmaxf(mx, zr[k]);
  }
  mx = wave_max(mx);
  float sum = 0.f;
#pragma unroll
  for (int k = 0; k < NJ; ++k) {
    zr[k] = exp2f(zr[k] - mx);  // 0 for j >= L
    sum += zr[k];
  }
  sum = wave_sum(sum);
  const float inv = 1.0f / sum;
#pragma unroll
  for (int k = 0; k < NJ; ++k) {
    zr[k] *= inv;
    const int j = lane + 64 * k;
    if (j < L) z[j] = zr[k];
  }
  Grp::sync();

  if constexpr (STABLE) {
    // Stable mode: slots stay in ascending position, so the slots behind the victim move down by
    // one and the new token takes the last one.  The victim depends on the scores only, so it is
    // chosen BEFORE the V sweep: scores, positions and K rows (re-read: the K sweep is over) are
    // shifted first, and the V rows are written one slot down as the V sweep loads them, which
    // saves reading them a second time.
    float s_new[NJ];
#pragma unroll
    for (int k = 0; k < NJ; ++k) s_new[k] = fmaf(alpha, s_old[k], zr[k]);
    const int excess = L - (select + recent);
    int v = -1;  // >= 0: the slot that is evicted
    if (excess == 1) {
      const int thr = t_pos - recent;
      int cnt = 0;
      unsigned long long best = ~0ull;
#pragma unroll
      for (int k = 0; k < NJ; ++k) {
        const int j = lane + 64 * k;
        if (j < L) {
          if (pos[k] > thr) {
            ++cnt;
          } else {
            const unsigned long long key = evict_key(s_new[k], pos[k]);
            best = key < best ? key : best;
          }
        }
      }
      cnt = wave_sum_i(cnt);
      if (cnt == recent) {
        const unsigned long long win = wave_min_u64(best);
#pragma unroll
        for (int k = 0; k < NJ; ++k) {
          const int j = lane + 64 * k;
          if (j < L && pos[k] <= thr && evict_key(s_new[k], pos[k]) == win) v = j;
        }
        v = wave_max_i(v);
      }
    }
    if (v >= 0) {
      float* sz = szs[wave];
      int* pz = pzs[wave];
#pragma unroll
      for (int k = 0; k < NJ; ++k) {
        const int j = lane + 64 * k;
        if (j < L) { sz[j] = s_new[k]; pz[j] = pos[k]; }   // slot n_old there is the new token
      }
      Grp::sync();
#pragma unroll
      for (int k = 0; k < NJ; ++k) {
        const int j = lane + 64 * k;
        if (j < n_old) {
          const int src = j < v ? j : j + 1;
          Sg[j] = sz[src];
          if (j >= v) Pg[j] = pz[src];
        }
      }
      shift_rows_down<T, D, kWaveUnroll>(Kg, knew, v, n_old);
      // len stays n_old
    } else {
      // room left, or a step the single shift cannot do (several evictions, gaps in the newest
      // positions): the token is appended; the selection and compaction kernels that follow
      // bring the head down to its budget
#pragma unroll
      for (int k = 0; k < NJ; ++k) {
        const int j = lane + 64 * k;
        if (j < L) Sg[j] = s_new[k];
      }
      if (lane == 0) { Pg[n_old] = t_pos; len[g] = L; }
      if (lane < Gm::LPR) store16(Kg + (size_t)n_old * D + lane * Gm::EPL, load16(knew + lane * Gm::EPL));
    }
    // V sweep; with a victim, every row behind it is written one slot down as it passes
    constexpr int VROWS = Gm::RPW * kWaveUnroll;
    float acc[Gm::EPL];
#pragma unroll
    for (int e = 0; e < Gm::EPL; ++e) acc[e] = 0.f;
    for (int base = 0; base < L; base += VROWS) {
      uint4 x[kWaveUnroll];
#pragma unroll
      for (int u = 0; u < kWaveUnroll; ++u) {
        const int r = base + u * Gm::RPW + rgrp;
        const T* p = (r == n_old) ? vnew : Vg + (size_t)(r < L ? r : 0) * D;
        x[u] = load16_stream(p + sub * Gm::EPL);
      }
#pragma unroll
      for (int u = 0; u < kWaveUnroll; ++u) {
        const int r = base + u * Gm::RPW + rgrp;
        const float wr = r < L ? z[r] : 0.f;
        float f[Gm::EPL];
        Elem<T>::unpack(x[u], f);
#pragma unroll
        for (int e = 0; e < Gm::EPL; ++e) acc[e] = fmaf(wr, f[e], acc[e]);
        // rows v+1 .. n_old (the new token) go to slots v .. n_old-1; without a victim the new
        // token's row goes to slot n_old
        if (v >= 0 ? (r > v && r <= n_old) : r == n_old)
          store16(Vg + (size_t)(v >= 0 ? r - 1 : r) * D + sub * Gm::EPL, x[u]);
      }
    }
    v_fold_row_groups<T, D>(acc);
    if (rgrp == 0) store16(o + (size_t)g * D + sub * Gm::EPL, pack16(acc, T()));
    return;
  }

  float acc[Gm::EPL];
  sweep_v<Grp, kWaveUnroll, true, T, D>(Vg, vnew, n_old, 0, L, z, 0, acc);
  if (rgrp == 0) store16(o + (size_t)g * D + sub * Gm::EPL, pack16(acc, T()));

  wave_update_and_evict<T, D, NJ>(s_old, zr, pos, z, n_old, Kg, Vg, Sg, Pg, len + g, knew, vnew, t_pos,
                                  alpha, select, recent, evict_here != kEvictNone, sm);
}

// ---- one wave per head, several heads per wave ----------------------------------------------
// The fast-mode step of decode_wave_kernel for launches with several times more heads than the
// chip holds waves.  The few small writes of a step (score row, output row, the new token's two
// rows) cost far more than their bytes when they trickle into the K/V read stream.  Here 256
// persistent workgroups of 16 waves each work through the heads; a wave holds what its heads'
// steps write in LDS and writes it out every HP heads and at the end, in bursts.  (Measured with
// the stand-alone probe of the step's memory traffic: 284 us per step with the writes in place,
// 274 us held back like this.)
constexpr int kLoopWaves = 16;
constexpr int kLoopGrid = 256;        // one workgroup per compute unit
constexpr int kLoopMinHeads = 8192;   // at least two heads per wave
template <typename T, int D, int NJ, int HP>
__global__ __launch_bounds__(kLoopWaves * 64) void decode_wave_loop_kernel(
    const T* __restrict__ q, const T* __restrict__ k_new, const T* __restrict__ v_new, int t_pos,
    T* K, T* V, float* S, int32_t* P, int32_t* len, int G, int capacity, float alpha,
    const float* __restrict__ alpha_heads, int select, int recent, T* __restrict__ o,
    float scale_log2e) {
  using Gm = RowGeom<T, D>;
  using Grp = WaveGroup;
  constexpr int NS = NJ * 64, REC = HeldStep::floats<NJ>();
  extern __shared__ __attribute__((aligned(16))) float lds[];  // [16][NS] logits | [16][HP][REC] held steps
  __shared__ StepSmem sms[kLoopWaves];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  float* z = lds + wave * NS;
  float* held0 = lds + kLoopWaves * NS + wave * HP * REC;
  StepSmem& sm = sms[wave];
  const int sub = lane % Gm::LPR, rgrp = lane / Gm::LPR;
  const int stride = gridDim.x * kLoopWaves;

  // writes out the first `cnt` held steps of this wave
  auto flush = [&](int cnt) {
    Grp::sync();
    for (int r = 0; r < cnt; ++r) {
      const float* rec = held0 + r * REC;
      const int* meta = reinterpret_cast<const int*>(rec + NS + HeldStep::kOutFloats);
      const int g = meta[0], slot = meta[1], nscores = meta[2], new_len = meta[3];
      float* Sg = S + (size_t)g * capacity;
#pragma unroll
      for (int k = 0; k < NJ; ++k) {
        const int j = lane + 64 * k;
        if (j < nscores) Sg[j] = rec[j];
      }
      if (lane < Gm::LPR)
        store16(o + (size_t)g * D + lane * Gm::EPL, *reinterpret_cast<const uint4*>(rec + NS + 4 * lane));
      if (slot >= 0) {
        T* Kg = K + (size_t)g * capacity * D;
        T* Vg = V + (size_t)g * capacity * D;
        copy_kv_row<Grp, T, D>(Kg + (size_t)slot * D, k_new + (size_t)g * D, Vg + (size_t)slot * D,
                               v_new + (size_t)g * D);
        if (lane == 63) P[(size_t)g * capacity + slot] = t_pos;
      }
      if (new_len >= 0 && lane == 0) len[g] = new_len;
    }
    Grp::sync();
  };

  int cnt = 0;
  for (int g = blockIdx.x * kLoopWaves + wave; g < G; g += stride) {
    const int n_old = len[g];
    if (n_old < 0 || n_old >= capacity) {
      flag_bad_head<T, D>(o + (size_t)g * D, lane, kWave);
      continue;
    }
    const int L = n_old + 1;
    const float alpha_g = alpha_heads ? alpha_heads[g] : alpha;
    T* Kg = K + (size_t)g * capacity * D;
    T* Vg = V + (size_t)g * capacity * D;
    float* Sg = S + (size_t)g * capacity;
    int32_t* Pg = P + (size_t)g * capacity;
    const T* knew = k_new + (size_t)g * D;
    const T* vnew = v_new + (size_t)g * D;

    float s_old[NJ];
    int pos[NJ];
#pragma unroll
    for (int k = 0; k < NJ; ++k) {
      const int j = lane + 64 * k;
      s_old[k] = j < n_old ? Sg[j] : 0.f;
      pos[k] = j < n_old ? Pg[j] : t_pos;
    }
    float qv[Gm::EPL];
    load_query<T, D>(q + (size_t)g * D, scale_log2e, qv);
    sweep_k<Grp, kWaveUnroll, true, T, D>(Kg, knew, n_old, 0, L, qv, z, 0);
    Grp::sync();

    float zr[NJ];
    float mx = -INFINITY;
#pragma unroll
    for (int k = 0; k < NJ; ++k) {
      const int j = lane + 64 * k;
      zr[k] = j < L ? z[j] : -INFINITY;
      mx = fmaxf(mx, zr[k]);
    }
    mx = wave_max(mx);
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < NJ; ++k) {
      zr[k] = exp2f(zr[k] - mx);  // 0 for j >= L
      sum += zr[k];
    }
    sum = wave_sum(sum);
    const float inv = 1.0f / sum;
#pragma unroll
    for (int k = 0; k < NJ; ++k) {
      zr[k] *= inv;
      const int j = lane + 64 * k;
      if (j < L) z[j] = zr[k];
    }
    Grp::sync();

    float acc[Gm::EPL];
    sweep_v<Grp, kWaveUnroll, true, T, D>(Vg, vnew, n_old, 0, L, z, 0, acc);
    float* rec = held0 + cnt * REC;
    if (rgrp == 0) *reinterpret_cast<uint4*>(rec + NS + 4 * sub) = pack16(acc, T());
    if (lane == 0) reinterpret_cast<int*>(rec + NS + HeldStep::kOutFloats)[0] = g;

    wave_update_and_evict<T, D, NJ, true>(s_old, zr, pos, z, n_old, Kg, Vg, Sg, Pg, len + g, knew, vnew, t_pos,
                                          alpha_g, select, recent, true, sm, rec);
    if (++cnt == HP) {
      flush(cnt);
      cnt = 0;
    }
  }
  flush(cnt);
}

// ---- grouped-query heads, one wave per K/V head ------------------------------------------
// Many K/V heads with short caches (capacity <= 64*NJ): as decode_wave_kernel, no workgroup
// barrier; a K row loaded once gives R logits, a V row R output contributions.  The R
// probability rows live in the wave's LDS strip, their sum per slot in registers.
// Registers: 160 (R = 2) and 200 (R = 4) per lane when the compiler is left alone; bounding
// them to raise the occupancy spills into the sweeps and is slower (R = 4: 182 us per step
// instead of 100 at 4096 K/V heads x 201 slots); R = 8 is held to 256, which two waves per SIMD
// need, and is faster for it (76 us instead of 99 at 2048 K/V heads).  bf16 with d = 128 and
// R = 4 or 8 runs decode_gqa_mfma_kernel below instead.
template <typename T, int D, int NJ, int R, bool STREAM>
__global__ __launch_bounds__(kThreads, R <= 4 ? 1 : 2) void decode_gqa_wave_kernel(
    const T* __restrict__ q, const T* __restrict__ k_new, const T* __restrict__ v_new, int t_pos,
    T* K, T* V, float* S, int32_t* P, int32_t* len, int G, int capacity, float alpha, int select,
    int recent, int evict_here, T* __restrict__ o, float scale_log2e) {
  using Gm = RowGeom<T, D>;
  using Grp = WaveGroup;
  constexpr int U = kWaveUnroll, ROWS = Gm::RPW * U, NS = NJ * 64;
  __shared__ float zs[kWaves][R][NS];
  __shared__ StepSmem sms[kWaves];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = blockIdx.x * kWaves + wave;
  if (g >= G) return;
  const int n_old = len[g];
  if (n_old < 0 || n_old >= capacity) {
    for (int r = 0; r < R; ++r) flag_bad_head<T, D>(o + ((size_t)g * R + r) * D, lane, kWave);
    return;
  }
  const int L = n_old + 1;
  float (*z)[NS] = zs[wave];
  T* Kg = K + (size_t)g * capacity * D;
  T* Vg = V + (size_t)g * capacity * D;
  float* Sg = S + (size_t)g * capacity;
  int32_t* Pg = P + (size_t)g * capacity;
  const T* knew = k_new + (size_t)g * D;
  const T* vnew = v_new + (size_t)g * D;
  const int sub = lane % Gm::LPR, rgrp = lane / Gm::LPR;

  float s_old[NJ];
  int pos[NJ];
#pragma unroll
  for (int k = 0; k < NJ; ++k) {
    const int j = lane + 64 * k;
    s_old[k] = j < n_old ? Sg[j] : 0.f;
    pos[k] = j < n_old ? Pg[j] : t_pos;
  }
  float qv[R][Gm::EPL];
#pragma unroll
  for (int r = 0; r < R; ++r) load_query<T, D>(q + ((size_t)g * R + r) * D, scale_log2e, qv[r]);

  // ---- K sweep: R logits per row
  for (int base = 0; base < L; base += ROWS) {
    uint4 x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = base + u * Gm::RPW + rgrp;
      const T* p = (row == n_old) ? knew : Kg + (size_t)(row < L ? row : 0) * D;
      x[u] = load16_as<STREAM>(p + sub * Gm::EPL);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = base + u * Gm::RPW + rgrp;
      float f[Gm::EPL];
      Elem<T>::unpack(x[u], f);
#pragma unroll
      for (int r = 0; r < R; ++r) {
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < Gm::EPL; ++e) dot = fmaf(qv[r][e], f[e], dot);
        dot = group_sum<Gm::LPR>(dot);
        if (sub == 0 && row < L) z[r][row] = dot;
      }
    }
  }
  Grp::sync();

  // ---- R softmaxes; psum = the group's probability of each slot
  float psum[NJ];
#pragma unroll
  for (int k = 0; k < NJ; ++k) psum[k] = 0.f;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    float zr[NJ];
    float mx = -INFINITY;
#pragma unroll
    for (int k = 0; k < NJ; ++k) {
      const int j = lane + 64 * k;
      zr[k] = j < L ? z[r][j] : -INFINITY;
      mx = fmaxf(mx, zr[k]);
    }
    mx = wave_max(mx);
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < NJ; ++k) {
      zr[k] = exp2f(zr[k] - mx);  // 0 for j >= L
      sum += zr[k];
    }
    sum = wave_sum(sum);
    const float inv = 1.0f / sum;
#pragma unroll
    for (int k = 0; k < NJ; ++k) {
      zr[k] *= inv;
      psum[k] += zr[k];
      const int j = lane + 64 * k;
      if (j < L) z[r][j] = zr[k];
    }
  }
  Grp::sync();

  // ---- V sweep: R output rows
  float acc[R][Gm::EPL];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int e = 0; e < Gm::EPL; ++e) acc[r][e] = 0.f;
  for (int base = 0; base < L; base += ROWS) {
    uint4 x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = base + u * Gm::RPW + rgrp;
      const T* p = (row == n_old) ? vnew : Vg + (size_t)(row < L ? row : 0) * D;
      x[u] = load16_as<STREAM>(p + sub * Gm::EPL);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = base + u * Gm::RPW + rgrp;
      float f[Gm::EPL];
      Elem<T>::unpack(x[u], f);
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const float wr = row < L ? z[r][row] : 0.f;
#pragma unroll
        for (int e = 0; e < Gm::EPL; ++e) acc[r][e] = fmaf(wr, f[e], acc[r][e]);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < R; ++r) {
    v_fold_row_groups<T, D>(acc[r]);
    if (rgrp == 0) store16(o + ((size_t)g * R + r) * D + sub * Gm::EPL, pack16(acc[r], T()));
  }
  Grp::sync();  // the strip's first row is reused by the rare general eviction

  wave_update_and_evict<T, D, NJ>(s_old, psum, pos, z[0], n_old, Kg, Vg, Sg, Pg, len + g, knew, vnew,
                                  t_pos, alpha, select, recent, evict_here != 0, sms[wave]);
}

// Waves per SIMD the registers are held to: four (128 registers) where that needs no spill, else
// three (two for the one form that would still spill).  Four loads of 16 bytes in flight per lane: with eight the kernel needs 136 registers
// and up, and at 16 384 query heads x 201 slots a step took 101 us (R = 4) / 50 us (R = 8)
// instead of 92 / 47.  The vector form above takes 91 / 72 us there; at four times the heads
// 348 / 301 us against 300 / 173 us here.
template <int NJ, int R, bool STREAM>
__global__ __launch_bounds__(kThreads, (R <= 4 && NJ <= 4) ? 4 : ((R > 4 && NJ == 4 && !STREAM) ? 2 : 3))
void decode_gqa_mfma_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k_new, const bf16_t* __restrict__ v_new,
    int t_pos, bf16_t* K, bf16_t* V, float* S, int32_t* P, int32_t* len, int G, int capacity,
    float alpha, int select, int recent, int evict_here, bf16_t* __restrict__ o, float scale_log2e) {
  using T = bf16_t;
  // U = loads of 16 bytes in flight per lane = row groups of four rows per round of a sweep
  constexpr int D = 128, U = 4, ROWS = 4 * U, NS = NJ * 64, ZS = NS + 4, HB = (R + 3) / 4;
  static_assert(R >= 2 && R <= 8, "one or two matrix blocks of four query heads (the last one may be partly idle)");
  static_assert(U % 4 == 0, "the block sum halves the registers twice");
  using Grp = WaveGroup;
  __shared__ __align__(16) float zs[kWaves][R][ZS];
  __shared__ StepSmem sms[kWaves];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = blockIdx.x * kWaves + wave;
  if (g >= G) return;
  const int n_old = len[g];
  if (n_old < 0 || n_old >= capacity) {
    for (int r = 0; r < R; ++r) flag_bad_head<T, D>(o + ((size_t)g * R + r) * D, lane, kWave);
    return;
  }
  const int L = n_old + 1;
  float (*z)[ZS] = zs[wave];
  T* Kg = K + (size_t)g * capacity * D;
  T* Vg = V + (size_t)g * capacity * D;
  float* Sg = S + (size_t)g * capacity;
  int32_t* Pg = P + (size_t)g * capacity;
  const T* knew = k_new + (size_t)g * D;
  const T* vnew = v_new + (size_t)g * D;
  const int blk = lane >> 2, jl = lane & 3;     // matrix block, row / head inside it
  const int sub = lane & 15, rgrp = lane >> 4;  // V sweep: 16-byte piece of a row, row group

  float s_old[NJ];
  int pos[NJ];
#pragma unroll
  for (int k = 0; k < NJ; ++k) {
    const int j = lane + 64 * k;
    s_old[k] = j < n_old ? Sg[j] : 0.f;
    pos[k] = j < n_old ? Pg[j] : t_pos;
  }
  uint4 qb[HB];  // elements 8*blk .. 8*blk+7 of query head 4h + jl
#pragma unroll
  for (int h = 0; h < HB; ++h) qb[h] = load16(q + ((size_t)g * R + min(4 * h + jl, R - 1)) * D + 8 * blk);

  // ---- K sweep
  for (int base = 0; base < L; base += ROWS) {
    uint4 x[U];
    gqa_request_rows<U, STREAM>(Kg, knew, base, jl, 8 * blk, n_old, x);
#pragma unroll
    for (int h = 0; h < HB; ++h) {
      float w[U / 4][4];
      gqa_block_logits<U>(x, qb[h], scale_log2e, w);
      // rows past L hold row 0's logits; the strip has room (base + ROWS <= NS), nobody reads them
      if (sub < 4 && 4 * h + jl < R) {
        float* zp = &z[4 * h + jl][base + U * rgrp];
#pragma unroll
        for (int c = 0; c < U / 4; ++c)
          *reinterpret_cast<float4*>(zp + 4 * c) = make_float4(w[c][0], w[c][1], w[c][2], w[c][3]);
      }
    }
  }
  Grp::sync();

  // ---- R softmaxes; psum = the group's probability of each slot.  The strip gets a 0 for
  // every slot from L on, so that the V sweep reads it without a bound.
  float psum[NJ];
#pragma unroll
  for (int k = 0; k < NJ; ++k) psum[k] = 0.f;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    float zr[NJ];
    float mx = -INFINITY;
#pragma unroll
    for (int k = 0; k < NJ; ++k) {
      const int j = lane + 64 * k;
      zr[k] = j < L ? z[r][j] : -INFINITY;
      mx = fmaxf(mx, zr[k]);
    }
    mx = wave_max(mx);
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < NJ; ++k) {
      zr[k] = exp2f(zr[k] - mx);  // 0 for j >= L
      sum += zr[k];
    }
    sum = wave_sum(sum);
    const float inv = 1.0f / sum;
#pragma unroll
    for (int k = 0; k < NJ; ++k) {
      zr[k] *= inv;
      psum[k] += zr[k];
      z[r][lane + 64 * k] = zr[k];
    }
  }
  Grp::sync();

  // ---- V sweep: acc[h][e][i] = o[head 4h+i][8*sub + e], partial over this lane's row group
  f32x4_t acc[HB][8];
#pragma unroll
  for (int h = 0; h < HB; ++h)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[h][e] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  for (int base = 0; base < L; base += ROWS) {
    uint4 x[U];
    gqa_request_rows<U, STREAM>(Vg, vnew, base, rgrp, 8 * sub, n_old, x);
    float pa[U][HB];  // probability of head 4h + jl for the row of load u
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int h = 0; h < HB; ++h) pa[u][h] = 4 * h + jl < R ? z[4 * h + jl][base + 4 * u + rgrp] : 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int h = 0; h < HB; ++h) gqa_outer_products(x[u], pa[u][h], acc[h]);
  }
#pragma unroll
  for (int h = 0; h < HB; ++h)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (4 * h + i >= R) continue;
      float out[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) out[e] = acc[h][e][i];
      v_fold_row_groups<T, D>(out);
      if (rgrp == 0) store16(o + ((size_t)g * R + 4 * h + i) * D + 8 * sub, pack16(out, T()));
    }
  Grp::sync();  // the strip's first row is reused by the rare general eviction

  wave_update_and_evict<T, D, NJ>(s_old, psum, pos, z[0], n_old, Kg, Vg, Sg, Pg, len + g, knew, vnew,
                                  t_pos, alpha, select, recent, evict_here != 0, sms[wave]);
}

// ---- split over tokens ----------------------------------------------------------------
// workspace layout (floats): z[G][capacity] | ml[G][nsplit][2] | po[G][nsplit][D]
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void decode_partial_kernel(
    const T* __restrict__ q, const T* __restrict__ k_new, const T* __restrict__ v_new,
    const T* __restrict__ K, const T* __restrict__ V, const int32_t* __restrict__ len, int capacity,
    int nsplit, int rows_per_split, float* __restrict__ zbuf, float* __restrict__ ml,
    float* __restrict__ po, float scale_log2e) {
  extern __shared__ float z[];  // [rows_per_split]
  __shared__ StepSmem sm;
  __shared__ float part[kWaves][128];
  const int g = blockIdx.x / nsplit, c = blockIdx.x % nsplit, tid = threadIdx.x;
  const int n_old = len[g];
  if (n_old < 0 || n_old >= capacity) return;
  const int L = n_old + 1;
  const int r0 = c * rows_per_split;
  const int r1 = min(L, r0 + rows_per_split);
  float* mlo = ml + ((size_t)g * nsplit + c) * 2;
  float* poo = po + ((size_t)g * nsplit + c) * D;
  if (r0 >= r1) {
    if (tid == 0) { mlo[0] = -INFINITY; mlo[1] = 0.f; }
    if (tid < D) poo[tid] = 0.f;
    return;
  }
  const T* Kg = K + (size_t)g * capacity * D;
  const T* Vg = V + (size_t)g * capacity * D;
  float qv[RowGeom<T, D>::EPL];
  load_query<T, D>(q + (size_t)g * D, scale_log2e, qv);
  sweep_k<BlockGroup, kBlockUnroll, true, T, D>(Kg, k_new + (size_t)g * D, n_old, r0, r1, qv, z, r0);
  __syncthreads();
  float mx = -INFINITY;
  for (int j = r0 + tid; j < r1; j += kThreads) {
    const float zz = z[j - r0];
    zbuf[(size_t)g * capacity + j] = zz;
    mx = fmaxf(mx, zz);
  }
  mx = block_max(mx, sm.redf);
  float sum = 0.f;
  for (int j = r0 + tid; j < r1; j += kThreads) {
    const float p = exp2f(z[j - r0] - mx);
    z[j - r0] = p;
    sum += p;
  }
  sum = block_sum(sum, sm.redf);
  float acc[RowGeom<T, D>::EPL];
  sweep_v<BlockGroup, kBlockUnroll, true, T, D>(Vg, v_new + (size_t)g * D, n_old, r0, r1, z, r0, acc);
  reduce_output<T, D>(acc, part);
  if (tid == 0) { mlo[0] = mx; mlo[1] = sum; }
  if (tid < D) poo[tid] = part[0][tid];
}

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void decode_combine_kernel(
    const T* __restrict__ k_new, const T* __restrict__ v_new, int t_pos, T* K, T* V, float* S,
    int32_t* P, int32_t* len, int capacity, int nsplit, const float* __restrict__ zbuf,
    const float* __restrict__ ml, const float* __restrict__ po, float alpha,
    const float* __restrict__ alpha_heads, int select, int recent, int evict_here,
    T* __restrict__ o) {
  extern __shared__ float a[];  // [capacity]
  __shared__ StepSmem sm;
  const int g = blockIdx.x, tid = threadIdx.x;
  if (alpha_heads) alpha = alpha_heads[g];
  const int n_old = len[g];
  if (n_old < 0 || n_old >= capacity) { flag_bad_head<T, D>(o + (size_t)g * D, tid, kThreads); return; }
  // everything the merge reads is requested at once: the per-split (max, sum), the first
  // slots' logits, scores and positions, the per-split outputs
  const float* zg = zbuf + (size_t)g * capacity;
  float* Sg = S + (size_t)g * capacity;
  int32_t* Pg = P + (size_t)g * capacity;
  const float* mlg = ml + (size_t)g * nsplit * 2;
  const float mc = tid < nsplit ? mlg[2 * tid] : -INFINITY;       // nsplit <= 64
  const float lc = tid < nsplit ? mlg[2 * tid + 1] : 0.f;
  const auto logit = [&](int j) { return zg[j]; };
  SlotBatch first;
  load_slot_batch(first, logit, Sg, Pg, tid, n_old, t_pos);
  __shared__ float wsplit[kWave];
  if (tid < kWave) {  // one lane per split, wave reductions
    const float mw = wave_max(mc);
    const float w = exp2f(mc - mw);  // 0 for empty splits
    const float sw = wave_sum(lc * w);
    wsplit[tid] = w;
    if (tid == 0) { sm.redf[6] = mw; sm.redf[7] = sw; }
  }
  __syncthreads();
  const float mx = sm.redf[6];
  const float inv = 1.0f / sm.redf[7];
  if (tid < D) {
    float acc = 0.f;
#pragma unroll 4
    for (int c = 0; c < nsplit; ++c) acc = fmaf(po[((size_t)g * nsplit + c) * D + tid], wsplit[c], acc);
    Elem<T>::store(o + (size_t)g * D + tid, acc * inv);
  }
  update_and_evict<T, D, true>(logit, [&](int, float z) { return exp2f(z - mx) * inv; }, first, a, n_old,
                               K + (size_t)g * capacity * D, V + (size_t)g * capacity * D, Sg, Pg,
                               len + g, k_new + (size_t)g * D, v_new + (size_t)g * D, t_pos, alpha,
                               select, recent, evict_here != 0, sm);
}

template <typename T, int D>
void launch_typed(const void* q, const void* k_new, const void* v_new, int t_pos,
                  const a2sf_cache& c, float alpha, const float* alpha_heads, int select,
                  int recent, bool evict_here, void* o, void* ws, const DecodePlan& plan,
                  hipStream_t st) {
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)D);
  if (plan.nsplit <= 1 && plan.loop && evict_here) {
    // several heads per wave, their small writes held back in LDS (up to 256 slots: with 512 the
    // kernel no longer fits the 128 registers that 16 waves per compute unit leave a lane)
#define A2SF_LOOP(NJ, HP)                                                                              \
  do {                                                                                                 \
    constexpr int kLds = kLoopWaves * (NJ * 64 + HP * HeldStep::floats<NJ>()) * (int)sizeof(float);    \
    static const hipError_t raised = hipFuncSetAttribute(                                              \
        (const void*)decode_wave_loop_kernel<T, D, NJ, HP>, hipFuncAttributeMaxDynamicSharedMemorySize, \
        kLds);                                                                                         \
    (void)raised;                                                                                      \
    hipLaunchKernelGGL((decode_wave_loop_kernel<T, D, NJ, HP>), dim3(kLoopGrid), dim3(kLoopWaves * 64), \
                       kLds, st, (const T*)q, (const T*)k_new, (const T*)v_new, t_pos, (T*)c.k,        \
                       (T*)c.v, c.scores, c.pos, c.len, c.G, c.capacity, alpha, alpha_heads, select,   \
                       recent, (T*)o, scale_log2e);                                                    \
  } while (0)
    if (plan.wave_slots == 2) A2SF_LOOP(2, 4);
    else A2SF_LOOP(4, 4);
#undef A2SF_LOOP
    return;
  }
  if (plan.nsplit <= 1 && plan.wave_slots > 0) {
    const dim3 grid((c.G + kWaves - 1) / kWaves);
#define A2SF_WAVE_(NJ, STABLE)                                                                        \
  hipLaunchKernelGGL((decode_wave_kernel<T, D, NJ, STABLE>), grid, dim3(kThreads), 0, st, (const T*)q, \
                     (const T*)k_new, (const T*)v_new, t_pos, (T*)c.k, (T*)c.v, c.scores, c.pos,       \
                     c.len, c.G, c.capacity, alpha, alpha_heads, select, recent,                       \
                     evict_here ? kEvictInSlot : kEvictShift, (T*)o, scale_log2e)
#define A2SF_WAVE(NJ)                       \
  do {                                      \
    if (evict_here) A2SF_WAVE_(NJ, false);  \
    else A2SF_WAVE_(NJ, true);              \
  } while (0)
    if (plan.wave_slots == 2) A2SF_WAVE(2);
    else if (plan.wave_slots == 4) A2SF_WAVE(4);
    else A2SF_WAVE(8);
#undef A2SF_WAVE
#undef A2SF_WAVE_
    return;
  }
  // the kernels that keep one float per slot in LDS may ask for more than the default 64 KB
  constexpr int kMaxLds = A2SF_MAX_CAPACITY * (int)sizeof(float);
  if (plan.nsplit <= 1) {
#define A2SF_FUSED(STREAM)                                                                          \
  do {                                                                                              \
    static const hipError_t raised = hipFuncSetAttribute(                                           \
        (const void*)decode_fused_kernel<T, D, STREAM>, hipFuncAttributeMaxDynamicSharedMemorySize, \
        kMaxLds);                                                                                   \
    (void)raised;                                                                                   \
    hipLaunchKernelGGL((decode_fused_kernel<T, D, STREAM>), dim3(c.G), dim3(kThreads),              \
                       (size_t)c.capacity * sizeof(float), st, (const T*)q, (const T*)k_new,        \
                       (const T*)v_new, t_pos, (T*)c.k, (T*)c.v, c.scores, c.pos, c.len,            \
                       c.capacity, alpha, alpha_heads, select, recent, (int)evict_here, (T*)o,      \
                       scale_log2e);                                                                \
  } while (0)
    if (plan.stream) A2SF_FUSED(true);
    else A2SF_FUSED(false);
#undef A2SF_FUSED
    return;
  }
  float* zbuf = (float*)ws;
  float* ml = zbuf + (size_t)c.G * c.capacity;
  float* po = ml + (size_t)c.G * plan.nsplit * 2;
  hipLaunchKernelGGL((decode_partial_kernel<T, D>), dim3((unsigned)c.G * plan.nsplit),
                     dim3(kThreads), (size_t)plan.rows_per_split * sizeof(float), st,
                     (const T*)q, (const T*)k_new, (const T*)v_new, (const T*)c.k,
                     (const T*)c.v, c.len, c.capacity, plan.nsplit, plan.rows_per_split, zbuf, ml,
                     po, scale_log2e);
  static const hipError_t raised = hipFuncSetAttribute(
      (const void*)decode_combine_kernel<T, D>, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds);
  (void)raised;
  hipLaunchKernelGGL((decode_combine_kernel<T, D>), dim3(c.G), dim3(kThreads),
                     (size_t)c.capacity * sizeof(float), st, (const T*)k_new, (const T*)v_new,
                     t_pos, (T*)c.k, (T*)c.v, c.scores, c.pos, c.len, c.capacity, plan.nsplit,
                     zbuf, ml, po, alpha, alpha_heads, select, recent, (int)evict_here, (T*)o);
}

// ---- grouped-query heads, tokens of a K/V head split over workgroups -------------------
// Few K/V heads with long caches (a layer of a grouped-query model at batch 1 has 8 of them):
// one workgroup per head leaves the chip idle, as in the ungrouped case.  bf16, d = 128, R = 4 or
// 8: workgroup (g, c) runs the matrix-instruction rounds over rows [c * rows_per_split, ...) for
// all R query heads, leaves their logits, per-split (max, sum) and unnormalised outputs in the
// workspace; one combine workgroup per K/V head merges the R softmaxes, writes the R outputs,
// sums the R probability rows per slot and runs the usual score update and eviction.
// workspace (floats): z[G*R][capacity] | ml[G*R][nsplit][2] | po[G*R][nsplit][128]
template <int R>
__global__ __launch_bounds__(kThreads) void decode_gqa_partial_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k_new, const bf16_t* __restrict__ v_new,
    const bf16_t* __restrict__ K, const bf16_t* __restrict__ V, const int32_t* __restrict__ len,
    int capacity, int nsplit, int rows_per_split, float* __restrict__ zbuf, float* __restrict__ ml,
    float* __restrict__ po, float scale_log2e) {
  using T = bf16_t;
  // a wave takes 16 consecutive rows of a round of 64 (the smallest split), and the workgroup
  // meets at three barriers only: a split is too short to pay for more
  constexpr int D = 128, UM = 4, HB = (R + 3) / 4, MROWS = 4 * UM;
  static_assert(R >= 2 && R <= 8, "one or two matrix blocks of four query heads");
  extern __shared__ float z[];  // [R][rows_per_split]
  __shared__ float part[kWaves][R][D];
  const int g = blockIdx.x / nsplit, c = blockIdx.x % nsplit, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int blk = lane >> 2, jl = lane & 3, sub = lane & 15, rgrp = lane >> 4;
  const int n_old = len[g];
  if (n_old < 0 || n_old >= capacity) return;
  const int L = n_old + 1;
  const int r0 = c * rows_per_split;
  const int r1 = min(L, r0 + rows_per_split);
  if (r0 >= r1) {
    for (int r = 0; r < R; ++r) {
      float* mlo = ml + (((size_t)g * R + r) * nsplit + c) * 2;
      if (tid == 0) { mlo[0] = -INFINITY; mlo[1] = 0.f; }
      if (tid < D) po[(((size_t)g * R + r) * nsplit + c) * D + tid] = 0.f;
    }
    return;
  }
  const T* Kg = K + (size_t)g * capacity * D;
  const T* Vg = V + (size_t)g * capacity * D;
  const T* knew = k_new + (size_t)g * D;
  const T* vnew = v_new + (size_t)g * D;
  uint4 qb[HB];
#pragma unroll
  for (int h = 0; h < HB; ++h) qb[h] = load16(q + ((size_t)g * R + min(4 * h + jl, R - 1)) * D + 8 * blk);

  for (int base = r0 + wave * MROWS; base < r1; base += kWaves * MROWS) {
    uint4 x[UM];
    gqa_request_rows<UM, true>(Kg, knew, base, jl, 8 * blk, n_old, x);
#pragma unroll
    for (int h = 0; h < HB; ++h) {
      float w[UM / 4][4];
      gqa_block_logits<UM>(x, qb[h], scale_log2e, w);
      if (sub < 4) {
#pragma unroll
        for (int cc = 0; cc < UM / 4; ++cc)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int row = base + UM * rgrp + 4 * cc + v;
            if (row < r1 && 4 * h + jl < R) z[(4 * h + jl) * rows_per_split + row - r0] = w[cc][v];
          }
      }
    }
  }
  __syncthreads();
  // a query head's softmax over the split is one wave's work
  for (int r = wave; r < R; r += kWaves) {
    float* zr = z + r * rows_per_split;
    float* zg = zbuf + ((size_t)g * R + r) * capacity;
    float mx = -INFINITY;
    for (int j = r0 + lane; j < r1; j += kWave) {
      const float zz = zr[j - r0];
      zg[j] = zz;
      mx = fmaxf(mx, zz);
    }
    mx = wave_max(mx);
    float sum = 0.f;
    for (int j = r0 + lane; j < r1; j += kWave) {
      const float pr = exp2f(zr[j - r0] - mx);
      zr[j - r0] = pr;
      sum += pr;
    }
    sum = wave_sum(sum);
    if (lane == 0) {
      float* mlo = ml + (((size_t)g * R + r) * nsplit + c) * 2;
      mlo[0] = mx;
      mlo[1] = sum;
    }
  }
  __syncthreads();

  f32x4_t macc[HB][8];
#pragma unroll
  for (int h = 0; h < HB; ++h)
#pragma unroll
    for (int e = 0; e < 8; ++e) macc[h][e] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  for (int base = r0 + wave * MROWS; base < r1; base += kWaves * MROWS) {
    uint4 x[UM];
    gqa_request_rows<UM, true>(Vg, vnew, base, rgrp, 8 * sub, n_old, x);
    float pa[UM][HB];
#pragma unroll
    for (int u = 0; u < UM; ++u) {
      const int row = base + 4 * u + rgrp;
#pragma unroll
      for (int h = 0; h < HB; ++h) pa[u][h] = (row < r1 && 4 * h + jl < R) ? z[(4 * h + jl) * rows_per_split + row - r0] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < UM; ++u)
#pragma unroll
      for (int h = 0; h < HB; ++h) gqa_outer_products(x[u], pa[u][h], macc[h]);
  }
  // every wave's partial outputs of all R heads side by side, then one sum over the waves
#pragma unroll
  for (int h = 0; h < HB; ++h)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (4 * h + i >= R) continue;
      float out[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) out[e] = macc[h][e][i];
      v_fold_row_groups<T, D>(out);
      if (rgrp == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) part[wave][4 * h + i][8 * sub + e] = out[e];
      }
    }
  __syncthreads();
  for (int idx = tid; idx < R * D; idx += kThreads) {
    const int r = idx / D, col = idx % D;
    po[(((size_t)g * R + r) * nsplit + c) * D + col] =
        (part[0][r][col] + part[1][r][col]) + (part[2][r][col] + part[3][r][col]);
  }
}

template <int R>
__global__ __launch_bounds__(kThreads) void decode_gqa_combine_kernel(
    const bf16_t* __restrict__ k_new, const bf16_t* __restrict__ v_new, int t_pos, bf16_t* K, bf16_t* V,
    float* S, int32_t* P, int32_t* len, int capacity, int nsplit, const float* __restrict__ zbuf,
    const float* __restrict__ ml, const float* __restrict__ po, float alpha, int select, int recent,
    int evict_here, bf16_t* __restrict__ o) {
  using T = bf16_t;
  constexpr int D = 128;
  extern __shared__ float a[];  // [capacity]: the group's summed probability of each slot
  __shared__ StepSmem sm;
  __shared__ float wsplit[R][kWave];
  __shared__ float mx_s[R], inv_s[R];
  const int g = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int n_old = len[g];
  if (n_old < 0 || n_old >= capacity) {
    for (int r = 0; r < R; ++r) flag_bad_head<T, D>(o + ((size_t)g * R + r) * D, tid, kThreads);
    return;
  }
  const int L = n_old + 1;
  float* Sg = S + (size_t)g * capacity;
  int32_t* Pg = P + (size_t)g * capacity;
  const auto no_aux = [](int) { return 0.f; };
  SlotBatch first;
  load_slot_batch(first, no_aux, Sg, Pg, tid, n_old, t_pos);
  // per query head: the splits' (max, sum) merged by one wave, one lane per split (nsplit <= 64)
  for (int r = wave; r < R; r += kWaves) {
    const float* mlg = ml + ((size_t)g * R + r) * nsplit * 2;
    const float mc = lane < nsplit ? mlg[2 * lane] : -INFINITY;
    const float lc = lane < nsplit ? mlg[2 * lane + 1] : 0.f;
    const float mw = wave_max(mc);
    const float w = exp2f(mc - mw);  // 0 for empty splits
    const float sw = wave_sum(lc * w);
    wsplit[r][lane] = w;
    if (lane == 0) { mx_s[r] = mw; inv_s[r] = 1.0f / sw; }
  }
  __syncthreads();
  {
    // a thread's R * D / kThreads outputs side by side, so that their loads are in flight together
    constexpr int PER = (R * D + kThreads - 1) / kThreads;
    float acc[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) acc[i] = 0.f;
#pragma unroll 8
    for (int c = 0; c < nsplit; ++c) {
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const int idx = min(tid + i * kThreads, R * D - 1), r = idx / D, col = idx % D;
        acc[i] = fmaf(po[(((size_t)g * R + r) * nsplit + c) * D + col], wsplit[r][c], acc[i]);
      }
    }
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int idx = tid + i * kThreads, r = idx / D, col = idx % D;
      if (idx < R * D) Elem<T>::store(o + ((size_t)g * R + r) * D + col, acc[i] * inv_s[r]);
    }
  }
  for (int j = tid; j < L; j += kThreads) {
    float p = 0.f;
#pragma unroll
    for (int r = 0; r < R; ++r) p += exp2f(zbuf[((size_t)g * R + r) * capacity + j] - mx_s[r]) * inv_s[r];
    a[j] = p;
  }
  __syncthreads();
  update_and_evict<T, D, true>(no_aux, [&](int j, float) { return a[j]; }, first, a, n_old,
                               K + (size_t)g * capacity * D, V + (size_t)g * capacity * D, Sg, Pg,
                               len + g, k_new + (size_t)g * D, v_new + (size_t)g * D, t_pos, alpha,
                               select, recent, evict_here != 0, sm);
}

// f(std::integral_constant<int, R>) for the run-time group size R = 2 .. 8
template <typename F>
void with_group(int group, F f) {
  switch (group) {
    case 2: f(std::integral_constant<int, 2>()); break;
    case 3: f(std::integral_constant<int, 3>()); break;
    case 4: f(std::integral_constant<int, 4>()); break;
    case 5: f(std::integral_constant<int, 5>()); break;
    case 6: f(std::integral_constant<int, 6>()); break;
    case 7: f(std::integral_constant<int, 7>()); break;
    default: f(std::integral_constant<int, 8>()); break;
  }
}

template <typename T, int D>
void launch_gqa_typed(const void* q, const void* k_new, const void* v_new, int t_pos,
                      const a2sf_cache& c, int group, float alpha, int select, int recent,
                      bool evict_here, void* o, void* ws, size_t ws_bytes, hipStream_t st) {
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)D);
  const size_t lds = (size_t)group * c.capacity * sizeof(float);
  const bool stream = 4.0 * c.G * c.capacity * D > 512e6;   // as in plan_decode
  constexpr bool kMatrixType = std::is_same<T, bf16_t>::value && D == 128;   // the forms on the 4x4 matrix instructions
  // Few K/V heads with long caches: tokens split over workgroups where plan_decode would split
  // the same cache with ungrouped heads, as far as the scratch memory the caller gave allows.
  if constexpr (kMatrixType) {
    const DecodePlan kv = plan_decode(c.G, c.capacity, D);
    if (group >= 2 && kv.nsplit > 1 && ws) {
      const size_t heads = (size_t)c.G * group;
      const size_t fixed = heads * c.capacity * sizeof(float);              // the logits
      const size_t per_split = heads * (2 + D) * sizeof(float);             // (max, sum) and output
      int ns = ws_bytes > fixed ? (int)std::min<size_t>((ws_bytes - fixed) / per_split, (size_t)kv.nsplit) : 0;
      if (ns >= 2) {
        int rows = (c.capacity + ns - 1) / ns;
        rows = (rows + 63) / 64 * 64;
        ns = (c.capacity + rows - 1) / rows;
        float* zbuf = (float*)ws;
        float* ml = zbuf + heads * c.capacity;
        float* po = ml + heads * ns * 2;
        const size_t lds_p = (size_t)group * rows * sizeof(float);
        const size_t lds_c = (size_t)c.capacity * sizeof(float);
        constexpr int kMaxLds = A2SF_MAX_CAPACITY * (int)sizeof(float);
        with_group(group, [&](auto rc) {
          constexpr int R = decltype(rc)::value;
          if constexpr (R >= 2) {
            static const hipError_t raised = hipFuncSetAttribute(
                (const void*)decode_gqa_combine_kernel<R>, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds);
            (void)raised;
            hipLaunchKernelGGL((decode_gqa_partial_kernel<R>), dim3((unsigned)c.G * ns), dim3(kThreads), lds_p,
                               st, (const T*)q, (const T*)k_new, (const T*)v_new, (const T*)c.k, (const T*)c.v,
                               c.len, c.capacity, ns, rows, zbuf, ml, po, scale_log2e);
            hipLaunchKernelGGL((decode_gqa_combine_kernel<R>), dim3(c.G), dim3(kThreads), lds_c, st,
                               (const T*)k_new, (const T*)v_new, t_pos, (T*)c.k, (T*)c.v, c.scores, c.pos, c.len,
                               c.capacity, ns, zbuf, ml, po, alpha, select, recent, (int)evict_here, (T*)o);
          }
        });
        return;
      }
    }
  }
  // Many K/V heads with short caches: one wave per K/V head (its strip of R probability rows
  // must fit: 4 waves x R x 64*NJ floats <= 32 KB)
  const int nj = c.capacity <= 128 ? 2 : (c.capacity <= 256 ? 4 : 8);
  if (c.G >= 1024 && c.capacity <= 512 && group * nj <= 32) {
    const dim3 grid((c.G + kWaves - 1) / kWaves);
    bool launched = false;
    with_group(group, [&](auto rc) {
      constexpr int R = decltype(rc)::value;
      auto with_nj = [&](auto f) {   // f(std::integral_constant<int, NJ>) for the forms that exist (R * NJ <= 32)
        if (nj == 2) f(std::integral_constant<int, 2>());
        else if (nj == 4) f(std::integral_constant<int, 4>());
        else if constexpr (R <= 4) f(std::integral_constant<int, 8>());
      };
      if constexpr (kMatrixType && R >= 2) {   // both products on the matrix pipe
        with_nj([&](auto njc) {
          constexpr int NJ = decltype(njc)::value;
          if (stream)
            hipLaunchKernelGGL((decode_gqa_mfma_kernel<NJ, R, true>), grid, dim3(kThreads), 0, st, (const T*)q,
                               (const T*)k_new, (const T*)v_new, t_pos, (T*)c.k, (T*)c.v, c.scores, c.pos, c.len,
                               c.G, c.capacity, alpha, select, recent, (int)evict_here, (T*)o, scale_log2e);
          else
            hipLaunchKernelGGL((decode_gqa_mfma_kernel<NJ, R, false>), grid, dim3(kThreads), 0, st, (const T*)q,
                               (const T*)k_new, (const T*)v_new, t_pos, (T*)c.k, (T*)c.v, c.scores, c.pos, c.len,
                               c.G, c.capacity, alpha, select, recent, (int)evict_here, (T*)o, scale_log2e);
          launched = true;
        });
      } else if constexpr (R == 2 || R == 4 || R == 8) {   // the vector form exists for these group sizes
        with_nj([&](auto njc) {
          constexpr int NJ = decltype(njc)::value;
          if (stream)
            hipLaunchKernelGGL((decode_gqa_wave_kernel<T, D, NJ, R, true>), grid, dim3(kThreads), 0, st,
                               (const T*)q, (const T*)k_new, (const T*)v_new, t_pos, (T*)c.k, (T*)c.v, c.scores,
                               c.pos, c.len, c.G, c.capacity, alpha, select, recent, (int)evict_here, (T*)o,
                               scale_log2e);
          else
            hipLaunchKernelGGL((decode_gqa_wave_kernel<T, D, NJ, R, false>), grid, dim3(kThreads), 0, st,
                               (const T*)q, (const T*)k_new, (const T*)v_new, t_pos, (T*)c.k, (T*)c.v, c.scores,
                               c.pos, c.len, c.G, c.capacity, alpha, select, recent, (int)evict_here, (T*)o,
                               scale_log2e);
          launched = true;
        });
      }
    });
    if (launched) return;   // other group sizes of other types take the workgroup kernel
  }
  with_group(group, [&](auto rc) {
    constexpr int R = decltype(rc)::value;
    if (stream)
      hipLaunchKernelGGL((decode_gqa_kernel<T, D, R, true>), dim3(c.G), dim3(kThreads), lds, st, (const T*)q,
                         (const T*)k_new, (const T*)v_new, t_pos, (T*)c.k, (T*)c.v, c.scores, c.pos, c.len,
                         c.capacity, alpha, select, recent, (int)evict_here, (T*)o, scale_log2e);
    else
      hipLaunchKernelGGL((decode_gqa_kernel<T, D, R, false>), dim3(c.G), dim3(kThreads), lds, st, (const T*)q,
                         (const T*)k_new, (const T*)v_new, t_pos, (T*)c.k, (T*)c.v, c.scores, c.pos, c.len,
                         c.capacity, alpha, select, recent, (int)evict_here, (T*)o, scale_log2e);
  });
}

}  // namespace

void launch_decode_gqa(const void* q, const void* k_new, const void* v_new, int t_pos,
                       const a2sf_cache& c, int group, float alpha, int select, int recent,
                       bool evict_here, void* o, void* ws, size_t ws_bytes, hipStream_t st) {
  if (c.dtype == A2SF_F32) {
    if (c.d == 64) launch_gqa_typed<float, 64>(q, k_new, v_new, t_pos, c, group, alpha, select, recent, evict_here, o, ws, ws_bytes, st);
    else launch_gqa_typed<float, 128>(q, k_new, v_new, t_pos, c, group, alpha, select, recent, evict_here, o, ws, ws_bytes, st);
  } else {
    if (c.d == 64) launch_gqa_typed<bf16_t, 64>(q, k_new, v_new, t_pos, c, group, alpha, select, recent, evict_here, o, ws, ws_bytes, st);
    else launch_gqa_typed<bf16_t, 128>(q, k_new, v_new, t_pos, c, group, alpha, select, recent, evict_here, o, ws, ws_bytes, st);
  }
}

DecodePlan plan_decode(int G, int capacity, int d) {
  DecodePlan p;
  // Token split: enough workgroups to cover the 256 compute units a few times over; a split
  // never gets fewer than 64 rows.  It costs a second kernel (the combine), which only pays
  // when one workgroup per head would leave most of the chip idle for long.  Measured GPU
  // time per step (steps replayed from a HIP graph, bf16, d = 128), one kernel / split:
  // 32 heads x 205 slots 8.1 / 8.7 us, 8 x 512 11.2 / 9.0, 128 x 512 14.7 / 12.2,
  // 64 x 1024 23.0 / 13.3, 256 x 1024 28.0 / 27.4, 320 x 410 17.0 / 18.2, 512 x 512 23.8 / 27.1,
  // 900 x 256 21.2 / 26.5, 700 x 4096 257 / 291.
  const bool one_kernel = capacity <= 256 || (G >= 256 && capacity <= 1024) || G >= 640;
  int want = one_kernel ? 1 : (1024 + G - 1) / G;
  int max_split = (capacity + 63) / 64;
  int ns = want < max_split ? want : max_split;
  if (ns < 1) ns = 1;
  if (ns > 64) ns = 64;
  int rows = (capacity + ns - 1) / ns;
  rows = (rows + 63) / 64 * 64;
  ns = (capacity + rows - 1) / rows;
  p.nsplit = ns;
  p.rows_per_split = rows;
  // Many heads with short caches: one wave per head (slots held as 64 * wave_slots registers).
  p.wave_slots = 0;
  if (ns == 1 && G >= 4096 && capacity <= 512) p.wave_slots = capacity <= 128 ? 2 : (capacity <= 256 ? 4 : 8);
  p.loop = p.wave_slots > 0 && p.wave_slots <= 4 && G >= kLoopMinHeads;
  p.wave_heads = p.loop ? (G + kLoopGrid * kLoopWaves - 1) / (kLoopGrid * kLoopWaves) : 1;
  // Cache rows carry the non-temporal hint when the K/V working set cannot stay in the 256 MB
  // last-level cache from one step to the next anyway (320 heads x 410 slots, 69 MB, resident:
  // 17.2 us per step without the hint, 20.8 with it; 16384 x 201, 1.7 GB: 317 without, 291 with).
  p.stream = 4.0 * G * capacity * d > 512e6;   // K and V rows of >= 2 bytes per element
  p.ws_bytes = ns <= 1 ? 0
                       : sizeof(float) * ((size_t)G * capacity + (size_t)G * ns * 2 + (size_t)G * ns * d);
  return p;
}

void launch_decode(const void* q, const void* k_new, const void* v_new, int t_pos,
                   const a2sf_cache& c, float alpha, const float* alpha_heads, int select,
                   int recent, bool evict_here, void* o, void* ws, const DecodePlan& plan,
                   hipStream_t st) {
  if (c.dtype == A2SF_F32) {
    if (c.d == 64) launch_typed<float, 64>(q, k_new, v_new, t_pos, c, alpha, alpha_heads, select, recent, evict_here, o, ws, plan, st);
    else launch_typed<float, 128>(q, k_new, v_new, t_pos, c, alpha, alpha_heads, select, recent, evict_here, o, ws, plan, st);
  } else {
    if (c.d == 64) launch_typed<bf16_t, 64>(q, k_new, v_new, t_pos, c, alpha, alpha_heads, select, recent, evict_here, o, ws, plan, st);
    else launch_typed<bf16_t, 128>(q, k_new, v_new, t_pos, c, alpha, alpha_heads, select, recent, evict_here, o, ws, plan, st);
  }
}

}  // namespace a2sf
