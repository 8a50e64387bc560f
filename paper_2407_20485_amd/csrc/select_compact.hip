// Per-head token selection (top-k with a protected recent window) and compaction of the
// KV cache.  Section 2.2 / Section 3.1 of the paper: the tokens with the smallest
// accumulated score leave the cache; Section 4.1: the budget has a score-selected and a
// most-recent part.  Ties go to the lower original position.
//
// One workgroup (256 threads) per head.  Selection is a radix select (four 8-bit digits,
// histograms in LDS) on order-preserving integer keys, used up to three times:
//   1. the `recent`-th largest position           -> who is in the recent window
//   2. the `select`-th largest score of the rest  -> score threshold
//   3. among scores equal to the threshold, the position below which ties are kept
// followed by an ordered emission (block prefix sum) of the surviving slot indices.
#include "a2sf_dev.h"
#include "a2sf_internal.h"

namespace a2sf {
namespace {

struct SelectSmem {
  int hist[256];
  int wave_tot[kWaves];
  uint32_t prefix;
  int k;
  int red[8];
};

// k-th largest (k >= 1) of the keys f(j).key over the j in [0, L) with f(j).valid.
// Must be reached by all 256 threads.  Requires that at least k elements are valid.
template <typename F>
__device__ uint32_t radix_kth_largest(F f, int L, int k, SelectSmem& sm) {
  const int tid = threadIdx.x;
  if (tid == 0) { sm.prefix = 0u; sm.k = k; }
  uint32_t known_mask = 0u;
  for (int shift = 24; shift >= 0; shift -= 8) {
    sm.hist[tid] = 0;
    __syncthreads();
    const uint32_t prefix = sm.prefix;
    const int kk = sm.k;
    for (int j = tid; j < L; j += kThreads) {
      uint32_t key;
      if (f(j, key) && (key & known_mask) == prefix) atomicAdd(&sm.hist[(key >> shift) & 255u], 1);
    }
    __syncthreads();
    // suffix sums: above(t) = sum of hist[b] for b > t.  Inside a wave by shuffles, then the
    // totals of the waves above: one barrier instead of a 256-wide scan through LDS.
    const int v = sm.hist[tid];
    const int lane = tid & 63, wave = tid >> 6;
    int incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int y = __shfl_down(incl, o, 64);
      if (lane + o < 64) incl += y;
    }
    if (lane == 0) sm.wave_tot[wave] = incl;
    __syncthreads();
    for (int w = wave + 1; w < kWaves; ++w) incl += sm.wave_tot[w];  // sum over b >= tid
    const int above = incl - v;
    if (above < kk && kk <= incl) {  // exactly one thread
      sm.prefix = prefix | ((uint32_t)tid << shift);
      sm.k = kk - above;
    }
    known_mask |= 255u << shift;
    __syncthreads();
  }
  const uint32_t res = sm.prefix;
  __syncthreads();
  return res;
}

__global__ __launch_bounds__(kThreads) void select_kernel(
    const float* __restrict__ scores, const int32_t* __restrict__ pos,
    const int32_t* __restrict__ len, int L, int stride, int select, int recent,
    int32_t* __restrict__ keep_idx, int32_t* __restrict__ n_keep) {
  __shared__ SelectSmem sm;
  const int g = blockIdx.x, tid = threadIdx.x;
  const int B = select + recent;
  int Lg = len ? len[g] : L;
  Lg = Lg < 0 ? 0 : (Lg > L ? L : Lg);
  const float* sc = scores + (size_t)g * stride;
  const int32_t* ps = pos ? pos + (size_t)g * stride : nullptr;
  int32_t* out = keep_idx + (size_t)g * B;

  if (Lg <= B) {
    for (int j = tid; j < Lg; j += kThreads) out[j] = j;
    if (tid == 0) n_keep[g] = Lg;
    return;
  }
  auto position = [&](int j) -> int { return ps ? ps[j] : j; };

  // 1. recent window: positions >= p_recent
  int p_recent = 0x7FFFFFFF;  // nothing is recent
  bool none_recent = true;
  if (recent > 0) {
    none_recent = false;
    if (!ps) {
      p_recent = Lg - recent;
    } else {
      uint32_t r = radix_kth_largest(
          [&](int j, uint32_t& key) { key = (uint32_t)ps[j]; return true; }, Lg, recent, sm);
      p_recent = (int)r;
    }
  }
  auto is_recent = [&](int j) -> bool { return !none_recent && position(j) >= p_recent; };

  // 2. score threshold among the others
  uint32_t key_cut = 0xFFFFFFFFu;
  int p_tie = -1;  // ties (key == key_cut) are kept when position <= p_tie
  bool any_selected = select > 0;
  if (any_selected) {
    key_cut = radix_kth_largest(
        [&](int j, uint32_t& key) { key = ordered_key(sc[j]); return !is_recent(j); }, Lg, select, sm);
    int gt = 0, eq = 0;
    for (int j = tid; j < Lg; j += kThreads) {
      if (is_recent(j)) continue;
      const uint32_t key = ordered_key(sc[j]);
      gt += key > key_cut;
      eq += key == key_cut;
    }
    gt = block_sum_i(gt, sm.red);
    __syncthreads();
    eq = block_sum_i(eq, sm.red);
    const int need = select - gt;  // 1 <= need <= eq
    if (need >= eq) {
      p_tie = 0x7FFFFFFF;
    } else {
      // need-th smallest position among the ties = need-th largest of ~position
      uint32_t r = radix_kth_largest(
          [&](int j, uint32_t& key) {
            key = ~(uint32_t)position(j);
            return !is_recent(j) && ordered_key(sc[j]) == key_cut;
          },
          Lg, need, sm);
      p_tie = (int)(~r);
    }
  }

  // 3. ordered emission
  int base = 0;
  for (int j0 = 0; j0 < Lg; j0 += kThreads) {
    const int j = j0 + tid;
    bool keep = false;
    if (j < Lg) {
      if (is_recent(j)) keep = true;
      else if (any_selected) {
        const uint32_t key = ordered_key(sc[j]);
        keep = key > key_cut || (key == key_cut && position(j) <= p_tie);
      }
    }
    const unsigned long long ballot = __ballot(keep);
    const int lane = tid & 63, wave = tid >> 6;
    const int before = __popcll(ballot & ((1ull << lane) - 1ull));
    __syncthreads();
    if (lane == 0) sm.wave_tot[wave] = __popcll(ballot);
    __syncthreads();
    int off = base;
    for (int w = 0; w < wave; ++w) off += sm.wave_tot[w];
    if (keep && off + before < B) out[off + before] = j;  // bound holds for valid input; guards bad input
    base += sm.wave_tot[0] + sm.wave_tot[1] + sm.wave_tot[2] + sm.wave_tot[3];
  }
  if (tid == 0) n_keep[g] = B;
}

// ---------------------------------------------------------------------------------------
// In-place stable compaction.  keep[] is strictly ascending, so destination r <= source
// keep[r].  Rows are processed in ascending chunks; inside a chunk every source row is in
// registers before (barrier) any destination row is written.  A later chunk's sources lie
// at or beyond its own destinations, i.e. beyond everything written so far.
// Second source (kin != null): the K/V rows of the slots from off_heads[g] on have not been
// stored in the cache yet; they are rows 0 .. m-1 of kin / vin [G, m, ...] (a chunk of a
// prompt).  Kept rows among them are copied in; they follow every kept cached row, so no
// cached row that is still to be moved lies at or behind their destinations.
template <int ROW_UNITS>  // 16-byte units per K (or V) row
__global__ __launch_bounds__(kThreads) void compact_kernel(
    uint4* __restrict__ K, uint4* __restrict__ V, float* __restrict__ S, int32_t* __restrict__ P,
    int32_t* __restrict__ len, int capacity, const int32_t* __restrict__ keep_idx, int keep_stride,
    const int32_t* __restrict__ n_keep, const uint4* __restrict__ kin, const uint4* __restrict__ vin,
    int m, const int32_t* __restrict__ off_heads) {
  constexpr int U = 4;                                  // units per thread per chunk
  constexpr int CH = kThreads * U / ROW_UNITS;          // rows per chunk
  const int g = blockIdx.x, tid = threadIdx.x;
  int nk = n_keep[g];
  nk = nk < 0 ? 0 : (nk > capacity ? capacity : nk);
  nk = nk > keep_stride ? keep_stride : nk;
  const int off = kin ? off_heads[g] : capacity;  // slots from here on live in the second source
  if (off < 0) return;                            // a head the chunk did not fit into: untouched
  // as many strictly ascending indices of valid slots as there are valid slots: the identity
  if (!kin && nk == len[g]) return;
  const uint4* king = kin ? kin + (size_t)g * m * ROW_UNITS : nullptr;
  const uint4* ving = kin ? vin + (size_t)g * m * ROW_UNITS : nullptr;
  const int32_t* keep = keep_idx + (size_t)g * keep_stride;
  uint4* Kg = K + (size_t)g * capacity * ROW_UNITS;
  uint4* Vg = V + (size_t)g * capacity * ROW_UNITS;
  float* Sg = S + (size_t)g * capacity;
  int32_t* Pg = P + (size_t)g * capacity;

  for (int r0 = 0; r0 < nk; r0 += CH) {
    uint4 kr[U], vr[U];
    int dst[U];
    bool mv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int unit = tid + u * kThreads;
      const int r = r0 + unit / ROW_UNITS, c = unit % ROW_UNITS;
      dst[u] = r * ROW_UNITS + c;
      mv[u] = false;
      if (r < nk) {
        int src = keep[r];
        src = src < 0 ? 0 : (src >= capacity ? capacity - 1 : src);
        if (src >= off) {
          const int r2 = src - off < m ? src - off : m - 1;
          mv[u] = true;
          kr[u] = king[r2 * ROW_UNITS + c];
          vr[u] = ving[r2 * ROW_UNITS + c];
        } else if (src != r) {
          mv[u] = true;
          kr[u] = Kg[src * ROW_UNITS + c];
          vr[u] = Vg[src * ROW_UNITS + c];
        }
      }
    }
    float s_val = 0.f;
    int p_val = 0;
    bool mv_s = false;
    if (tid < CH && r0 + tid < nk) {
      int src = keep[r0 + tid];
      src = src < 0 ? 0 : (src >= capacity ? capacity - 1 : src);
      if (src != r0 + tid) { mv_s = true; s_val = Sg[src]; p_val = Pg[src]; }
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (mv[u]) { Kg[dst[u]] = kr[u]; Vg[dst[u]] = vr[u]; }
    if (mv_s) { Sg[r0 + tid] = s_val; Pg[r0 + tid] = p_val; }
  }
  if (tid == 0) len[g] = nk;
}

// Out-of-place gather of surviving prompt rows.  grid = G * chunks (head-major).
template <int ROW_UNITS>
__global__ __launch_bounds__(kThreads) void gather_prompt_kernel(
    const uint4* __restrict__ Kin, const uint4* __restrict__ Vin, const float* __restrict__ Sfull,
    int n, const int32_t* __restrict__ keep_idx, int keep_stride, const int32_t* __restrict__ n_keep,
    uint4* __restrict__ K, uint4* __restrict__ V, float* __restrict__ S, int32_t* __restrict__ P,
    int32_t* __restrict__ len, int capacity, int chunks) {
  constexpr int ROWS = kThreads / ROW_UNITS;
  const int g = blockIdx.x / chunks, chunk = blockIdx.x % chunks, tid = threadIdx.x;
  const int nk = n_keep[g];
  const int r = chunk * ROWS + tid / ROW_UNITS, c = tid % ROW_UNITS;
  if (chunk == 0 && tid == 0) len[g] = nk;
  if (r >= nk || r >= capacity || r >= keep_stride) return;
  int src = keep_idx[(size_t)g * keep_stride + r];
  src = src < 0 ? 0 : (src >= n ? n - 1 : src);
  const size_t in = ((size_t)g * n + src) * ROW_UNITS + c;
  const size_t out = ((size_t)g * capacity + r) * ROW_UNITS + c;
  K[out] = Kin[in];
  V[out] = Vin[in];
  if (c == 0) {
    S[(size_t)g * capacity + r] = Sfull[(size_t)g * n + src];
    P[(size_t)g * capacity + r] = src;
  }
}

inline int row_units(int d, int dtype) { return d * (dtype == A2SF_BF16 ? 2 : 4) / 16; }

}  // namespace

void launch_select(const float* scores, const int32_t* pos, const int32_t* len, int G, int L,
                   int stride, int select, int recent, int32_t* keep_idx, int32_t* n_keep,
                   hipStream_t st) {
  hipLaunchKernelGGL(select_kernel, dim3(G), dim3(kThreads), 0, st, scores, pos, len, L, stride,
                     select, recent, keep_idx, n_keep);
}

void launch_compact(const a2sf_cache& c, const int32_t* keep_idx, int keep_stride,
                    const int32_t* n_keep, hipStream_t st, const void* k2, const void* v2, int m2,
                    const int32_t* off_heads) {
  const int ru = row_units(c.d, c.dtype);
#define A2SF_COMPACT(RU)                                                                        \
  hipLaunchKernelGGL(compact_kernel<RU>, dim3(c.G), dim3(kThreads), 0, st, (uint4*)c.k,         \
                     (uint4*)c.v, c.scores, c.pos, c.len, c.capacity, keep_idx, keep_stride,    \
                     n_keep, (const uint4*)k2, (const uint4*)v2, m2, off_heads)
  if (ru == 8) A2SF_COMPACT(8);
  else if (ru == 16) A2SF_COMPACT(16);
  else A2SF_COMPACT(32);
#undef A2SF_COMPACT
}

void launch_gather_prompt(const void* k, const void* v, const float* scores_full, int n,
                          const int32_t* keep_idx, int keep_stride, const int32_t* n_keep,
                          const a2sf_cache& c, hipStream_t st) {
  const int ru = row_units(c.d, c.dtype);
  const int rows = kThreads / ru;
  const int max_rows = keep_stride < c.capacity ? keep_stride : c.capacity;
  const int chunks = (max_rows + rows - 1) / rows;
  dim3 grid((unsigned)chunks * (unsigned)c.G);
#define A2SF_GATHER(RU)                                                                          \
  hipLaunchKernelGGL(gather_prompt_kernel<RU>, grid, dim3(kThreads), 0, st, (const uint4*)k,     \
                     (const uint4*)v, scores_full, n, keep_idx, keep_stride, n_keep, (uint4*)c.k, \
                     (uint4*)c.v, c.scores, c.pos, c.len, c.capacity, chunks)
  if (ru == 8) A2SF_GATHER(8);
  else if (ru == 16) A2SF_GATHER(16);
  else A2SF_GATHER(32);
#undef A2SF_GATHER
}

}  // namespace a2sf
