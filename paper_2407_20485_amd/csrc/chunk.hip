// A prompt processed in chunks: the step that puts a chunk's K/V rows behind the tokens a head
// already caches.  (The paper evicts once per generation step, Section 3.1; a chunk of m tokens
// is m such steps with the eviction deferred to the end of the chunk, so that the rows can go
// through the matrix cores together.)  Attention of the chunk's rows over cache + chunk, the
// score update and the eviction are the general forms of the prompt-phase kernels and the
// selection / compaction kernels; only the append is specific.
#include "a2sf_dev.h"
#include "a2sf_internal.h"

namespace a2sf {
namespace {

// One workgroup per head: rows len .. len+m-1 of the cache receive the chunk's K/V rows, position
// pos0 + i and score 0; len grows by m; len_old[g] keeps the old length for the kernels that
// follow (-1 for a head without room for the chunk, which is left untouched).
// COPY_ROWS = false: positions, scores and lengths only; the kernels that follow read the
// chunk's rows from the call's inputs, and the compaction copies those that are kept.
template <int ROW_UNITS, bool COPY_ROWS>  // 16-byte units per K (or V) row
__global__ __launch_bounds__(kThreads) void chunk_append_kernel(
    const uint4* __restrict__ kin, const uint4* __restrict__ vin, int m, int pos0,
    uint4* __restrict__ K, uint4* __restrict__ V, float* __restrict__ S, int32_t* __restrict__ P,
    int32_t* __restrict__ len, int capacity, int32_t* __restrict__ len_old) {
  const int g = blockIdx.x, tid = threadIdx.x;
  const int L = len[g];
  const bool fits = L >= 0 && (long long)L + m <= capacity;
  __syncthreads();  // every thread has read len[g] before thread 0 changes it
  if (tid == 0) {
    len_old[g] = fits ? L : -1;
    if (fits) len[g] = L + m;
  }
  if (!fits) return;
  const size_t src0 = (size_t)g * m * ROW_UNITS;
  const size_t dst0 = ((size_t)g * capacity + L) * ROW_UNITS;
  const int units = m * ROW_UNITS;
  if (COPY_ROWS) {
    for (int u = tid; u < units; u += kThreads) {
      K[dst0 + u] = kin[src0 + u];
      V[dst0 + u] = vin[src0 + u];
    }
  }
  for (int i = tid; i < m; i += kThreads) {
    S[(size_t)g * capacity + L + i] = 0.f;
    P[(size_t)g * capacity + L + i] = pos0 + i;
  }
}

}  // namespace

void launch_chunk_append(const void* k, const void* v, int m, int pos0, const a2sf_cache& c,
                         int32_t* len_old, bool copy_rows, hipStream_t st) {
  const int ru = c.d * (c.dtype == A2SF_BF16 ? 2 : 4) / 16;
#define A2SF_APPEND_(RU, COPY)                                                                    \
  hipLaunchKernelGGL((chunk_append_kernel<RU, COPY>), dim3(c.G), dim3(kThreads), 0, st,           \
                     (const uint4*)k, (const uint4*)v, m, pos0, (uint4*)c.k, (uint4*)c.v,         \
                     c.scores, c.pos, c.len, c.capacity, len_old)
#define A2SF_APPEND(RU)                \
  do {                                 \
    if (copy_rows) A2SF_APPEND_(RU, true); \
    else A2SF_APPEND_(RU, false);      \
  } while (0)
  if (ru == 8) A2SF_APPEND(8);
  else if (ru == 16) A2SF_APPEND(16);
  else A2SF_APPEND(32);
#undef A2SF_APPEND
#undef A2SF_APPEND_
}

}  // namespace a2sf
