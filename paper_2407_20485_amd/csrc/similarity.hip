// Similarity of a pruning policy's attention row to the row of the Ideal mask (Section 4.3
// and Table 2 of the paper), one generation step, every head.
//
// The Ideal attends ALL tokens so far and keeps the entries of the tokens with the largest
// attention score; a pruning policy's row has entries on the tokens still in its cache and
// on the new token.  Both rows are softmaxes over their own token sets (Section 2.2: after
// pruning the denominator runs over what is left), so with u_j = exp(s_j - max) on a set the
// cosine of the two rows is  sum_{both} u_j w_j / sqrt(sum u_j^2 * sum w_j^2): the softmax
// denominators cancel.
//
// One workgroup per head.  The logits of all L = t_pos + 1 tokens are formed once (the keys
// are streamed from HBM exactly once, 16 bytes per lane) and stay in LDS (4 L bytes of dynamic
// LDS, so short rows leave room for several workgroups per CU); the Ideal's cut is an exact
// radix select over 64-bit keys (ordered logit, then lower position first), so ties need no
// special case; it stops as soon as every key that still matches is known to be kept.
#include "a2sf_dev.h"
#include "a2sf_internal.h"

namespace a2sf {
namespace {

constexpr int kSimMaxRows = A2SF_SIM_MAX_ROWS;  // 32768 logits = 128 KB of LDS

// larger key = kept first: higher logit, then lower position
__device__ __forceinline__ unsigned long long rank_key(float s, int j) {
  return ((unsigned long long)ordered_key(s) << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)j);
}

template <typename T, int D, bool STREAM>
__global__ __launch_bounds__(kThreads) void ideal_similarity_kernel(
    const T* __restrict__ Q, const T* __restrict__ Kall, int n_stride, int L,
    const int32_t* __restrict__ cache_pos, const int32_t* __restrict__ cache_len, int capacity,
    float* __restrict__ out) {
  constexpr int EPL = Elem<T>::kPerLane;  // elements per 16-byte access
  constexpr int LPR = D / EPL;            // lanes per row
  constexpr int RPW = kWave / LPR;        // rows per wave-wide load
  constexpr int U = 8;                    // loads in flight per lane
  extern __shared__ __attribute__((aligned(16))) float s[];  // L logits
  __shared__ int hist[256];
  __shared__ float redf[8];
  __shared__ unsigned long long pick[3];

  const int g = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPR, rgrp = lane / LPR;
  const T* Kg = Kall + (size_t)g * n_stride * D;

  // ---- logits of every token
  float qv[EPL];
  Elem<T>::unpack(load16(Q + (size_t)g * D + sub * EPL), qv);
  const float scale = rsqrtf((float)D);
  for (int base = 0; base < L; base += kWaves * RPW * U) {
    uint4 x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int r = base + (u * kWaves + wave) * RPW + rgrp;
      x[u] = load16_as<STREAM>(Kg + (size_t)(r < L ? r : L - 1) * D + sub * EPL);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int r = base + (u * kWaves + wave) * RPW + rgrp;
      float f[EPL], dot = 0.f;
      Elem<T>::unpack(x[u], f);
#pragma unroll
      for (int e = 0; e < EPL; ++e) dot = fmaf(qv[e], f[e], dot);
      dot = group_sum<LPR>(dot);
      if (sub == 0 && r < L) s[r] = dot * scale;
    }
  }
  __syncthreads();

  // ---- the policy's token set: its cache plus the new token (position L - 1)
  const int len = min(max(cache_len[g], 0), capacity);
  const int32_t* pg = cache_pos + (size_t)g * capacity;
  const int keep = min(len + 1, L);  // the Ideal keeps as many tokens as the policy's row has

  // ---- the Ideal's cut: the keep-th largest rank key (8 digits of 8 bits, top digit first)
  unsigned long long prefix = 0, cut = 0;
  if (keep < L) {
    int want = keep;  // rank, among the keys that match the prefix so far
    for (int shift = 56; shift >= 0; shift -= 8) {
      hist[tid] = 0;
      __syncthreads();
      const unsigned long long mask = shift == 56 ? 0ull : ~0ull << (shift + 8);
      for (int j = tid; j < L; j += kThreads) {
        const unsigned long long key = rank_key(s[j], j);
        if ((key & mask) == prefix) atomicAdd(&hist[(int)((key >> shift) & 255)], 1);
      }
      __syncthreads();
      if (tid == 0) {
        int digit = 255, above = 0;
        while (above + hist[digit] < want) above += hist[digit--];
        pick[0] = (unsigned long long)digit;
        pick[1] = (unsigned long long)above;
        pick[2] = (unsigned long long)hist[digit];
      }
      __syncthreads();
      prefix |= pick[0] << shift;
      want -= (int)pick[1];
      const bool all_kept = (int)pick[2] == want;  // every key with this prefix is kept
      __syncthreads();
      if (all_kept) break;                         // (the digits left are 0 in `prefix`)
    }
    cut = prefix;  // keys are distinct: exactly `keep` of them are >= cut
  }

  // ---- sums of squares on either set and the overlap
  float top_i = -INFINITY;
  for (int j = tid; j < L; j += kThreads) top_i = fmaxf(top_i, s[j]);
  top_i = block_max(top_i, redf);  // the largest logit is always kept
  float top_m = -INFINITY;
  for (int c = tid; c <= len; c += kThreads) {
    const int p = c < len ? pg[c] : L - 1;
    if (p >= 0 && p < L) top_m = fmaxf(top_m, s[p]);
  }
  top_m = block_max(top_m, redf);
  float qi = 0.f, qm = 0.f, dot = 0.f;
  for (int j = tid; j < L; j += kThreads) {
    if (rank_key(s[j], j) >= cut) {
      const float w = expf(s[j] - top_i);
      qi = fmaf(w, w, qi);
    }
  }
  for (int c = tid; c <= len; c += kThreads) {
    const int p = c < len ? pg[c] : L - 1;
    if (p < 0 || p >= L || (c < len && p == L - 1)) continue;  // not a token of this sequence
    const float u = expf(s[p] - top_m);
    qm = fmaf(u, u, qm);
    if (rank_key(s[p], p) >= cut) dot = fmaf(u, expf(s[p] - top_i), dot);
  }
  qi = block_sum(qi, redf);
  qm = block_sum(qm, redf);
  dot = block_sum(dot, redf);
  if (tid == 0) out[g] = dot / sqrtf(qi * qm);
}

// Mean of cos[first_step .. steps) x [0 .. G): the figure Table 2 reports (average over the
// steps past the budget and over heads).  One workgroup; fp64 accumulation, fixed order.
__global__ __launch_bounds__(kThreads) void similarity_mean_kernel(const float* __restrict__ cos,
                                                                   long long begin, long long end,
                                                                   float* __restrict__ out) {
  __shared__ double part[kThreads];
  double acc = 0.0;
  for (long long i = begin + threadIdx.x; i < end; i += kThreads) acc += (double)cos[i];
  part[threadIdx.x] = acc;
  __syncthreads();
  for (int w = kThreads / 2; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = end > begin ? (float)(part[0] / (double)(end - begin)) : 1.0f;
}

}  // namespace

void launch_similarity_mean(const float* cos, long long begin, long long end, float* out,
                            hipStream_t st) {
  hipLaunchKernelGGL(similarity_mean_kernel, dim3(1), dim3(kThreads), 0, st, cos, begin, end, out);
}

void launch_ideal_similarity(const void* q, const void* k_all, int n_stride, int L,
                             const a2sf_cache& c, float* out, hipStream_t st) {
  const size_t lds = ((size_t)L * 4 + 1023) & ~(size_t)1023;
  // keys that cannot stay in the 256 MB last-level cache until the next step are read with the
  // non-temporal hint (see load16_stream)
  const bool stream = (double)c.G * L * c.d * (c.dtype == A2SF_F32 ? 4 : 2) > 512e6;
#define A2SF_SIM_(T, D, S)                                                                         \
  do {                                                                                             \
    static const hipError_t raised = hipFuncSetAttribute(                                          \
        (const void*)ideal_similarity_kernel<T, D, S>, hipFuncAttributeMaxDynamicSharedMemorySize, \
        kSimMaxRows * 4);                                                                          \
    (void)raised;                                                                                  \
    hipLaunchKernelGGL((ideal_similarity_kernel<T, D, S>), dim3(c.G), dim3(kThreads), lds, st,     \
                       (const T*)q, (const T*)k_all, n_stride, L, c.pos, c.len, c.capacity, out);  \
  } while (0)
#define A2SF_SIM(T, D)              \
  do {                              \
    if (stream) A2SF_SIM_(T, D, true); \
    else A2SF_SIM_(T, D, false);    \
  } while (0)
  if (c.dtype == A2SF_F32) {
    if (c.d == 64) A2SF_SIM(float, 64); else A2SF_SIM(float, 128);
  } else {
    if (c.d == 64) A2SF_SIM(bf16_t, 64); else A2SF_SIM(bf16_t, 128);
  }
#undef A2SF_SIM
#undef A2SF_SIM_
}

}  // namespace a2sf
