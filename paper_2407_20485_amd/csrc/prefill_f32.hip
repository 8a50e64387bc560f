// fp32 prompt phase (small-shape path): masked attention rows with their log-sum-exp
// (Section 3.1 Eq.3 of the paper) and the forgotten column scores of Section 3.3 Eq.5,
//   S_j = sum_{i>=j} alpha^(n-1-i) * exp(s_ij - lse_i),
// with plain fp32 FMA arithmetic.  One workgroup per attention row, then one per column.
// The probability matrix is recomputed, never stored.  The bf16 matrix-core path lives in
// prefill_bf16.hip; this one exists for fp32 inputs, where exact fp32 products are wanted.
#include <math.h>

#include "a2sf_dev.h"
#include "a2sf_internal.h"

namespace a2sf {
namespace {

constexpr int kChunk = 2048;  // logits held in LDS at a time

template <int D>
__device__ __forceinline__ float dot_row(const float* __restrict__ a, const float* __restrict__ b) {
  float acc = 0.f;
#pragma unroll
  for (int c = 0; c < D; c += 4) {
    const float4 x = *reinterpret_cast<const float4*>(a + c);
    const float4 y = *reinterpret_cast<const float4*>(b + c);
    acc = fmaf(x.x, y.x, acc); acc = fmaf(x.y, y.y, acc);
    acc = fmaf(x.z, y.z, acc); acc = fmaf(x.w, y.w, acc);
  }
  return acc;
}

template <int D>
__global__ __launch_bounds__(kThreads) void attn_rows_f32_kernel(
    const float* __restrict__ q, const float* __restrict__ k, const float* __restrict__ v, int n,
    float* __restrict__ o, float* __restrict__ lse2, float scale_log2e) {
  __shared__ float z[kChunk];
  __shared__ float part[kThreads / D][D];
  __shared__ float red[8];
  const int g = blockIdx.x / n, i = blockIdx.x % n, tid = threadIdx.x;
  const float* qi = q + ((size_t)g * n + i) * D;
  const float* kg = k + (size_t)g * n * D;
  const float* vg = v + (size_t)g * n * D;
  constexpr int PARTS = kThreads / D;
  const int c = tid % D, part_id = tid / D;

  float m = -INFINITY, l = 0.f, acc = 0.f;
  for (int c0 = 0; c0 <= i; c0 += kChunk) {
    const int c1 = min(i + 1, c0 + kChunk);
    float mx = -INFINITY;
    for (int j = c0 + tid; j < c1; j += kThreads) {
      const float s = dot_row<D>(qi, kg + (size_t)j * D) * scale_log2e;
      z[j - c0] = s;
      mx = fmaxf(mx, s);
    }
    mx = block_max(mx, red);
    const float m_new = fmaxf(m, mx);
    const float corr = exp2f(m - m_new);  // 0 on the first chunk (m = -inf)
    float sum = 0.f;
    for (int j = c0 + tid; j < c1; j += kThreads) {
      const float p = exp2f(z[j - c0] - m_new);
      z[j - c0] = p;
      sum += p;
    }
    sum = block_sum(sum, red);
    l = l * corr + sum;
    m = m_new;
    if (o) {
      acc *= corr;
      for (int j = c0 + part_id; j < c1; j += PARTS) acc = fmaf(z[j - c0], vg[(size_t)j * D + c], acc);
    }
    __syncthreads();
  }
  if (o) {
    part[part_id][c] = acc;
    __syncthreads();
    if (tid < D) {
      float t = 0.f;
#pragma unroll
      for (int p = 0; p < PARTS; ++p) t += part[p][tid];
      o[((size_t)g * n + i) * D + tid] = t / l;
    }
  }
  if (tid == 0) lse2[(size_t)g * n + i] = m + log2f(l);
}

template <int D>
__global__ __launch_bounds__(kThreads) void scores_f32_kernel(
    const float* __restrict__ q, const float* __restrict__ k, const float* __restrict__ lse2, int n,
    int first_row, float log2_alpha, const float* __restrict__ alpha_heads,
    float* __restrict__ scores, float scale_log2e) {
  __shared__ float red[8];
  const int g = blockIdx.x / n, j = blockIdx.x % n, tid = threadIdx.x;
  head_window(alpha_heads, g, n, first_row, log2_alpha);
  const float* kj = k + ((size_t)g * n + j) * D;
  const float* qg = q + (size_t)g * n * D;
  const float* lg = lse2 + (size_t)g * n;
  float sum = 0.f;
  for (int i = max(j, first_row) + tid; i < n; i += kThreads) {
    const float s = dot_row<D>(qg + (size_t)i * D, kj) * scale_log2e;
    sum += exp2f(s - lg[i] + (float)(n - 1 - i) * log2_alpha);
  }
  sum = block_sum(sum, red);
  if (tid == 0) scores[(size_t)g * n + j] = sum;
}

}  // namespace

int first_contributing_row(int n, float alpha, float* log2_alpha) {
  if (alpha <= 0.f) { *log2_alpha = 0.f; return n - 1; }
  if (alpha >= 1.f) { *log2_alpha = 0.f; return 0; }
  const float l2 = log2f(alpha);  // < 0
  *log2_alpha = l2;
  // weight 2^((n-1-i)*l2) <= 2^-160 rounds to 0 in fp32 whatever the probability (<= 1)
  const double rows = 160.0 / (double)(-l2);
  if (rows >= (double)n) return 0;
  const int w = (int)rows + 1;
  return n - w < 0 ? 0 : n - w;
}

void launch_prefill_f32(const float* q, const float* k, const float* v, int G, int n, int d,
                        float* o, float* lse2, hipStream_t st) {
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)d);
  dim3 grid((unsigned)G * (unsigned)n);
  if (d == 64)
    hipLaunchKernelGGL(attn_rows_f32_kernel<64>, grid, dim3(kThreads), 0, st, q, k, v, n, o, lse2, scale_log2e);
  else
    hipLaunchKernelGGL(attn_rows_f32_kernel<128>, grid, dim3(kThreads), 0, st, q, k, v, n, o, lse2, scale_log2e);
}

void launch_scores_f32(const float* q, const float* k, const float* lse2, int G, int n, int d,
                       float alpha, const float* alpha_heads, float* scores, hipStream_t st) {
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)d);
  float l2a;
  const int first = first_contributing_row(n, alpha, &l2a);
  dim3 grid((unsigned)G * (unsigned)n);
  if (d == 64)
    hipLaunchKernelGGL(scores_f32_kernel<64>, grid, dim3(kThreads), 0, st, q, k, lse2, n, first, l2a, alpha_heads, scores, scale_log2e);
  else
    hipLaunchKernelGGL(scores_f32_kernel<128>, grid, dim3(kThreads), 0, st, q, k, lse2, n, first, l2a, alpha_heads, scores, scale_log2e);
}

}  // namespace a2sf
