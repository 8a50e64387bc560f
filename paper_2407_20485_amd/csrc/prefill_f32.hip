// fp32 prompt phase (small-shape path): masked attention rows with their log-sum-exp
// (Section 3.1 Eq.3 of the paper) and the forgotten column scores of Section 3.3 Eq.5,
//   S_j = sum_{i>=j} alpha^(n-1-i) * exp(s_ij - lse_i),
// with plain fp32 FMA arithmetic.  One workgroup per attention row, then one per column.
// The probability matrix is recomputed, never stored.  The bf16 matrix-core path lives in
// prefill_bf16.hip; this one exists for fp32 inputs, where exact fp32 products are wanted.
//
// Both kernels take the geometry of a2sf_internal.h's AttnRect: m query rows per head against
// keys that lie kv_stride rows apart from head to head; row i sees keys 0 .. off + i, where
// off (per head, or 0) is the number of older tokens in front of the rows' own.  The prompt
// phase is the square case (off = 0, kv_stride = m); a chunk of a prompt runs against the
// head's cache (off = tokens cached before the chunk).
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
    const float* __restrict__ q, const float* __restrict__ k, const float* __restrict__ v,
    AttnRect rc, float* __restrict__ o, float* __restrict__ lse2, float scale_log2e) {
  __shared__ float z[kChunk];
  __shared__ float part[kThreads / D][D];
  __shared__ float red[8];
  const int n = rc.m;
  const int g = blockIdx.x / n, i = blockIdx.x % n, tid = threadIdx.x;
  const int gk = g / rc.kv_group;  // the K/V head this query head reads
  const int off = rc.off_heads ? rc.off_heads[gk] : 0;
  if (off < 0) {  // a head the caller's precondition excludes: its rows are flagged
    if (o && tid < D) o[((size_t)g * n + i) * D + tid] = __int_as_float(0x7FC00000);
    return;
  }
  const float* qi = q + ((size_t)g * n + i) * D;
  const float* kg = k + (size_t)gk * rc.kv_stride * D;
  const float* vg = v + (size_t)gk * rc.kv_stride * D;
  constexpr int PARTS = kThreads / D;
  const int c = tid % D, part_id = tid / D;
  const int last = off + i;  // newest key this row sees

  float m = -INFINITY, l = 0.f, acc = 0.f;
  for (int c0 = 0; c0 <= last; c0 += kChunk) {
    const int c1 = min(last + 1, c0 + kChunk);
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

// `accumulate`: the result is added to `decay` times what scores[] holds (a chunk: the cached
// tokens' older scores, decayed by alpha^m); otherwise it replaces it.
template <int D>
__global__ __launch_bounds__(kThreads) void scores_f32_kernel(
    const float* __restrict__ q, const float* __restrict__ k, const float* __restrict__ lse2,
    AttnRect rc, int keys_per_head, int first_row, float log2_alpha,
    const float* __restrict__ alpha_heads, float* __restrict__ scores, int s_stride, bool accumulate,
    float decay, float scale_log2e) {
  __shared__ float red[8];
  const int n = rc.m;
  const int g = blockIdx.x / keys_per_head, j = blockIdx.x % keys_per_head, tid = threadIdx.x;
  const int off = rc.off_heads ? rc.off_heads[g] : 0;
  if (off < 0 || j >= off + n) return;
  head_window(alpha_heads, g, n, first_row, log2_alpha);
  const float* kj = k + ((size_t)g * rc.kv_stride + j) * D;
  float sum = 0.f;
  for (int hq = 0; hq < rc.kv_group; ++hq) {  // the query heads that share this K/V head
    const float* qg = q + ((size_t)g * rc.kv_group + hq) * n * D;
    const float* lg = lse2 + ((size_t)g * rc.kv_group + hq) * n;
    for (int i = max(max(j - off, first_row), 0) + tid; i < n; i += kThreads) {
      const float s = dot_row<D>(qg + (size_t)i * D, kj) * scale_log2e;
      sum += exp2f(s - lg[i] + (float)(n - 1 - i) * log2_alpha);
    }
  }
  sum = block_sum(sum, red);
  if (tid == 0) {
    float* out = scores + (size_t)g * s_stride + j;
    *out = accumulate ? fmaf(decay, *out, sum) : sum;
  }
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

void launch_attn_f32(const float* q, const float* k, const float* v, int G, const AttnRect& rc,
                     int d, float* o, float* lse2, hipStream_t st) {
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)d);
  dim3 grid((unsigned)G * (unsigned)rc.kv_group * (unsigned)rc.m);
  if (d == 64)
    hipLaunchKernelGGL(attn_rows_f32_kernel<64>, grid, dim3(kThreads), 0, st, q, k, v, rc, o, lse2, scale_log2e);
  else
    hipLaunchKernelGGL(attn_rows_f32_kernel<128>, grid, dim3(kThreads), 0, st, q, k, v, rc, o, lse2, scale_log2e);
}

void launch_colscores_f32(const float* q, const float* k, const float* lse2, int G,
                          const AttnRect& rc, int keys_per_head, int d, float alpha,
                          const float* alpha_heads, float* scores, int s_stride, bool accumulate,
                          float decay, hipStream_t st) {
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)d);
  float l2a;
  const int first = first_contributing_row(rc.m, alpha, &l2a);
  dim3 grid((unsigned)G * (unsigned)keys_per_head);
  if (d == 64)
    hipLaunchKernelGGL(scores_f32_kernel<64>, grid, dim3(kThreads), 0, st, q, k, lse2, rc, keys_per_head,
                       first, l2a, alpha_heads, scores, s_stride, accumulate, decay, scale_log2e);
  else
    hipLaunchKernelGGL(scores_f32_kernel<128>, grid, dim3(kThreads), 0, st, q, k, lse2, rc, keys_per_head,
                       first, l2a, alpha_heads, scores, s_stride, accumulate, decay, scale_log2e);
}

void launch_prefill_f32(const float* q, const float* k, const float* v, int G, int n, int d,
                        float* o, float* lse2, hipStream_t st) {
  launch_attn_f32(q, k, v, G, AttnRect{n, n, nullptr}, d, o, lse2, st);
}

void launch_scores_f32(const float* q, const float* k, const float* lse2, int G, int n, int d,
                       float alpha, const float* alpha_heads, float* scores, hipStream_t st) {
  launch_colscores_f32(q, k, lse2, G, AttnRect{n, n, nullptr}, n, d, alpha, alpha_heads, scores, n,
                       false, 0.f, st);
}

}  // namespace a2sf
