// Host-side launch functions of the kernel files, called by the C-ABI entry points.
// Every launcher only enqueues on `st`; shapes have been validated by the caller.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/a2sf.h"

namespace a2sf {

// select_compact.hip
void launch_select(const float* scores, const int32_t* pos, const int32_t* len, int G, int L,
                   int stride, int select, int recent, int32_t* keep_idx, int32_t* n_keep,
                   hipStream_t st);
// k2 / v2 [G, m2, d] set: the rows of the slots from off_heads[g] on are taken from there
// (a chunk whose rows were not copied into the cache)
void launch_compact(const a2sf_cache& c, const int32_t* keep_idx, int keep_stride,
                    const int32_t* n_keep, hipStream_t st, const void* k2 = nullptr,
                    const void* v2 = nullptr, int m2 = 0, const int32_t* off_heads = nullptr);
// Out-of-place gather of the prompt's surviving rows into the cache.
void launch_gather_prompt(const void* k, const void* v, const float* scores_full, int n,
                          const int32_t* keep_idx, int keep_stride, const int32_t* n_keep,
                          const a2sf_cache& c, hipStream_t st);

// decode.hip
struct DecodePlan {
  int nsplit;          // workgroups per head (1 = single fused kernel)
  int rows_per_split;  // multiple of 64
  int wave_slots;      // > 0: wave-per-head kernel holding 64*wave_slots slots in registers
  bool loop;           // wave-per-head path, fast mode: persistent workgroups, a wave works through several heads
  int wave_heads;      // ... that many (1 otherwise)
  bool stream;         // single-kernel paths: load the cache rows with the non-temporal hint
  size_t ws_bytes;     // split-K scratch
};
DecodePlan plan_decode(int G, int capacity, int d);
void launch_decode(const void* q, const void* k_new, const void* v_new, int t_pos,
                   const a2sf_cache& c, float alpha, const float* alpha_heads, int select,
                   int recent, bool evict_here, void* o, void* ws, const DecodePlan& plan,
                   hipStream_t st);

// Generation step of G K/V heads with `group` (2 .. 8) query heads each: q, o are
// [G, group, d]; group * capacity floats of LDS per workgroup.  ws (may be null) / ws_bytes:
// scratch memory for the token-split form that few K/V heads with long caches take.
void launch_decode_gqa(const void* q, const void* k_new, const void* v_new, int t_pos,
                       const a2sf_cache& c, int group, float alpha, int select, int recent,
                       bool evict_here, void* o, void* ws, size_t ws_bytes, hipStream_t st);

// chunk.hip: the chunk's K/V rows go behind each head's cached tokens (len grows by m, the old
// lengths are left in len_old, -1 where the chunk does not fit)
void launch_chunk_append(const void* k, const void* v, int m, int pos0, const a2sf_cache& c,
                         int32_t* len_old, bool copy_rows, hipStream_t st);

// similarity.hip: cosine between the policy's attention row (cache positions + the new token)
// and the Ideal row over the first L rows of k_all, per head.
void launch_ideal_similarity(const void* q, const void* k_all, int n_stride, int L,
                             const a2sf_cache& c, float* out, hipStream_t st);

void launch_similarity_mean(const float* cos, long long begin, long long end, float* out,
                            hipStream_t st);

// Geometry of one attention call: m query rows per head against keys that lie kv_stride rows
// apart from head to head; row i sees keys 0 .. off + i.  The prompt phase is the square case
// (off = 0, kv_stride = m); a chunk of a prompt runs against the head's cache, off = the tokens
// cached before the chunk (off_heads[g] < 0 marks a head to be skipped).
// kv_group > 1: grouped-query heads.  The attention kernels then run over G * kv_group query
// heads, query head g reading the K/V rows of head g / kv_group; the column-score kernels run
// over the G K/V heads and sum the scores of each head's kv_group query heads.
struct AttnRect {
  int m;
  int kv_stride;
  const int32_t* off_heads;  // [G] device, or null: 0 for every head
  int kv_group = 1;
  // Second source of key / value rows (bf16, d = 128, kv_group = 1 only): when set, a head's
  // keys 0 .. off-1 are rows of k / v and its keys off .. off+m-1 are the m rows [G, m, d] of
  // k2 / v2 -- a chunk whose rows have not been copied behind the cached ones.
  const void* k2 = nullptr;
  const void* v2 = nullptr;
  // Calls without outputs (bf16, d = 128): the log-sum-exp of the rows before first_row is not
  // needed (the score kernel that follows skips them), so their row blocks are not computed.
  int first_row = 0;
};
// true when launch_attn_bf16 / launch_colscores_bf16 serve these sizes with kernels that read a
// second key / value source
bool bf16_two_source_ok(int d, const AttnRect& rc, float alpha);

// prefill_f32.hip / prefill_bf16.hip
// lse2[g][i] = log2(sum_j exp(s_ij)) of the masked row i (s already scaled by 1/sqrt(d)).
void launch_prefill_f32(const float* q, const float* k, const float* v, int G, int n, int d,
                        float* o, float* lse2, hipStream_t st);
// alpha_heads (device [G]) may be null: then every head uses `alpha`; otherwise `alpha` is an
// upper bound of the per-head factors.
void launch_scores_f32(const float* q, const float* k, const float* lse2, int G, int n, int d,
                       float alpha, const float* alpha_heads, float* scores, hipStream_t st);
// The general (rectangular) forms, used for chunks of a prompt.  keys_per_head: upper bound of
// off + m over the heads (the grid is sized by it).  accumulate: the new column sums are added
// to decay * scores[] (the cached tokens' older scores) instead of replacing it.
void launch_attn_f32(const float* q, const float* k, const float* v, int G, const AttnRect& rc,
                     int d, float* o, float* lse2, hipStream_t st);
void launch_colscores_f32(const float* q, const float* k, const float* lse2, int G,
                          const AttnRect& rc, int keys_per_head, int d, float alpha,
                          const float* alpha_heads, float* scores, int s_stride, bool accumulate,
                          float decay, hipStream_t st);
void launch_attn_bf16(const void* q, const void* k, const void* v, int G, const AttnRect& rc, int d,
                      void* o, float* lse2, hipStream_t st);
void launch_colscores_bf16(const void* q, const void* k, const float* lse2, int G,
                           const AttnRect& rc, int keys_per_head, int d, float alpha, float* scores,
                           int s_stride, bool accumulate, float decay, hipStream_t st);
// first_row > 0 (only with o == null): rows before it need no log-sum-exp
void launch_prefill_bf16(const void* q, const void* k, const void* v, int G, int n, int d,
                         void* o, float* lse2, hipStream_t st, int first_row = 0);
// First prompt row whose log-sum-exp launch_scores_bf16 reads for these sizes (Section 3.3: the
// forgetting factor takes older rows' contributions to 0; exactly 0 in fp32 before that row).
int bf16_first_lse_row(int n, int d, float alpha_max);
// tol > 0 (d = 128 only): rows whose whole remaining contribution is provably below tol * S_j
// are skipped (see RowWindow in prefill_bf16.hip); tol = 0 computes every row of nonzero weight.
void launch_scores_bf16(const void* q, const void* k, const float* lse2, int G, int n, int d,
                        float alpha, const float* alpha_heads, float tol, float* scores,
                        hipStream_t st);

// Rows i < first_row contribute exactly 0 to every fp32 score (their weight alpha^(n-1-i)
// is below the smallest fp32 subnormal while P <= 1), so the score kernels skip them.
// Also returns log2(alpha) as used in the exponent (0 for alpha == 0, whose only row is n-1).
int first_contributing_row(int n, float alpha, float* log2_alpha);

}  // namespace a2sf
