/*
 * a2sf.h - C ABI of the MI355X (gfx950) A2SF hot path.
 *
 * A2SF = Accumulative Attention Score with Forgetting Factor (arxiv 2407.20485).
 * The library computes, for G independent heads (one head = one (layer, batch, head)
 * triple; the paper keeps a separate score per layer and per head, Section 2.2 and
 * Section 3.1 Eq.2):
 *
 *   prompt phase      masked self-attention (Section 1, Section 3.1 Eq.3), the forgotten
 *                     accumulated score of every prompt token (Section 3.3 Eq.5/Eq.6)
 *                     S_j = sum_{i>=j} alpha^(n-1-i) * softmax(Q K^T / sqrt(d))[i, j],
 *                     and one selection of the budgeted token set into a KV cache;
 *   generation step   attention of one new query over the retained tokens only
 *                     (Section 2.2: pruning changes the softmax denominator), the update
 *                     S <- alpha * S + a_t on every retained token (abstract, Section 3.3),
 *                     and eviction of the lowest-score tokens so that the budget holds
 *                     (Section 2.2, Section 3.1 after Eq.2, Section 4.1 for the split of
 *                     the budget into a score-selected and a most-recent part).
 *
 * Conventions shared by every call
 *  - All data pointers are DEVICE pointers owned by the caller; the library never
 *    allocates, frees or keeps them.  a2sf_cache itself is a small HOST struct.
 *  - Every call only enqueues work on `hip_stream` (a hipStream_t passed as void*;
 *    NULL = the default stream) and never synchronises.  Results are valid once the
 *    stream reaches the end of the enqueued work.
 *  - Arguments are validated on the host before anything is launched; an argument
 *    error returns its status and launches nothing (so it is testable without a GPU).
 *    A failed launch returns A2SF_EHIP.
 *  - Row-major everywhere, head dimension d contiguous.  d is 64 or 128.  dtype is
 *    fp32 or bf16 for Q/K/V/O; scores are always fp32, positions int32.
 *  - Data pointers must be 16-byte aligned.
 *  - 0 <= alpha <= 1 and finite.  The paper states 0 < alpha < 1 (Section 3.3) but
 *    evaluates alpha = 0 (Section 4.4) and alpha = 1 is the plain accumulated score of
 *    Section 3.1 Eq.4; both ends are accepted, with 0^0 = 1.
 *  - Budget B = select + recent >= 1.  recent = 0 is the paper's own A2SF setting and
 *    select = 0 is its local-attention baseline (Section 4.1).
 *  - "Position" is the 0-based index of a token in the sequence.  Ties between equal
 *    scores are resolved in favour of the lower position (the higher one is evicted).
 *  - Original positions stored in a cache must be distinct and >= 0.
 */
#ifndef A2SF_H
#define A2SF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  A2SF_OK = 0,
  A2SF_EINVAL = 1,     /* null pointer, misaligned pointer, alpha outside [0,1] or not finite,
                          negative count, unknown mode */
  A2SF_ESHAPE = 2,     /* d not in {64,128}, n < 1, G < 1, L < 1 ... */
  A2SF_EDTYPE = 3,     /* dtype not A2SF_F32 / A2SF_BF16 */
  A2SF_ECAPACITY = 4,  /* cache capacity too small for budget + 1, or above the supported maximum */
  A2SF_EWORKSPACE = 5, /* workspace missing or smaller than a2sf_workspace_bytes() */
  A2SF_EHIP = 6        /* the HIP runtime reported an error at launch */
} a2sf_status;

typedef enum { A2SF_F32 = 0, A2SF_BF16 = 1 } a2sf_dtype;

/* How a generation step makes the cache dense again after an eviction. */
typedef enum {
  A2SF_EVICT_FAST = 0,   /* the new token's row is written into the evicted slot: no row
                            moves; slot order becomes arbitrary, the set of (pos, K, V, S)
                            tuples is what is defined */
  A2SF_EVICT_STABLE = 1  /* slots stay in ascending position (select + in-place compaction) */
} a2sf_evict_mode;

/* Section 4.1: the cache ratio is split into a score-selected and a most-recent part. */
typedef struct {
  int32_t select; /* tokens kept for their score, >= 0 */
  int32_t recent; /* newest tokens always kept, >= 0 */
} a2sf_budget;

/* The KV cache of G heads plus the A2SF bookkeeping (host struct, device pointers). */
typedef struct {
  void* k;        /* [G, capacity, d] dtype */
  void* v;        /* [G, capacity, d] dtype */
  float* scores;  /* [G, capacity] accumulated score of each slot */
  int32_t* pos;   /* [G, capacity] original position of each slot */
  int32_t* len;   /* [G] number of valid slots of each head */
  int32_t G;
  int32_t capacity; /* slots per head; needs >= select + recent + 1; at most A2SF_MAX_CAPACITY */
  int32_t d;
  int32_t dtype;  /* a2sf_dtype */
} a2sf_cache;

/* One float per slot is kept in the 160 KB of LDS of a compute unit by the generation step. */
#define A2SF_MAX_CAPACITY 36864

/* Bytes of device workspace that any of the calls below may need for these sizes
 * (n_max = longest prompt, 0 if a2sf_prefill is not used; capacity as in a2sf_cache).
 * Returns 0 on invalid arguments.  The content of the workspace need not be preserved
 * between calls; calls that share a workspace must not overlap in time. */
size_t a2sf_workspace_bytes(int32_t G, int32_t n_max, int32_t capacity, int32_t d,
                            int32_t dtype, a2sf_budget budget);

/* Prompt phase (Section 3.1 Eq.3, Section 3.3 Eq.5, one selection as in Section 2.2).
 *   q, k, v      [G, n, d] dtype, read only.
 *   cache        out: for every head the min(n, B) surviving tokens in ascending
 *                position: K, V rows, their Eq.5 score, their position; len = min(n, B).
 *                Survivors: the `recent` last positions, plus of the others the `select`
 *                with the largest score (tie -> lower position).
 *   o            out [G, n, d] dtype: attention output rows; may be NULL: then no P*V
 *                work is done, and (bf16, d = 128) rows whose weight alpha^(n-1-i) is
 *                exactly 0 in fp32 are not visited at all where the scores do not need them.
 *   scores_full  out [G, n] fp32: the Eq.5 score of every prompt token; may be NULL.
 * The n x n probability matrix is never written to memory. */
a2sf_status a2sf_prefill(const void* q, const void* k, const void* v, int32_t n, float alpha,
                         a2sf_budget budget, const a2sf_cache* cache, void* o,
                         float* scores_full, void* workspace, size_t workspace_bytes,
                         void* hip_stream);

/* a2sf_prefill with a relative tolerance on the Eq.5 scores (Section 3.3: the forgetting
 * factor sends the contribution of old rows to 0, so for alpha < 1 only the newest rows of
 * the prompt matter).  Rows whose whole remaining contribution to S_j is PROVABLY at most
 * score_rel_tol * S_j are not computed.  The bound needs nothing but the newest row: all rows
 * before n - W together add at most alpha^W / (1 - alpha) to any score (probabilities are
 * <= 1) while S_j >= P[n-1, j]; the kernel reads the smallest P[n-1, j] of each group of 64
 * keys off the newest row, which it processes first, and walks back W rows with
 * alpha^W <= score_rel_tol * (1 - alpha) * min_j P[n-1, j].
 *   score_rel_tol  in [0, 1); 0 = every row of nonzero fp32 weight, exactly a2sf_prefill.
 * Everything else as in a2sf_prefill.  The window is applied to bf16 prompts with d = 128;
 * other shapes compute every row (the result is then a2sf_prefill's).  alpha = 1 has no
 * window, alpha = 0 only the newest row either way. */
a2sf_status a2sf_prefill_windowed(const void* q, const void* k, const void* v, int32_t n,
                                  float alpha, float score_rel_tol, a2sf_budget budget,
                                  const a2sf_cache* cache, void* o, float* scores_full,
                                  void* workspace, size_t workspace_bytes, void* hip_stream);

/* A further chunk of a prompt that is too long to be processed at once (beyond the paper,
 * which evicts once per generation step, Section 3.1): the chunk's m tokens are m generation
 * steps whose eviction is deferred to the end of the chunk, so that their rows go through the
 * matrix cores together.
 *   q, k, v   [G, m, d] dtype: the chunk's queries, keys and values; its tokens have
 *             positions pos0 .. pos0 + m - 1 (larger than every cached one).
 *   cache     in/out; requires len[g] + m <= capacity (so capacity > m).  Row i of the chunk
 *             attends the head's cached tokens and the chunk's tokens 0 .. i (softmax over
 *             exactly those, Section 2.2); o_i is that row's output; every cached token's score
 *             becomes alpha^m * S + sum_i alpha^(m-1-i) P[i, .] and a chunk token gets
 *             sum_{i >= its own row} alpha^(m-1-i) P[i, .] (Section 3.3 Eq.5 over the rows
 *             that exist); then ONE eviction as in a2sf_decode_step's stable mode brings the
 *             head down to min(len + m, B) tokens, slot order preserved.
 *             A head without room for the chunk is left untouched, its rows of o are NaN.
 *   o         out [G, m, d] dtype, may be NULL.
 * The first chunk of a prompt is a2sf_prefill (or this call on an empty cache, len = 0).
 * Workspace: a2sf_workspace_bytes(G, m, capacity, d, dtype, budget). */
a2sf_status a2sf_prefill_chunk(const void* q, const void* k, const void* v, int32_t m, int32_t pos0,
                               float alpha, a2sf_budget budget, const a2sf_cache* cache, void* o,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/* One generation step (abstract; Section 2.2; Section 3.3).
 *   q, k_new, v_new  [G, d] dtype: the new token's query, key and value.
 *   t_pos            original position of the new token (larger than every cached one).
 *   cache            in/out.  Requires 0 <= len[g] and len[g] + 1 <= capacity; a head that
 *                    violates this is left untouched and its row of o is filled with NaN
 *                    (the lengths live on the device, so the host cannot check them).
 *                    The new token joins with
 *                    score 0; a = softmax(K_c q / sqrt(d)) over the len+1 cached tokens;
 *                    o = a^T V_c; every score becomes alpha*S + a; then, if len+1 > B,
 *                    the len+1-B lowest-score tokens outside the `recent` newest
 *                    positions are evicted (tie -> the higher position goes) and
 *                    len = B; else len = len+1.
 *   mode             a2sf_evict_mode.
 *   o                out [G, d] dtype. */
a2sf_status a2sf_decode_step(const void* q, const void* k_new, const void* v_new, int32_t t_pos,
                             const a2sf_cache* cache, float alpha, a2sf_budget budget,
                             int32_t mode, void* o, void* workspace, size_t workspace_bytes,
                             void* hip_stream);

/* Grouped-query heads (beyond the paper, whose models are all multi-head): `group` query heads
 * share each of the G K/V heads of the cache, so a token is kept or evicted for the whole
 * group.  The group's score of a token is the SUM of its query heads' accumulated scores -- as
 * the paper's Eq.1 sums over the heads that one pruning decision serves.  Every query head has
 * its own softmax and its own output.
 *   group        1 .. 8 (1 = the plain calls).
 *   q            prefill: [G, group, n, d]; decode: [G, group, d].
 *   k, v / k_new, v_new   as in the plain calls: one row per K/V head.
 *   o            prefill: [G, group, n, d] (may be NULL); decode: [G, group, d].
 *   scores_full  [G, n] (prefill, may be NULL): the summed scores.
 * Workspace: a2sf_workspace_bytes(G * group, n, capacity, d, dtype, budget) for the prefill
 * (one log-sum-exp row per query head); the decode step needs one only in stable mode
 * (a2sf_workspace_bytes(G, 0, capacity, ...) is enough for that).  Given a larger one -- the
 * prefill's, or a2sf_workspace_bytes(G * group, 0, capacity, ...) plus
 * 4 * G * group * 64 * (d + 2) bytes -- a step over few K/V heads with long caches (bf16,
 * d = 128) splits each head's tokens over as many workgroups as its scratch
 * memory allows; results do not depend on that beyond fp32 summation order.  The decode step
 * holds group * capacity logits in LDS: group * capacity <= A2SF_GQA_MAX_LOGITS. */
#define A2SF_GQA_MAX_LOGITS 16384
a2sf_status a2sf_prefill_gqa(const void* q, const void* k, const void* v, int32_t n, int32_t group,
                             float alpha, a2sf_budget budget, const a2sf_cache* cache, void* o,
                             float* scores_full, void* workspace, size_t workspace_bytes,
                             void* hip_stream);
a2sf_status a2sf_decode_step_gqa(const void* q, const void* k_new, const void* v_new, int32_t t_pos,
                                 const a2sf_cache* cache, int32_t group, float alpha,
                                 a2sf_budget budget, int32_t mode, void* o, void* workspace,
                                 size_t workspace_bytes, void* hip_stream);

/* a2sf_prefill_chunk for grouped-query heads (the two extensions above together): a chunk of m
 * tokens of G K/V heads with `group` query heads each.  Every query head attends as a plain
 * head's chunk does, with its own softmax and output; a cached token's score becomes
 * alpha^m * S + the sum over the group's heads of sum_i alpha^(m-1-i) P_h[i, .]; one eviction
 * per K/V head.
 *   q, o      [G, group, m, d] (o may be NULL);  k, v  [G, m, d].
 * Everything else as in a2sf_prefill_chunk.
 * Workspace: a2sf_workspace_bytes(G * group, m, capacity, d, dtype, budget). */
a2sf_status a2sf_prefill_chunk_gqa(const void* q, const void* k, const void* v, int32_t m,
                                   int32_t pos0, int32_t group, float alpha, a2sf_budget budget,
                                   const a2sf_cache* cache, void* o, void* workspace,
                                   size_t workspace_bytes, void* hip_stream);

/* a2sf_decode_step for callers that cannot provide or allocate a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  Identical in every
 * other respect (same kernels, same results); the scratch memory that a2sf_decode_step takes
 * as `workspace` is a fixed array of A2SF_STATIC_WS_BYTES inside the library instead, one per
 * GPU, held until the process ends.  Nothing is allocated or freed by this call.
 *  - Returns A2SF_EWORKSPACE, launching nothing, when
 *    a2sf_workspace_bytes(G, 0, capacity, d, dtype, budget) exceeds A2SF_STATIC_WS_BYTES.
 *  - Every call on one GPU uses the same array: calls that overlap in time on one GPU (on
 *    different streams) race.  The array keeps the previous call's content; every kernel
 *    writes what it later reads, so nothing has to be cleared.
 *  - The first call on a device looks the array's address up (hipGetSymbolAddress); make that
 *    first call outside any stream capture. */
#define A2SF_STATIC_WS_BYTES (16u << 20)
a2sf_status a2sf_decode_step_static_ws(const void* q, const void* k_new, const void* v_new,
                                       int32_t t_pos, const a2sf_cache* cache, float alpha,
                                       a2sf_budget budget, int32_t mode, void* o, void* hip_stream);

/* The same two calls with one forgetting factor per head (Section 6 of the paper names a
 * distinct factor per layer and head as the way to lift its limitation of a single one).
 *   alpha_heads  [G] fp32, device: head g uses alpha_heads[g], each in [0, 1].
 *   alpha_max    (prefill only) an upper bound of alpha_heads, checked like alpha; it sizes
 *                the row window of the score pass.  A head whose factor exceeds it is
 *                computed with alpha_max instead of its own factor.
 * Everything else as in a2sf_prefill / a2sf_decode_step. */
a2sf_status a2sf_prefill_alpha_per_head(const void* q, const void* k, const void* v, int32_t n,
                                        const float* alpha_heads, float alpha_max,
                                        a2sf_budget budget, const a2sf_cache* cache, void* o,
                                        float* scores_full, void* workspace,
                                        size_t workspace_bytes, void* hip_stream);
a2sf_status a2sf_decode_step_alpha_per_head(const void* q, const void* k_new, const void* v_new,
                                            int32_t t_pos, const a2sf_cache* cache,
                                            const float* alpha_heads, a2sf_budget budget,
                                            int32_t mode, void* o, void* workspace,
                                            size_t workspace_bytes, void* hip_stream);

/* Selection alone (Section 2.2, Section 4.1): which of the L tokens of each head survive.
 *   scores    [G, stride] fp32 (no NaN);  pos [G, stride] int32 or NULL (position = slot).
 *   len       [G] device, valid slots per head (<= L), or NULL: every head has L.
 *   keep_idx  out [G, B]: surviving slot indices in ascending slot order, first n_keep[g]
 *             entries valid;  n_keep out [G] = min(len, B).
 * Survivors: the `recent` largest positions plus the `select` best scores of the rest
 * (tie -> lower position); everything if len <= B. */
a2sf_status a2sf_select(const float* scores, const int32_t* pos, const int32_t* len, int32_t G,
                        int32_t L, int32_t stride, a2sf_budget budget, int32_t* keep_idx,
                        int32_t* n_keep, void* hip_stream);

/* Removal of the tokens that were not selected (Section 2.2: tokens with a small accumulated
 * score are removed from the KV cache; Section 3.1 after Eq.2), as an in-place stable
 * compaction: for every head, row keep_idx[g][r] of K, V, scores and pos moves to row r for
 * r < n_keep[g], and len[g] = n_keep[g].
 *   keep_idx  [G, keep_stride] strictly ascending indices of valid slots, i.e. below len[g]
 *             (as a2sf_select writes).
 *   n_keep    [G] device. */
a2sf_status a2sf_compact(const a2sf_cache* cache, const int32_t* keep_idx, int32_t keep_stride,
                         const int32_t* n_keep, void* hip_stream);

/* Diagnostic of Section 4.3 / Table 2: how close a pruning policy's attention row is to the
 * row of the Ideal mask, for one generation step of every head.  The Ideal attends ALL
 * tokens so far (nothing is ever removed) and keeps the entries of the tokens with the
 * largest attention score (tie -> lower position), as many as the policy's row has; the
 * policy's row has entries on the tokens in its cache and on the new token.  Either row is
 * the softmax over its own tokens (Section 2.2), zero elsewhere; the result is their cosine.
 *   q        [G, d] dtype: the step's query.
 *   k_all    [G, n_stride, d] dtype, read only: the keys of all tokens so far, row = position,
 *            rows 0 .. t_pos valid (row t_pos is the new token's key).
 *   t_pos    position of the new token; t_pos + 1 <= A2SF_SIM_MAX_ROWS, t_pos < n_stride.
 *   cache    the policy's cache BEFORE this step; only pos, len, capacity, G, d and dtype
 *            are read.  Cached positions must be < t_pos.
 *   cos_out  out [G] fp32, in [0, 1]; 1 when the two rows select the same tokens.
 * Call it right before the a2sf_decode_step of the same token. */
#define A2SF_SIM_MAX_ROWS 32768
a2sf_status a2sf_ideal_similarity(const void* q, const void* k_all, int32_t n_stride,
                                  int32_t t_pos, const a2sf_cache* cache, float* cos_out,
                                  void* hip_stream);

/* Average of the similarities over the steps from first_step on and over all heads: the
 * figure Table 2 reports (Section 4.3; steps before the budget is reached prune nothing and
 * are left out by the caller through first_step).
 *   cos       [steps, G] fp32, device, as successive a2sf_ideal_similarity calls wrote it.
 *   mean_out  out [1] fp32, device; 1 when no step is left to average. */
a2sf_status a2sf_similarity_mean(const float* cos, int32_t steps, int32_t G, int32_t first_step,
                                 float* mean_out, void* hip_stream);

/* How a2sf_decode_step will launch for these sizes (host only, launches nothing; for
 * benchmarks and profiles that have to name the kernels they measure).  Any out pointer may
 * be NULL.
 *   nsplit          workgroups per head; 1 = one fused kernel, > 1 = the tokens of a head are
 *                   split over that many workgroups and a second kernel combines them.
 *   rows_per_split  cached tokens per workgroup when nsplit > 1.
 *   wave_slots      > 0: a wave works on a whole head (64 * wave_slots slots in registers).
 *   wave_heads      heads a wave works through in the fast eviction mode: 1, or more in the
 *                   form for launches with several times more heads than the chip holds waves
 *                   (persistent workgroups; a step's small writes are held back in LDS). */
a2sf_status a2sf_decode_plan(int32_t G, int32_t capacity, int32_t d, int32_t* nsplit,
                             int32_t* rows_per_split, int32_t* wave_slots, int32_t* wave_heads);

const char* a2sf_status_string(int32_t status);

#ifdef __cplusplus
}
#endif
#endif /* A2SF_H */
