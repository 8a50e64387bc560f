// C-ABI entry points: argument validation on the host, workspace carving, launches.
// Nothing here allocates, synchronises or falls back to the CPU.
#include <math.h>
#include <stdint.h>

#include <mutex>

#include "a2sf_internal.h"

using namespace a2sf;

// Scratch memory of a2sf_decode_step_static_ws: one array per GPU, alive for the life of the
// process.  In host code this name is only a handle for hipGetSymbolAddress; the device
// address it yields (one per device) is what kernels and the carving code below are given.
static __device__ __align__(256) unsigned char scratch[A2SF_STATIC_WS_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each device, once known

// Device address of this device's copy of `scratch` (looked up once per device).
a2sf_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return A2SF_EHIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return A2SF_EHIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return A2SF_OK;
}

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }
inline bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

struct WsLayout {
  size_t lse2, s_full, keep_idx, n_keep, split, total;
};

// One layout serves every call: the regions a call does not use are simply not touched.
WsLayout ws_layout(int G, int n_max, int capacity, int d, a2sf_budget b) {
  WsLayout w;
  size_t off = 0;
  const size_t Gn = (size_t)G * (size_t)(n_max > 0 ? n_max : 0);
  w.lse2 = off;     off += align_up(Gn * sizeof(float));
  w.s_full = off;   off += align_up(Gn * sizeof(float));
  w.keep_idx = off; off += align_up((size_t)G * (size_t)(b.select + b.recent) * sizeof(int32_t));
  w.n_keep = off;   off += align_up((size_t)G * sizeof(int32_t));
  w.split = off;    off += align_up(capacity > 0 ? plan_decode(G, capacity, d).ws_bytes : 0);
  w.total = off;
  return w;
}

a2sf_status check_budget(a2sf_budget b) {
  if (b.select < 0 || b.recent < 0) return A2SF_EINVAL;
  if ((long long)b.select + (long long)b.recent < 1) return A2SF_EINVAL;
  if ((long long)b.select + (long long)b.recent > 0x3FFFFFFF) return A2SF_EINVAL;
  return A2SF_OK;
}

a2sf_status check_alpha(float alpha) {
  if (!(alpha >= 0.0f && alpha <= 1.0f)) return A2SF_EINVAL;  // also rejects NaN
  return A2SF_OK;
}

a2sf_status check_cache(const a2sf_cache* c, a2sf_budget b) {
  if (!c) return A2SF_EINVAL;
  if (c->dtype != A2SF_F32 && c->dtype != A2SF_BF16) return A2SF_EDTYPE;
  if (c->d != 64 && c->d != 128) return A2SF_ESHAPE;
  if (c->G < 1) return A2SF_ESHAPE;
  if (!c->k || !c->v || !c->scores || !c->pos || !c->len) return A2SF_EINVAL;
  if (misaligned(c->k) || misaligned(c->v) || misaligned(c->scores) || misaligned(c->pos))
    return A2SF_EINVAL;
  if (c->capacity < 1 || c->capacity > A2SF_MAX_CAPACITY) return A2SF_ECAPACITY;
  if ((long long)c->capacity < (long long)b.select + b.recent + 1) return A2SF_ECAPACITY;
  return A2SF_OK;
}

// A launch error is read with hipGetLastError(), which also returns (and clears) an error an
// unrelated earlier call left behind on this thread: every entry point clears that stale
// state before its first launch, so A2SF_EHIP speaks of this call's launches only.
inline void clear_stale_error() { (void)hipGetLastError(); }
inline a2sf_status launch_status() {
  return hipGetLastError() == hipSuccess ? A2SF_OK : A2SF_EHIP;
}

constexpr int kPrefillPartHeads = 2048;

a2sf_status prefill_impl(const void* q, const void* k, const void* v, int32_t n, float alpha,
                         const float* alpha_heads, float tol, a2sf_budget budget, const a2sf_cache* cache,
                         void* o, float* scores_full, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
  a2sf_status s;
  if ((s = check_budget(budget)) != A2SF_OK) return s;
  if ((s = check_alpha(alpha)) != A2SF_OK) return s;
  if ((s = check_cache(cache, budget)) != A2SF_OK) return s;
  if (!q || !k || !v) return A2SF_EINVAL;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(scores_full))
    return A2SF_EINVAL;
  if (n < 1) return A2SF_ESHAPE;
  if ((long long)cache->G * n > 0x7FFFFFFFLL) return A2SF_ESHAPE;
  const WsLayout w = ws_layout(cache->G, n, 0, cache->d, budget);
  if (!workspace || misaligned(workspace) || workspace_bytes < w.total) return A2SF_EWORKSPACE;

  hipStream_t st = (hipStream_t)hip_stream;
  clear_stale_error();
  char* ws = (char*)workspace;
  float* lse2 = (float*)(ws + w.lse2);
  float* s_full = scores_full ? scores_full : (float*)(ws + w.s_full);
  int32_t* keep_idx = (int32_t*)(ws + w.keep_idx);
  int32_t* n_keep = (int32_t*)(ws + w.n_keep);
  const int G = cache->G, d = cache->d;
  const int B = budget.select + budget.recent;

  // A large launch goes through in parts of kPrefillPartHeads heads, each part's four kernels
  // back to back.  The attention kernel gains most: the tiles its row blocks share stay in the
  // L2 of the die that works on them (16384 heads of n = 2048, bf16: it reads 34 GB instead of
  // 52 GB and takes 18.0 ms instead of 18.7; the whole call 20.3 ms instead of 21.0).  Parts of
  // 512 to 2048 heads measure the same within 0.1 ms, also when the three kernels that follow
  // the attention run on larger groups of heads (then 0.2 to 0.5 ms slower); 256 heads: 21.2 ms.
  const size_t e = cache->dtype == A2SF_F32 ? 4 : 2;
  const int part = (cache->dtype == A2SF_BF16 && G >= 2 * kPrefillPartHeads) ? kPrefillPartHeads : G;
  for (int g0 = 0; g0 < G; g0 += part) {
    const int Gp = G - g0 < part ? G - g0 : part;
    const size_t row0 = (size_t)g0 * n;  // first prompt row of the part
    const char* qp = (const char*)q + row0 * d * e;
    const char* kp = (const char*)k + row0 * d * e;
    const char* vp = (const char*)v + row0 * d * e;
    void* op = o ? (char*)o + row0 * d * e : nullptr;
    float* lp = lse2 + row0;
    float* sp = s_full + row0;
    const float* ap = alpha_heads ? alpha_heads + g0 : nullptr;
    int32_t* kip = keep_idx + (size_t)g0 * B;
    int32_t* nkp = n_keep + g0;
    a2sf_cache cp = *cache;
    cp.G = Gp;
    cp.k = (char*)cache->k + (size_t)g0 * cache->capacity * d * e;
    cp.v = (char*)cache->v + (size_t)g0 * cache->capacity * d * e;
    cp.scores = cache->scores + (size_t)g0 * cache->capacity;
    cp.pos = cache->pos + (size_t)g0 * cache->capacity;
    cp.len = cache->len + g0;
    if (cache->dtype == A2SF_F32) {
      launch_prefill_f32((const float*)qp, (const float*)kp, (const float*)vp, Gp, n, d, (float*)op, lp, st);
      launch_scores_f32((const float*)qp, (const float*)kp, lp, Gp, n, d, alpha, ap, sp, st);
    } else {
      // without outputs only the rows the score kernel will read need their log-sum-exp
      launch_prefill_bf16(qp, kp, vp, Gp, n, d, op, lp, st, op ? 0 : bf16_first_lse_row(n, d, alpha));
      launch_scores_bf16(qp, kp, lp, Gp, n, d, alpha, ap, tol, sp, st);
    }
    launch_select(sp, nullptr, nullptr, Gp, n, n, budget.select, budget.recent, kip, nkp, st);
    launch_gather_prompt(kp, vp, sp, n, kip, B, nkp, cp, st);
  }
  return launch_status();
}

a2sf_status decode_impl(const void* q, const void* k_new, const void* v_new, int32_t t_pos,
                        const a2sf_cache* cache, float alpha, const float* alpha_heads,
                        a2sf_budget budget, int32_t mode, void* o, void* workspace,
                        size_t workspace_bytes, void* hip_stream) {
  a2sf_status s;
  if ((s = check_budget(budget)) != A2SF_OK) return s;
  if ((s = check_alpha(alpha)) != A2SF_OK) return s;
  if ((s = check_cache(cache, budget)) != A2SF_OK) return s;
  if (!q || !k_new || !v_new || !o) return A2SF_EINVAL;
  if (misaligned(q) || misaligned(k_new) || misaligned(v_new) || misaligned(o)) return A2SF_EINVAL;
  if (t_pos < 0) return A2SF_EINVAL;
  if (mode != A2SF_EVICT_FAST && mode != A2SF_EVICT_STABLE) return A2SF_EINVAL;
  const WsLayout w = ws_layout(cache->G, 0, cache->capacity, cache->d, budget);
  const DecodePlan plan = plan_decode(cache->G, cache->capacity, cache->d);
  const bool needs_ws = plan.ws_bytes > 0 || mode == A2SF_EVICT_STABLE;
  if (needs_ws && (!workspace || misaligned(workspace) || workspace_bytes < w.total))
    return A2SF_EWORKSPACE;

  hipStream_t st = (hipStream_t)hip_stream;
  clear_stale_error();
  char* ws = (char*)workspace;
  launch_decode(q, k_new, v_new, t_pos, *cache, alpha, alpha_heads, budget.select, budget.recent,
                mode == A2SF_EVICT_FAST, o, ws ? ws + w.split : nullptr, plan, st);
  if (mode == A2SF_EVICT_STABLE) {
    int32_t* keep_idx = (int32_t*)(ws + w.keep_idx);
    int32_t* n_keep = (int32_t*)(ws + w.n_keep);
    launch_select(cache->scores, cache->pos, cache->len, cache->G, cache->capacity,
                  cache->capacity, budget.select, budget.recent, keep_idx, n_keep, st);
    launch_compact(*cache, keep_idx, budget.select + budget.recent, n_keep, st);
  }
  return launch_status();
}

}  // namespace

extern "C" {

size_t a2sf_workspace_bytes(int32_t G, int32_t n_max, int32_t capacity, int32_t d, int32_t dtype,
                            a2sf_budget budget) {
  if (G < 1 || n_max < 0 || capacity < 0 || (d != 64 && d != 128)) return 0;
  if (dtype != A2SF_F32 && dtype != A2SF_BF16) return 0;
  if (check_budget(budget) != A2SF_OK) return 0;
  if (capacity > A2SF_MAX_CAPACITY) return 0;
  return ws_layout(G, n_max, capacity, d, budget).total;
}

a2sf_status a2sf_prefill(const void* q, const void* k, const void* v, int32_t n, float alpha,
                         a2sf_budget budget, const a2sf_cache* cache, void* o,
                         float* scores_full, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
  return prefill_impl(q, k, v, n, alpha, nullptr, 0.0f, budget, cache, o, scores_full, workspace,
                      workspace_bytes, hip_stream);
}

a2sf_status a2sf_prefill_windowed(const void* q, const void* k, const void* v, int32_t n,
                                  float alpha, float score_rel_tol, a2sf_budget budget,
                                  const a2sf_cache* cache, void* o, float* scores_full,
                                  void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!(score_rel_tol >= 0.0f && score_rel_tol < 1.0f)) return A2SF_EINVAL;   // also rejects NaN
  return prefill_impl(q, k, v, n, alpha, nullptr, score_rel_tol, budget, cache, o, scores_full,
                      workspace, workspace_bytes, hip_stream);
}

namespace {
inline bool bad_group(int32_t group) { return group < 1 || group > 8; }

// A chunk of a prompt for G K/V heads with `group` query heads each (1 = plain heads).
a2sf_status chunk_impl(const void* q, const void* k, const void* v, int32_t m, int32_t pos0, int32_t group,
                       float alpha, a2sf_budget budget, const a2sf_cache* cache, void* o, void* workspace,
                       size_t workspace_bytes, void* hip_stream) {
  a2sf_status s;
  if ((s = check_budget(budget)) != A2SF_OK) return s;
  if ((s = check_alpha(alpha)) != A2SF_OK) return s;
  if ((s = check_cache(cache, budget)) != A2SF_OK) return s;
  if (!q || !k || !v) return A2SF_EINVAL;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o)) return A2SF_EINVAL;
  if (bad_group(group)) return A2SF_ESHAPE;
  if (m < 1 || pos0 < 0 || (long long)pos0 + m > 0x7FFFFFFFLL) return A2SF_ESHAPE;
  if (m >= cache->capacity) return A2SF_ECAPACITY;   // a chunk needs room beside at least one slot
  if ((long long)cache->G * group * m > 0x7FFFFFFFLL) return A2SF_ESHAPE;
  const WsLayout w = ws_layout(cache->G * group, m, 0, cache->d, budget);   // one log-sum-exp row per QUERY head
  if (!workspace || misaligned(workspace) || workspace_bytes < w.total) return A2SF_EWORKSPACE;

  hipStream_t st = (hipStream_t)hip_stream;
  clear_stale_error();
  char* ws = (char*)workspace;
  float* lse2 = (float*)(ws + w.lse2);
  int32_t* len_old = (int32_t*)(ws + w.s_full);   // G ints fit where G * group * m floats would go
  int32_t* keep_idx = (int32_t*)(ws + w.keep_idx);
  int32_t* n_keep = (int32_t*)(ws + w.n_keep);
  const int G = cache->G, d = cache->d, C = cache->capacity;
  AttnRect rc{m, C, len_old};
  rc.kv_group = group;
  const float decay = alpha > 0.f ? powf(alpha, (float)m) : 0.f;   // 0^m = 0 for m >= 1
  // Where the kernels can read the chunk's K/V rows from the call's inputs, the rows are not
  // copied behind the cached ones first: the compaction copies in those that are kept.
  const bool two_source = cache->dtype == A2SF_BF16 && bf16_two_source_ok(d, rc, alpha);
  if (two_source) { rc.k2 = k; rc.v2 = v; }

  launch_chunk_append(k, v, m, pos0, *cache, len_old, !two_source, st);
  if (cache->dtype == A2SF_F32) {
    launch_attn_f32((const float*)q, (const float*)cache->k, (const float*)cache->v, G, rc, d,
                    (float*)o, lse2, st);
    launch_colscores_f32((const float*)q, (const float*)cache->k, lse2, G, rc, C, d, alpha, nullptr,
                         cache->scores, C, true, decay, st);
  } else {
    launch_attn_bf16(q, cache->k, cache->v, G, rc, d, o, lse2, st);
    launch_colscores_bf16(q, cache->k, lse2, G, rc, C, d, alpha, cache->scores, C, true, decay, st);
  }
  launch_select(cache->scores, cache->pos, cache->len, G, C, C, budget.select, budget.recent,
                keep_idx, n_keep, st);
  if (two_source)
    launch_compact(*cache, keep_idx, budget.select + budget.recent, n_keep, st, k, v, m, len_old);
  else
    launch_compact(*cache, keep_idx, budget.select + budget.recent, n_keep, st);
  return launch_status();
}
}  // namespace

a2sf_status a2sf_prefill_chunk(const void* q, const void* k, const void* v, int32_t m, int32_t pos0,
                               float alpha, a2sf_budget budget, const a2sf_cache* cache, void* o,
                               void* workspace, size_t workspace_bytes, void* hip_stream) {
  return chunk_impl(q, k, v, m, pos0, 1, alpha, budget, cache, o, workspace, workspace_bytes, hip_stream);
}

a2sf_status a2sf_prefill_chunk_gqa(const void* q, const void* k, const void* v, int32_t m, int32_t pos0,
                                   int32_t group, float alpha, a2sf_budget budget, const a2sf_cache* cache,
                                   void* o, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return chunk_impl(q, k, v, m, pos0, group, alpha, budget, cache, o, workspace, workspace_bytes, hip_stream);
}

a2sf_status a2sf_prefill_gqa(const void* q, const void* k, const void* v, int32_t n, int32_t group,
                             float alpha, a2sf_budget budget, const a2sf_cache* cache, void* o,
                             float* scores_full, void* workspace, size_t workspace_bytes,
                             void* hip_stream) {
  a2sf_status s;
  if ((s = check_budget(budget)) != A2SF_OK) return s;
  if ((s = check_alpha(alpha)) != A2SF_OK) return s;
  if ((s = check_cache(cache, budget)) != A2SF_OK) return s;
  if (!q || !k || !v) return A2SF_EINVAL;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(scores_full))
    return A2SF_EINVAL;
  if (n < 1 || bad_group(group)) return A2SF_ESHAPE;
  if ((long long)cache->G * group * n > 0x7FFFFFFFLL) return A2SF_ESHAPE;
  const int G = cache->G, d = cache->d;
  const WsLayout w = ws_layout(G * group, n, 0, d, budget);   // one log-sum-exp row per QUERY head
  if (!workspace || misaligned(workspace) || workspace_bytes < w.total) return A2SF_EWORKSPACE;

  hipStream_t st = (hipStream_t)hip_stream;
  clear_stale_error();
  char* ws = (char*)workspace;
  float* lse2 = (float*)(ws + w.lse2);
  float* s_full = scores_full ? scores_full : (float*)(ws + w.s_full);
  int32_t* keep_idx = (int32_t*)(ws + w.keep_idx);
  int32_t* n_keep = (int32_t*)(ws + w.n_keep);
  AttnRect rc{n, n, nullptr};
  rc.kv_group = group;
  // without outputs only the rows the score kernel will read need their log-sum-exp
  if (!o && cache->dtype == A2SF_BF16) rc.first_row = bf16_first_lse_row(n, cache->d, alpha);
  // in parts of kPrefillPartHeads query heads, as the plain prompt phase and for the same reason
  const size_t e = cache->dtype == A2SF_F32 ? 4 : 2;
  const int B = budget.select + budget.recent;
  const int part_kv = kPrefillPartHeads / group;   // K/V heads per part
  const int part = (cache->dtype == A2SF_BF16 && G >= 2 * part_kv) ? part_kv : G;
  for (int g0 = 0; g0 < G; g0 += part) {
    const int Gp = G - g0 < part ? G - g0 : part;
    const size_t kv0 = (size_t)g0 * n;          // first K/V row of the part
    const size_t q0 = kv0 * group;              // first query / output / log-sum-exp row
    const char* qp = (const char*)q + q0 * d * e;
    const char* kp = (const char*)k + kv0 * d * e;
    const char* vp = (const char*)v + kv0 * d * e;
    void* op = o ? (char*)o + q0 * d * e : nullptr;
    float* lp = lse2 + q0;
    float* sp = s_full + kv0;
    int32_t* kip = keep_idx + (size_t)g0 * B;
    int32_t* nkp = n_keep + g0;
    a2sf_cache cp = *cache;
    cp.G = Gp;
    cp.k = (char*)cache->k + (size_t)g0 * cache->capacity * d * e;
    cp.v = (char*)cache->v + (size_t)g0 * cache->capacity * d * e;
    cp.scores = cache->scores + (size_t)g0 * cache->capacity;
    cp.pos = cache->pos + (size_t)g0 * cache->capacity;
    cp.len = cache->len + g0;
    if (cache->dtype == A2SF_F32) {
      launch_attn_f32((const float*)qp, (const float*)kp, (const float*)vp, Gp, rc, d, (float*)op, lp, st);
      launch_colscores_f32((const float*)qp, (const float*)kp, lp, Gp, rc, n, d, alpha, nullptr, sp, n,
                           false, 0.f, st);
    } else {
      launch_attn_bf16(qp, kp, vp, Gp, rc, d, op, lp, st);
      launch_colscores_bf16(qp, kp, lp, Gp, rc, n, d, alpha, sp, n, false, 0.f, st);
    }
    launch_select(sp, nullptr, nullptr, Gp, n, n, budget.select, budget.recent, kip, nkp, st);
    launch_gather_prompt(kp, vp, sp, n, kip, B, nkp, cp, st);
  }
  return launch_status();
}

a2sf_status a2sf_decode_step_gqa(const void* q, const void* k_new, const void* v_new, int32_t t_pos,
                                 const a2sf_cache* cache, int32_t group, float alpha,
                                 a2sf_budget budget, int32_t mode, void* o, void* workspace,
                                 size_t workspace_bytes, void* hip_stream) {
  if (group == 1)
    return decode_impl(q, k_new, v_new, t_pos, cache, alpha, nullptr, budget, mode, o, workspace,
                       workspace_bytes, hip_stream);
  a2sf_status s;
  if ((s = check_budget(budget)) != A2SF_OK) return s;
  if ((s = check_alpha(alpha)) != A2SF_OK) return s;
  if ((s = check_cache(cache, budget)) != A2SF_OK) return s;
  if (!q || !k_new || !v_new || !o) return A2SF_EINVAL;
  if (misaligned(q) || misaligned(k_new) || misaligned(v_new) || misaligned(o)) return A2SF_EINVAL;
  if (t_pos < 0) return A2SF_EINVAL;
  if (mode != A2SF_EVICT_FAST && mode != A2SF_EVICT_STABLE) return A2SF_EINVAL;
  if (bad_group(group)) return A2SF_ESHAPE;
  if ((long long)group * cache->capacity > A2SF_GQA_MAX_LOGITS) return A2SF_ECAPACITY;
  const WsLayout w = ws_layout(cache->G, 0, cache->capacity, cache->d, budget);
  if (mode == A2SF_EVICT_STABLE && (!workspace || misaligned(workspace) || workspace_bytes < w.total))
    return A2SF_EWORKSPACE;

  hipStream_t st = (hipStream_t)hip_stream;
  clear_stale_error();
  // the split region of the workspace, as far as the caller's buffer reaches into it
  const bool has_split = workspace && !misaligned(workspace) && workspace_bytes > w.split;
  launch_decode_gqa(q, k_new, v_new, t_pos, *cache, group, alpha, budget.select, budget.recent,
                    mode == A2SF_EVICT_FAST, o, has_split ? (char*)workspace + w.split : nullptr,
                    has_split ? workspace_bytes - w.split : 0, st);
  if (mode == A2SF_EVICT_STABLE) {
    char* ws = (char*)workspace;
    int32_t* keep_idx = (int32_t*)(ws + w.keep_idx);
    int32_t* n_keep = (int32_t*)(ws + w.n_keep);
    launch_select(cache->scores, cache->pos, cache->len, cache->G, cache->capacity, cache->capacity,
                  budget.select, budget.recent, keep_idx, n_keep, st);
    launch_compact(*cache, keep_idx, budget.select + budget.recent, n_keep, st);
  }
  return launch_status();
}

a2sf_status a2sf_prefill_alpha_per_head(const void* q, const void* k, const void* v, int32_t n,
                                        const float* alpha_heads, float alpha_max,
                                        a2sf_budget budget, const a2sf_cache* cache, void* o,
                                        float* scores_full, void* workspace,
                                        size_t workspace_bytes, void* hip_stream) {
  if (!alpha_heads || ((uintptr_t)alpha_heads & 3u)) return A2SF_EINVAL;
  return prefill_impl(q, k, v, n, alpha_max, alpha_heads, 0.0f, budget, cache, o, scores_full,
                      workspace, workspace_bytes, hip_stream);
}

a2sf_status a2sf_decode_step(const void* q, const void* k_new, const void* v_new, int32_t t_pos,
                             const a2sf_cache* cache, float alpha, a2sf_budget budget,
                             int32_t mode, void* o, void* workspace, size_t workspace_bytes,
                             void* hip_stream) {
  return decode_impl(q, k_new, v_new, t_pos, cache, alpha, nullptr, budget, mode, o, workspace,
                     workspace_bytes, hip_stream);
}

a2sf_status a2sf_decode_step_static_ws(const void* q, const void* k_new, const void* v_new,
                                       int32_t t_pos, const a2sf_cache* cache, float alpha,
                                       a2sf_budget budget, int32_t mode, void* o, void* hip_stream) {
  // size check first (host only): what a2sf_decode_step would ask of its workspace argument
  a2sf_status s;
  if ((s = check_budget(budget)) != A2SF_OK) return s;
  if ((s = check_cache(cache, budget)) != A2SF_OK) return s;
  if (ws_layout(cache->G, 0, cache->capacity, cache->d, budget).total > (size_t)A2SF_STATIC_WS_BYTES)
    return A2SF_EWORKSPACE;
  void* ws = nullptr;
  if ((s = static_scratch(&ws)) != A2SF_OK) return s;
  return decode_impl(q, k_new, v_new, t_pos, cache, alpha, nullptr, budget, mode, o, ws,
                     (size_t)A2SF_STATIC_WS_BYTES, hip_stream);
}

a2sf_status a2sf_decode_step_alpha_per_head(const void* q, const void* k_new, const void* v_new,
                                            int32_t t_pos, const a2sf_cache* cache,
                                            const float* alpha_heads, a2sf_budget budget,
                                            int32_t mode, void* o, void* workspace,
                                            size_t workspace_bytes, void* hip_stream) {
  if (!alpha_heads || ((uintptr_t)alpha_heads & 3u)) return A2SF_EINVAL;
  return decode_impl(q, k_new, v_new, t_pos, cache, 1.0f, alpha_heads, budget, mode, o, workspace,
                     workspace_bytes, hip_stream);
}

a2sf_status a2sf_select(const float* scores, const int32_t* pos, const int32_t* len, int32_t G,
                        int32_t L, int32_t stride, a2sf_budget budget, int32_t* keep_idx,
                        int32_t* n_keep, void* hip_stream) {
  a2sf_status s;
  if ((s = check_budget(budget)) != A2SF_OK) return s;
  if (!scores || !keep_idx || !n_keep) return A2SF_EINVAL;
  if (misaligned(scores) || ((uintptr_t)pos & 3u) || ((uintptr_t)len & 3u) ||
      ((uintptr_t)keep_idx & 3u) || ((uintptr_t)n_keep & 3u))
    return A2SF_EINVAL;
  if (G < 1 || L < 1 || stride < L) return A2SF_ESHAPE;
  if ((long long)G * stride > 0x7FFFFFFFLL) return A2SF_ESHAPE;   // slots are indexed with 32 bits
  clear_stale_error();
  launch_select(scores, pos, len, G, L, stride, budget.select, budget.recent, keep_idx, n_keep,
                (hipStream_t)hip_stream);
  return launch_status();
}

a2sf_status a2sf_compact(const a2sf_cache* cache, const int32_t* keep_idx, int32_t keep_stride,
                         const int32_t* n_keep, void* hip_stream) {
  a2sf_budget any = {1, 0};
  a2sf_status s;
  if ((s = check_cache(cache, any)) != A2SF_OK) return s;
  if (!keep_idx || !n_keep) return A2SF_EINVAL;
  if (keep_stride < 1) return A2SF_ESHAPE;
  if (((uintptr_t)keep_idx & 3u) || ((uintptr_t)n_keep & 3u)) return A2SF_EINVAL;
  clear_stale_error();
  launch_compact(*cache, keep_idx, keep_stride, n_keep, (hipStream_t)hip_stream);
  return launch_status();
}

a2sf_status a2sf_ideal_similarity(const void* q, const void* k_all, int32_t n_stride,
                                  int32_t t_pos, const a2sf_cache* cache, float* cos_out,
                                  void* hip_stream) {
  a2sf_budget any = {1, 0};
  a2sf_status s;
  if ((s = check_cache(cache, any)) != A2SF_OK) return s;
  if (!q || !k_all || !cos_out) return A2SF_EINVAL;
  if (misaligned(q) || misaligned(k_all)) return A2SF_EINVAL;
  if (t_pos < 0 || t_pos >= A2SF_SIM_MAX_ROWS || n_stride <= t_pos) return A2SF_ESHAPE;
  clear_stale_error();
  launch_ideal_similarity(q, k_all, n_stride, t_pos + 1, *cache, cos_out, (hipStream_t)hip_stream);
  return launch_status();
}

a2sf_status a2sf_similarity_mean(const float* cos, int32_t steps, int32_t G, int32_t first_step,
                                 float* mean_out, void* hip_stream) {
  if (!cos || !mean_out || ((uintptr_t)cos & 3u) || ((uintptr_t)mean_out & 3u)) return A2SF_EINVAL;
  if (steps < 1 || G < 1 || first_step < 0 || first_step > steps) return A2SF_ESHAPE;
  clear_stale_error();
  launch_similarity_mean(cos, (long long)first_step * G, (long long)steps * G, mean_out,
                         (hipStream_t)hip_stream);
  return launch_status();
}

a2sf_status a2sf_decode_plan(int32_t G, int32_t capacity, int32_t d, int32_t* nsplit,
                             int32_t* rows_per_split, int32_t* wave_slots, int32_t* wave_heads) {
  if (G < 1 || (d != 64 && d != 128)) return A2SF_ESHAPE;
  if (capacity < 1 || capacity > A2SF_MAX_CAPACITY) return A2SF_ECAPACITY;
  const DecodePlan p = plan_decode(G, capacity, d);
  if (nsplit) *nsplit = p.nsplit;
  if (rows_per_split) *rows_per_split = p.rows_per_split;
  if (wave_slots) *wave_slots = p.wave_slots;
  if (wave_heads) *wave_heads = p.wave_heads;
  return A2SF_OK;
}

const char* a2sf_status_string(int32_t status) {
  switch (status) {
    case A2SF_OK: return "ok";
    case A2SF_EINVAL: return "invalid argument";
    case A2SF_ESHAPE: return "unsupported shape";
    case A2SF_EDTYPE: return "unsupported dtype";
    case A2SF_ECAPACITY: return "cache capacity too small or too large";
    case A2SF_EWORKSPACE: return "workspace missing or too small";
    case A2SF_EHIP: return "HIP launch error";
    default: return "unknown status";
  }
}

}  // extern "C"
