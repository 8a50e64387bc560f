"""MI355X-native A2SF hot path: masked attention fused with forgotten-score bookkeeping and
budgeted KV-cache eviction (arxiv 2407.20485).  All compute runs in liba2sf.so (HIP, gfx950)
behind the C ABI of include/a2sf.h; `binding` marshals arguments, `synth` draws workloads."""
from .binding import (A2SF_BF16, A2SF_EVICT_FAST, A2SF_EVICT_STABLE, A2SF_F32, A2SF_MAX_CAPACITY,
                      A2SFError, Cache, a2sf_compact, a2sf_decode_step, a2sf_prefill, a2sf_select,
                      a2sf_status_string, a2sf_workspace_bytes, a2sf_prefill_alpha_per_head,
                      a2sf_decode_step_alpha_per_head, a2sf_ideal_similarity,
                      a2sf_decode_step_static_ws, A2SF_STATIC_WS_BYTES, a2sf_similarity_mean,
                      a2sf_decode_plan, a2sf_prefill_windowed, a2sf_prefill_chunk,
                      a2sf_prefill_gqa, a2sf_decode_step_gqa, a2sf_prefill_chunk_gqa)

__all__ = ["A2SF_BF16", "A2SF_F32", "A2SF_EVICT_FAST", "A2SF_EVICT_STABLE", "A2SF_MAX_CAPACITY",
           "A2SFError", "Cache", "a2sf_compact", "a2sf_decode_step", "a2sf_prefill", "a2sf_select",
           "a2sf_status_string", "a2sf_workspace_bytes", "a2sf_prefill_alpha_per_head",
           "a2sf_decode_step_alpha_per_head", "a2sf_ideal_similarity", "a2sf_decode_step_static_ws",
           "A2SF_STATIC_WS_BYTES", "a2sf_similarity_mean", "a2sf_decode_plan", "a2sf_prefill_windowed", "a2sf_prefill_chunk",
           "a2sf_prefill_gqa", "a2sf_decode_step_gqa", "a2sf_prefill_chunk_gqa"]
