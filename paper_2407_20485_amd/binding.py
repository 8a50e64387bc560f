"""ctypes binding of liba2sf.so - argument marshalling only.

Every function has the name and the arguments of its C entry point (include/a2sf.h).
torch tensors are accepted wherever the C side takes a device pointer; torch is used for
device memory and for the current stream handle, nothing else.  There is no CPU fallback:
if the shared library is missing the import of a symbol fails loudly.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liba2sf.so")

A2SF_OK, A2SF_EINVAL, A2SF_ESHAPE, A2SF_EDTYPE, A2SF_ECAPACITY, A2SF_EWORKSPACE, A2SF_EHIP = range(7)
A2SF_F32, A2SF_BF16 = 0, 1
A2SF_EVICT_FAST, A2SF_EVICT_STABLE = 0, 1
A2SF_MAX_CAPACITY = 36864
A2SF_STATIC_WS_BYTES = 16 << 20

EXPORTS = ("a2sf_workspace_bytes", "a2sf_prefill", "a2sf_decode_step", "a2sf_select",
           "a2sf_compact", "a2sf_status_string", "a2sf_prefill_alpha_per_head",
           "a2sf_decode_step_alpha_per_head", "a2sf_ideal_similarity", "a2sf_decode_step_static_ws",
           "a2sf_similarity_mean", "a2sf_decode_plan", "a2sf_prefill_windowed",
           "a2sf_prefill_chunk", "a2sf_prefill_gqa", "a2sf_decode_step_gqa", "a2sf_prefill_chunk_gqa")


class Budget(ctypes.Structure):
    _fields_ = [("select", ctypes.c_int32), ("recent", ctypes.c_int32)]


class CacheStruct(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("scores", ctypes.c_void_p),
                ("pos", ctypes.c_void_p), ("len", ctypes.c_void_p), ("G", ctypes.c_int32),
                ("capacity", ctypes.c_int32), ("d", ctypes.c_int32), ("dtype", ctypes.c_int32)]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2407_20485_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
        L.a2sf_workspace_bytes.restype = sz
        L.a2sf_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, Budget]
        L.a2sf_prefill.restype = i32
        L.a2sf_prefill.argtypes = [vp, vp, vp, i32, f32, Budget, ctypes.POINTER(CacheStruct), vp, vp,
                                   vp, sz, vp]
        L.a2sf_prefill_windowed.restype = i32
        L.a2sf_prefill_windowed.argtypes = [vp, vp, vp, i32, f32, f32, Budget, ctypes.POINTER(CacheStruct), vp,
                                            vp, vp, sz, vp]
        L.a2sf_prefill_chunk.restype = i32
        L.a2sf_prefill_chunk.argtypes = [vp, vp, vp, i32, i32, f32, Budget, ctypes.POINTER(CacheStruct), vp,
                                         vp, sz, vp]
        L.a2sf_prefill_chunk_gqa.restype = i32
        L.a2sf_prefill_chunk_gqa.argtypes = [vp, vp, vp, i32, i32, i32, f32, Budget, ctypes.POINTER(CacheStruct),
                                             vp, vp, sz, vp]
        L.a2sf_prefill_gqa.restype = i32
        L.a2sf_prefill_gqa.argtypes = [vp, vp, vp, i32, i32, f32, Budget, ctypes.POINTER(CacheStruct), vp, vp,
                                       vp, sz, vp]
        L.a2sf_decode_step_gqa.restype = i32
        L.a2sf_decode_step_gqa.argtypes = [vp, vp, vp, i32, ctypes.POINTER(CacheStruct), i32, f32, Budget, i32,
                                           vp, vp, sz, vp]
        L.a2sf_decode_step.restype = i32
        L.a2sf_decode_step.argtypes = [vp, vp, vp, i32, ctypes.POINTER(CacheStruct), f32, Budget, i32,
                                       vp, vp, sz, vp]
        L.a2sf_decode_step_static_ws.restype = i32
        L.a2sf_decode_step_static_ws.argtypes = [vp, vp, vp, i32, ctypes.POINTER(CacheStruct), f32, Budget,
                                                 i32, vp, vp]
        L.a2sf_prefill_alpha_per_head.restype = i32
        L.a2sf_prefill_alpha_per_head.argtypes = [vp, vp, vp, i32, vp, f32, Budget,
                                                  ctypes.POINTER(CacheStruct), vp, vp, vp, sz, vp]
        L.a2sf_decode_step_alpha_per_head.restype = i32
        L.a2sf_decode_step_alpha_per_head.argtypes = [vp, vp, vp, i32, ctypes.POINTER(CacheStruct), vp,
                                                      Budget, i32, vp, vp, sz, vp]
        L.a2sf_select.restype = i32
        L.a2sf_select.argtypes = [vp, vp, vp, i32, i32, i32, Budget, vp, vp, vp]
        L.a2sf_compact.restype = i32
        L.a2sf_compact.argtypes = [ctypes.POINTER(CacheStruct), vp, i32, vp, vp]
        L.a2sf_ideal_similarity.restype = i32
        L.a2sf_ideal_similarity.argtypes = [vp, vp, i32, i32, ctypes.POINTER(CacheStruct), vp, vp]
        L.a2sf_similarity_mean.restype = i32
        L.a2sf_similarity_mean.argtypes = [vp, i32, i32, i32, vp, vp]
        L.a2sf_decode_plan.restype = i32
        L.a2sf_decode_plan.argtypes = [i32, i32, i32, ctypes.POINTER(i32), ctypes.POINTER(i32),
                                       ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.a2sf_status_string.restype = ctypes.c_char_p
        L.a2sf_status_string.argtypes = [i32]
        _lib = L
    return _lib


class A2SFError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"a2sf status {status}: {a2sf_status_string(status)}")


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, torch.Tensor):
        return x.data_ptr()
    return int(x)


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    return int(stream)


def _check(status: int):
    if status != A2SF_OK:
        raise A2SFError(status)


def dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return A2SF_F32
    if t == torch.bfloat16:
        return A2SF_BF16
    raise A2SFError(A2SF_EDTYPE)


class Cache:
    """Device buffers of a KV cache for G heads plus the matching C struct."""

    def __init__(self, G: int, capacity: int, d: int, dtype: torch.dtype, device="cuda"):
        self.G, self.capacity, self.d, self.dtype = G, capacity, d, dtype
        self.k = torch.zeros((G, capacity, d), dtype=dtype, device=device)
        self.v = torch.zeros((G, capacity, d), dtype=dtype, device=device)
        self.scores = torch.zeros((G, capacity), dtype=torch.float32, device=device)
        self.pos = torch.zeros((G, capacity), dtype=torch.int32, device=device)
        self.len = torch.zeros((G,), dtype=torch.int32, device=device)

    def struct(self) -> CacheStruct:
        return CacheStruct(self.k.data_ptr(), self.v.data_ptr(), self.scores.data_ptr(),
                           self.pos.data_ptr(), self.len.data_ptr(), self.G, self.capacity, self.d,
                           dtype_code(self.dtype))

    def tensors(self):
        return (self.k, self.v, self.scores, self.pos, self.len)

    def snapshot(self):
        return [t.clone() for t in self.tensors()]

    def restore(self, snap):
        for t, s in zip(self.tensors(), snap):
            t.copy_(s)


def _cache_struct(cache):
    return cache.struct() if isinstance(cache, Cache) else cache


def a2sf_status_string(status: int) -> str:
    return lib().a2sf_status_string(int(status)).decode()


def a2sf_workspace_bytes(G, n_max, capacity, d, dtype, select, recent) -> int:
    return int(lib().a2sf_workspace_bytes(G, n_max, capacity, d, dtype, Budget(select, recent)))


def a2sf_prefill(q, k, v, n, alpha, select, recent, cache, o=None, scores_full=None,
                 workspace=None, workspace_bytes=None, stream=None):
    cs = _cache_struct(cache)
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().a2sf_prefill(_ptr(q), _ptr(k), _ptr(v), n, alpha, Budget(select, recent),
                              ctypes.byref(cs), _ptr(o), _ptr(scores_full), _ptr(workspace),
                              workspace_bytes, _stream(stream)))


def a2sf_prefill_windowed(q, k, v, n, alpha, score_rel_tol, select, recent, cache, o=None, scores_full=None,
                          workspace=None, workspace_bytes=None, stream=None):
    cs = _cache_struct(cache)
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().a2sf_prefill_windowed(_ptr(q), _ptr(k), _ptr(v), n, alpha, score_rel_tol,
                                       Budget(select, recent), ctypes.byref(cs), _ptr(o), _ptr(scores_full),
                                       _ptr(workspace), workspace_bytes, _stream(stream)))


def a2sf_prefill_chunk(q, k, v, m, pos0, alpha, select, recent, cache, o=None, workspace=None,
                       workspace_bytes=None, stream=None):
    cs = _cache_struct(cache)
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().a2sf_prefill_chunk(_ptr(q), _ptr(k), _ptr(v), m, pos0, alpha, Budget(select, recent),
                                    ctypes.byref(cs), _ptr(o), _ptr(workspace), workspace_bytes,
                                    _stream(stream)))


def a2sf_prefill_chunk_gqa(q, k, v, m, pos0, group, alpha, select, recent, cache, o=None, workspace=None,
                           workspace_bytes=None, stream=None):
    cs = _cache_struct(cache)
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().a2sf_prefill_chunk_gqa(_ptr(q), _ptr(k), _ptr(v), m, pos0, group, alpha, Budget(select, recent),
                                        ctypes.byref(cs), _ptr(o), _ptr(workspace), workspace_bytes,
                                        _stream(stream)))


def a2sf_prefill_gqa(q, k, v, n, group, alpha, select, recent, cache, o=None, scores_full=None,
                     workspace=None, workspace_bytes=None, stream=None):
    cs = _cache_struct(cache)
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().a2sf_prefill_gqa(_ptr(q), _ptr(k), _ptr(v), n, group, alpha, Budget(select, recent),
                                  ctypes.byref(cs), _ptr(o), _ptr(scores_full), _ptr(workspace),
                                  workspace_bytes, _stream(stream)))


def a2sf_decode_step_gqa(q, k_new, v_new, t_pos, cache, group, alpha, select, recent, o,
                         mode=A2SF_EVICT_FAST, workspace=None, workspace_bytes=None, stream=None):
    cs = _cache_struct(cache)
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().a2sf_decode_step_gqa(_ptr(q), _ptr(k_new), _ptr(v_new), t_pos, ctypes.byref(cs), group,
                                      alpha, Budget(select, recent), mode, _ptr(o), _ptr(workspace),
                                      workspace_bytes, _stream(stream)))


def a2sf_decode_step(q, k_new, v_new, t_pos, cache, alpha, select, recent, o,
                     mode=A2SF_EVICT_FAST, workspace=None, workspace_bytes=None, stream=None):
    cs = _cache_struct(cache)
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().a2sf_decode_step(_ptr(q), _ptr(k_new), _ptr(v_new), t_pos, ctypes.byref(cs), alpha,
                                  Budget(select, recent), mode, _ptr(o), _ptr(workspace),
                                  workspace_bytes, _stream(stream)))


def a2sf_decode_step_static_ws(q, k_new, v_new, t_pos, cache, alpha, select, recent, o,
                               mode=A2SF_EVICT_FAST, stream=None):
    cs = _cache_struct(cache)
    _check(lib().a2sf_decode_step_static_ws(_ptr(q), _ptr(k_new), _ptr(v_new), t_pos, ctypes.byref(cs),
                                            alpha, Budget(select, recent), mode, _ptr(o), _stream(stream)))


def a2sf_prefill_alpha_per_head(q, k, v, n, alpha_heads, alpha_max, select, recent, cache, o=None,
                                scores_full=None, workspace=None, workspace_bytes=None, stream=None):
    cs = _cache_struct(cache)
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().a2sf_prefill_alpha_per_head(_ptr(q), _ptr(k), _ptr(v), n, _ptr(alpha_heads), alpha_max,
                                             Budget(select, recent), ctypes.byref(cs), _ptr(o),
                                             _ptr(scores_full), _ptr(workspace), workspace_bytes,
                                             _stream(stream)))


def a2sf_decode_step_alpha_per_head(q, k_new, v_new, t_pos, cache, alpha_heads, select, recent, o,
                                    mode=A2SF_EVICT_FAST, workspace=None, workspace_bytes=None,
                                    stream=None):
    cs = _cache_struct(cache)
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().a2sf_decode_step_alpha_per_head(_ptr(q), _ptr(k_new), _ptr(v_new), t_pos,
                                                 ctypes.byref(cs), _ptr(alpha_heads),
                                                 Budget(select, recent), mode, _ptr(o), _ptr(workspace),
                                                 workspace_bytes, _stream(stream)))


def a2sf_select(scores, pos, length, G, L, stride, select, recent, keep_idx, n_keep, stream=None):
    _check(lib().a2sf_select(_ptr(scores), _ptr(pos), _ptr(length), G, L, stride,
                             Budget(select, recent), _ptr(keep_idx), _ptr(n_keep), _stream(stream)))


def a2sf_ideal_similarity(q, k_all, n_stride, t_pos, cache, cos_out, stream=None):
    cs = _cache_struct(cache)
    _check(lib().a2sf_ideal_similarity(_ptr(q), _ptr(k_all), n_stride, t_pos, ctypes.byref(cs),
                                       _ptr(cos_out), _stream(stream)))


def a2sf_similarity_mean(cos, steps, G, first_step, mean_out, stream=None):
    _check(lib().a2sf_similarity_mean(_ptr(cos), steps, G, first_step, _ptr(mean_out), _stream(stream)))


def a2sf_decode_plan(G, capacity, d):
    """(nsplit, rows_per_split, wave_slots, wave_heads) of a2sf_decode_step for these sizes."""
    a, b, c, h = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    _check(lib().a2sf_decode_plan(G, capacity, d, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c),
                                  ctypes.byref(h)))
    return a.value, b.value, c.value, h.value


def a2sf_compact(cache, keep_idx, keep_stride, n_keep, stream=None):
    cs = _cache_struct(cache)
    _check(lib().a2sf_compact(ctypes.byref(cs), _ptr(keep_idx), keep_stride, _ptr(n_keep),
                              _stream(stream)))
