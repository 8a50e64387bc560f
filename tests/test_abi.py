"""CPU-only checks of the boundary: the shared library loads, exports every function that
include/a2sf.h declares, and rejects bad arguments on the host before any launch."""
import ctypes
import os
import re

import pytest

from paper_2407_20485_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "a2sf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(a2sf_[a-z_]+)\s*\(", text)))


def test_header_and_binding_agree():
    assert declared_functions() == sorted(B.EXPORTS)


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    for name in declared_functions():
        assert getattr(lib, name) is not None


def test_status_strings():
    assert B.a2sf_status_string(B.A2SF_OK) == "ok"
    assert "workspace" in B.a2sf_status_string(B.A2SF_EWORKSPACE)
    assert B.a2sf_status_string(99) == "unknown status"


def test_workspace_bytes():
    w = B.a2sf_workspace_bytes(4, 256, 65, 64, B.A2SF_F32, 32, 32)
    assert w >= 2 * 4 * 256 * 4 + 4 * 64 * 4
    assert B.a2sf_workspace_bytes(4, 256, 65, 96, B.A2SF_F32, 32, 32) == 0      # bad d
    assert B.a2sf_workspace_bytes(4, 256, 65, 64, 7, 32, 32) == 0               # bad dtype
    assert B.a2sf_workspace_bytes(4, 256, 65, 64, B.A2SF_F32, 0, 0) == 0        # empty budget
    assert B.a2sf_workspace_bytes(0, 256, 65, 64, B.A2SF_F32, 1, 1) == 0


FAKE = 0x10000  # a 16-byte aligned non-null "device pointer"; never dereferenced on these paths


def fake_cache(G=2, capacity=9, d=64, dtype=B.A2SF_F32, **over):
    f = dict(k=FAKE, v=FAKE, scores=FAKE, pos=FAKE, len=FAKE, G=G, capacity=capacity, d=d, dtype=dtype)
    f.update(over)
    return B.CacheStruct(**f)


def prefill_status(cache, n=16, alpha=0.3, select=4, recent=4, q=FAKE, ws=FAKE, ws_bytes=1 << 30):
    return B.lib().a2sf_prefill(q, FAKE, FAKE, n, alpha, B.Budget(select, recent), ctypes.byref(cache),
                                None, None, ws, ws_bytes, None)


def decode_status(cache, alpha=0.3, select=4, recent=4, mode=0, t_pos=5, o=FAKE, ws=FAKE, ws_bytes=1 << 30):
    return B.lib().a2sf_decode_step(FAKE, FAKE, FAKE, t_pos, ctypes.byref(cache), alpha,
                                    B.Budget(select, recent), mode, o, ws, ws_bytes, None)


@pytest.mark.parametrize("alpha", [-0.1, 1.5, float("nan"), float("inf")])
def test_alpha_domain(alpha):
    assert prefill_status(fake_cache(), alpha=alpha) == B.A2SF_EINVAL
    assert decode_status(fake_cache(), alpha=alpha) == B.A2SF_EINVAL


def test_prefill_argument_errors():
    assert prefill_status(fake_cache(), q=None) == B.A2SF_EINVAL
    assert prefill_status(fake_cache(), q=FAKE + 4) == B.A2SF_EINVAL            # misaligned
    assert prefill_status(fake_cache(), n=0) == B.A2SF_ESHAPE
    assert prefill_status(fake_cache(d=96)) == B.A2SF_ESHAPE
    assert prefill_status(fake_cache(dtype=5)) == B.A2SF_EDTYPE
    assert prefill_status(fake_cache(capacity=8)) == B.A2SF_ECAPACITY           # needs B+1 = 9
    assert prefill_status(fake_cache(capacity=B.A2SF_MAX_CAPACITY + 1)) == B.A2SF_ECAPACITY
    assert prefill_status(fake_cache(), select=0, recent=0) == B.A2SF_EINVAL
    assert prefill_status(fake_cache(), select=-1, recent=4) == B.A2SF_EINVAL
    assert prefill_status(fake_cache(), ws=None) == B.A2SF_EWORKSPACE
    assert prefill_status(fake_cache(), ws_bytes=16) == B.A2SF_EWORKSPACE
    assert prefill_status(fake_cache(k=None)) == B.A2SF_EINVAL


def test_decode_argument_errors():
    assert decode_status(fake_cache(), o=None) == B.A2SF_EINVAL
    assert decode_status(fake_cache(), mode=3) == B.A2SF_EINVAL
    assert decode_status(fake_cache(), t_pos=-1) == B.A2SF_EINVAL
    assert decode_status(fake_cache(capacity=8)) == B.A2SF_ECAPACITY
    # few heads with a long cache => split over tokens => needs the workspace; stable mode always does
    assert decode_status(fake_cache(G=2, capacity=700, select=50, recent=50), select=50, recent=50,
                         ws=None) == B.A2SF_EWORKSPACE
    assert decode_status(fake_cache(G=4096), mode=1, ws=None) == B.A2SF_EWORKSPACE


def test_static_workspace_entry_point_checks_its_limit_on_the_host():
    f = B.lib().a2sf_decode_step_static_ws
    big = fake_cache(G=4096, capacity=2049, d=128, dtype=B.A2SF_BF16)       # 33 MB of keep indices
    assert B.a2sf_workspace_bytes(4096, 0, 2049, 128, B.A2SF_BF16, 1024, 1024) > B.A2SF_STATIC_WS_BYTES
    assert f(FAKE, FAKE, FAKE, 5, ctypes.byref(big), 0.3, B.Budget(1024, 1024), 0, FAKE, None) == B.A2SF_EWORKSPACE
    assert f(FAKE, FAKE, FAKE, 5, ctypes.byref(fake_cache(capacity=8)), 0.3, B.Budget(4, 4), 0, FAKE,
             None) == B.A2SF_ECAPACITY
    assert f(FAKE, FAKE, FAKE, 5, None, 0.3, B.Budget(4, 4), 0, FAKE, None) == B.A2SF_EINVAL


def test_per_head_alpha_argument_errors():
    lib = B.lib()
    c = fake_cache()
    b = B.Budget(4, 4)
    assert lib.a2sf_prefill_alpha_per_head(FAKE, FAKE, FAKE, 16, None, 0.5, b, ctypes.byref(c), None,
                                           None, FAKE, 1 << 30, None) == B.A2SF_EINVAL
    assert lib.a2sf_prefill_alpha_per_head(FAKE, FAKE, FAKE, 16, FAKE, 1.5, b, ctypes.byref(c), None,
                                           None, FAKE, 1 << 30, None) == B.A2SF_EINVAL
    assert lib.a2sf_decode_step_alpha_per_head(FAKE, FAKE, FAKE, 5, ctypes.byref(c), None, b, 0, FAKE,
                                               FAKE, 1 << 30, None) == B.A2SF_EINVAL
    assert lib.a2sf_decode_step_alpha_per_head(FAKE, FAKE, FAKE, 5, ctypes.byref(c), FAKE + 2, b, 0, FAKE,
                                               FAKE, 1 << 30, None) == B.A2SF_EINVAL


def test_select_and_compact_argument_errors():
    lib = B.lib()
    assert lib.a2sf_select(None, None, None, 1, 8, 8, B.Budget(2, 2), FAKE, FAKE, None) == B.A2SF_EINVAL
    assert lib.a2sf_select(FAKE, None, None, 1, 8, 4, B.Budget(2, 2), FAKE, FAKE, None) == B.A2SF_ESHAPE
    assert lib.a2sf_select(FAKE, None, None, 1, 8, 8, B.Budget(0, 0), FAKE, FAKE, None) == B.A2SF_EINVAL
    c = fake_cache()
    assert lib.a2sf_compact(ctypes.byref(c), None, 8, FAKE, None) == B.A2SF_EINVAL
    assert lib.a2sf_compact(ctypes.byref(c), FAKE, 0, FAKE, None) == B.A2SF_ESHAPE


def test_select_rejects_misaligned_pointers_and_index_overflow():
    lib = B.lib()
    b = B.Budget(2, 2)
    assert lib.a2sf_select(FAKE + 4, None, None, 1, 8, 8, b, FAKE, FAKE, None) == B.A2SF_EINVAL     # scores: 16 bytes
    assert lib.a2sf_select(FAKE, FAKE + 2, None, 1, 8, 8, b, FAKE, FAKE, None) == B.A2SF_EINVAL     # pos: 4 bytes
    assert lib.a2sf_select(FAKE, None, None, 1, 8, 8, b, FAKE + 1, FAKE, None) == B.A2SF_EINVAL
    assert lib.a2sf_select(FAKE, None, None, 1 << 20, 1 << 12, 1 << 12, b, FAKE, FAKE, None) == B.A2SF_ESHAPE


def test_prefill_chunk_argument_errors():
    f = B.lib().a2sf_prefill_chunk
    c = fake_cache(capacity=40)
    b = B.Budget(4, 4)
    assert f(None, FAKE, FAKE, 8, 0, 0.3, b, ctypes.byref(c), None, FAKE, 1 << 30, None) == B.A2SF_EINVAL
    assert f(FAKE, FAKE, FAKE, 0, 0, 0.3, b, ctypes.byref(c), None, FAKE, 1 << 30, None) == B.A2SF_ESHAPE
    assert f(FAKE, FAKE, FAKE, 8, -1, 0.3, b, ctypes.byref(c), None, FAKE, 1 << 30, None) == B.A2SF_ESHAPE
    assert f(FAKE, FAKE, FAKE, 40, 0, 0.3, b, ctypes.byref(c), None, FAKE, 1 << 30, None) == B.A2SF_ECAPACITY
    assert f(FAKE, FAKE, FAKE, 8, 0, 1.3, b, ctypes.byref(c), None, FAKE, 1 << 30, None) == B.A2SF_EINVAL
    assert f(FAKE, FAKE, FAKE, 8, 0, 0.3, b, ctypes.byref(c), None, None, 0, None) == B.A2SF_EWORKSPACE
    assert f(FAKE, FAKE, FAKE, 8, 0, 0.3, b, ctypes.byref(c), None, FAKE, 64, None) == B.A2SF_EWORKSPACE


def test_grouped_query_argument_errors():
    lib = B.lib()
    c = fake_cache(capacity=40)
    b = B.Budget(4, 4)
    assert lib.a2sf_prefill_gqa(FAKE, FAKE, FAKE, 16, 9, 0.3, b, ctypes.byref(c), None, None, FAKE, 1 << 30,
                                None) == B.A2SF_ESHAPE                                   # group of 9
    assert lib.a2sf_prefill_gqa(FAKE, FAKE, FAKE, 16, 0, 0.3, b, ctypes.byref(c), None, None, FAKE, 1 << 30,
                                None) == B.A2SF_ESHAPE
    assert lib.a2sf_prefill_gqa(FAKE, FAKE, FAKE, 16, 4, 0.3, b, ctypes.byref(c), None, None, FAKE, 64,
                                None) == B.A2SF_EWORKSPACE
    assert lib.a2sf_prefill_gqa(None, FAKE, FAKE, 16, 4, 0.3, b, ctypes.byref(c), None, None, FAKE, 1 << 30,
                                None) == B.A2SF_EINVAL
    assert lib.a2sf_decode_step_gqa(FAKE, FAKE, FAKE, 5, ctypes.byref(c), 9, 0.3, b, 0, FAKE, None, 0,
                                    None) == B.A2SF_ESHAPE
    g = lib.a2sf_prefill_chunk_gqa
    assert g(FAKE, FAKE, FAKE, 8, 0, 9, 0.3, b, ctypes.byref(c), None, FAKE, 1 << 30, None) == B.A2SF_ESHAPE      # group of 9
    assert g(FAKE, FAKE, FAKE, 40, 0, 4, 0.3, b, ctypes.byref(c), None, FAKE, 1 << 30, None) == B.A2SF_ECAPACITY  # no room beside the chunk
    assert g(FAKE, FAKE, FAKE, 8, 0, 4, 0.3, b, ctypes.byref(c), None, FAKE, 64, None) == B.A2SF_EWORKSPACE
    assert g(FAKE, None, FAKE, 8, 0, 4, 0.3, b, ctypes.byref(c), None, FAKE, 1 << 30, None) == B.A2SF_EINVAL
    big = fake_cache(capacity=4096)
    assert lib.a2sf_decode_step_gqa(FAKE, FAKE, FAKE, 5, ctypes.byref(big), 8, 0.3, b, 0, FAKE, None, 0,
                                    None) == B.A2SF_ECAPACITY                            # 8 * 4096 logits
    assert lib.a2sf_decode_step_gqa(FAKE, FAKE, FAKE, 5, ctypes.byref(c), 4, 0.3, b, 1, FAKE, None, 0,
                                    None) == B.A2SF_EWORKSPACE                           # stable mode needs one
    assert lib.a2sf_decode_step_gqa(FAKE, FAKE, FAKE, 5, ctypes.byref(c), 4, 0.3, b, 0, None, None, 0,
                                    None) == B.A2SF_EINVAL


def test_decode_plan_is_a_host_query():
    assert B.a2sf_decode_plan(16384, 201, 128) == (1, 256, 4, 4)     # a wave per head, 256 slots in registers, four heads per wave
    assert B.a2sf_decode_plan(4200, 201, 128) == (1, 256, 4, 1)      # fewer heads: one head per wave
    assert B.a2sf_decode_plan(16384, 500, 128)[2:] == (8, 1)         # 512 slots: one head per wave
    nsplit, rows, wave, heads = B.a2sf_decode_plan(32, 3277, 128)     # few heads, long cache: tokens are split
    assert nsplit > 1 and rows % 64 == 0 and nsplit * rows >= 3277 and wave == 0 and heads == 1
    assert B.a2sf_decode_plan(320, 410, 128)[0] == 1
    lib = B.lib()
    assert lib.a2sf_decode_plan(0, 10, 128, None, None, None, None) == B.A2SF_ESHAPE
    assert lib.a2sf_decode_plan(4, 10, 100, None, None, None, None) == B.A2SF_ESHAPE
    assert lib.a2sf_decode_plan(4, B.A2SF_MAX_CAPACITY + 1, 128, None, None, None, None) == B.A2SF_ECAPACITY
    assert lib.a2sf_decode_plan(4, 10, 128, None, None, None, None) == B.A2SF_OK      # out pointers are optional


def test_similarity_mean_argument_errors():
    f = B.lib().a2sf_similarity_mean
    assert f(None, 4, 2, 1, FAKE, None) == B.A2SF_EINVAL
    assert f(FAKE, 4, 2, 1, None, None) == B.A2SF_EINVAL
    assert f(FAKE + 2, 4, 2, 1, FAKE, None) == B.A2SF_EINVAL
    assert f(FAKE, 0, 2, 0, FAKE, None) == B.A2SF_ESHAPE
    assert f(FAKE, 4, 2, 5, FAKE, None) == B.A2SF_ESHAPE


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/liba2sf.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        B.lib()


def test_ideal_similarity_argument_errors():
    f = B.lib().a2sf_ideal_similarity
    ok_cache = fake_cache()
    assert f(None, FAKE, 16, 3, ctypes.byref(ok_cache), FAKE, None) == B.A2SF_EINVAL
    assert f(FAKE, FAKE, 16, 3, ctypes.byref(ok_cache), None, None) == B.A2SF_EINVAL
    assert f(FAKE, FAKE + 4, 16, 3, ctypes.byref(ok_cache), FAKE, None) == B.A2SF_EINVAL      # misaligned
    assert f(FAKE, FAKE, 16, 16, ctypes.byref(ok_cache), FAKE, None) == B.A2SF_ESHAPE         # row outside k_all
    assert f(FAKE, FAKE, 1 << 20, 32768, ctypes.byref(ok_cache), FAKE, None) == B.A2SF_ESHAPE  # too long a row
    assert f(FAKE, FAKE, 16, -1, ctypes.byref(ok_cache), FAKE, None) == B.A2SF_ESHAPE
    assert f(FAKE, FAKE, 16, 3, ctypes.byref(fake_cache(d=96)), FAKE, None) == B.A2SF_ESHAPE
    assert f(FAKE, FAKE, 16, 3, None, FAKE, None) == B.A2SF_EINVAL
