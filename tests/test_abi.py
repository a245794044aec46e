"""Host-only checks of the C ABI: the library loads, exports every symbol include/fasth.h declares,
and validates its arguments before touching the GPU (so these run without one)."""
import ctypes
import os
import re

import pytest

from paper_2009_13977_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "fasth.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b((?:fasth|svd_layer|svd_sym|svd_rect)_\w+)\s*\(", text))


def test_library_exports_every_declared_symbol():
    lib = B.load_library()
    declared = _declared_symbols()
    assert declared == set(B.EXPORTED_SYMBOLS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_strerror_texts():
    for code in (0, -1, -2, -3, -4, -5):
        assert B.strerror(code)
    assert "unknown" in B.strerror(-99)


def test_workspace_bytes_and_shape_validation():
    assert B.fasth_workspace_bytes(1024, 1024, 32, 32) > 2 * 32 * 32 * 1024 * 4  # two sets of nb saved d x m matrices
    assert B.fasth_workspace_bytes(64, 64, 32, 7) == 0       # k does not divide n (Section 3.1)
    assert B.fasth_workspace_bytes(0, 64, 32, 32) == 0
    assert B.fasth_workspace_bytes(64, 64, 32, 256) == 0     # beyond the supported block size
    assert B.svd_layer_workspace_bytes(64, 64, 32, 32) > 2 * B.fasth_workspace_bytes(64, 64, 32, 32)
    assert B.fasth_sequential_workspace_bytes(64, 64, 32) >= 32 * 64 * 64 * 4


def _call_forward(shape, V=256, X=256, A=512, ws=1024, nbytes=1 << 40):
    return B.load_library().fasth_forward(ctypes.byref(shape), V, X, A, ws, nbytes, None)


def test_workspace_holds_the_hand_off_area_of_shared_columns():
    """Few long columns are shared by 2 to 8 workgroups that pass partial sums through the workspace: per column a
    256-byte head and np * 2 * np * 64 words of 8 bytes, which shapes outside that range do not pay for."""
    def area(d, n, m, k, np_):
        return m * (256 + np_ * 2 * np_ * 64 * 8)
    base = B.fasth_workspace_bytes(1024, 1024, 200, 32)   # too many columns for a team of 2: 400 workgroups
    team = B.fasth_workspace_bytes(1024, 1024, 100, 32)
    per_col = 2 * (1024 // 32) * 1024 * 4 + 2 * 1024 * 4  # saved inputs of both chains and both coefficient vectors
    assert team - (base - 100 * per_col) >= area(1024, 1024, 100, 32, 2)
    # more parts, more words: d = 4096 takes 8 parts
    w8 = B.fasth_workspace_bytes(4096, 64, 32, 64)
    w8_alone = B.fasth_workspace_bytes(4096, 64, 33, 64)  # 33 columns x 8 parts > 256 workgroups: no team
    assert w8 > area(4096, 64, 32, 64, 8)
    assert w8_alone < w8 + 2 * (2 * 4096 * 4 + 64 * 4) + 4096  # one more column, no hand-off area
    # steps of 128 rows (d = 1024 in four parts of 256): 64 words of 16 bytes per part and step, and per pair of
    # blocks of 64 rows the product of their rows and its transpose
    wide = B.fasth_workspace_bytes(1024, 1024, 64, 32)     # 256 workgroups
    narrow = B.fasth_workspace_bytes(1024, 1024, 65, 32)   # 260: two parts per column instead
    area_wide = 64 * (256 + 4 * 2 * 4 * 64 * 16)
    assert wide + per_col - narrow >= area_wide - area(1024, 1024, 65, 32, 2) + (1024 // 128) * 2 * 64 * 64 * 4


def test_wait_limit_is_host_state():
    B.fasth_set_wait_limit(0)
    B.fasth_set_wait_limit(-1)  # back to the default
    assert B.FASTH_ETIMEOUT == -6
    assert "gave up" in B.load_library().fasth_strerror(B.FASTH_ETIMEOUT).decode()


def test_forward_argument_errors_precede_any_gpu_call():
    ok = B.fasth_shape(64, 64, 32, 32, 0)
    assert _call_forward(B.fasth_shape(64, 64, 32, 7, 0)) == B.FASTH_EINVAL
    assert _call_forward(B.fasth_shape(64, 64, 0, 32, 0)) == B.FASTH_EINVAL
    assert _call_forward(B.fasth_shape(64, 64, 32, 32, 2)) == B.FASTH_EINVAL
    assert _call_forward(B.fasth_shape(64, 256, 32, 256, 0)) == B.FASTH_EUNSUPPORTED
    assert _call_forward(ok, V=None) == B.FASTH_EINVAL
    assert _call_forward(ok, X=260) == B.FASTH_EALIGN
    assert _call_forward(ok, nbytes=128) == B.FASTH_EWORKSPACE
    assert B.load_library().fasth_forward(None, 256, 256, 256, 256, 1 << 40, None) == B.FASTH_EINVAL


def test_static_forward_argument_errors_precede_any_gpu_call():
    lib = B.load_library()
    ok = B.fasth_shape(64, 64, 32, 32, 0)
    assert lib.fasth_forward_static(ctypes.byref(ok), None, 256, 256, None) == B.FASTH_EINVAL
    assert lib.fasth_forward_static(ctypes.byref(ok), 256, 260, 256, None) == B.FASTH_EALIGN
    assert lib.fasth_forward_static(ctypes.byref(B.fasth_shape(64, 64, 32, 7, 0)), 256, 256, 256, None) == B.FASTH_EINVAL
    # factors and partial Gram matrices of this shape need more than the fixed scratch array holds
    big = B.fasth_shape(16384, 16384, 32, 128, 0)
    assert lib.fasth_forward_static(ctypes.byref(big), 256, 256, 256, None) == B.FASTH_EUNSUPPORTED


def test_backward_and_layer_argument_errors():
    lib = B.load_library()
    ok = B.fasth_shape(64, 64, 32, 32, 0)
    assert lib.fasth_backward(ctypes.byref(ok), 256, 256, None, 256, 256, 1 << 40, None) == B.FASTH_EINVAL
    assert lib.fasth_backward(ctypes.byref(ok), 256, 256, 256, 256, 256, 16, None) == B.FASTH_EWORKSPACE
    assert lib.fasth_sequential_forward(ctypes.byref(ok), 256, None, 256, None) == B.FASTH_EINVAL
    assert lib.fasth_sequential_backward(ctypes.byref(ok), 256, 256, 256, 256, 256, 256, 16, None) == B.FASTH_EWORKSPACE
    s = B.fasth_svd_shape(64, 64, 32, 5)
    assert lib.svd_layer_apply(ctypes.byref(s), 256, 256, 256, 256, 256, 256, 1 << 40, None) == B.FASTH_EINVAL
    s = B.fasth_svd_shape(64, 64, 32, 32)
    assert lib.svd_layer_apply(ctypes.byref(s), 256, 256, 256, 256, 256, 256, 16, None) == B.FASTH_EWORKSPACE
    assert lib.svd_layer_inverse_apply(ctypes.byref(s), 256, 8, 256, 256, 256, 256, 1 << 40, None) == B.FASTH_EALIGN
    assert lib.svd_layer_apply_backward(ctypes.byref(s), 256, 256, 256, 256, 256, 256, 256, None, 256, 1 << 40,
                                        None) == B.FASTH_EINVAL


def test_binding_refuses_cpu_tensors():
    import torch
    t = torch.zeros(4, 4)
    with pytest.raises(ValueError):
        B.fasth_forward(t, t, t, t, 2)


def test_block_size_search_argument_errors():
    lib = B.load_library()
    ok = B.fasth_shape(64, 64, 32, 0, 0)
    best = ctypes.c_int(0)
    call = lambda **kw: lib.fasth_tune_block_size(ctypes.byref(kw.get("shape", ok)), None, 0, kw.get("reps", 3),
                                                  kw.get("V", 256), 256, 256, 256, 256, 256, 256, 1 << 40,
                                                  ctypes.byref(best), None, None)
    assert call(reps=0) == B.FASTH_EINVAL
    assert call(V=None) == B.FASTH_EINVAL
    assert call(V=260) == B.FASTH_EALIGN
    assert call(shape=B.fasth_shape(64, 64, 0, 0, 0)) == B.FASTH_EINVAL


def test_rectangular_layer_argument_errors():
    lib = B.load_library()
    ok = B.fasth_rect_shape(96, 64, 96, 64, 8, 32)
    assert B.svd_rect_workspace_bytes(96, 64, 96, 64, 8, 32) > 0
    assert B.svd_rect_workspace_bytes(96, 64, 96, 60, 8, 32) == 0      # k does not divide n_v
    assert B.svd_rect_workspace_bytes(96, 20000, 96, 64, 8, 32) == 0   # cols beyond the supported range
    bad = B.fasth_rect_shape(96, 64, 96, 60, 8, 32)
    assert lib.svd_rect_apply(ctypes.byref(bad), 256, 256, 256, 256, 256, 256, 1 << 40, None) == B.FASTH_EINVAL
    assert lib.svd_rect_apply(ctypes.byref(ok), 256, None, 256, 256, 256, 256, 1 << 40, None) == B.FASTH_EINVAL
    assert lib.svd_rect_apply(ctypes.byref(ok), 256, 256, 256, 260, 256, 256, 1 << 40, None) == B.FASTH_EALIGN
    assert lib.svd_rect_apply(ctypes.byref(ok), 256, 256, 256, 256, 256, 256, 16, None) == B.FASTH_EWORKSPACE
    assert lib.svd_rect_apply_backward(ctypes.byref(ok), 256, 256, 256, 256, 256, None, 256, 256, 256, 1 << 40,
                                       None) == B.FASTH_EINVAL
    assert lib.svd_rect_apply_backward(ctypes.byref(ok), 256, 256, 256, 256, 256, 256, 256, 256, 256, 16,
                                       None) == B.FASTH_EWORKSPACE
