"""ctypes binding of libfasth.so: the same entry points as include/fasth.h.

Argument marshalling only. torch supplies device memory and the current HIP
stream; every step of the computation runs in the library's kernels. There is
no fallback: if the shared library is missing or a call fails, an exception is
raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG_DIR, "libfasth.so")

FASTH_OK = 0
FASTH_EINVAL = -1
FASTH_EWORKSPACE = -2
FASTH_EALIGN = -3
FASTH_EHIP = -4
FASTH_EUNSUPPORTED = -5
FASTH_ETIMEOUT = -6

EXPORTED_SYMBOLS = (
    "fasth_strerror",
    "fasth_workspace_bytes",
    "fasth_forward",
    "fasth_forward_static",
    "fasth_prepare",
    "fasth_apply",
    "fasth_backward",
    "fasth_tune_block_size",
    "fasth_sequential_workspace_bytes",
    "fasth_sequential_forward",
    "fasth_sequential_backward",
    "svd_layer_workspace_bytes",
    "svd_layer_apply",
    "svd_layer_inverse_apply",
    "svd_layer_apply_backward",
    "svd_layer_inverse_apply_backward",
    "svd_sym_apply",
    "svd_sym_apply_backward",
    "svd_rect_workspace_bytes",
    "svd_rect_apply",
    "svd_rect_apply_backward",
    "svd_layer_log_abs_det",
    "fasth_kernel_name",
    "fasth_profile_enable",
    "fasth_profile_collect",
    "fasth_profile_variant",
    "fasth_measure_peaks",
    "fasth_wait_status",
    "fasth_set_wait_limit",
)


class fasth_shape(ctypes.Structure):
    _fields_ = [("d", ctypes.c_int), ("n", ctypes.c_int), ("m", ctypes.c_int), ("k", ctypes.c_int),
                ("transpose", ctypes.c_int)]


class fasth_svd_shape(ctypes.Structure):
    _fields_ = [("d", ctypes.c_int), ("n", ctypes.c_int), ("m", ctypes.c_int), ("k", ctypes.c_int)]


class fasth_rect_shape(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int), ("cols", ctypes.c_int), ("n_u", ctypes.c_int), ("n_v", ctypes.c_int),
                ("m", ctypes.c_int), ("k", ctypes.c_int)]


class FasthError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} (code {code})")


_lib: Optional[ctypes.CDLL] = None


def load_library() -> ctypes.CDLL:
    """Load libfasth.so (built by `python -m paper_2009_13977_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    path = os.environ.get("FASTH_LIBRARY_PATH", LIB_PATH)  # another build of the same library, e.g. for an A/B timing
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} is missing: build it with `python -m paper_2009_13977_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(path)
    P, S, I = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    shp, sshp = ctypes.POINTER(fasth_shape), ctypes.POINTER(fasth_svd_shape)
    lib.fasth_strerror.restype = ctypes.c_char_p
    lib.fasth_strerror.argtypes = [I]
    lib.fasth_workspace_bytes.restype = S
    lib.fasth_workspace_bytes.argtypes = [shp]
    lib.fasth_forward.restype = I
    lib.fasth_forward.argtypes = [shp, P, P, P, P, S, P]
    lib.fasth_forward_static.restype = I
    lib.fasth_forward_static.argtypes = [shp, P, P, P, P]
    lib.fasth_backward.restype = I
    lib.fasth_backward.argtypes = [shp, P, P, P, P, P, S, P]
    lib.fasth_tune_block_size.restype = I
    lib.fasth_tune_block_size.argtypes = [shp, ctypes.POINTER(ctypes.c_int), I, I, P, P, P, P, P, P, P, S,
                                          ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_float), P]
    lib.fasth_prepare.restype = I
    lib.fasth_prepare.argtypes = [shp, P, P, S, P]
    lib.fasth_apply.restype = I
    lib.fasth_apply.argtypes = [shp, P, P, P, P, S, I, P]
    lib.fasth_sequential_workspace_bytes.restype = S
    lib.fasth_sequential_workspace_bytes.argtypes = [shp]
    lib.fasth_sequential_forward.restype = I
    lib.fasth_sequential_forward.argtypes = [shp, P, P, P, P]
    lib.fasth_sequential_backward.restype = I
    lib.fasth_sequential_backward.argtypes = [shp, P, P, P, P, P, P, S, P]
    lib.svd_layer_workspace_bytes.restype = S
    lib.svd_layer_workspace_bytes.argtypes = [sshp]
    for name in ("svd_layer_apply", "svd_layer_inverse_apply"):
        fn = getattr(lib, name)
        fn.restype = I
        fn.argtypes = [sshp, P, P, P, P, P, P, S, P]
    for name in ("svd_layer_apply_backward", "svd_layer_inverse_apply_backward"):
        fn = getattr(lib, name)
        fn.restype = I
        fn.argtypes = [sshp, P, P, P, P, P, P, P, P, P, S, P]
    lib.svd_sym_apply.restype = I
    lib.svd_sym_apply.argtypes = [sshp, I, P, P, P, P, P, S, P]
    lib.svd_sym_apply_backward.restype = I
    lib.svd_sym_apply_backward.argtypes = [sshp, I, P, P, P, P, P, P, P, S, P]
    rshp = ctypes.POINTER(fasth_rect_shape)
    lib.svd_rect_workspace_bytes.restype = S
    lib.svd_rect_workspace_bytes.argtypes = [rshp]
    lib.svd_rect_apply.restype = I
    lib.svd_rect_apply.argtypes = [rshp, P, P, P, P, P, P, S, P]
    lib.svd_rect_apply_backward.restype = I
    lib.svd_rect_apply_backward.argtypes = [rshp, P, P, P, P, P, P, P, P, P, S, P]
    lib.svd_layer_log_abs_det.restype = I
    lib.svd_layer_log_abs_det.argtypes = [I, P, P, P, P]
    lib.fasth_kernel_name.restype = ctypes.c_char_p
    lib.fasth_kernel_name.argtypes = [I]
    lib.fasth_profile_enable.restype = I
    lib.fasth_profile_enable.argtypes = [I]
    lib.fasth_profile_collect.restype = I
    lib.fasth_profile_collect.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int)]
    lib.fasth_profile_variant.restype = ctypes.c_char_p
    lib.fasth_profile_variant.argtypes = [I]
    lib.fasth_wait_status.restype = I
    lib.fasth_wait_status.argtypes = [P]
    lib.fasth_set_wait_limit.restype = I
    lib.fasth_set_wait_limit.argtypes = [I]
    lib.fasth_measure_peaks.restype = I
    lib.fasth_measure_peaks.argtypes = [P, S, I, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float),
                                        ctypes.POINTER(ctypes.c_float), P]
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load_library().fasth_strerror(int(code)).decode()


def _check(code: int, where: str) -> None:
    if code != FASTH_OK:
        raise FasthError(code, where)


def _ptr(t, name: str) -> int:
    import torch
    if not isinstance(t, torch.Tensor):
        raise TypeError(f"{name}: expected a torch.Tensor")
    if not t.is_cuda:
        raise ValueError(f"{name}: must live in GPU memory")
    if t.dtype != torch.float32 and name != "workspace":
        raise ValueError(f"{name}: must be float32")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    return t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _shape(d, n, m, k, transpose=False) -> fasth_shape:
    return fasth_shape(int(d), int(n), int(m), int(k), 1 if transpose else 0)


def fasth_workspace_bytes(d: int, n: int, m: int, k: int) -> int:
    return int(load_library().fasth_workspace_bytes(ctypes.byref(_shape(d, n, m, k))))


def fasth_sequential_workspace_bytes(d: int, n: int, m: int) -> int:
    return int(load_library().fasth_sequential_workspace_bytes(ctypes.byref(_shape(d, n, m, 1))))


def svd_layer_workspace_bytes(d: int, n: int, m: int, k: int) -> int:
    return int(load_library().svd_layer_workspace_bytes(ctypes.byref(fasth_svd_shape(int(d), int(n), int(m), int(k)))))


def new_workspace(nbytes: int, device="cuda"):
    import torch
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)


def fasth_forward(V, X, A, workspace, k: int, transpose: bool = False) -> None:
    n, d = V.shape
    m = X.shape[1]
    assert X.shape == (d, m) and A.shape == (d, m)
    shape = _shape(d, n, m, k, transpose)
    rc = load_library().fasth_forward(ctypes.byref(shape), _ptr(V, "V"), _ptr(X, "X"), _ptr(A, "A"),
                                      _ptr(workspace, "workspace"), workspace.numel(), _stream())
    _check(rc, "fasth_forward")


def fasth_forward_static(V, X, A, k: int, transpose: bool = False) -> None:
    n, d = V.shape
    m = X.shape[1]
    assert X.shape == (d, m) and A.shape == (d, m)
    shape = _shape(d, n, m, k, transpose)
    rc = load_library().fasth_forward_static(ctypes.byref(shape), _ptr(V, "V"), _ptr(X, "X"), _ptr(A, "A"), _stream())
    _check(rc, "fasth_forward_static")


def fasth_prepare(V, m: int, workspace, k: int) -> None:
    n, d = V.shape
    shape = _shape(d, n, m, k, False)
    rc = load_library().fasth_prepare(ctypes.byref(shape), _ptr(V, "V"), _ptr(workspace, "workspace"),
                                      workspace.numel(), _stream())
    _check(rc, "fasth_prepare")


def fasth_apply(V, X, A, workspace, k: int, transpose: bool = False, save_for_backward: bool = False) -> None:
    n, d = V.shape
    m = X.shape[1]
    assert X.shape == (d, m) and A.shape == (d, m)
    shape = _shape(d, n, m, k, transpose)
    rc = load_library().fasth_apply(ctypes.byref(shape), _ptr(V, "V"), _ptr(X, "X"), _ptr(A, "A"),
                                    _ptr(workspace, "workspace"), workspace.numel(),
                                    1 if save_for_backward else 0, _stream())
    _check(rc, "fasth_apply")


def fasth_backward(V, G, dV, dX, workspace, k: int, transpose: bool = False) -> None:
    n, d = V.shape
    m = G.shape[1]
    assert G.shape == (d, m) and dX.shape == (d, m) and dV.shape == (n, d)
    shape = _shape(d, n, m, k, transpose)
    rc = load_library().fasth_backward(ctypes.byref(shape), _ptr(V, "V"), _ptr(G, "G"), _ptr(dV, "dV"),
                                       _ptr(dX, "dX"), _ptr(workspace, "workspace"), workspace.numel(), _stream())
    _check(rc, "fasth_backward")


def fasth_tune_block_size(V, X, G, A, dV, dX, workspace, candidates=None, repetitions: int = 5,
                          transpose: bool = False):
    """Returns (best k, milliseconds per forward+backward pass at that k)."""
    n, d = V.shape
    m = X.shape[1]
    shape = _shape(d, n, m, 1, transpose)
    if candidates is None:
        cand, ncand = None, 0
    else:
        cand = (ctypes.c_int * len(candidates))(*[int(c) for c in candidates])
        ncand = len(candidates)
    best_k = ctypes.c_int(0)
    best_ms = ctypes.c_float(0.0)
    rc = load_library().fasth_tune_block_size(ctypes.byref(shape), cand, ncand, int(repetitions), _ptr(V, "V"),
                                              _ptr(X, "X"), _ptr(G, "G"), _ptr(A, "A"), _ptr(dV, "dV"),
                                              _ptr(dX, "dX"), _ptr(workspace, "workspace"), workspace.numel(),
                                              ctypes.byref(best_k), ctypes.byref(best_ms), _stream())
    _check(rc, "fasth_tune_block_size")
    return best_k.value, best_ms.value


def fasth_sequential_forward(V, X, A, transpose: bool = False) -> None:
    n, d = V.shape
    m = X.shape[1]
    shape = _shape(d, n, m, 1, transpose)
    rc = load_library().fasth_sequential_forward(ctypes.byref(shape), _ptr(V, "V"), _ptr(X, "X"), _ptr(A, "A"),
                                                 _stream())
    _check(rc, "fasth_sequential_forward")


def fasth_sequential_backward(V, A, G, dV, dX, workspace, transpose: bool = False) -> None:
    """A is the product fasth_sequential_forward wrote for the same V and X."""
    n, d = V.shape
    m = A.shape[1]
    shape = _shape(d, n, m, 1, transpose)
    rc = load_library().fasth_sequential_backward(ctypes.byref(shape), _ptr(V, "V"), _ptr(A, "A"), _ptr(G, "G"),
                                                  _ptr(dV, "dV"), _ptr(dX, "dX"), _ptr(workspace, "workspace"),
                                                  workspace.numel(), _stream())
    _check(rc, "fasth_sequential_backward")


def _svd_forward(name, Uv, sigma, Vv, X, Y, workspace, k):
    n, d = Uv.shape
    m = X.shape[1]
    assert Vv.shape == (n, d) and sigma.shape == (d,) and X.shape == (d, m) and Y.shape == (d, m)
    shape = fasth_svd_shape(d, n, m, int(k))
    rc = getattr(load_library(), name)(ctypes.byref(shape), _ptr(Uv, "Uv"), _ptr(sigma, "sigma"), _ptr(Vv, "Vv"),
                                       _ptr(X, "X"), _ptr(Y, "Y"), _ptr(workspace, "workspace"), workspace.numel(),
                                       _stream())
    _check(rc, name)


def _svd_backward(name, Uv, sigma, Vv, G, dUv, dsigma, dVv, dX, workspace, k):
    n, d = Uv.shape
    m = G.shape[1]
    shape = fasth_svd_shape(d, n, m, int(k))
    rc = getattr(load_library(), name)(ctypes.byref(shape), _ptr(Uv, "Uv"), _ptr(sigma, "sigma"), _ptr(Vv, "Vv"),
                                       _ptr(G, "G"), _ptr(dUv, "dUv"), _ptr(dsigma, "dsigma"), _ptr(dVv, "dVv"),
                                       _ptr(dX, "dX"), _ptr(workspace, "workspace"), workspace.numel(), _stream())
    _check(rc, name)


def svd_layer_apply(Uv, sigma, Vv, X, Y, workspace, k: int) -> None:
    _svd_forward("svd_layer_apply", Uv, sigma, Vv, X, Y, workspace, k)


def svd_layer_inverse_apply(Uv, sigma, Vv, X, Y, workspace, k: int) -> None:
    _svd_forward("svd_layer_inverse_apply", Uv, sigma, Vv, X, Y, workspace, k)


def svd_layer_apply_backward(Uv, sigma, Vv, G, dUv, dsigma, dVv, dX, workspace, k: int) -> None:
    _svd_backward("svd_layer_apply_backward", Uv, sigma, Vv, G, dUv, dsigma, dVv, dX, workspace, k)


def svd_layer_inverse_apply_backward(Uv, sigma, Vv, G, dUv, dsigma, dVv, dX, workspace, k: int) -> None:
    _svd_backward("svd_layer_inverse_apply_backward", Uv, sigma, Vv, G, dUv, dsigma, dVv, dX, workspace, k)


DIAG_FUNCTIONS = {"identity": 0, "exp": 1, "cayley": 2}


def svd_sym_apply(Uv, sigma, X, Y, workspace, k: int, function: str = "identity") -> None:
    n, d = Uv.shape
    m = X.shape[1]
    assert sigma.shape == (d,) and X.shape == (d, m) and Y.shape == (d, m)
    shape = fasth_svd_shape(d, n, m, int(k))
    rc = load_library().svd_sym_apply(ctypes.byref(shape), DIAG_FUNCTIONS[function], _ptr(Uv, "Uv"),
                                      _ptr(sigma, "sigma"), _ptr(X, "X"), _ptr(Y, "Y"),
                                      _ptr(workspace, "workspace"), workspace.numel(), _stream())
    _check(rc, "svd_sym_apply")


def svd_sym_apply_backward(Uv, sigma, G, dUv, dsigma, dX, workspace, k: int, function: str = "identity") -> None:
    n, d = Uv.shape
    m = G.shape[1]
    shape = fasth_svd_shape(d, n, m, int(k))
    rc = load_library().svd_sym_apply_backward(ctypes.byref(shape), DIAG_FUNCTIONS[function], _ptr(Uv, "Uv"),
                                               _ptr(sigma, "sigma"), _ptr(G, "G"), _ptr(dUv, "dUv"),
                                               _ptr(dsigma, "dsigma"), _ptr(dX, "dX"),
                                               _ptr(workspace, "workspace"), workspace.numel(), _stream())
    _check(rc, "svd_sym_apply_backward")


def _rect_shape(Uv, Vv, m, k) -> fasth_rect_shape:
    return fasth_rect_shape(int(Uv.shape[1]), int(Vv.shape[1]), int(Uv.shape[0]), int(Vv.shape[0]), int(m), int(k))


def svd_rect_workspace_bytes(rows: int, cols: int, n_u: int, n_v: int, m: int, k: int) -> int:
    shape = fasth_rect_shape(int(rows), int(cols), int(n_u), int(n_v), int(m), int(k))
    return int(load_library().svd_rect_workspace_bytes(ctypes.byref(shape)))


def svd_rect_apply(Uv, sigma, Vv, X, Y, workspace, k: int) -> None:
    m = X.shape[1]
    shape = _rect_shape(Uv, Vv, m, k)
    assert sigma.shape == (min(shape.rows, shape.cols),) and X.shape == (shape.cols, m) and Y.shape == (shape.rows, m)
    rc = load_library().svd_rect_apply(ctypes.byref(shape), _ptr(Uv, "Uv"), _ptr(sigma, "sigma"), _ptr(Vv, "Vv"),
                                       _ptr(X, "X"), _ptr(Y, "Y"), _ptr(workspace, "workspace"), workspace.numel(),
                                       _stream())
    _check(rc, "svd_rect_apply")


def svd_rect_apply_backward(Uv, sigma, Vv, G, dUv, dsigma, dVv, dX, workspace, k: int) -> None:
    m = G.shape[1]
    shape = _rect_shape(Uv, Vv, m, k)
    assert G.shape == (shape.rows, m) and dX.shape == (shape.cols, m) and dsigma.shape == sigma.shape
    assert dUv.shape == Uv.shape and dVv.shape == Vv.shape
    rc = load_library().svd_rect_apply_backward(ctypes.byref(shape), _ptr(Uv, "Uv"), _ptr(sigma, "sigma"),
                                                _ptr(Vv, "Vv"), _ptr(G, "G"), _ptr(dUv, "dUv"),
                                                _ptr(dsigma, "dsigma"), _ptr(dVv, "dVv"), _ptr(dX, "dX"),
                                                _ptr(workspace, "workspace"), workspace.numel(), _stream())
    _check(rc, "svd_rect_apply_backward")


def svd_layer_log_abs_det(sigma, out, dsigma=None) -> None:
    rc = load_library().svd_layer_log_abs_det(int(sigma.shape[0]), _ptr(sigma, "sigma"), _ptr(out, "out"),
                                              _ptr(dsigma, "dsigma") if dsigma is not None else None, _stream())
    _check(rc, "svd_layer_log_abs_det")


FASTH_KERNEL_COUNT = 9


def fasth_profile_enable(on: bool) -> None:
    _check(load_library().fasth_profile_enable(1 if on else 0), "fasth_profile_enable")


def fasth_profile_collect() -> dict:
    """{kernel name: (total milliseconds, launches)} since profiling was enabled or last collected."""
    lib = load_library()
    ms = (ctypes.c_float * FASTH_KERNEL_COUNT)()
    cnt = (ctypes.c_int * FASTH_KERNEL_COUNT)()
    _check(lib.fasth_profile_collect(ms, cnt), "fasth_profile_collect")
    return {lib.fasth_kernel_name(i).decode(): (float(ms[i]), int(cnt[i])) for i in range(FASTH_KERNEL_COUNT)}


def fasth_profile_variants() -> dict:
    """{kernel name: instantiation last launched in that slot since profiling was switched on}."""
    lib = load_library()
    return {lib.fasth_kernel_name(i).decode(): lib.fasth_profile_variant(i).decode() for i in range(FASTH_KERNEL_COUNT)}


def fasth_measure_peaks(buffer, repetitions: int = 3) -> dict:
    """Measured fp32 matrix-instruction rate (TFLOP/s) and streaming read / copy rates (GB/s) of this GPU."""
    mf, rd, cp = ctypes.c_float(0.0), ctypes.c_float(0.0), ctypes.c_float(0.0)
    rc = load_library().fasth_measure_peaks(_ptr(buffer, "workspace"), buffer.numel() * buffer.element_size(),
                                            int(repetitions), ctypes.byref(mf), ctypes.byref(rd), ctypes.byref(cp),
                                            _stream())
    _check(rc, "fasth_measure_peaks")
    return {"fp32_mfma_tflops": mf.value, "hbm_read_gbs": rd.value, "hbm_copy_gbs": cp.value}


def fasth_wait_status() -> int:
    """Waits for the current stream; FASTH_OK, or FASTH_ETIMEOUT if a kernel's wait for another workgroup gave up
    on this GPU since the last check."""
    return int(load_library().fasth_wait_status(_stream()))


def fasth_set_wait_limit(polls: int) -> None:
    _check(load_library().fasth_set_wait_limit(int(polls)), "fasth_set_wait_limit")
