"""Thin ctypes binding to libgivens_rr.so (the C ABI of include/givens_rr.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.
PyTorch tensors are used as device buffers (data_ptr) and for the current HIP stream.
There is no CPU fallback: if the library is not built, loading raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgivens_rr.so")

KERNEL_AUTO, KERNEL_LDS, KERNEL_CAROUSEL, KERNEL_COLUMN = 0, 1, 2, 3
FORM_AUTO, FORM_STANDARD, FORM_SCALED, FORM_LIFTED, FORM_RANGE = 0, 1, 2, 3, 4
REDUCTION_AUTO, REDUCTION_TWO_STAGE, REDUCTION_GRAM = 0, 1, 3
PREPARE_FORWARD, PREPARE_BACKWARD, PREPARE_BACKWARD_WIDE = 1, 2, 4
ERR_STALE = -8

EXPORTS = [
    "rr_schedule", "givens_forward", "givens_build", "givens_backward",
    "givens_forward_f64", "givens_build_f64", "givens_backward_f64",
    "givens_forward_transposed", "givens_forward_transposed_f64", "givens_forward_noalloc",
    "givens_forward_ex", "givens_backward_ex",
    "givens_prepare", "givens_prepare_restricted", "givens_prepare_ex", "givens_forward_prepared", "givens_build_prepared",
    "givens_backward_prepared",
    "givens_release", "givens_last_hip_error", "givens_error_string",
    "givens_set_kernel", "givens_last_kernel", "givens_set_timing", "givens_last_timing",
    "givens_set_rotation_form", "givens_last_rotation_form",
    "givens_set_reduction", "givens_last_reduction", "givens_last_chains",
    "givens_num_angles", "rr_schedule_restricted",
    "givens_forward_restricted", "givens_build_restricted", "givens_backward_restricted",
    "givens_forward_restricted_f64", "givens_build_restricted_f64", "givens_backward_restricted_f64",
    "givens_unitary_forward", "givens_unitary_build", "givens_unitary_backward",
    "givens_unitary_forward_f64", "givens_unitary_build_f64", "givens_unitary_backward_f64",
]

_lib = None


class GivensError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        L = _lib
        text = L.givens_error_string(code).decode() if L is not None else "?"
        hip = L.givens_last_hip_error() if L is not None else 0
        super().__init__(f"{where}: error {code} ({text}); last HIP error {hip}")


def lib():
    """Load the library once.  Raises if it has not been built (python -m ... build or __graft_entry__.build())."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python paper_2106_00003_amd/build.py` "
            "(there is no fallback path)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    L.rr_schedule.argtypes = [i32, vp]
    for name in ("givens_forward", "givens_forward_f64", "givens_forward_transposed", "givens_forward_transposed_f64",
                 "givens_forward_noalloc"):
        getattr(L, name).argtypes = [i32, i64, vp, vp, vp, vp]
    for name in ("givens_build", "givens_build_f64"):
        getattr(L, name).argtypes = [i32, vp, vp, vp]
    for name in ("givens_backward", "givens_backward_f64"):
        getattr(L, name).argtypes = [i32, i64, vp, vp, vp, vp, vp, vp]
    L.givens_forward_ex.argtypes = [i32, i32, i64, vp, vp, vp, vp, vp]
    L.givens_backward_ex.argtypes = [i32, i32, i64, vp, vp, vp, vp, vp, vp, vp]
    L.givens_prepare.argtypes = [i32, vp, i32, vp]
    L.givens_prepare_restricted.argtypes = [i32, i32, vp, i32, vp]
    L.givens_prepare_ex.argtypes = [i32, i32, vp, i32, i64, vp, vp]
    L.givens_forward_prepared.argtypes = [i64, i64, vp, vp, vp]
    L.givens_build_prepared.argtypes = [i64, vp, vp]
    L.givens_backward_prepared.argtypes = [i64, i64, vp, vp, vp, vp, vp]
    L.givens_num_angles.argtypes = [i32, i32]
    L.rr_schedule_restricted.argtypes = [i32, i32, vp]
    for name in ("givens_forward_restricted", "givens_forward_restricted_f64"):
        getattr(L, name).argtypes = [i32, i32, i64, vp, vp, vp, vp]
    for name in ("givens_build_restricted", "givens_build_restricted_f64"):
        getattr(L, name).argtypes = [i32, i32, vp, vp, vp]
    for name in ("givens_backward_restricted", "givens_backward_restricted_f64"):
        getattr(L, name).argtypes = [i32, i32, i64, vp, vp, vp, vp, vp, vp]
    for name in ("givens_unitary_forward", "givens_unitary_forward_f64"):
        getattr(L, name).argtypes = [i32, i64, vp, vp, vp, vp, vp]
    for name in ("givens_unitary_build", "givens_unitary_build_f64"):
        getattr(L, name).argtypes = [i32, vp, vp, vp, vp]
    for name in ("givens_unitary_backward", "givens_unitary_backward_f64"):
        getattr(L, name).argtypes = [i32, i64, vp, vp, vp, vp, vp, vp, vp, vp]
    L.givens_error_string.argtypes = [i32]
    L.givens_error_string.restype = ctypes.c_char_p
    L.givens_set_kernel.argtypes = [i32]
    L.givens_set_rotation_form.argtypes = [i32]
    L.givens_set_reduction.argtypes = [i32]
    L.givens_set_timing.argtypes = [i32]
    L.givens_last_timing.argtypes = [ctypes.POINTER(ctypes.c_float)]
    for name in EXPORTS:
        if name not in ("givens_error_string", "givens_num_angles", "givens_prepare", "givens_prepare_restricted",
                        "givens_prepare_ex"):
            getattr(L, name).restype = i32
    for name in ("givens_num_angles", "givens_prepare", "givens_prepare_restricted", "givens_prepare_ex"):
        getattr(L, name).restype = i64
    _lib = L
    return L


def _check(rc: int, where: str):
    if rc != 0:
        raise GivensError(rc, where)


def _stream_ptr(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _suffix(t) -> str:
    import torch
    if t.dtype == torch.float32:
        return ""
    if t.dtype == torch.float64:
        return "_f64"
    raise TypeError(f"unsupported dtype {t.dtype}")


def _dev(t, name, dtype=None):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} has dtype {t.dtype}, expected {dtype}")
    return ctypes.c_void_p(t.data_ptr())


def rr_schedule(n: int) -> np.ndarray:
    """Host call: (n-1, n/2, 2) int32 array of pairs (i < j) in block order."""
    if n < 2 or n % 2:
        _check(lib().rr_schedule(n, None), "rr_schedule")
    out = np.empty((n - 1, n // 2, 2), dtype=np.int32)
    _check(lib().rr_schedule(n, out.ctypes.data_as(ctypes.c_void_p)), "rr_schedule")
    return out


def givens_forward(theta, X, Y=None, stream=None):
    """Y = U(theta) X on the device.  Y=None allocates; Y may be X (in place)."""
    import torch
    n, B = X.shape
    if theta.numel() != n * (n - 1) // 2:
        raise ValueError("theta must have n(n-1)/2 entries")
    if Y is None:
        Y = torch.empty_like(X)
    fn = getattr(lib(), "givens_forward" + _suffix(X))
    _check(fn(n, B, _dev(theta, "theta", X.dtype), _dev(X, "X"), _dev(Y, "Y", X.dtype), _stream_ptr(stream)),
           "givens_forward")
    return Y


NOALLOC_MAX_N = 1024


def givens_forward_noalloc(theta, X, Y, stream=None):
    """givens_forward through the entry point that allocates nothing; the caller brings Y (float32 only)."""
    import torch
    n, B = X.shape
    if theta.numel() != n * (n - 1) // 2:
        raise ValueError("theta must have n(n-1)/2 entries")
    _check(lib().givens_forward_noalloc(n, B, _dev(theta, "theta", torch.float32), _dev(X, "X", torch.float32),
                                        _dev(Y, "Y", torch.float32), _stream_ptr(stream)),
           "givens_forward_noalloc")
    return Y


class Options(ctypes.Structure):
    """givens_options of the C header: per-call kernel family, rotation form and reduction."""
    _fields_ = [("kernel", ctypes.c_int), ("rotation_form", ctypes.c_int), ("reduction", ctypes.c_int)]


def _options(kernel, form, reduction):
    return ctypes.byref(Options(kernel, form, reduction))


def givens_forward_ex(theta, X, m=None, Y=None, n=None, kernel=KERNEL_AUTO, form=FORM_AUTO,
                      reduction=REDUCTION_AUTO, stream=None):
    """givens_forward (X given) or givens_build (X=None, n given) with per-call options; float32."""
    import torch
    if X is None:
        B = n
        if Y is None:
            Y = torch.empty((n, n), dtype=torch.float32, device=theta.device)
    else:
        n, B = X.shape
        if Y is None:
            Y = torch.empty_like(X)
    m = n - 1 if m is None else m
    _check(lib().givens_forward_ex(n, m, B, _dev(theta, "theta", torch.float32), _dev(X, "X", torch.float32),
                                   _dev(Y, "Y", torch.float32), _stream_ptr(stream),
                                   _options(kernel, form, reduction)), "givens_forward_ex")
    return Y


def givens_backward_ex(theta, Y, G, m=None, dX=None, dtheta=None, want_dx=True, kernel=KERNEL_AUTO,
                       form=FORM_AUTO, reduction=REDUCTION_AUTO, stream=None):
    """givens_backward with per-call options; float32.  Returns (dX or None, dtheta)."""
    import torch
    n, B = Y.shape
    m = n - 1 if m is None else m
    if dtheta is None:
        dtheta = torch.empty_like(theta)
    if want_dx and dX is None:
        dX = torch.empty_like(G)
    _check(lib().givens_backward_ex(n, m, B, _dev(theta, "theta", torch.float32), _dev(Y, "Y", torch.float32),
                                    _dev(G, "G", torch.float32), _dev(dX if want_dx else None, "dX", torch.float32),
                                    _dev(dtheta, "dtheta", torch.float32), _stream_ptr(stream),
                                    _options(kernel, form, reduction)), "givens_backward_ex")
    return (dX if want_dx else None), dtheta


def givens_prepare(theta, n: int, m=None, directions=PREPARE_FORWARD | PREPARE_BACKWARD, stream=None,
                   batch=None) -> int:
    """Builds the coefficient tables of theta once in the stream's workspace; returns the token.
    batch: the number of columns the tables will be used with, if known (the default rotation form depends on it)."""
    import torch
    th = _dev(theta, "theta", torch.float32)
    if batch is not None:
        tok = lib().givens_prepare_ex(n, (n - 1) if m is None else m, th, directions, int(batch), _stream_ptr(stream),
                                      None)
    elif m is None:
        tok = lib().givens_prepare(n, th, directions, _stream_ptr(stream))
    else:
        tok = lib().givens_prepare_restricted(n, m, th, directions, _stream_ptr(stream))
    if tok <= 0:
        raise GivensError(int(tok), "givens_prepare")
    return int(tok)


def givens_forward_prepared(token: int, X, Y=None, stream=None):
    import torch
    n, B = X.shape
    if Y is None:
        Y = torch.empty_like(X)
    _check(lib().givens_forward_prepared(token, B, _dev(X, "X", torch.float32), _dev(Y, "Y", torch.float32),
                                         _stream_ptr(stream)), "givens_forward_prepared")
    return Y


def givens_build_prepared(token: int, n: int, device, U=None, stream=None):
    import torch
    if U is None:
        U = torch.empty((n, n), dtype=torch.float32, device=device)
    _check(lib().givens_build_prepared(token, _dev(U, "U", torch.float32), _stream_ptr(stream)),
           "givens_build_prepared")
    return U


def givens_backward_prepared(token: int, Y, G, ntheta: int, dX=None, dtheta=None, want_dx=True, stream=None):
    """Returns (dX or None, dtheta); ntheta = number of angles (size of dtheta)."""
    import torch
    n, B = Y.shape
    if dtheta is None:
        dtheta = torch.empty(ntheta, dtype=torch.float32, device=Y.device)
    if want_dx and dX is None:
        dX = torch.empty_like(G)
    _check(lib().givens_backward_prepared(token, B, _dev(Y, "Y", torch.float32), _dev(G, "G", torch.float32),
                                          _dev(dX if want_dx else None, "dX", torch.float32),
                                          _dev(dtheta, "dtheta", torch.float32), _stream_ptr(stream)),
           "givens_backward_prepared")
    return (dX if want_dx else None), dtheta


def givens_forward_transposed(theta, X, Y=None, stream=None):
    """Y = U(theta)^T X (the inverse transform) on the device.  Y=None allocates; Y may be X."""
    import torch
    n, B = X.shape
    if theta.numel() != n * (n - 1) // 2:
        raise ValueError("theta must have n(n-1)/2 entries")
    if Y is None:
        Y = torch.empty_like(X)
    fn = getattr(lib(), "givens_forward_transposed" + _suffix(X))
    _check(fn(n, B, _dev(theta, "theta", X.dtype), _dev(X, "X"), _dev(Y, "Y", X.dtype), _stream_ptr(stream)),
           "givens_forward_transposed")
    return Y


def givens_build(theta, n: int, U=None, stream=None):
    """U = U(theta), n x n."""
    import torch
    if theta.numel() != n * (n - 1) // 2:
        raise ValueError("theta must have n(n-1)/2 entries")
    if U is None:
        U = torch.empty((n, n), dtype=theta.dtype, device=theta.device)
    fn = getattr(lib(), "givens_build" + _suffix(theta))
    _check(fn(n, _dev(theta, "theta"), _dev(U, "U", theta.dtype), _stream_ptr(stream)), "givens_build")
    return U


def givens_backward(theta, Y, G, dX=None, dtheta=None, want_dx: bool = True, stream=None):
    """Reverse sweep from the forward output Y and the upstream gradient G.  Returns (dX, dtheta)."""
    import torch
    n, B = Y.shape
    if theta.numel() != n * (n - 1) // 2:
        raise ValueError("theta must have n(n-1)/2 entries")
    if G.shape != Y.shape:
        raise ValueError("G must have the shape of Y")
    if dX is None and want_dx:
        dX = torch.empty_like(G)
    if dtheta is None:
        dtheta = torch.empty_like(theta)
    fn = getattr(lib(), "givens_backward" + _suffix(Y))
    _check(fn(n, B, _dev(theta, "theta", Y.dtype), _dev(Y, "Y"), _dev(G, "G", Y.dtype),
              _dev(dX, "dX", Y.dtype), _dev(dtheta, "dtheta", Y.dtype), _stream_ptr(stream)),
           "givens_backward")
    return dX, dtheta


def num_angles(n: int, m: int | None = None) -> int:
    """Free angles of the parametrisation restricted to pairs (i, j), i < min(j, m); m=None: unrestricted."""
    rc = lib().givens_num_angles(n, n - 1 if m is None else m)
    if rc < 0:
        raise GivensError(int(rc), "givens_num_angles")
    return int(rc)


def rr_schedule_restricted(n: int, m: int | None = None) -> np.ndarray:
    """Host call: (N, 2) int32 array of the free pairs (i < j) in E order; any n >= 2."""
    m = n - 1 if m is None else m
    count = num_angles(n, m)
    out = np.empty((count, 2), dtype=np.int32)
    _check(lib().rr_schedule_restricted(n, m, out.ctypes.data_as(ctypes.c_void_p)), "rr_schedule_restricted")
    return out


def givens_forward_restricted(theta, X, m: int, Y=None, stream=None):
    """Y = U(theta) X with only the pairs (i, j), i < m, free (any n >= 2)."""
    import torch
    n, B = X.shape
    if theta.numel() != num_angles(n, m):
        raise ValueError("theta must have m n - m (m + 1) / 2 entries")
    if Y is None:
        Y = torch.empty_like(X)
    fn = getattr(lib(), "givens_forward_restricted" + _suffix(X))
    _check(fn(n, m, B, _dev(theta, "theta", X.dtype), _dev(X, "X"), _dev(Y, "Y", X.dtype), _stream_ptr(stream)),
           "givens_forward_restricted")
    return Y


def givens_build_restricted(theta, n: int, m: int, U=None, stream=None):
    import torch
    if theta.numel() != num_angles(n, m):
        raise ValueError("theta must have m n - m (m + 1) / 2 entries")
    if U is None:
        U = torch.empty((n, n), dtype=theta.dtype, device=theta.device)
    fn = getattr(lib(), "givens_build_restricted" + _suffix(theta))
    _check(fn(n, m, _dev(theta, "theta"), _dev(U, "U", theta.dtype), _stream_ptr(stream)),
           "givens_build_restricted")
    return U


def givens_backward_restricted(theta, Y, G, m: int, dX=None, dtheta=None, want_dx: bool = True, stream=None):
    import torch
    n, B = Y.shape
    if theta.numel() != num_angles(n, m):
        raise ValueError("theta must have m n - m (m + 1) / 2 entries")
    if G.shape != Y.shape:
        raise ValueError("G must have the shape of Y")
    if dX is None and want_dx:
        dX = torch.empty_like(G)
    if dtheta is None:
        dtheta = torch.empty_like(theta)
    fn = getattr(lib(), "givens_backward_restricted" + _suffix(Y))
    _check(fn(n, m, B, _dev(theta, "theta", Y.dtype), _dev(Y, "Y"), _dev(G, "G", Y.dtype),
              _dev(dX, "dX", Y.dtype), _dev(dtheta, "dtheta", Y.dtype), _stream_ptr(stream)),
           "givens_backward_restricted")
    return dX, dtheta


def _real_dtype(t):
    import torch
    return {torch.complex64: torch.float32, torch.complex128: torch.float64}[t.dtype]


def _csuffix(t) -> str:
    import torch
    if t.dtype == torch.complex64:
        return ""
    if t.dtype == torch.complex128:
        return "_f64"
    raise TypeError(f"unsupported dtype {t.dtype}")


def givens_unitary_forward(theta, phi, X, Y=None, stream=None):
    """Y = U(theta, phi) X for a complex X of shape (n, B) (complex64 or complex128 device tensor)."""
    import torch
    n, B = X.shape
    if theta.numel() != n * (n - 1) // 2 or phi.numel() != theta.numel():
        raise ValueError("theta and phi must have n(n-1)/2 entries")
    if Y is None:
        Y = torch.empty_like(X)
    rd = _real_dtype(X)
    fn = getattr(lib(), "givens_unitary_forward" + _csuffix(X))
    _check(fn(n, B, _dev(theta, "theta", rd), _dev(phi, "phi", rd), _dev(X, "X"), _dev(Y, "Y", X.dtype),
              _stream_ptr(stream)), "givens_unitary_forward")
    return Y


def givens_unitary_build(theta, phi, n: int, U=None, stream=None):
    import torch
    if theta.numel() != n * (n - 1) // 2 or phi.numel() != theta.numel():
        raise ValueError("theta and phi must have n(n-1)/2 entries")
    cd = torch.complex64 if theta.dtype == torch.float32 else torch.complex128
    if U is None:
        U = torch.empty((n, n), dtype=cd, device=theta.device)
    fn = getattr(lib(), "givens_unitary_build" + _csuffix(U))
    _check(fn(n, _dev(theta, "theta"), _dev(phi, "phi", theta.dtype), _dev(U, "U", cd), _stream_ptr(stream)),
           "givens_unitary_build")
    return U


def givens_unitary_backward(theta, phi, Y, G, dX=None, dtheta=None, dphi=None, want_dx: bool = True, stream=None):
    """Returns (dX, dtheta, dphi) from the forward output Y and the upstream gradient G (complex)."""
    import torch
    n, B = Y.shape
    if theta.numel() != n * (n - 1) // 2 or phi.numel() != theta.numel():
        raise ValueError("theta and phi must have n(n-1)/2 entries")
    if G.shape != Y.shape:
        raise ValueError("G must have the shape of Y")
    rd = _real_dtype(Y)
    if dX is None and want_dx:
        dX = torch.empty_like(G)
    if dtheta is None:
        dtheta = torch.empty_like(theta)
    if dphi is None:
        dphi = torch.empty_like(phi)
    fn = getattr(lib(), "givens_unitary_backward" + _csuffix(Y))
    _check(fn(n, B, _dev(theta, "theta", rd), _dev(phi, "phi", rd), _dev(Y, "Y"), _dev(G, "G", Y.dtype),
              _dev(dX, "dX", Y.dtype), _dev(dtheta, "dtheta", rd), _dev(dphi, "dphi", rd), _stream_ptr(stream)),
           "givens_unitary_backward")
    return dX, dtheta, dphi


def set_kernel(which: int) -> int:
    rc = lib().givens_set_kernel(which)
    if rc < 0:
        raise GivensError(rc, "givens_set_kernel")
    return rc


def last_kernel() -> int:
    return lib().givens_last_kernel()


def set_rotation_form(which: int) -> int:
    rc = lib().givens_set_rotation_form(which)
    if rc < 0:
        raise GivensError(rc, "givens_set_rotation_form")
    return rc


def last_rotation_form() -> int:
    rc = lib().givens_last_rotation_form()
    if rc < 0:
        raise GivensError(rc, "givens_last_rotation_form")
    return rc


def set_reduction(which: int) -> int:
    rc = lib().givens_set_reduction(which)
    if rc < 0:
        raise GivensError(rc, "givens_set_reduction")
    return rc


def last_reduction() -> int:
    return lib().givens_last_reduction()


def last_chains() -> int:
    return lib().givens_last_chains()


def set_timing(on: bool) -> int:
    return lib().givens_set_timing(1 if on else 0)


def last_timing():
    """(table_ms, sweep_ms, reduce_ms, gram_ms) of the last call on this thread; waits for its events."""
    buf = (ctypes.c_float * 4)()
    _check(lib().givens_last_timing(buf), "givens_last_timing")
    return float(buf[0]), float(buf[1]), float(buf[2]), float(buf[3])


def release():
    _check(lib().givens_release(), "givens_release")
