"""ctypes loader for the C oracle (oracle/givens_oracle.c).  Test infrastructure only.

Inputs of any float dtype are promoted to float64 before the call, so fp32 workloads
are evaluated on exactly the fp32 input values, in float64 arithmetic.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build_oracle

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = build_oracle.build(force=False)
        L = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        L.oracle_schedule.argtypes = [ctypes.c_int, ip]
        L.oracle_forward.argtypes = [ctypes.c_int, ctypes.c_long, dp, ip, dp, dp, ctypes.c_int]
        L.oracle_grad_operand.argtypes = [ctypes.c_int, ctypes.c_long, dp, ip, dp, dp, ctypes.c_int]
        L.oracle_reverse_sweep.argtypes = [ctypes.c_int, ctypes.c_long, dp, ip, dp, dp, dp, dp, dp,
                                           ctypes.c_int]
        L.oracle_grad_theta_alg3.argtypes = [ctypes.c_int, dp, ip, dp, dp, dp, ctypes.c_int]
        L.oracle_forward_pairs.argtypes = [ctypes.c_int, ctypes.c_long, ctypes.c_long, dp, ip, dp, dp, ctypes.c_int]
        L.oracle_grad_operand_pairs.argtypes = [ctypes.c_int, ctypes.c_long, ctypes.c_long, dp, ip, dp, dp,
                                                ctypes.c_int]
        L.oracle_reverse_sweep_pairs.argtypes = [ctypes.c_int, ctypes.c_long, ctypes.c_long, dp, ip, dp, dp, dp,
                                                 dp, dp, ctypes.c_int]
        L.oracle_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _d(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"{what} failed with code {rc}")


def schedule(n: int) -> np.ndarray:
    out = np.empty((n - 1, n // 2, 2), dtype=np.int32)
    _check(lib().oracle_schedule(n, out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))), "oracle_schedule")
    return out


def _pairs_ptr(n, pairs):
    if pairs is None:
        pairs = schedule(n)
    pairs = np.ascontiguousarray(pairs, dtype=np.int32)
    return pairs, pairs.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def forward(theta, X, n=None, pairs=None, threads: int = 0) -> np.ndarray:
    """Algorithm 1 from operand X (n x B); X=None builds U from I_n."""
    theta = _f64(theta).reshape(-1)
    if X is None:
        B = n
        x64 = None
    else:
        x64 = _f64(X)
        n, B = x64.shape
    keep, pp = _pairs_ptr(n, pairs)
    Y = np.empty((n, B), dtype=np.float64)
    _check(lib().oracle_forward(n, B, _d(theta), pp, _d(x64), _d(Y), threads), "oracle_forward")
    return Y


def grad_operand(theta, G, pairs=None, threads: int = 0) -> np.ndarray:
    theta = _f64(theta).reshape(-1)
    g64 = _f64(G)
    n, B = g64.shape
    keep, pp = _pairs_ptr(n, pairs)
    dX = np.empty((n, B), dtype=np.float64)
    _check(lib().oracle_grad_operand(n, B, _d(theta), pp, _d(g64), _d(dX), threads), "oracle_grad_operand")
    return dX


def reverse_sweep(theta, Y, G, pairs=None, threads: int = 0, want_dx=True, want_x=True):
    """Returns (dtheta, dX or None, X_recovered or None)."""
    theta = _f64(theta).reshape(-1)
    y64, g64 = _f64(Y), _f64(G)
    n, B = y64.shape
    keep, pp = _pairs_ptr(n, pairs)
    dth = np.empty(theta.size, dtype=np.float64)
    dX = np.empty((n, B), dtype=np.float64) if want_dx else None
    Xr = np.empty((n, B), dtype=np.float64) if want_x else None
    _check(lib().oracle_reverse_sweep(n, B, _d(theta), pp, _d(y64), _d(g64), _d(dth), _d(dX), _d(Xr),
                                      threads), "oracle_reverse_sweep")
    return dth, dX, Xr


def grad_theta_alg3(theta, U, Gamma, pairs=None, threads: int = 0) -> np.ndarray:
    theta = _f64(theta).reshape(-1)
    u64, g64 = _f64(U), _f64(Gamma)
    n = u64.shape[0]
    keep, pp = _pairs_ptr(n, pairs)
    dth = np.empty(theta.size, dtype=np.float64)
    _check(lib().oracle_grad_theta_alg3(n, _d(theta), pp, _d(u64), _d(g64), _d(dth), threads),
           "oracle_grad_theta_alg3")
    return dth


# ---- any sequence E of pairs, any n >= 2 (restricted parametrisation, odd n)
def _free(pairs):
    pairs = np.ascontiguousarray(pairs, dtype=np.int32).reshape(-1, 2)
    return pairs, pairs.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def forward_pairs(theta, X, pairs, n=None, threads: int = 0) -> np.ndarray:
    """Algorithm 1 over the listed pairs (E order) from operand X; X=None builds U from I_n."""
    theta = _f64(theta).reshape(-1)
    if X is None:
        B, x64 = n, None
    else:
        x64 = _f64(X)
        n, B = x64.shape
    keep, pp = _free(pairs)
    assert keep.shape[0] == theta.size
    Y = np.empty((n, B), dtype=np.float64)
    _check(lib().oracle_forward_pairs(n, B, theta.size, _d(theta), pp, _d(x64), _d(Y), threads),
           "oracle_forward_pairs")
    return Y


def grad_operand_pairs(theta, G, pairs, threads: int = 0) -> np.ndarray:
    theta = _f64(theta).reshape(-1)
    g64 = _f64(G)
    n, B = g64.shape
    keep, pp = _free(pairs)
    assert keep.shape[0] == theta.size
    dX = np.empty((n, B), dtype=np.float64)
    _check(lib().oracle_grad_operand_pairs(n, B, theta.size, _d(theta), pp, _d(g64), _d(dX), threads),
           "oracle_grad_operand_pairs")
    return dX


def reverse_sweep_pairs(theta, Y, G, pairs, threads: int = 0, want_dx=True, want_x=True):
    """Returns (dtheta, dX or None, X_recovered or None) for the listed pairs."""
    theta = _f64(theta).reshape(-1)
    y64, g64 = _f64(Y), _f64(G)
    n, B = y64.shape
    keep, pp = _free(pairs)
    assert keep.shape[0] == theta.size
    dth = np.empty(theta.size, dtype=np.float64)
    dX = np.empty((n, B), dtype=np.float64) if want_dx else None
    Xr = np.empty((n, B), dtype=np.float64) if want_x else None
    _check(lib().oracle_reverse_sweep_pairs(n, B, theta.size, _d(theta), pp, _d(y64), _d(g64), _d(dth), _d(dX),
                                            _d(Xr), threads), "oracle_reverse_sweep_pairs")
    return dth, dX, Xr


def num_threads() -> int:
    return int(lib().oracle_num_threads())
