"""Pins for the C oracle: it must agree with the NumPy oracle (pinned to the paper elsewhere)
and keep the invariants at sizes NumPy does not reach in test time."""
import math

import numpy as np
import pytest

from oracle import c_oracle as C
from oracle import givens_oracle as O


def _case(n, b, seed):
    rng = np.random.default_rng(seed)
    th = rng.uniform(-math.pi, math.pi, n * (n - 1) // 2)
    return th, rng.standard_normal((n, b)), rng.standard_normal((n, b))


@pytest.mark.parametrize("n", [2, 4, 6, 8, 64, 256])
def test_schedule_equals_numpy_oracle(n):
    assert np.array_equal(C.schedule(n), O.circle_method_schedule(n))


def test_schedule_invariants_at_n4096():
    n = 4096
    s = C.schedule(n)
    assert s.shape == (n - 1, n // 2, 2)
    assert np.all(s[:, :, 0] < s[:, :, 1])
    # every block is a perfect matching
    flat = np.sort(s.reshape(n - 1, n), axis=1)
    assert np.array_equal(flat, np.broadcast_to(np.arange(n), (n - 1, n)))
    # every pair exactly once
    key = s[:, :, 0].astype(np.int64) * n + s[:, :, 1]
    assert np.unique(key).size == n * (n - 1) // 2
    # arc 0 of block k joins 0 with n-1-k
    assert np.array_equal(s[:, 0, 1], n - 1 - np.arange(n - 1))


@pytest.mark.parametrize("n,b", [(8, 4), (16, 37), (64, 70)])
def test_forward_and_operand_gradient_equal_numpy_oracle(n, b):
    th, x, g = _case(n, b, n * b)
    y = C.forward(th, x, threads=3)
    assert np.allclose(y, O.forward_sequential(th, x), atol=1e-13)
    assert np.allclose(C.forward(th, None, n=n), O.build_u(th, n), atol=1e-13)
    assert np.allclose(C.grad_operand(th, g), O.grad_operand(th, g), atol=1e-13)


@pytest.mark.parametrize("n,b", [(8, 4), (16, 37), (64, 70)])
def test_both_gradient_routines_equal_numpy_oracle(n, b):
    th, x, g = _case(n, b, n + 3 * b)
    u = O.build_u(th, n)
    y = u @ x
    want, want_dx, want_x = O.reverse_sweep(th, y, g)
    d, dx, xr = C.reverse_sweep(th, y, g, threads=2)
    scale = np.linalg.norm(want)
    assert np.linalg.norm(d - want) < 1e-13 * scale
    assert np.allclose(dx, want_dx, atol=1e-13)
    assert np.allclose(xr, want_x, atol=1e-13)
    d3 = C.grad_theta_alg3(th, u, g @ x.T, threads=3)
    assert np.linalg.norm(d3 - O.grad_theta_alg3(th, u, g @ x.T)) < 1e-13 * scale
    assert np.linalg.norm(d3 - want) < 1e-12 * scale


def test_fp32_inputs_are_promoted_exactly():
    th, x, g = _case(16, 8, 3)
    th32, x32 = th.astype(np.float32), x.astype(np.float32)
    y = C.forward(th32, x32)
    assert np.allclose(y, O.forward_sequential(th32.astype(np.float64), x32.astype(np.float64)), atol=1e-13)


def test_invariants_at_n512():
    n, b = 512, 96
    th, x, _ = _case(n, b, 512)
    u = C.forward(th, None, n=n)
    assert np.allclose(u.T @ u, np.eye(n), atol=1e-11)
    sign, logdet = np.linalg.slogdet(u)
    assert sign == 1.0 and abs(logdet) < 1e-9
    y = C.forward(th, x)
    assert np.allclose(y, u @ x, atol=1e-11)
    d, dx, xr = C.reverse_sweep(th, y, y)
    assert np.max(np.abs(d)) < 1e-9            # G = Y: gradient of a constant
    assert np.allclose(xr, x, atol=1e-11)
    assert np.allclose(dx, x, atol=1e-11)
