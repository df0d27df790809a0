"""Pins for oracle/unitary_oracle.py (the paper's appendix on U(n))."""
import numpy as np
import pytest

from oracle import givens_oracle as O
from oracle import unitary_oracle as V


def _data(n, B, seed):
    rng = np.random.default_rng(seed)
    count = n * (n - 1) // 2
    theta = rng.uniform(-np.pi, np.pi, count)
    phi = rng.uniform(-np.pi, np.pi, count)
    x = rng.standard_normal((n, B)) + 1j * rng.standard_normal((n, B))
    g = rng.standard_normal((n, B)) + 1j * rng.standard_normal((n, B))
    return theta, phi, x, g


def test_factor_entries_and_unitarity():
    g = V.unitary_factor(5, 1, 3, 0.7, -0.4)
    w = np.exp(-0.4j)
    want = np.eye(5, dtype=complex)
    want[1, 1], want[1, 3], want[3, 1], want[3, 3] = w * np.cos(0.7), -np.sin(0.7), w * np.sin(0.7), np.cos(0.7)
    assert np.allclose(g, want, atol=0, rtol=0)
    assert np.allclose(g.conj().T @ g, np.eye(5), atol=1e-15)
    # the appendix's derivative entries, against differences of the explicit factor
    eps = 1e-6
    d_th = (V.unitary_factor(5, 1, 3, 0.7 + eps, -0.4) - V.unitary_factor(5, 1, 3, 0.7 - eps, -0.4)) / (2 * eps)
    d_ph = (V.unitary_factor(5, 1, 3, 0.7, -0.4 + eps) - V.unitary_factor(5, 1, 3, 0.7, -0.4 - eps)) / (2 * eps)
    q = d_th @ g.conj().T
    p = d_ph @ g.conj().T
    want_q = np.zeros((5, 5), dtype=complex)
    want_q[1, 3], want_q[3, 1] = -1, 1
    c, s = np.cos(0.7), np.sin(0.7)
    want_p = np.zeros((5, 5), dtype=complex)
    want_p[1, 1], want_p[3, 3], want_p[1, 3], want_p[3, 1] = 1j * c * c, 1j * s * s, 1j * s * c, 1j * s * c
    assert np.allclose(q, want_q, atol=1e-9) and np.allclose(p, want_p, atol=1e-9)


def test_n2_closed_form():
    th, ph = 0.3, 1.1
    u = V.dense_product(2, [th], [ph])
    w = np.exp(1j * ph)
    assert np.allclose(u, [[w * np.cos(th), -np.sin(th)], [w * np.sin(th), np.cos(th)]], atol=1e-16)


@pytest.mark.parametrize("n", [2, 4, 6, 8])
def test_zero_phases_give_the_real_oracle(n):
    theta, _, x, g = _data(n, 3, n)
    zero = np.zeros_like(theta)
    assert V.rel_fro(V.dense_product(n, theta, zero).real, O.dense_product(n, theta)) < 1e-15
    assert np.abs(V.dense_product(n, theta, zero).imag).max() == 0.0
    y = V.forward(theta, zero, x.real)
    assert V.rel_fro(y.real, O.forward_sequential(theta, x.real)) < 1e-15
    dth, dph, dx, _ = V.reverse_sweep(theta, zero, y, g.real)
    want_dth, want_dx, _ = O.reverse_sweep(theta, y.real, g.real)
    assert V.rel_fro(dth, want_dth) < 1e-13 and V.rel_fro(dx.real, want_dx) < 1e-13
    assert np.abs(dph).max() < 1e-12                          # real data: the phase gradient vanishes


@pytest.mark.parametrize("n,B,seed", [(2, 3, 1), (4, 2, 2), (6, 5, 3), (8, 4, 4)])
def test_product_forward_unitarity_and_determinant(n, B, seed):
    theta, phi, x, _ = _data(n, B, seed)
    u = V.dense_product(n, theta, phi)
    assert np.allclose(u.conj().T @ u, np.eye(n), atol=1e-13)
    assert np.allclose(np.linalg.det(u), np.exp(1j * np.sum(phi)), atol=1e-12)
    assert np.allclose(V.forward(theta, phi, x), u @ x, atol=1e-13)
    assert np.allclose(V.forward(theta, phi, np.eye(n)), u, atol=1e-13)


@pytest.mark.parametrize("n,B,seed", [(2, 3, 11), (4, 3, 12), (6, 4, 13), (8, 4, 14)])
def test_gradients_against_central_differences(n, B, seed):
    theta, phi, x, g = _data(n, B, seed)
    y = V.forward(theta, phi, x)
    dth, dph, dx, x_back = V.reverse_sweep(theta, phi, y, g)
    fd_th, fd_ph = V.finite_differences(theta, phi, x, g)
    assert V.rel_fro(dth, fd_th) < 1e-7
    assert V.rel_fro(dph, fd_ph) < 1e-7
    assert np.allclose(x_back, x, atol=1e-12)
    u = V.dense_product(n, theta, phi)
    assert np.allclose(dx, u.conj().T @ g, atol=1e-12)
    assert np.allclose(V.grad_operand(theta, phi, g), u.conj().T @ g, atol=1e-12)
    x2 = np.random.default_rng(seed + 50).standard_normal((n, B)) * (1 + 0.5j)
    assert abs(np.real(np.vdot(g, u @ x2)) - np.real(np.vdot(dx, x2))) < 1e-10     # adjoint identity


def test_upstream_equal_to_output_gives_zero_gradients():
    theta, phi, x, _ = _data(8, 5, 21)
    y = V.forward(theta, phi, x)
    dth, dph, dx, _ = V.reverse_sweep(theta, phi, y, y)
    assert np.abs(dth).max() < 1e-12 and np.abs(dph).max() < 1e-12
    assert np.allclose(dx, x, atol=1e-12)


@pytest.mark.parametrize("n,B,seed", [(4, 3, 31), (16, 5, 32), (34, 7, 33)])
def test_block_vectorised_versions_equal_the_per_pair_ones(n, B, seed):
    theta, phi, x, g = _data(n, B, seed)
    y = V.forward(theta, phi, x)
    assert np.allclose(V.forward_blocks(theta, phi, x), y, atol=1e-13)
    a = V.reverse_sweep(theta, phi, y, g)
    b = V.reverse_sweep_blocks(theta, phi, y, g)
    for u, v in zip(a, b):
        assert np.allclose(u, v, atol=1e-11)
