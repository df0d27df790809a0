"""CPU oracle for the unitary extension (the paper's appendix "Adaptations to U(n)").

TEST INFRASTRUCTURE ONLY (see oracle/givens_oracle.py): only tests/, the smoke check and the
benchmark's cpu_baseline leg may import it; it shares no code with the HIP path.

Parametrisation.  For e = (i, j), i < j, the elementary factor G^e(theta_e, phi_e) is the identity
except for
    G_ii = exp(i phi) cos(theta),  G_ij = -sin(theta),
    G_ji = exp(i phi) sin(theta),  G_jj =  cos(theta),
i.e. the real rotation times diag(exp(i phi), 1) on (i, j).  Reading taken here: the appendix's display
prints G_jj = exp(i phi) cos(theta), but its forward algorithm (r_j = exp(i phi) sin U_i + cos U_j), its
list of derivatives ([dG/dtheta]_jj = -sin, no (j, j) entry in dG/dphi) and unitarity all require
G_jj = cos(theta); the display is taken as a misprint.
U = G^{e_1} ... G^{e_N} with E the round-robin sequence, G^{e_N} applied first, as in the real case.

Gradient convention.  The loss is real; the upstream gradient G collects dL/dRe(Y) + i dL/dIm(Y), so
that dL = Re <G, dY> = Re sum(conj(G) * dY).  Then
    dL/dtheta_e = Re <G, (dU/dtheta_e) X>,  dL/dphi_e = Re <G, (dU/dphi_e) X>,  dL/dX = U^dagger G.
With U^fwd = U^{1:k-1}, U^bck = U^{k:n-1} for e in b_k the appendix gives dU/dtheta_e = U^fwd Q_e U^bck
and dU/dphi_e = U^fwd P_e U^bck, where Q_e has -1 at (i, j), +1 at (j, i) and P_e has i cos^2 at (i, i),
i sin^2 at (j, j) and i sin cos at (i, j) and (j, i).  The appendix stops there ("can then follow an
analogous path ... albeit more tediously"); the operand-side sweep below is the analogue of the real
one: z = U^bck X and gbar = U^fwd^dagger G are carried, the two derivatives are contracted per pair,
then block k is undone with the adjoint factors.

  unitary_factor           the explicit n x n factor
  dense_product            Eq. (2) with these factors
  forward                  the appendix's forward algorithm, started from any operand
  grad_operand             U^dagger G by adjoint factors in E order
  reverse_sweep            (dtheta, dphi, dX, X recovered)
  forward_blocks / reverse_sweep_blocks   the same two, vectorised over the pairs of a block (for sizes
                           where the per-pair loops are too slow); pinned to the per-pair versions
  loss / finite_differences   L = Re sum(conj(G) * (U X)) and central differences in theta and phi

Pins (tests/test_oracle_unitary.py): phi = 0 gives the real oracle; n = 2 closed form; entries of the
factor and of Q_e, P_e against differences of the explicit factor; dense product = forward algorithm;
U^dagger U = I and det U = exp(i sum phi); per-parameter central differences of the loss; adjoint
identity for dX; G = Y gives dtheta = 0 and dphi = 0 (the loss is then the constant ||X||^2).
The appendix prints no gradient algorithm to compare the sweep with: the per-parameter central differences of
the loss through the explicit product (every theta and phi at small n) are what pins it.
"""
from __future__ import annotations

import numpy as np

from oracle.givens_oracle import circle_method_schedule


def _pairs(n, pairs):
    if pairs is None:
        pairs = circle_method_schedule(n)
    return np.asarray(pairs).reshape(n - 1, n // 2, 2)


def unitary_factor(n: int, i: int, j: int, theta: float, phi: float) -> np.ndarray:
    assert 0 <= i < j < n
    g = np.eye(n, dtype=np.complex128)
    w = np.exp(1j * phi)
    g[i, i] = w * np.cos(theta)
    g[i, j] = -np.sin(theta)
    g[j, i] = w * np.sin(theta)
    g[j, j] = np.cos(theta)
    return g


def dense_product(n: int, theta, phi, pairs=None) -> np.ndarray:
    e_list = _pairs(n, pairs).reshape(-1, 2)
    theta = np.asarray(theta, dtype=np.float64).reshape(-1)
    phi = np.asarray(phi, dtype=np.float64).reshape(-1)
    u = np.eye(n, dtype=np.complex128)
    for (i, j), th, ph in zip(e_list, theta, phi):
        u = u @ unitary_factor(n, int(i), int(j), float(th), float(ph))
    return u


def forward(theta, phi, operand, pairs=None) -> np.ndarray:
    """The appendix's forward algorithm from `operand`: blocks in reverse order, per pair
    r_i = exp(i phi) cos U_i - sin U_j,  r_j = exp(i phi) sin U_i + cos U_j."""
    state = np.array(operand, dtype=np.complex128, copy=True)
    n = state.shape[0]
    blocks = _pairs(n, pairs)
    theta = np.asarray(theta, dtype=np.float64).reshape(n - 1, n // 2)
    phi = np.asarray(phi, dtype=np.float64).reshape(n - 1, n // 2)
    for k in range(n - 2, -1, -1):
        for p in range(n // 2):
            i, j = int(blocks[k, p, 0]), int(blocks[k, p, 1])
            c, s, w = np.cos(theta[k, p]), np.sin(theta[k, p]), np.exp(1j * phi[k, p])
            r_i = w * c * state[i] - s * state[j]
            r_j = w * s * state[i] + c * state[j]
            state[i] = r_i
            state[j] = r_j
    return state


def _undo(state, i, j, c, s, w):
    """Rows (i, j) <- G^dagger rows: G^dagger = [[conj(w) c, conj(w) s], [-s, c]]."""
    a = np.conj(w) * (c * state[i] + s * state[j])
    b = -s * state[i] + c * state[j]
    state[i] = a
    state[j] = b


def grad_operand(theta, phi, upstream, pairs=None) -> np.ndarray:
    state = np.array(upstream, dtype=np.complex128, copy=True)
    n = state.shape[0]
    blocks = _pairs(n, pairs)
    theta = np.asarray(theta, dtype=np.float64).reshape(n - 1, n // 2)
    phi = np.asarray(phi, dtype=np.float64).reshape(n - 1, n // 2)
    for k in range(n - 1):
        for p in range(n // 2):
            i, j = int(blocks[k, p, 0]), int(blocks[k, p, 1])
            _undo(state, i, j, np.cos(theta[k, p]), np.sin(theta[k, p]), np.exp(1j * phi[k, p]))
    return state


def reverse_sweep(theta, phi, y, upstream, pairs=None):
    """Returns (dtheta, dphi, dX, X recovered).  For e = (i, j) in block k, with z = U^{k:n-1} X and
    gbar = (U^{1:k-1})^dagger G:
        dtheta_e = Re <gbar, Q_e z> = Re sum_b ( conj(gbar_j) z_i - conj(gbar_i) z_j ),
        dphi_e   = Re <gbar, P_e z> = Re sum_b i ( conj(gbar_i) (c^2 z_i + c s z_j) + conj(gbar_j) (c s z_i + s^2 z_j) ),
    then z and gbar are multiplied by the adjoint factor."""
    z = np.array(y, dtype=np.complex128, copy=True)
    gbar = np.array(upstream, dtype=np.complex128, copy=True)
    n = z.shape[0]
    blocks = _pairs(n, pairs)
    theta = np.asarray(theta, dtype=np.float64).reshape(n - 1, n // 2)
    phi = np.asarray(phi, dtype=np.float64).reshape(n - 1, n // 2)
    dtheta = np.zeros((n - 1, n // 2))
    dphi = np.zeros((n - 1, n // 2))
    for k in range(n - 1):
        for p in range(n // 2):
            i, j = int(blocks[k, p, 0]), int(blocks[k, p, 1])
            c, s, w = np.cos(theta[k, p]), np.sin(theta[k, p]), np.exp(1j * phi[k, p])
            dtheta[k, p] = float(np.real(np.sum(np.conj(gbar[j]) * z[i] - np.conj(gbar[i]) * z[j])))
            pz_i = 1j * (c * c * z[i] + c * s * z[j])
            pz_j = 1j * (c * s * z[i] + s * s * z[j])
            dphi[k, p] = float(np.real(np.sum(np.conj(gbar[i]) * pz_i + np.conj(gbar[j]) * pz_j)))
            _undo(z, i, j, c, s, w)
            _undo(gbar, i, j, c, s, w)
    return dtheta.reshape(-1), dphi.reshape(-1), gbar, z


def forward_blocks(theta, phi, operand, pairs=None) -> np.ndarray:
    """forward() with each block's disjoint pairs updated in one vectorised step (same arithmetic per pair;
    the pairs of a block touch different rows, so their order is immaterial)."""
    state = np.array(operand, dtype=np.complex128, copy=True)
    n = state.shape[0]
    blocks = _pairs(n, pairs)
    theta = np.asarray(theta, dtype=np.float64).reshape(n - 1, n // 2)
    phi = np.asarray(phi, dtype=np.float64).reshape(n - 1, n // 2)
    for k in range(n - 2, -1, -1):
        i, j = blocks[k, :, 0], blocks[k, :, 1]
        c, s, w = np.cos(theta[k])[:, None], np.sin(theta[k])[:, None], np.exp(1j * phi[k])[:, None]
        ri, rj = state[i], state[j]
        state[i] = w * c * ri - s * rj
        state[j] = w * s * ri + c * rj
    return state


def reverse_sweep_blocks(theta, phi, y, upstream, pairs=None):
    """reverse_sweep() block by block, vectorised over the block's pairs."""
    z = np.array(y, dtype=np.complex128, copy=True)
    gbar = np.array(upstream, dtype=np.complex128, copy=True)
    n = z.shape[0]
    blocks = _pairs(n, pairs)
    theta = np.asarray(theta, dtype=np.float64).reshape(n - 1, n // 2)
    phi = np.asarray(phi, dtype=np.float64).reshape(n - 1, n // 2)
    dtheta = np.zeros((n - 1, n // 2))
    dphi = np.zeros((n - 1, n // 2))
    for k in range(n - 1):
        i, j = blocks[k, :, 0], blocks[k, :, 1]
        c, s, w = np.cos(theta[k])[:, None], np.sin(theta[k])[:, None], np.exp(1j * phi[k])[:, None]
        zi, zj, gi, gj = z[i], z[j], gbar[i], gbar[j]
        dtheta[k] = np.real(np.sum(np.conj(gj) * zi - np.conj(gi) * zj, axis=1))
        pz_i = 1j * (c * c * zi + c * s * zj)
        pz_j = 1j * (c * s * zi + s * s * zj)
        dphi[k] = np.real(np.sum(np.conj(gi) * pz_i + np.conj(gj) * pz_j, axis=1))
        z[i] = np.conj(w) * (c * zi + s * zj)
        z[j] = -s * zi + c * zj
        gbar[i] = np.conj(w) * (c * gi + s * gj)
        gbar[j] = -s * gi + c * gj
    return dtheta.reshape(-1), dphi.reshape(-1), gbar, z


def loss(theta, phi, operand, upstream, pairs=None) -> float:
    y = forward(theta, phi, operand, pairs)
    return float(np.real(np.sum(np.conj(np.asarray(upstream, dtype=np.complex128)) * y)))


def finite_differences(theta, phi, operand, upstream, eps: float = 1e-6, pairs=None):
    """Central differences of the loss in every theta_e and every phi_e (tiny n only)."""
    theta = np.asarray(theta, dtype=np.float64).reshape(-1).copy()
    phi = np.asarray(phi, dtype=np.float64).reshape(-1).copy()
    out = []
    for vec in (theta, phi):
        g = np.empty_like(vec)
        for a in range(vec.size):
            keep = vec[a]
            vec[a] = keep + eps
            lp = loss(theta, phi, operand, upstream, pairs)
            vec[a] = keep - eps
            lm = loss(theta, phi, operand, upstream, pairs)
            vec[a] = keep
            g[a] = (lp - lm) / (2.0 * eps)
        out.append(g)
    return out[0], out[1]


def rel_fro(a, b) -> float:
    """||a - b||_F / ||b||_F for complex (or real) arrays, in complex128 (b is the reference)."""
    a = np.asarray(a, dtype=np.complex128)
    b = np.asarray(b, dtype=np.complex128)
    den = float(np.linalg.norm(b.ravel()))
    num = float(np.linalg.norm((a - b).ravel()))
    return num / den if den > 0 else num
