"""CPU oracle for angle-parametrised orthogonal matrices under the round-robin order.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file;
only tests/, the smoke check and the benchmark's cpu_baseline leg use it.  It
shares no code with the HIP kernels and never receives a value computed by them.

Everything is plain NumPy in float64 (inputs are promoted on entry), written so
that each function can be compared with the paper by eye:

  circle_method_schedule   Section 3, circle method; Figure 1; worked example Eq. (3)
  givens_matrix            Section 2, entries of G^e
  dense_product            Eq. (2): U = G^{e_1} G^{e_2} ... G^{e_N}, explicit n x n factors
  forward_sequential       Algorithm 1 ("Forward U"), started from any operand
  forward_block_parallel   Algorithm 2 ("Parallel Forward U"), one vectorised step per block
  grad_operand             dL/dX = U^T G, by transposed rotations taken in E order
  grad_theta_alg3          Algorithm 3 ("Parallel JVP"), as printed: U^fwd column updates,
                           M row updates, A matrix, row sums
  reverse_sweep            the operand-side form of the same gradient (Section 4.1,
                           dU/dtheta_e = U^{1:k-1} Q_e U^{k:n-1}, contracted with the
                           upstream gradient on the operand's side)
  apply_block_range        partial products U^{a:b} of Section 4.1 applied to an operand
  grad_theta_single        one component of the gradient from the rank-2 Jacobian
                           dU/dtheta_e = u_j v_i^T - u_i v_j^T (Section 4.1), O(n^2 + nB)
  loss / finite_difference_grad_theta   L = sum(G * (U X)) and its central differences

Readings of the paper taken here (each is also listed in the design notes):
  * the circle method starts from (0, 1, ..., n-1), holds element 0 and moves the last
    element to position 1 at each shift, as the five sequences of Figure 1 print it;
  * pairs inside a block are in arc order, outermost arc first (Eq. (3));
  * every pair is written (i, j) with i < j; G_ij = -sin, G_ji = +sin;
  * theta is indexed by E = b_1 ++ b_2 ++ ... ++ b_{n-1} (block-major, arc-minor);
  * G^{e_N} applies first, so the loops run over reversed(E) / reversed(B);
  * in Algorithm 3 the indices are 0-based and A is (n/2) x n;
  * in Algorithm 3, u_{lj} is entry (l, j) of U^fwd, i.e. entry l of column u_j;
  * with a general operand X the upstream gradient with respect to U is
    Gamma = G X^T (chain rule through Y = U X); the paper treats only Y = U.

Parity pins (tests/test_oracle_*.py): Eq. (3) and Figure 1 literally, perfect
matching / each pair once, dense product vs Algorithm 1 vs Algorithm 2,
theta = 0, single angle, n = 2 closed form, U^T U = I, det U = +1, norm
preservation, finite differences per angle, G = Y gives zero gradient,
Algorithm 3 vs the operand-side sweep, adjoint identity for dX.
No function in this file is "parity unpinned".
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------
# Section 3: the round-robin sequence by the circle method
# --------------------------------------------------------------------------
def circle_method_sequences(n: int) -> np.ndarray:
    """The n-1 dimension sequences of Figure 1 (left column), one per block."""
    if n < 2 or n % 2:
        raise ValueError("n must be even and >= 2")
    seq = list(range(n))
    rows = []
    for _ in range(n - 1):
        rows.append(list(seq))
        # hold the first element, shift the other n-1 cyclically: last -> position 1
        seq = [seq[0], seq[-1]] + seq[1:-1]
    return np.asarray(rows, dtype=np.int64)


def circle_method_schedule(n: int) -> np.ndarray:
    """Blocks b_1..b_{n-1}; result[k, p] = (i, j), i < j, arc p of block k+1."""
    seqs = circle_method_sequences(n)
    half = n // 2
    out = np.empty((n - 1, half, 2), dtype=np.int32)
    for k in range(n - 1):
        for p in range(half):
            a, b = int(seqs[k, p]), int(seqs[k, n - 1 - p])
            out[k, p, 0] = min(a, b)
            out[k, p, 1] = max(a, b)
    return out


def _as_blocks(n: int, pairs) -> np.ndarray:
    if pairs is None:
        return circle_method_schedule(n)
    pairs = np.asarray(pairs)
    return pairs.reshape(n - 1, n // 2, 2)


# --------------------------------------------------------------------------
# Section 2: Givens matrices and the product that defines U
# --------------------------------------------------------------------------
def givens_matrix(n: int, i: int, j: int, theta: float) -> np.ndarray:
    """G^e for e = (i, j), i < j: identity except four entries."""
    assert 0 <= i < j < n
    g = np.eye(n, dtype=np.float64)
    g[i, i] = np.cos(theta)
    g[j, j] = np.cos(theta)
    g[i, j] = -np.sin(theta)
    g[j, i] = np.sin(theta)
    return g


def dense_product(n: int, theta, pairs=None) -> np.ndarray:
    """Eq. (2): multiply the explicit n x n factors left to right in E order."""
    blocks = _as_blocks(n, pairs)
    theta = np.asarray(theta, dtype=np.float64).reshape(-1)
    e_list = blocks.reshape(-1, 2)
    assert theta.size == e_list.shape[0]
    u = np.eye(n, dtype=np.float64)
    for (i, j), th in zip(e_list, theta):
        u = u @ givens_matrix(n, int(i), int(j), float(th))
    return u


# --------------------------------------------------------------------------
# Algorithm 1 and Algorithm 2: forward
# --------------------------------------------------------------------------
def forward_sequential(theta, operand, pairs=None) -> np.ndarray:
    """Algorithm 1, started from `operand` instead of I_n (in-place row operations)."""
    state = np.array(operand, dtype=np.float64, copy=True)
    n = state.shape[0]
    e_list = _as_blocks(n, pairs).reshape(-1, 2)
    theta = np.asarray(theta, dtype=np.float64).reshape(-1)
    for idx in range(e_list.shape[0] - 1, -1, -1):        # reversed(E)
        i, j = int(e_list[idx, 0]), int(e_list[idx, 1])
        c, s = np.cos(theta[idx]), np.sin(theta[idx])
        r_i = c * state[i] - s * state[j]
        r_j = s * state[i] + c * state[j]
        state[i] = r_i
        state[j] = r_j
    return state


def forward_block_parallel(theta, operand, pairs=None) -> np.ndarray:
    """Algorithm 2: outer loop over reversed(B); each block's pairs are updated together."""
    state = np.array(operand, dtype=np.float64, copy=True)
    n = state.shape[0]
    blocks = _as_blocks(n, pairs)
    theta = np.asarray(theta, dtype=np.float64).reshape(n - 1, n // 2)
    for k in range(n - 2, -1, -1):                        # reversed(B)
        i = blocks[k, :, 0]
        j = blocks[k, :, 1]
        c = np.cos(theta[k])[:, None]
        s = np.sin(theta[k])[:, None]
        rows_i = state[i]
        rows_j = state[j]
        state[i] = c * rows_i - s * rows_j
        state[j] = s * rows_i + c * rows_j
    return state


def build_u(theta, n: int, pairs=None) -> np.ndarray:
    """Algorithm 2 exactly as printed: U <- I_n, then the block sweeps."""
    return forward_block_parallel(theta, np.eye(n, dtype=np.float64), pairs)


# --------------------------------------------------------------------------
# Gradients
# --------------------------------------------------------------------------
def grad_operand(theta, upstream, pairs=None) -> np.ndarray:
    """dL/dX = U^T G.  U^T = G^{e_N}^T ... G^{e_1}^T, so G^{e_1}^T applies first:
    the transposed rotations are taken in E order."""
    state = np.array(upstream, dtype=np.float64, copy=True)
    n = state.shape[0]
    blocks = _as_blocks(n, pairs)
    theta = np.asarray(theta, dtype=np.float64).reshape(n - 1, n // 2)
    for k in range(n - 1):
        i = blocks[k, :, 0]
        j = blocks[k, :, 1]
        c = np.cos(theta[k])[:, None]
        s = np.sin(theta[k])[:, None]
        rows_i = state[i]
        rows_j = state[j]
        state[i] = c * rows_i + s * rows_j                # row i of G^T: ( c, +s)
        state[j] = -s * rows_i + c * rows_j               # row j of G^T: (-s,  c)
    return state


def grad_theta_alg3(theta, u, gamma, pairs=None) -> np.ndarray:
    """Algorithm 3.  u = U(theta) from the forward pass, gamma = dL/dU (n x n)."""
    u_fwd = np.array(u, dtype=np.float64, copy=True)
    m = np.array(gamma, dtype=np.float64).T.copy()
    n = u_fwd.shape[0]
    blocks = _as_blocks(n, pairs)
    theta = np.asarray(theta, dtype=np.float64).reshape(n - 1, n // 2)
    grad = np.zeros((n - 1, n // 2), dtype=np.float64)
    a = np.empty((n // 2, n), dtype=np.float64)
    for k in range(n - 2, -1, -1):                        # reversed(B)
        i = blocks[k, :, 0]
        j = blocks[k, :, 1]
        c = np.cos(theta[k])
        s = np.sin(theta[k])
        # U^fwd column update
        col_i = u_fwd[:, i]
        col_j = u_fwd[:, j]
        u_fwd[:, i] = c[None, :] * col_i - s[None, :] * col_j
        u_fwd[:, j] = s[None, :] * col_i + c[None, :] * col_j
        # M row update
        row_i = m[i]
        row_j = m[j]
        m[i] = c[:, None] * row_i - s[:, None] * row_j
        m[j] = s[:, None] * row_i + c[:, None] * row_j
        # A assignment: A[m(e), l] = M[i, l] u[l, j] - M[j, l] u[l, i]
        a[:, :] = m[i] * u_fwd[:, j].T - m[j] * u_fwd[:, i].T
        # row sums, scattered to the block's angles
        grad[k] = a @ np.ones(n)
    return grad.reshape(-1)


def reverse_sweep(theta, y, upstream, pairs=None):
    """Operand-side gradient: returns (d_theta, dX, X_recovered).

    For e in b_k, dL/dtheta_e = <Gbar, Q_e Z>, where Z = U^{k:n-1} X is the state
    right after block k was applied in the forward pass, Gbar = (U^{1:k-1})^T G is
    the upstream gradient carried back to that point, and Q_e is -1 at (i, j),
    +1 at (j, i) (Section 4.1).  Q_e Z has row i = -Z_j and row j = +Z_i.
    """
    z = np.array(y, dtype=np.float64, copy=True)
    gbar = np.array(upstream, dtype=np.float64, copy=True)
    n = z.shape[0]
    blocks = _as_blocks(n, pairs)
    theta = np.asarray(theta, dtype=np.float64).reshape(n - 1, n // 2)
    grad = np.zeros((n - 1, n // 2), dtype=np.float64)
    for k in range(n - 1):
        i = blocks[k, :, 0]
        j = blocks[k, :, 1]
        c = np.cos(theta[k])[:, None]
        s = np.sin(theta[k])[:, None]
        zi, zj = z[i], z[j]
        gi, gj = gbar[i], gbar[j]
        grad[k] = np.sum(gj * zi - gi * zj, axis=1)
        z[i] = c * zi + s * zj
        z[j] = -s * zi + c * zj
        gbar[i] = c * gi + s * gj
        gbar[j] = -s * gi + c * gj
    return grad.reshape(-1), gbar, z


def apply_block_range(theta, operand, k_lo: int, k_hi: int, transpose: bool = False, pairs=None):
    """U^{k_lo+1 : k_hi} . operand (0-based block indices k_lo..k_hi-1 are used), or its transpose.

    U^{a:b} = G^{b_a} ... G^{b_b} (Section 4.1); the rightmost block applies first, so the plain
    product sweeps the blocks downwards and the transposed one upwards with transposed rotations.
    """
    state = np.array(operand, dtype=np.float64, copy=True)
    n = state.shape[0]
    blocks = _as_blocks(n, pairs)
    theta = np.asarray(theta, dtype=np.float64).reshape(n - 1, n // 2)
    order = range(k_lo, k_hi) if transpose else range(k_hi - 1, k_lo - 1, -1)
    for k in order:
        i = blocks[k, :, 0]
        j = blocks[k, :, 1]
        c = np.cos(theta[k])
        s = np.sin(theta[k])
        if state.ndim == 2:
            c, s = c[:, None], s[:, None]
        rows_i = state[i]
        rows_j = state[j]
        if transpose:
            state[i] = c * rows_i + s * rows_j
            state[j] = -s * rows_i + c * rows_j
        else:
            state[i] = c * rows_i - s * rows_j
            state[j] = s * rows_i + c * rows_j
    return state


def grad_theta_single(theta, operand, upstream, e: int, pairs=None) -> float:
    """dL/dtheta_e for one angle, straight from the rank-2 form of Section 4.1:

        dU/dtheta_e = u_j v_i^T - u_i v_j^T,   u = columns of U^fwd = U^{1:k-1},
                                                v^T = rows of U^bck = U^{k:n-1},  e in b_k,

    contracted with dL/dU = G X^T:  dL/dtheta_e = u_j^T G (v_i^T X)^T - u_i^T G (v_j^T X)^T.
    Cost O(n^2 + nB): this is what full-size tests use for sampled angles.
    """
    x = np.asarray(operand)
    g = np.asarray(upstream)
    n = x.shape[0]
    half = n // 2
    blocks = _as_blocks(n, pairs)
    k, p = divmod(int(e), half)
    i, j = int(blocks[k, p, 0]), int(blocks[k, p, 1])
    unit = np.zeros((n, 2), dtype=np.float64)
    unit[i, 0] = 1.0
    unit[j, 1] = 1.0
    u_cols = apply_block_range(theta, unit, 0, k, transpose=False, pairs=pairs)          # U^{1:k-1} e_i, e_j
    v_rows = apply_block_range(theta, unit, k, n - 1, transpose=True, pairs=pairs)       # (U^{k:n-1})^T e_i, e_j
    z_i = v_rows[:, 0] @ x.astype(np.float64, copy=False)                                # row i of U^bck X
    z_j = v_rows[:, 1] @ x.astype(np.float64, copy=False)
    g_i = u_cols[:, 0] @ g.astype(np.float64, copy=False)                                # row i of U^fwd^T G
    g_j = u_cols[:, 1] @ g.astype(np.float64, copy=False)
    return float(g_j @ z_i - g_i @ z_j)


def loss(theta, operand, upstream, pairs=None) -> float:
    """L = sum(G * (U X))."""
    y = forward_block_parallel(theta, operand, pairs)
    return float(np.sum(np.asarray(upstream, dtype=np.float64) * y))


def finite_difference_grad_theta(theta, operand, upstream, eps: float = 1e-6,
                                 pairs=None, forward=None) -> np.ndarray:
    """Central differences of L, one angle at a time (tiny n only)."""
    theta = np.asarray(theta, dtype=np.float64).reshape(-1).copy()
    fwd = forward or (lambda th: forward_block_parallel(th, operand, pairs))
    g64 = np.asarray(upstream, dtype=np.float64)
    out = np.empty_like(theta)
    for a in range(theta.size):
        keep = theta[a]
        theta[a] = keep + eps
        lp = float(np.sum(g64 * fwd(theta)))
        theta[a] = keep - eps
        lm = float(np.sum(g64 * fwd(theta)))
        theta[a] = keep
        out[a] = (lp - lm) / (2.0 * eps)
    return out


def rel_fro(a, b) -> float:
    """||a - b||_F / ||b||_F in float64 (b is the reference)."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = float(np.linalg.norm(b.ravel()))
    num = float(np.linalg.norm((a - b).ravel()))
    return num / den if den > 0 else num
