"""CPU oracle for the two adaptations the paper describes on top of the round-robin algorithms:
the restricted parametrisation (Section 5, "Restricting the Parametrization": no rotation among
the coordinates m..n-1) and odd n (end of Section 3: an extra, inactive dimension).

TEST INFRASTRUCTURE ONLY, like oracle/givens_oracle.py: only tests/, the smoke check and the
benchmark's cpu_baseline leg may import it; it shares no code with the HIP path.

Both adaptations are taken literally: the blocks are still those of the circle method (on n
dimensions, or on n + 1 when n is odd), and the loops *bypass* a pair
  * when i >= m (with i < j by convention, so both coordinates are in m..n-1), Section 5;
  * when j = n, the added dimension, end of Section 3 (forward) and end of Section 4.2 (gradient).
The free angles are the pairs that are not bypassed, in the order in which E lists them; theta and
dtheta have one entry per free angle (N = m n - m (m + 1) / 2 of them, Section 5).  m = n - 1 is the
unrestricted case (no pair lies inside a set of one coordinate).

Everything is float64 NumPy with explicit loops over pairs, in the paper's order:

  padded_dimension        n, or n + 1 for odd n
  restricted_blocks       the blocks b_1.. with the bypassed pairs left out
  free_pairs              their concatenation: the sequence E of free pairs
  num_free_angles         Section 5's closed form for N
  dense_product           Eq. (2) over the free pairs, explicit n x n factors
  forward                 Algorithm 1 / 2 with the bypass conditions (block by block)
  grad_operand            dL/dX = U^T G
  reverse_sweep           operand-side gradient with the bypass conditions
  scatter_to_full / pad_operand   embed a restricted / odd problem into the unrestricted even one
                          (bypassed pairs get angle 0, the added row is zero) -- used by the pins

Pins (tests/test_oracle_restricted.py): the n = 8, m = 4 example of Section 5 (which pairs go, 22
remain), the count formula, every free pair exactly once and disjoint pairs per block, a
hand-derived n = 3 schedule, m = n - 1 equal to the unrestricted oracle, dense product = Algorithm 1
with bypass = the unrestricted oracle with zero angles at the bypassed pairs (and a zero row for
odd n), orthogonality and det = +1, central differences of the loss for every free angle.
No function in this file is "parity unpinned".
"""
from __future__ import annotations

import numpy as np


def padded_dimension(n: int) -> int:
    """Number of dimensions the circle method runs on: n itself, or n + 1 when n is odd."""
    if n < 2:
        raise ValueError("n must be >= 2")
    return n + (n % 2)


def _check(n: int, m):
    if n < 2:
        raise ValueError("n must be >= 2")
    if m is None:
        m = n - 1
    if not 1 <= m <= n - 1:
        raise ValueError("m must satisfy 1 <= m <= n - 1")
    return m


def restricted_blocks(n: int, m=None):
    """List of blocks; block k is the list of free pairs (i, j), i < j, of b_{k+1} in arc order."""
    m = _check(n, m)
    size = padded_dimension(n)
    seq = list(range(size))                       # Section 3: start from (0, 1, ..., size-1)
    blocks = []
    for _ in range(size - 1):
        block = []
        for p in range(size // 2):
            a, b = seq[p], seq[size - 1 - p]      # position p with its mirror position
            i, j = (a, b) if a < b else (b, a)
            if j >= n:                            # the added dimension: bypass (odd n)
                continue
            if i >= m:                            # both coordinates in m..n-1: bypass (Section 5)
                continue
            block.append((i, j))
        blocks.append(block)
        seq = [seq[0], seq[-1]] + seq[1:-1]       # hold the first, last moves to position 1
    return blocks


def free_pairs(n: int, m=None) -> np.ndarray:
    """E restricted to the free pairs, shape (N, 2), int32."""
    flat = [pair for block in restricted_blocks(n, m) for pair in block]
    return np.asarray(flat, dtype=np.int32).reshape(-1, 2)


def num_free_angles(n: int, m=None) -> int:
    """Section 5: N = m n - m (m + 1) / 2."""
    m = _check(n, m)
    return m * n - m * (m + 1) // 2


def _givens(n, i, j, th):
    g = np.eye(n, dtype=np.float64)
    g[i, i] = np.cos(th)
    g[j, j] = np.cos(th)
    g[i, j] = -np.sin(th)
    g[j, i] = np.sin(th)
    return g


def dense_product(n: int, theta, m=None) -> np.ndarray:
    """Eq. (2) over the free pairs: U = G^{e_1} G^{e_2} ... (explicit factors, tiny n only)."""
    pairs = free_pairs(n, m)
    theta = np.asarray(theta, dtype=np.float64).reshape(-1)
    assert theta.size == pairs.shape[0]
    u = np.eye(n, dtype=np.float64)
    for (i, j), th in zip(pairs, theta):
        u = u @ _givens(n, int(i), int(j), float(th))
    return u


def _block_offsets(blocks):
    offsets, total = [], 0
    for block in blocks:
        offsets.append(total)
        total += len(block)
    return offsets, total


def forward(theta, operand, m=None) -> np.ndarray:
    """Algorithm 2 with the bypass conditions: blocks in reverse order, each free pair's two-row update."""
    state = np.array(operand, dtype=np.float64, copy=True)
    n = state.shape[0]
    blocks = restricted_blocks(n, m)
    offsets, total = _block_offsets(blocks)
    theta = np.asarray(theta, dtype=np.float64).reshape(-1)
    assert theta.size == total
    for k in range(len(blocks) - 1, -1, -1):                   # reversed(B)
        for q, (i, j) in enumerate(blocks[k]):
            th = theta[offsets[k] + q]
            c, s = np.cos(th), np.sin(th)
            r_i = c * state[i] - s * state[j]
            r_j = s * state[i] + c * state[j]
            state[i] = r_i
            state[j] = r_j
    return state


def grad_operand(theta, upstream, m=None) -> np.ndarray:
    """dL/dX = U^T G: transposed rotations of the free pairs in E order."""
    state = np.array(upstream, dtype=np.float64, copy=True)
    n = state.shape[0]
    blocks = restricted_blocks(n, m)
    offsets, _ = _block_offsets(blocks)
    theta = np.asarray(theta, dtype=np.float64).reshape(-1)
    for k in range(len(blocks)):
        for q, (i, j) in enumerate(blocks[k]):
            th = theta[offsets[k] + q]
            c, s = np.cos(th), np.sin(th)
            r_i = c * state[i] + s * state[j]
            r_j = -s * state[i] + c * state[j]
            state[i] = r_i
            state[j] = r_j
    return state


def reverse_sweep(theta, y, upstream, m=None):
    """Operand-side gradient with the bypass conditions: (dtheta over the free angles, dX, X recovered).
    Per free pair of block k, first dtheta_e = sum_b (gbar_j z_i - gbar_i z_j) (Section 4.1: Q_e Z has
    row i = -Z_j, row j = +Z_i), then the transposed rotation of z and gbar."""
    z = np.array(y, dtype=np.float64, copy=True)
    gbar = np.array(upstream, dtype=np.float64, copy=True)
    n = z.shape[0]
    blocks = restricted_blocks(n, m)
    offsets, total = _block_offsets(blocks)
    theta = np.asarray(theta, dtype=np.float64).reshape(-1)
    grad = np.zeros(total, dtype=np.float64)
    for k in range(len(blocks)):
        for q, (i, j) in enumerate(blocks[k]):
            e = offsets[k] + q
            c, s = np.cos(theta[e]), np.sin(theta[e])
            grad[e] = float(np.sum(gbar[j] * z[i] - gbar[i] * z[j]))
            zi = c * z[i] + s * z[j]
            zj = -s * z[i] + c * z[j]
            z[i], z[j] = zi, zj
            gi = c * gbar[i] + s * gbar[j]
            gj = -s * gbar[i] + c * gbar[j]
            gbar[i], gbar[j] = gi, gj
    return grad, gbar, z


def scatter_to_full(n: int, theta, m=None) -> np.ndarray:
    """Angles of the unrestricted problem on padded_dimension(n) dimensions, in its E order, with the
    free angles in place and 0 at every bypassed pair."""
    m = _check(n, m)
    size = padded_dimension(n)
    theta = np.asarray(theta, dtype=np.float64).reshape(-1)
    full = np.zeros((size - 1) * (size // 2), dtype=np.float64)
    seq = list(range(size))
    e_full, e_free = 0, 0
    for _ in range(size - 1):
        for p in range(size // 2):
            a, b = seq[p], seq[size - 1 - p]
            i, j = (a, b) if a < b else (b, a)
            if j < n and i < m:
                full[e_full] = theta[e_free]
                e_free += 1
            e_full += 1
        seq = [seq[0], seq[-1]] + seq[1:-1]
    assert e_free == theta.size
    return full


def pad_operand(operand) -> np.ndarray:
    """The operand with a zero row appended when its row count is odd."""
    x = np.asarray(operand, dtype=np.float64)
    if x.shape[0] % 2 == 0:
        return x.copy()
    return np.vstack([x, np.zeros((1,) + x.shape[1:], dtype=np.float64)])
