"""Pins for oracle/restricted_oracle.py (restricted parametrisation, Section 5; odd n, end of Section 3)."""
import itertools
import os

import numpy as np
import pytest

from oracle import givens_oracle as O
from oracle import restricted_oracle as R

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, val = line.split(":", 1)
        out[key.strip()] = val.strip()
    return out


def test_section5_example_n8_m4():
    gold = _read("restricted_n8_m4.txt")
    removed = {tuple(int(v) for v in tok.split("-")) for tok in gold["removed"].split()}
    free = {tuple(p) for p in R.free_pairs(8, 4).tolist()}
    every = set(itertools.combinations(range(8), 2))
    assert every - free == removed
    assert len(free) == int(gold["free"]) == R.num_free_angles(8, 4)


def test_hand_derived_schedule_for_n3():
    gold = _read("odd_n3_schedule.txt")
    blocks = R.restricted_blocks(3)
    assert len(blocks) == int(gold["blocks"])
    for k, block in enumerate(blocks):
        want = [tuple(int(v) for v in tok.split("-")) for tok in gold[f"b{k + 1}"].split()]
        assert block == want


@pytest.mark.parametrize("n", [2, 3, 4, 5, 6, 7, 8, 9, 16, 17, 33, 64, 101])
def test_counts_and_matching_structure(n):
    size = R.padded_dimension(n)
    for m in sorted({1, 2, n // 2, n - 2, n - 1} & set(range(1, n))):
        blocks = R.restricted_blocks(n, m)
        assert len(blocks) == size - 1                         # still one block per round of the circle method
        flat = [p for b in blocks for p in b]
        assert len(flat) == R.num_free_angles(n, m) == m * n - m * (m + 1) // 2
        assert len(set(flat)) == len(flat)                     # every free pair once
        assert set(flat) == {(i, j) for i, j in itertools.combinations(range(n), 2) if i < m}
        for b in blocks:                                       # pairs of a block are disjoint: they commute
            used = [v for p in b for v in p]
            assert len(set(used)) == len(used)


@pytest.mark.parametrize("n", [4, 6, 8, 12])
def test_m_equal_n_minus_1_is_the_unrestricted_case(n):
    assert np.array_equal(R.free_pairs(n, n - 1), O.circle_method_schedule(n).reshape(-1, 2))
    rng = np.random.default_rng(n)
    theta = rng.uniform(-np.pi, np.pi, n * (n - 1) // 2)
    x, g = rng.standard_normal((n, 5)), rng.standard_normal((n, 5))
    y = R.forward(theta, x)
    assert np.array_equal(y, O.forward_sequential(theta, x)) or O.rel_fro(y, O.forward_sequential(theta, x)) < 1e-15
    gt, gx, _ = R.reverse_sweep(theta, y, g, n - 1)
    wt, wx, _ = O.reverse_sweep(theta, y, g)
    assert O.rel_fro(gt, wt) < 1e-13 and O.rel_fro(gx, wx) < 1e-13


@pytest.mark.parametrize("n,m", [(4, 1), (6, 2), (8, 4), (8, 7), (5, 2), (5, 4), (7, 3), (9, 8), (3, 1), (3, 2)])
def test_dense_product_bypass_and_embedding_agree(n, m):
    rng = np.random.default_rng(100 * n + m)
    count = R.num_free_angles(n, m)
    theta = rng.uniform(-np.pi, np.pi, count)
    x, g = rng.standard_normal((n, 6)), rng.standard_normal((n, 6))
    u = R.dense_product(n, theta, m)                                   # the definition, Eq. (2)
    assert O.rel_fro(u.T @ u, np.eye(n)) < 1e-14
    assert abs(np.linalg.det(u) - 1.0) < 1e-12
    y = R.forward(theta, x, m)
    assert O.rel_fro(y, u @ x) < 1e-14
    assert O.rel_fro(R.forward(theta, np.eye(n), m), u) < 1e-14
    # the same problem inside the unrestricted even one: zero angles at the bypassed pairs
    size = R.padded_dimension(n)
    full = R.scatter_to_full(n, theta, m)
    y_full = O.forward_sequential(full, R.pad_operand(x))
    assert O.rel_fro(y_full[:n], y) < 1e-14
    if size != n:
        assert np.all(y_full[n] == 0.0)                                # the added row is never touched
    # gradients
    dth, dx, x_back = R.reverse_sweep(theta, y, g, m)
    assert O.rel_fro(x_back, x) < 1e-13
    assert O.rel_fro(dx, u.T @ g) < 1e-14
    assert O.rel_fro(R.grad_operand(theta, g, m), u.T @ g) < 1e-14
    full_dth, _, _ = O.reverse_sweep(full, y_full, R.pad_operand(g))
    free_mask = R.scatter_to_full(n, np.ones(count), m) == 1.0
    assert O.rel_fro(dth, full_dth[free_mask]) < 1e-12
    fd = np.empty(count)
    for a in range(count):
        tp, tm = theta.copy(), theta.copy()
        tp[a] += 1e-6
        tm[a] -= 1e-6
        fd[a] = (np.sum(g * (R.dense_product(n, tp, m) @ x)) - np.sum(g * (R.dense_product(n, tm, m) @ x))) / 2e-6
    assert O.rel_fro(dth, fd) < 1e-7


def test_coordinates_outside_the_subset_only_mix_through_the_subset():
    """Section 5: no rotation acts inside m..n-1.  With all angles zero except those of pairs (i, j)
    with j < m, rows m..n-1 of the operand are untouched."""
    n, m = 8, 3
    pairs = R.free_pairs(n, m)
    rng = np.random.default_rng(7)
    theta = np.where(pairs[:, 1] < m, rng.uniform(-1, 1, pairs.shape[0]), 0.0)
    x = rng.standard_normal((n, 4))
    y = R.forward(theta, x, m)
    assert np.array_equal(y[m:], x[m:])
    assert not np.allclose(y[:m], x[:m])


@pytest.mark.parametrize("n,m,B", [(8, 4, 5), (9, 8, 40), (33, 10, 70), (64, 63, 33), (127, 126, 20)])
def test_c_oracle_on_free_pairs_equals_the_numpy_oracle(n, m, B):
    from oracle import c_oracle as C
    rng = np.random.default_rng(n * 1000 + m)
    pairs = R.free_pairs(n, m)
    theta = rng.uniform(-np.pi, np.pi, pairs.shape[0])
    x, g = rng.standard_normal((n, B)), rng.standard_normal((n, B))
    y = R.forward(theta, x, m)
    assert O.rel_fro(C.forward_pairs(theta, x, pairs), y) < 1e-14
    assert O.rel_fro(C.forward_pairs(theta, None, pairs, n=n), R.forward(theta, np.eye(n), m)) < 1e-14
    dth, dx, xr = R.reverse_sweep(theta, y, g, m)
    c_dth, c_dx, c_xr = C.reverse_sweep_pairs(theta, y, g, pairs)
    assert O.rel_fro(c_dth, dth) < 1e-12 and O.rel_fro(c_dx, dx) < 1e-14 and O.rel_fro(c_xr, xr) < 1e-14
    assert O.rel_fro(C.grad_operand_pairs(theta, g, pairs), dx) < 1e-14


def test_invalid_arguments():
    for bad in [(1, None), (4, 0), (4, 4), (5, 5)]:
        with pytest.raises(ValueError):
            R.restricted_blocks(*bad)
