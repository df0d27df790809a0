"""Seeded synthetic inputs for the round-robin Givens workloads.

This module only draws random numbers and shapes them; it holds none of the
method's arithmetic (no rotations, no schedule).  Both the CPU oracle's tests
and the HIP path's tests/bench feed on the arrays it returns, so the two sides
always see bit-identical inputs.

The paper's own workload is "an orthogonal matrix of size n built from random
angles" (Results section); it uses no dataset, so nothing external is being
stood in for.  The five workloads below are the ones the benchmark names:

  id  n     B      dtype  theta                X, G
  1   8     4      f64    Uniform[-pi, pi)     N(0,1)
  2   256   256    f32    Uniform[-pi, pi)     N(0,1)
  3   1024  1024   f32    Uniform[-pi, pi)     X = I (never materialised), G ~ N(0,1)
  4   4096  4096   f32    N(0, 0.1^2)          N(0,1)   (near-identity initialisation)
  5   2048  65536  f32    Uniform[-pi, pi)     N(0,1)   (batch-heavy layer)

theta has n(n-1)/2 entries.  Each array comes from its own NumPy PCG64 stream
(seed = 20210600 + id, spawned per array), drawn directly in the workload's
dtype, so a column subset of X or G can be generated without the rest only by
slicing the full array.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    id: int
    n: int
    B: int
    dtype: str          # "f64" or "f32"
    theta_dist: str     # "uniform" or "normal0.1"
    x_identity: bool    # True: the operand is I_n (build U), X is not generated

    @property
    def num_angles(self) -> int:
        return self.n * (self.n - 1) // 2

    @property
    def np_dtype(self):
        return np.float64 if self.dtype == "f64" else np.float32

    @property
    def name(self) -> str:
        return f"config{self.id}_n{self.n}_B{self.B}_{self.dtype}"


WORKLOADS = {
    1: Workload(1, 8, 4, "f64", "uniform", False),
    2: Workload(2, 256, 256, "f32", "uniform", False),
    3: Workload(3, 1024, 1024, "f32", "uniform", True),
    4: Workload(4, 4096, 4096, "f32", "normal0.1", False),
    5: Workload(5, 2048, 65536, "f32", "uniform", False),
}

BASE_SEED = 20210600


def _streams(seed: int, count: int):
    return [np.random.Generator(np.random.PCG64(s))
            for s in np.random.SeedSequence(seed).spawn(count)]


def draw_theta(rng: np.random.Generator, count: int, dist: str, dtype) -> np.ndarray:
    """Angles in the workload's dtype.  'uniform' is Uniform[-pi, pi)."""
    if dist == "uniform":
        u = rng.random(count, dtype=dtype)                # [0, 1)
        th = (u * dtype(2.0 * math.pi) - dtype(math.pi)).astype(dtype)
        # the fp32 product can round up to +pi; fold that single value back
        th[th >= dtype(math.pi)] = -dtype(math.pi)
        return th
    if dist == "normal0.1":
        return (rng.standard_normal(count, dtype=dtype) * dtype(0.1)).astype(dtype)
    raise ValueError(f"unknown theta distribution {dist!r}")


def make_inputs(workload_id: int, *, want_x: bool = True, want_g: bool = True) -> dict:
    """Return {'theta', 'X', 'G', 'workload'} for one of the five named workloads.

    X is None for the build workload (operand = identity).  Arrays are C-order,
    n x B with the batch along the second axis.
    """
    wl = WORKLOADS[workload_id]
    s_theta, s_x, s_g = _streams(BASE_SEED + wl.id, 3)
    dt = wl.np_dtype
    out = {"workload": wl}
    out["theta"] = draw_theta(s_theta, wl.num_angles, wl.theta_dist, dt)
    out["X"] = None
    if want_x and not wl.x_identity:
        out["X"] = s_x.standard_normal((wl.n, wl.B), dtype=dt)
    out["G"] = s_g.standard_normal((wl.n, wl.B), dtype=dt) if want_g else None
    return out


def make_custom(n: int, B: int, *, seed: int, dtype=np.float32,
                theta_dist: str = "uniform") -> dict:
    """Same recipe for an arbitrary (n, B): used by parity tests at ragged sizes."""
    s_theta, s_x, s_g = _streams(seed, 3)
    dt = np.dtype(dtype).type
    return {
        "theta": draw_theta(s_theta, n * (n - 1) // 2, theta_dist, dt),
        "X": s_x.standard_normal((n, B), dtype=dt),
        "G": s_g.standard_normal((n, B), dtype=dt),
    }


def make_restricted(n: int, m: int, B: int, *, seed: int, dtype=np.float32,
                    theta_dist: str = "uniform") -> dict:
    """Same recipe with one angle per free pair of the parametrisation restricted to pairs (i, j),
    i < m (m n - m (m + 1) / 2 of them); n may be odd."""
    s_theta, s_x, s_g = _streams(seed, 3)
    dt = np.dtype(dtype).type
    return {
        "theta": draw_theta(s_theta, m * n - m * (m + 1) // 2, theta_dist, dt),
        "X": s_x.standard_normal((n, B), dtype=dt),
        "G": s_g.standard_normal((n, B), dtype=dt),
    }
