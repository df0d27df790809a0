#!/usr/bin/env python3
"""Benchmark of the round-robin Givens hot path on one MI355X.

One "step" = one forward (cos/sin table + Algorithm-2 sweep, Y = U(theta) X) and one backward
(table + reverse sweep + dtheta second-stage reduction, giving dX and dtheta) on the workload
n = 4096, B = 4096, fp32, theta ~ N(0, 0.1^2), X, G ~ N(0, 1), all resident in HBM before the
timed region.  `value` is Givens row-pair column updates per second over the whole step:
N * B / (time of one step), N = n(n-1)/2 (one "update" = one rotation applied to one column in
the forward pass; the backward pass does two rotations and one two-term product per update).

Prints ONE JSON line.  Besides the contract fields it carries
  roofline      forward sweep kernel against the vector-FP32 peak (6 flop per update)
  roofline_bwd  reverse sweep kernel against the same peak (16 flop per update)
  cpu_baseline  the fp64 C oracle (oracle/givens_oracle.c) timed on the host cores on the first
                `sample` columns of the same workload
Kernel durations come from HIP events that the library records on the launch stream around each
kernel (givens_set_timing), during the timed steps themselves.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_VECTOR_TFLOPS = 157.3      # MI355X published vector FP32 peak (256 CU x 2.4 GHz x 256 flop/clk)
FWD_FLOP_PER_UPDATE = 6              # 4 mul + 2 add (Algorithm 1's two row updates)
BWD_FLOP_PER_UPDATE = 16             # two transposed rotations (12) + two-term product and sum (4)
CPU_SAMPLE_COLUMNS = 4096


def _traffic_from_profiles(kernel_tag: str):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE), if a summary
    for this kernel has been committed under profiles/ (a line 'traffic_bytes_per_launch: N')."""
    path = os.path.join(ROOT, "profiles", f"{kernel_tag}_pmc.txt")
    try:
        text = open(path).read()
    except OSError:
        return None
    m = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", text)
    return float(m.group(1)) if m else None


def _bench_unitary(args, binding, torch, np) -> int:
    """Forward + backward of the unitary extension on synthetic complex64 data (LDS strip kernels)."""
    n, B = (int(v) for v in args.unitary.split(","))
    N = n * (n - 1) // 2
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20210699)
    theta = (torch.rand(N, device="cuda", generator=gen) * 2 - 1) * np.pi
    phi = (torch.rand(N, device="cuda", generator=gen) * 2 - 1) * np.pi
    x = torch.randn(n, B, 2, device="cuda", generator=gen)
    g = torch.randn(n, B, 2, device="cuda", generator=gen)
    x, g = torch.view_as_complex(x), torch.view_as_complex(g)
    y, dx = torch.empty_like(x), torch.empty_like(x)
    dth, dph = torch.empty_like(theta), torch.empty_like(phi)

    def step():
        binding.givens_unitary_forward(theta, phi, x, Y=y)
        t_f = binding.last_timing()
        binding.givens_unitary_backward(theta, phi, y, g, dX=dx, dtheta=dth, dphi=dph)
        return t_f, binding.last_timing()

    binding.set_timing(True)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    times = [step() for _ in range(args.steps)]
    torch.cuda.synchronize()
    ms = 1e3 * (time.perf_counter() - t0) / args.steps
    binding.set_timing(False)
    print(json.dumps({
        "metric": "unitary_row_pair_complex_column_updates_per_s_fwd_bwd", "value": float(N) * B / (ms * 1e-3),
        "unit": "updates/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "dtype": "c64", "data": "synthetic",
        "config": {"workload": f"unitary_n{n}_B{B}_c64", "n": n, "B": B, "angles": 2 * N},
        "kernel_ms": {"fwd_table": float(np.mean([t[0][0] for t in times])),
                      "fwd_sweep": float(np.mean([t[0][1] for t in times])),
                      "bwd_sweep": float(np.mean([t[1][1] for t in times])),
                      "bwd_reduce": float(np.mean([t[1][2] for t in times]))}}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=4, choices=[2, 4, 5],
                    help="benchmark workload id (default 4: n=4096, B=4096)")
    ap.add_argument("--restricted", type=str, default=None, metavar="ROWS,M",
                    help="time the restricted entry points instead: ROWS coordinates (may be odd), pairs (i, j) "
                         "with i < M free, the chosen workload's B and angle distribution; not the headline metric")
    ap.add_argument("--unitary", type=str, default=None, metavar="N,B",
                    help="time the unitary (complex) entry points on an N x B complex64 operand instead and print a "
                         "short JSON line; not the headline metric")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-copy", action="store_true",
                    help="after the steps, run one plain device copy of X into Y (n*B*4 bytes read and "
                         "written) so that a rocprofv3 --pmc run has a kernel of known traffic to scale by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (columns of X shard trivially across GPUs; "
              "that path is design-only here). Use --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2106_00003_amd import binding, inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    binding.lib()
    binding.set_kernel(binding.KERNEL_AUTO)

    if args.unitary:
        return _bench_unitary(args, binding, torch, np)

    data = inputs.make_inputs(args.workload)
    wl = data["workload"]
    n, B = wl.n, wl.B
    N = wl.num_angles
    name = wl.name
    restricted_m = None
    if args.restricted:
        n, restricted_m = (int(v) for v in args.restricted.split(","))
        data = inputs.make_restricted(n, restricted_m, B, seed=inputs.BASE_SEED + 100 + args.workload,
                                      theta_dist=wl.theta_dist)
        N = data["theta"].size
        name = f"restricted_n{n}_m{restricted_m}_B{B}_f32"
        args.no_cpu_baseline = True
    th_d = torch.from_numpy(data["theta"]).cuda()
    x_d = torch.from_numpy(data["X"]).cuda()
    g_d = torch.from_numpy(data["G"]).cuda()
    y_d = torch.empty_like(x_d)
    dx_d = torch.empty_like(x_d)
    dth_d = torch.empty_like(th_d)

    def step():
        if restricted_m is None:
            binding.givens_forward(th_d, x_d, Y=y_d)
        else:
            binding.givens_forward_restricted(th_d, x_d, restricted_m, Y=y_d)
        t_f = binding.last_timing()
        if restricted_m is None:
            binding.givens_backward(th_d, y_d, g_d, dX=dx_d, dtheta=dth_d)
        else:
            binding.givens_backward_restricted(th_d, y_d, g_d, restricted_m, dX=dx_d, dtheta=dth_d)
        t_b = binding.last_timing()
        return t_f, t_b

    binding.set_timing(True)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    kernel_times = [step() for _ in range(args.steps)]
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    binding.set_timing(False)
    families = binding.last_kernel()

    ms_per_step = 1e3 * elapsed / args.steps
    updates = float(N) * float(B)
    fwd_table = float(np.mean([t[0][0] for t in kernel_times]))
    fwd_sweep = float(np.mean([t[0][1] for t in kernel_times]))
    bwd_table = float(np.mean([t[1][0] for t in kernel_times]))
    bwd_sweep = float(np.mean([t[1][1] for t in kernel_times]))
    bwd_reduce = float(np.mean([t[1][2] for t in kernel_times]))

    # one build (operand = I_n) outside the timed region, for the record
    binding.set_timing(True)
    u_d = torch.empty((n, n), dtype=torch.float32, device="cuda")
    if restricted_m is None:
        binding.givens_build(th_d, n, U=u_d)
    else:
        binding.givens_build_restricted(th_d, n, restricted_m, U=u_d)
    build_ms = binding.last_timing()[1]
    binding.set_timing(False)
    del u_d

    if args.pmc_copy:
        y_d.copy_(x_d)
        torch.cuda.synchronize()

    fwd_tflops = FWD_FLOP_PER_UPDATE * updates / (fwd_sweep * 1e-3) / 1e12
    bwd_tflops = BWD_FLOP_PER_UPDATE * updates / (bwd_sweep * 1e-3) / 1e12
    result = {
        "metric": "givens_row_pair_column_updates_per_s_fwd_bwd",
        "value": updates / (ms_per_step * 1e-3),
        "unit": "updates/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": name, "n": n, "B": B, "angles": N, "theta": wl.theta_dist,
                   "step": "givens_forward + givens_backward", "kernel_family": families},
        "fwd_updates_per_s": updates / ((fwd_table + fwd_sweep) * 1e-3),
        "fwd_ms": fwd_table + fwd_sweep,
        "bwd_ms": bwd_table + bwd_sweep + bwd_reduce,
        "kernel_ms": {"fwd_table": fwd_table, "fwd_sweep": fwd_sweep, "bwd_table": bwd_table,
                      "bwd_sweep": bwd_sweep, "bwd_reduce": bwd_reduce, "build_sweep": build_ms},
        "roofline": {"kernel": "carousel_forward_kernel", "bound": "alu", "achieved": fwd_tflops,
                     "peak": PEAK_FP32_VECTOR_TFLOPS, "unit": "TFLOP/s",
                     "frac": fwd_tflops / PEAK_FP32_VECTOR_TFLOPS,
                     "traffic": _traffic_from_profiles(f"carousel_forward_{name}")},
        "roofline_bwd": {"kernel": "carousel_backward_kernel", "bound": "alu", "achieved": bwd_tflops,
                         "peak": PEAK_FP32_VECTOR_TFLOPS, "unit": "TFLOP/s",
                         "frac": bwd_tflops / PEAK_FP32_VECTOR_TFLOPS,
                         "traffic": _traffic_from_profiles(f"carousel_backward_{name}")},
    }

    if not args.no_cpu_baseline:
        from oracle import c_oracle
        cols = min(CPU_SAMPLE_COLUMNS, B)
        xs = np.ascontiguousarray(data["X"][:, :cols])
        gs = np.ascontiguousarray(data["G"][:, :cols])
        pairs = c_oracle.schedule(n)
        t0 = time.perf_counter()
        ys = c_oracle.forward(data["theta"], xs, pairs=pairs)
        t_f = time.perf_counter() - t0
        t0 = time.perf_counter()
        c_oracle.reverse_sweep(data["theta"], ys, gs, pairs=pairs, want_x=False)
        t_b = time.perf_counter() - t0
        result["cpu_baseline"] = {
            "value": float(N) * cols / (t_f + t_b), "unit": "updates/s", "cores": c_oracle.num_threads(),
            "kind": "oracle",
            "sample": f"fp64 C oracle, forward + reverse sweep on the first {cols} of {B} columns, n={n}",
            "fwd_s": t_f, "bwd_s": t_b,
        }
        # the paper's own CPU baseline was single-threaded: the same forward on one thread, fewer columns
        one_cols = min(64, cols)
        t0 = time.perf_counter()
        c_oracle.forward(data["theta"], np.ascontiguousarray(xs[:, :one_cols]), pairs=pairs, threads=1)
        t_1 = time.perf_counter() - t0
        result["cpu_baseline"]["fwd_1thread_updates_per_s"] = float(N) * one_cols / t_1
        result["cpu_baseline"]["fwd_1thread_sample"] = f"forward on the first {one_cols} columns, 1 thread"

    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
