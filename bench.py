#!/usr/bin/env python3
"""Benchmark of the round-robin Givens hot path on one MI355X.

One "step" = one forward (coefficient tables + Algorithm-2 sweep, Y = U(theta) X, or U itself for the
workload whose operand is I_n) and one backward (tables + reverse sweep + dtheta reduction, giving dtheta
and, unless the operand is I_n, dX), all inputs resident in HBM before the timed region.  `value` is Givens
row-pair column updates per second over the whole step: N * B / (time of one step), N = n(n-1)/2 (one
"update" = one rotation applied to one column in the forward pass; the backward pass does two rotations and
one two-term product per update).

Default workload: n = 4096, B = 4096, fp32, theta ~ N(0, 0.1^2), X, G ~ N(0, 1) (--workload 4).  The other
workloads of the parity tests can be timed with --workload 1|2|3|5; --theta uniform draws the default
workload's angles from U[-pi, pi) instead (general angles: the three-FMA rotation form) and --form standard
switches the device-side choice of the rotation form off; --prepared times givens_prepare +
givens_forward_prepared + givens_backward_prepared instead of the plain calls.

Prints ONE JSON line.  Besides the contract fields it carries
  roofline      forward sweep kernel against the vector-FP32 peak (6 flop per update); `frac_with_tables`
                counts the coefficient kernels of the forward call into the time
  roofline_bwd  reverse sweep kernel(s) against the same peak (16 flop per update over the columns they sweep)
  roofline_gram the Gram-matrix contraction against the dense float32 MFMA peak, when the backward call used it
  cpu_baseline  the fp64 C oracle (oracle/givens_oracle.c) timed on the host cores on a bounded sample of
                the same workload's columns
Kernel durations come from HIP events that the library records on the launch stream around each group of
kernels (givens_set_timing), during the timed steps themselves.
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
PEAK_FP64_VECTOR_TFLOPS = 78.6       # same for FP64
PEAK_FP32_MFMA_TFLOPS = 157.3        # dense float32 MFMA peak
FWD_FLOP_PER_UPDATE = 6              # 4 mul + 2 add (Algorithm 1's two row updates)
BWD_FLOP_PER_UPDATE = 16             # two transposed rotations (12) + two-term product and sum (4)
CPU_SAMPLE_UPDATES = 4.0e10          # the oracle's sample: about this many (pair, column) updates forward


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
    """Forward + backward of the unitary extension on synthetic complex64 data (carousel family where the shape
    allows it, LDS strip kernels otherwise or with --family lds)."""
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

    binding.set_kernel({"auto": binding.KERNEL_AUTO, "lds": binding.KERNEL_LDS,
                        "carousel": binding.KERNEL_CAROUSEL}[args.family])
    binding.set_timing(True)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    times = [step() for _ in range(args.steps)]
    torch.cuda.synchronize()
    ms = 1e3 * (time.perf_counter() - t0) / args.steps
    binding.set_timing(False)
    family = {binding.KERNEL_LDS: "lds", binding.KERNEL_CAROUSEL: "carousel"}.get(binding.last_kernel(), "?")
    # 9 FMA per (pair, complex column) forward and 26 in the reverse sweep in the carousel family
    fwd_sweep = float(np.mean([t[0][1] for t in times]))
    bwd_sweep = float(np.mean([t[1][1] for t in times]))
    print(json.dumps({
        "metric": "unitary_row_pair_complex_column_updates_per_s_fwd_bwd", "value": float(N) * B / (ms * 1e-3),
        "unit": "updates/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "dtype": "c64", "data": "synthetic",
        "config": {"workload": f"unitary_n{n}_B{B}_c64", "n": n, "B": B, "angles": 2 * N,
                   "kernel_family": family},
        "kernel_ms": {"fwd_table": float(np.mean([t[0][0] for t in times])),
                      "fwd_sweep": fwd_sweep,
                      "bwd_table": float(np.mean([t[1][0] for t in times])),
                      "bwd_sweep": bwd_sweep,
                      "bwd_reduce": float(np.mean([t[1][2] for t in times]))},
        "executed_tflops": {"fwd_sweep": 18.0 * N * B / (fwd_sweep * 1e-3) / 1e12,
                            "bwd_sweep": 52.0 * N * B / (bwd_sweep * 1e-3) / 1e12} if family == "carousel" else None}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--settle", type=int, default=25,
                    help="untimed steps before the warm-up steps, so that a short --warmup still times the steady state")
    ap.add_argument("--warmup", type=int, default=30,
                    help="untimed steps first (the shader clock and the caches need some tens of launches to settle)")
    ap.add_argument("--workload", type=int, default=4, choices=[1, 2, 3, 4, 5],
                    help="benchmark workload id (default 4: n=4096, B=4096)")
    ap.add_argument("--theta", type=str, default=None, choices=["uniform", "normal0.1"],
                    help="draw the workload's angles from this distribution instead of its own")
    ap.add_argument("--form", type=str, default="auto", choices=["auto", "standard", "lifted"],
                    help="rotation form of the float carousel kernels (auto: chosen on the device from max |theta|)")
    ap.add_argument("--reduction", type=str, default="auto", choices=["auto", "two_stage", "gram"])
    ap.add_argument("--prepared", nargs="?", const="step", default=None, choices=["step", "frozen"],
                    help="float32 only. step: a step is givens_prepare + givens_forward_prepared + "
                         "givens_backward_prepared (angles change every step, as in training). frozen: the token is "
                         "prepared once before the warmup and a step is the two prepared calls (angles fixed)")
    ap.add_argument("--restricted", type=str, default=None, metavar="ROWS,M",
                    help="time the restricted entry points instead: ROWS coordinates (may be odd), pairs (i, j) "
                         "with i < M free, the chosen workload's B and angle distribution; not the headline metric")
    ap.add_argument("--unitary", type=str, default=None, metavar="N,B",
                    help="time the unitary (complex) entry points on an N x B complex64 operand instead and print a "
                         "short JSON line; not the headline metric")
    ap.add_argument("--enqueue-only", action="store_true",
                    help="time the steps with the library's per-kernel event timing switched off, so that the host "
                         "only enqueues (no wait between calls); the per-kernel figures then come from a second, "
                         "untimed pass of at most 20 steps.  For the small workloads, where the host's wait after "
                         "every call is a visible part of the step")
    ap.add_argument("--graph", action="store_true",
                    help="record one step into a HIP graph after the warm-up and time replays of it (the launch-bound "
                         "small workloads); implies --enqueue-only for the per-kernel figures")
    ap.add_argument("--build", type=int, default=None, metavar="N",
                    help="the paper's own experiment at size N: build U(theta) from N(N-1)/2 uniform random angles "
                         "(givens_build) and take the gradient of a loss on U (dtheta-only givens_backward with a "
                         "random N x N upstream gradient); workload 3 is this at N = 1024; not the headline metric")
    ap.add_argument("--family", type=str, default="auto", choices=["auto", "lds", "carousel"],
                    help="with --unitary: kernel family")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-copy", action="store_true",
                    help="after the steps, run one plain device copy of G into a scratch tensor (n*B*4 bytes read "
                         "and written) so that a rocprofv3 --pmc run has a kernel of known traffic to scale by")
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
    binding.set_rotation_form({"auto": binding.FORM_AUTO, "standard": binding.FORM_STANDARD,
                               "lifted": binding.FORM_LIFTED}[args.form])
    binding.set_reduction({"auto": binding.REDUCTION_AUTO, "two_stage": binding.REDUCTION_TWO_STAGE,
                           "gram": binding.REDUCTION_GRAM}[args.reduction])

    if args.unitary:
        return _bench_unitary(args, binding, torch, np)
    if args.graph:
        # graphs are recorded on a stream other than the null stream (default priority); the whole run uses it, so
        # that the workspace and any prepared coefficients belong to it
        side = torch.cuda.Stream()
        torch.cuda.set_stream(side)

    wl = inputs.WORKLOADS[args.workload]
    if args.build:
        wl = inputs.Workload(3, args.build, args.build, "f32", "uniform", True)
    n, B = wl.n, wl.B
    name = wl.name if not args.build else f"build_n{n}_f32"
    theta_dist = args.theta or wl.theta_dist
    restricted_m = None
    if args.restricted:
        n, restricted_m = (int(v) for v in args.restricted.split(","))
        data = inputs.make_restricted(n, restricted_m, B, seed=inputs.BASE_SEED + 100 + args.workload,
                                      theta_dist=theta_dist)
        name = f"restricted_n{n}_m{restricted_m}_B{B}_f32"
        args.no_cpu_baseline = True
    elif args.build:
        data = inputs.make_custom(n, n, seed=inputs.BASE_SEED + 200 + (n % 997), theta_dist=theta_dist)
        args.no_cpu_baseline = args.no_cpu_baseline or n > 2048
    else:
        data = inputs.make_inputs(args.workload)
        if theta_dist != wl.theta_dist:
            rng = np.random.default_rng(inputs.BASE_SEED + 50 + args.workload)
            data["theta"] = inputs.draw_theta(rng, wl.num_angles, theta_dist, wl.np_dtype)
            name += "_theta_" + theta_dist
    if args.form != "auto":
        name += "_form_" + args.form
    identity = wl.x_identity and restricted_m is None
    N = int(data["theta"].size)
    th_d = torch.from_numpy(data["theta"]).cuda()
    x_d = None if identity else torch.from_numpy(data["X"]).cuda()
    g_d = torch.from_numpy(data["G"]).cuda()
    y_d = torch.empty_like(g_d)
    dx_d = None if identity else torch.empty_like(g_d)
    dth_d = torch.empty_like(th_d)
    prepared = args.prepared if wl.dtype == "f32" else None
    directions = binding.PREPARE_FORWARD | (binding.PREPARE_BACKWARD_WIDE if B >= 2 * n else binding.PREPARE_BACKWARD)
    frozen_token = binding.givens_prepare(th_d, n, restricted_m, directions, batch=B) if prepared == "frozen" else None

    timing_on = [True]
    zeros = (0.0, 0.0, 0.0, 0.0)
    last_timing = lambda: binding.last_timing() if timing_on[0] else zeros  # noqa: E731

    def step():
        if prepared:
            if frozen_token is None:
                token = binding.givens_prepare(th_d, n, restricted_m, directions, batch=B)
                t_p = last_timing()
            else:
                token, t_p = frozen_token, (0.0, 0.0, 0.0, 0.0)
            if identity:
                binding.givens_build_prepared(token, n, th_d.device, U=y_d)
            else:
                binding.givens_forward_prepared(token, x_d, Y=y_d)
            t_f = last_timing()
            binding.givens_backward_prepared(token, y_d, g_d, N, dX=dx_d, dtheta=dth_d, want_dx=not identity)
            t_b = last_timing()
            return (t_p[0] + t_f[0], t_f[1], 0.0, 0.0), t_b
        if restricted_m is not None:
            binding.givens_forward_restricted(th_d, x_d, restricted_m, Y=y_d)
            t_f = last_timing()
            binding.givens_backward_restricted(th_d, y_d, g_d, restricted_m, dX=dx_d, dtheta=dth_d)
            return t_f, last_timing()
        if identity:
            binding.givens_build(th_d, n, U=y_d)
        else:
            binding.givens_forward(th_d, x_d, Y=y_d)
        t_f = last_timing()
        binding.givens_backward(th_d, y_d, g_d, dX=dx_d, dtheta=dth_d, want_dx=not identity)
        return t_f, last_timing()

    args.enqueue_only = args.enqueue_only or args.graph
    timing_on[0] = not args.enqueue_only
    binding.set_timing(timing_on[0])
    # the shader clock and the caches take some 25 launches to reach their steady state; a short --warmup would time
    # that ramp instead of the kernels, so the same untimed steps run first whatever --warmup says (reported as
    # config.settle_steps)
    for _ in range(args.settle + args.warmup):
        step()
    torch.cuda.synchronize()
    if args.graph:
        # the stream's workspace is warm, so a step allocates nothing: record it and replay it
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        for _ in range(3):
            graph.replay()
        side.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        side.synchronize()
        elapsed = time.perf_counter() - t0
        kernel_times = []
    else:
        t0 = time.perf_counter()
        kernel_times = [step() for _ in range(args.steps)]
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    if args.enqueue_only:
        timing_on[0] = True
        binding.set_timing(True)
        kernel_times = [step() for _ in range(min(args.steps, 20))]
        torch.cuda.synchronize()
    binding.set_timing(False)
    family = binding.last_kernel()
    form = binding.last_rotation_form() if wl.dtype == "f32" else binding.FORM_STANDARD
    reduction = binding.last_reduction()

    if args.pmc_copy:
        scratch = torch.empty_like(g_d)
        scratch.copy_(g_d)
        torch.cuda.synchronize()
        del scratch

    ms_per_step = 1e3 * elapsed / args.steps
    updates = float(N) * float(B)
    mean = lambda which, slot: float(np.mean([t[which][slot] for t in kernel_times]))  # noqa: E731
    fwd_table, fwd_sweep = mean(0, 0), mean(0, 1)
    bwd_table, bwd_sweep, bwd_reduce, bwd_gram = mean(1, 0), mean(1, 1), mean(1, 2), mean(1, 3)
    peak = PEAK_FP64_VECTOR_TFLOPS if wl.dtype == "f64" else PEAK_FP32_VECTOR_TFLOPS
    family_name = {binding.KERNEL_LDS: "lds", binding.KERNEL_CAROUSEL: "carousel", binding.KERNEL_COLUMN: "column"}[family]
    fwd_kernel = {"lds": "lds_forward_kernel", "carousel": "carousel_forward_kernel",
                  "column": "column_forward_kernel"}[family_name]
    chains = binding.last_chains() if family_name == "carousel" and wl.dtype == "f32" else 0
    bwd_kernel = ("lds_backward_kernel" if family_name == "lds"
                  else "carousel_backward_chain_kernel" if chains else "carousel_backward_kernel")

    fwd_tflops = FWD_FLOP_PER_UPDATE * updates / (fwd_sweep * 1e-3) / 1e12
    gram = reduction == binding.REDUCTION_GRAM
    if gram:
        # the sweeps of the Gram form: the reverse sweep over the n columns of C = Y G^T (16 flop per update) and,
        # when dX is wanted, a forward-type sweep over the B columns of G (6 flop per update)
        bwd_flops = BWD_FLOP_PER_UPDATE * float(N) * n + (0 if identity else FWD_FLOP_PER_UPDATE * updates)
    else:
        bwd_flops = BWD_FLOP_PER_UPDATE * updates
    bwd_tflops = bwd_flops / (bwd_sweep * 1e-3) / 1e12
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
        "dtype": wl.dtype,
        "data": "synthetic",
        "config": {"workload": name, "n": n, "B": B, "angles": N, "theta": theta_dist,
                   "settle_steps": args.settle,
                   "step": ("givens_prepare + givens_forward_prepared + givens_backward_prepared" if prepared == "step"
                            else "givens_forward_prepared + givens_backward_prepared (token prepared once)"
                            if prepared == "frozen"
                            else ("givens_build" if identity else "givens_forward") + " + givens_backward"),
                   "host": ("replays a HIP graph of one step; kernel_ms from a second, eager pass" if args.graph
                            else "enqueues only; kernel_ms from a second pass" if args.enqueue_only
                            else "waits for each call's timing events"),
                   "kernel_family": family_name,
                   "rotation_form": {binding.FORM_STANDARD: "standard", binding.FORM_SCALED: "scaled",
                                     binding.FORM_LIFTED: "lifted"}[form],
                   "reduction": {binding.REDUCTION_TWO_STAGE: "two_stage", binding.REDUCTION_GRAM: "gram"}[reduction]},
        "fwd_updates_per_s": updates / ((fwd_table + fwd_sweep) * 1e-3),
        "fwd_ms": fwd_table + fwd_sweep,
        "bwd_ms": bwd_table + bwd_sweep + bwd_reduce + bwd_gram,
        "kernel_ms": {"fwd_table": fwd_table, "fwd_sweep": fwd_sweep, "bwd_table": bwd_table,
                      "bwd_sweep": bwd_sweep, "bwd_reduce": bwd_reduce, "bwd_gram": bwd_gram},
        "roofline": {"kernel": fwd_kernel, "bound": "alu", "achieved": fwd_tflops,
                     "peak": peak, "unit": "TFLOP/s", "frac": fwd_tflops / peak,
                     "frac_with_tables": FWD_FLOP_PER_UPDATE * updates / ((fwd_table + fwd_sweep) * 1e-3) / 1e12 / peak,
                     "traffic": _traffic_from_profiles(f"{fwd_kernel.replace('_kernel', '')}_{name}")},
        "roofline_bwd": {"kernel": bwd_kernel + (" (on C = Y G^T) + " + fwd_kernel + " (dX)" if gram and not identity
                                                 else (" (on C = Y G^T)" if gram else "")),
                         "bound": "alu", "achieved": bwd_tflops, "peak": peak, "unit": "TFLOP/s",
                         "frac": bwd_tflops / peak,
                         "traffic": _traffic_from_profiles(
                             f"{bwd_kernel.replace('_chain', '').replace('_kernel', '')}_{name}")},
    }
    if gram and bwd_gram > 0:
        gram_tflops = 2.0 * n * n * B / (bwd_gram * 1e-3) / 1e12
        result["roofline_gram"] = {"kernel": "gram_tile_kernel", "bound": "mfma", "achieved": gram_tflops,
                                   "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                                   "frac": gram_tflops / PEAK_FP32_MFMA_TFLOPS,
                                   "traffic": _traffic_from_profiles(f"gram_tile_{name}")}

    if not args.no_cpu_baseline:
        from oracle import c_oracle
        cols = int(max(1, min(B, CPU_SAMPLE_UPDATES // N)))
        pairs = c_oracle.schedule(n)
        gs = np.ascontiguousarray(data["G"][:, :cols])
        t0 = time.perf_counter()
        if identity:
            ys = c_oracle.forward(data["theta"], None, n=n, pairs=pairs)[:, :cols]
            t_f = (time.perf_counter() - t0) * cols / n     # the oracle builds all n columns of U
        else:
            ys = c_oracle.forward(data["theta"], np.ascontiguousarray(data["X"][:, :cols]), pairs=pairs)
            t_f = time.perf_counter() - t0
        t0 = time.perf_counter()
        c_oracle.reverse_sweep(data["theta"], np.ascontiguousarray(ys), gs, pairs=pairs, want_x=False)
        t_b = time.perf_counter() - t0
        result["cpu_baseline"] = {
            "value": float(N) * cols / (t_f + t_b), "unit": "updates/s", "cores": c_oracle.num_threads(),
            "kind": "oracle",
            "sample": f"fp64 C oracle, forward + reverse sweep on the first {cols} of {B} columns, n={n}",
            "fwd_s": t_f, "bwd_s": t_b,
        }
        # the paper's own CPU baseline was single-threaded: the same forward on one thread, fewer columns
        if not identity:
            one_cols = min(64, cols)
            t0 = time.perf_counter()
            c_oracle.forward(data["theta"], np.ascontiguousarray(data["X"][:, :one_cols]), pairs=pairs, threads=1)
            t_1 = time.perf_counter() - t0
            result["cpu_baseline"]["fwd_1thread_updates_per_s"] = float(N) * one_cols / t_1
            result["cpu_baseline"]["fwd_1thread_sample"] = f"forward on the first {one_cols} columns, 1 thread"

    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
