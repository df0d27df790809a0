"""Builds the HIP library in-tree: paper_2106_00003_amd/libgivens_rr.so (gfx950 only).

Every .hip file under csrc/ is one translation unit; they are compiled in parallel into _build/ and
linked into one shared library.  The carousel kernels are spread over one unit per rotation form
and sweep direction because their many template instances dominate the compile time.
"""
from __future__ import annotations

import concurrent.futures
import glob
import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libgivens_rr.so")

# Packed-FP32 VALU forms are switched off for every translation unit of this library.
HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


# translation units in the order of their compile times (measured; the rest take under 45 s each)
SLOWEST_FIRST = ("carousel_bwd_m4", "carousel_bwd_m8", "carousel_fwd_m8", "carousel_fwd_m8_large", "carousel_bwd_m7",
                 "carousel_fwd_m7", "carousel_fwd_m4", "carousel_bwd_m5")


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + res.stdout + res.stderr)
    return res


def build_library(verbose: bool = False, extra_flags=(), jobs: int | None = None, only=()) -> str:
    """Compiles every translation unit and links the library.  `only` (names without the suffix) restricts
    the compile step to those units and links them with the other units' existing objects."""
    hipcc = hipcc_path()
    sources = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    if not sources:
        raise RuntimeError(f"no sources under {CSRC}")
    os.makedirs(OBJ, exist_ok=True)
    objects = [os.path.join(OBJ, os.path.basename(s)[:-4] + ".o") for s in sources]
    todo = [(s, o) for s, o in zip(sources, objects)
            if not only or os.path.basename(s)[:-4] in only or not os.path.exists(o)]
    # the units that take longest start first, so that none of them is left running alone at the end
    todo.sort(key=lambda so: SLOWEST_FIRST.index(os.path.basename(so[0])[:-4])
              if os.path.basename(so[0])[:-4] in SLOWEST_FIRST else len(SLOWEST_FIRST))
    jobs = jobs or max(1, min(len(sources), os.cpu_count() or 1, 16))
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
        futures = [pool.submit(_run, [hipcc, *HIPCC_FLAGS, *extra_flags, "-c", src, "-o", obj], verbose)
                   for src, obj in todo]
        for f in futures:
            f.result()
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objects], verbose)
    return LIB


if __name__ == "__main__":
    import sys
    print(build_library(verbose=True, only=tuple(sys.argv[1:])))
