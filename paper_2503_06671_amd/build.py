"""Build libesc_convattn.so for gfx950 with hipcc (cross-compiles without a GPU).

The forward kernel is instantiated once per large-kernel size in a translation unit of
its own (esc_variants.hip with -DESC_KS=<Ks>), so the units compile in parallel; the
host side and the C ABI are esc_api.hip.
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(CSRC, "_build")
LIB = os.path.join(CSRC, "libesc_convattn.so")

KERNEL_SIZES = (0,) + tuple(range(1, 32, 2))

# packed-fp32 instructions are switched off on purpose: some of their forms have
# produced silently wrong results on the target machines.  The compiler's wavefront-level
# rewrite of atomics is switched off too: it reads the atomic's result back at once, and
# the kernel issues its one returning atomic per block early precisely so as not to wait.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
    "-ffp-contract=off", "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _units(extra_sources=()):
    units = [(os.path.join(CSRC, "esc_api.hip"), [], "esc_api.o")]
    for ks in KERNEL_SIZES:
        units.append((os.path.join(CSRC, "esc_variants.hip"), [f"-DESC_KS={ks}"], f"esc_variants_ks{ks}.o"))
    for src in extra_sources:
        units.append((src, [], os.path.splitext(os.path.basename(src))[0] + ".o"))
    return units


def build(verbose: bool = False, extra=(), jobs: int | None = None) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    extra_sources = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC))
                     if f.endswith(".hip") and f not in ("esc_api.hip", "esc_variants.hip")]
    jobs = jobs or min(8, os.cpu_count() or 1)

    def compile_one(unit):
        src, defs, obj = unit
        cmd = [hipcc, *HIPCC_FLAGS, *extra, *defs, "-c", "-o", os.path.join(OBJ_DIR, obj), src]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return os.path.join(OBJ_DIR, obj)

    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(compile_one, _units(extra_sources)))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
