"""Builds libadaptra.so (gfx950) in-tree with hipcc.  Cross-compiles without a GPU."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
KERNEL_SIZES = (2, 4, 8, 12, 16, 24, 32, 48, 64)       # one translation unit per size of the on-chip kernels
SOURCES = [os.path.join(_HERE, "csrc", name)
           for name in ("adaptra.hip", "adaptra_zb.hip", "adaptra_search.hip", "adaptra_probe.hip",
                        *(f"adaptra_size_{n}.hip" for n in sorted(KERNEL_SIZES, reverse=True)))]
INCLUDE = os.path.join(ROOT, "include")
LIB = os.path.join(_HERE, "libadaptra.so")
OBJ_DIR = os.path.join(_HERE, "_build")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # No packed-FP32 instructions in device code (the device pass honours this: a float2
    # multiply-add compiles to v_pk_fma_f32 without it and to two v_fma_f32 with it; the path
    # itself is all int32).  The host pass does not know the feature and says so once per
    # function it compiles -- harmless.
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-Wno-int-to-pointer-cast",     # LDS addresses are 32-bit integers on purpose (address space 3)
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass's note about the device-only target feature is dropped, everything else shown
    out = "\n".join(l for l in p.stdout.splitlines() if "'-packed-fp32-ops' is not a recognized feature" not in l)
    if out.strip():
        print(out, flush=True)
    if p.returncode != 0:
        raise subprocess.CalledProcessError(p.returncode, cmd)


def build_library(verbose: bool = False, extra_flags=()) -> str:
    """Compiles every source (one hipcc per file, side by side), then links the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    objects = [os.path.join(OBJ_DIR, os.path.basename(s) + f".{os.getpid()}.o") for s in SOURCES]
    tmp = LIB + f".tmp{os.getpid()}"
    try:
        with ThreadPoolExecutor(max_workers=min(os.cpu_count() or 4, 8, len(SOURCES))) as pool:
            jobs = [pool.submit(_run, [hipcc, *HIPCC_FLAGS, *extra_flags, "-I", INCLUDE, "-c", s, "-o", o], verbose)
                    for s, o in zip(SOURCES, objects)]
            for j in jobs:
                j.result()
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objects, "-o", tmp], verbose)
        os.replace(tmp, LIB)
    finally:
        for o in objects + [tmp]:
            if os.path.exists(o):
                os.remove(o)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
