"""Compile the HIP library for gfx950 in-tree (``liblean_attn.so`` next to this file).

The decode kernels are compiled as six translation units (core family x dtype, ``csrc/lean_kernels.hip``
with two defines) next to the host side (``csrc/lean_attn.hip``), in parallel, and linked into one
shared library.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
SOURCE = os.path.join(CSRC, "lean_attn.hip")
KERNELS = os.path.join(CSRC, "lean_kernels.hip")
LIBRARY = os.path.join(_HERE, "liblean_attn.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]
_NOISE = "is not a recognized feature for this target"


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    log = "\n".join(line for line in proc.stdout.splitlines() if _NOISE not in line)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed ({proc.returncode}): {' '.join(cmd)}\n{log}")
    if verbose and log.strip():
        print(log, flush=True)


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    jobs = max(1, min(7, int(os.environ.get("MAX_JOBS", os.cpu_count() or 1))))
    work = tempfile.mkdtemp(prefix="lean_attn_build_")
    try:
        units = [(SOURCE, os.path.join(work, "lean_attn.o"), [])]
        for family in (0, 1, 2):
            for dt in (0, 1):
                units.append((KERNELS, os.path.join(work, f"lean_kernels_{family}_{dt}.o"),
                              [f"-DLEAN_TU_FAMILY={family}", f"-DLEAN_TU_DT={dt}"]))
        # the heaviest units (MFMA cores) first
        units.sort(key=lambda u: (0 if "FAMILY=1" in " ".join(u[2]) else 1 if "FAMILY=2" in " ".join(u[2]) else 2))
        with ThreadPoolExecutor(max_workers=jobs) as pool:
            list(pool.map(lambda u: _run([hipcc, *HIPCC_FLAGS, *u[2], "-c", "-o", u[1], u[0]], verbose), units))
        tmp = LIBRARY + f".tmp{os.getpid()}"
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *[u[1] for u in units]], verbose)
        os.replace(tmp, LIBRARY)
    finally:
        shutil.rmtree(work, ignore_errors=True)
    return LIBRARY


if __name__ == "__main__":
    print(build(verbose=True))
