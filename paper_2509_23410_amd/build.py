"""Build step: compile csrc/*.hip into the in-tree C-ABI shared library for gfx950."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpatch_hip.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
    # never let the compiler emit packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out:
        print(out)


def build_lib(verbose: bool = False, extra_flags=()) -> str:
    """Compile every source (each to an object of its own, side by side) and link the shared library."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    jobs = []
    for src in sources():
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        jobs.append((obj, [hipcc, *flags, *extra_flags, "-c", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", obj, src]))
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as pool:
        list(pool.map(lambda j: _run(j[1], verbose), jobs))
    _run([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *[j[0] for j in jobs]], verbose)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
    sys.exit(0)


def device_asm(source: str, out_path: str) -> str:
    """gfx950 assembly of one source file (what the compiler generated around the inline asm), for checks."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *[f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC")], "-S", "--cuda-device-only", "-I",
           os.path.join(ROOT, "include"), "-I", CSRC, "-o", out_path, os.path.join(CSRC, source)]
    subprocess.run(cmd, check=True, capture_output=True)
    return out_path
