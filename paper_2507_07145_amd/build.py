"""Builds libccq.so (the C-ABI library: HIP kernels for gfx950 + host layer) in-tree with hipcc.

Every source under csrc/ is compiled to an object file of its own (in parallel) and the objects are linked
into paper_2507_07145_amd/libccq.so.  `python -m paper_2507_07145_amd.build --incremental` recompiles only the
sources that are newer than their objects (headers count for every source).
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libccq.so")
OBJ_DIR = os.path.join(HERE, "_build")
ARCH = "gfx950"


def sources() -> list[str]:
    src = os.path.join(HERE, "csrc")
    return sorted(glob.glob(os.path.join(src, "*.hip")) + glob.glob(os.path.join(src, "*.cpp")))


def headers() -> list[str]:
    return sorted(glob.glob(os.path.join(HERE, "csrc", "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h")))


def compile_flags() -> list[str]:
    return ["-O3", f"--offload-arch={ARCH}", "-std=c++17",
            # keep the compiler from forming packed fp32 instructions
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-fPIC", "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc")]


def _run(cmd: list[str], verbose: bool) -> None:
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print("\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd[-3:]))


def build_lib(verbose: bool = False, incremental: bool = False) -> str:
    """Compile every source under csrc/ and link paper_2507_07145_amd/libccq.so."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    newest_header = max(os.path.getmtime(h) for h in headers())
    jobs = []
    objs = []
    for s in sources():
        obj = os.path.join(OBJ_DIR, os.path.basename(s) + ".o")
        objs.append(obj)
        stale = not os.path.exists(obj) or os.path.getmtime(obj) < max(os.path.getmtime(s), newest_header)
        if stale or not incremental:
            jobs.append([hipcc] + compile_flags() + ["-c", s, "-o", obj])
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as pool:
        list(pool.map(lambda c: _run(c, verbose), jobs))
    _run([hipcc, f"--offload-arch={ARCH}", "-shared", "-fPIC", "-o", LIB] + objs, verbose)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose="-v" in sys.argv, incremental="--incremental" in sys.argv))
