"""Builds libccq.so (the C-ABI library: HIP kernels for gfx950 + host layer) in-tree with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libccq.so")
ARCH = "gfx950"


def sources() -> list[str]:
    src = os.path.join(HERE, "csrc")
    return sorted(glob.glob(os.path.join(src, "*.hip")) + glob.glob(os.path.join(src, "*.cpp")))


def build_lib(verbose: bool = False) -> str:
    """Compile every source under csrc/ into paper_2507_07145_amd/libccq.so."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-O3", f"--offload-arch={ARCH}", "-std=c++17",
           # keep the compiler from forming packed fp32 instructions
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-shared", "-fPIC", "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
           "-o", LIB] + sources()
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print("\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libccq.so")
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
