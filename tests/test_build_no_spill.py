"""Build guard: no kernel of the library may spill registers to scratch memory (kernels that did
produced wrong results on the device in some launch shapes), and no packed-fp32
vector instruction may appear in the generated code."""
import glob
import os
import re
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2507_07145_amd", "csrc")


def _compile(src, *extra):
    cmd = ["/opt/rocm/bin/hipcc", "-O3", "--offload-arch=gfx950", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "--cuda-device-only", "-I", os.path.join(ROOT, "include"), "-I", CSRC, *extra, src]
    return subprocess.run(cmd, capture_output=True, text=True)


def _check_source(args):
    src, out = args
    res = _compile(src, "-S", "-o", str(out), "-Rpass-analysis=kernel-resource-usage")
    assert res.returncode == 0, res.stderr[-2000:]
    names = re.findall(r"Function Name: (\S+)", res.stderr)
    scratch = [int(v) for v in re.findall(r"ScratchSize \[bytes/lane\]: (\d+)", res.stderr)]
    assert names and len(names) == len(scratch), os.path.basename(src)
    spilling = [n for n, sz in zip(names, scratch) if sz != 0]
    assert not spilling, f"{os.path.basename(src)}: kernels using scratch: {spilling}"
    asm = open(out).read()
    assert "s_endpgm" in asm
    assert not re.search(r"\bv_pk_(add|mul|fma)_f32\b", asm)
    return len(names)


def test_no_spills_and_no_packed_fp32(tmp_path):
    """One device-only compile per source that holds kernels: the resource remarks give the scratch size of every kernel,
    the assembly is searched for packed-fp32 instructions."""
    from concurrent.futures import ThreadPoolExecutor
    srcs = [s for s in sorted(glob.glob(os.path.join(CSRC, "*.hip"))) if "__global__" in open(s).read()]
    assert len(srcs) >= 5
    with ThreadPoolExecutor(max_workers=6) as pool:
        counts = list(pool.map(_check_source, [(s, tmp_path / (os.path.basename(s) + ".s")) for s in srcs]))
    assert all(c > 0 for c in counts)
