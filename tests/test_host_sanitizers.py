"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer: the oracle (oracle/ccq_oracle.c) and the host side
of the library (every source under csrc/, host pass only: validation, layout accounting, the pack routines, launch-shape
logic) are built with -fsanitize=address,undefined and the oracle pin tests and the ABI tests run against those builds
in a child process.  Device code is not instrumented (and not built: the device images are empty stand-ins), so nothing
here launches a kernel."""
import glob
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2507_07145_amd", "csrc")
HIPCC = "/opt/rocm/bin/hipcc"
CLANG = "/opt/rocm/lib/llvm/bin/clang"
SAN_HOST = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]


def _run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert res.returncode == 0, " ".join(cmd[:3]) + "\n" + res.stderr[-3000:]
    return res


def _asan_runtime() -> str:
    path = _run([CLANG, "-print-file-name=libclang_rt.asan-x86_64.so"]).stdout.strip()
    assert os.path.isabs(path) and os.path.exists(path), path
    return path


def test_oracle_and_host_layer_under_asan_and_ubsan(tmp_path):
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "*.cpp")))
    objs = [str(tmp_path / (os.path.basename(s) + ".o")) for s in srcs]

    def compile_one(pair):
        src, obj = pair
        _run([HIPCC, "--cuda-host-only", "-O1", "-g", "-std=c++17", "-fPIC", *SAN_HOST, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
              "-c", src, "-o", obj])

    with ThreadPoolExecutor(max_workers=8) as pool:
        list(pool.map(compile_one, zip(srcs, objs)))
    # the host pass refers to the device image of every source; there is none in this build
    undefined = _run(["nm", "-u", *objs]).stdout
    images = sorted(set(re.findall(r"__hip_fatbin_[0-9a-f]+", undefined)))
    stub = tmp_path / "device_images.c"
    stub.write_text("".join(f"const char {name}[64] __attribute__((aligned(4096))) = {{0}};\n" for name in images))
    _run(["gcc", "-c", "-fPIC", str(stub), "-o", str(tmp_path / "device_images.o")])
    lib = tmp_path / "libccq_san.so"
    _run([HIPCC, "--cuda-host-only", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined", "-shared-libasan", "-o", str(lib), *objs,
          str(tmp_path / "device_images.o")])
    oracle = tmp_path / "libccq_oracle_san.so"
    _run([CLANG, "-O1", "-g", "-std=c11", "-fopenmp=libgomp", "-fPIC", "-shared", "-ffp-contract=off", "-fsanitize=address,undefined",
          "-fno-sanitize-recover=undefined", "-shared-libasan", "-o", str(oracle), os.path.join(ROOT, "oracle", "ccq_oracle.c"), "-lm"])
    for built in (lib, oracle):
        assert "__asan_init" in _run(["nm", "-D", str(built)]).stdout, f"{built} is not instrumented"

    env = dict(os.environ)
    env.update({"LD_PRELOAD": _asan_runtime(), "ASAN_OPTIONS": "detect_leaks=0:halt_on_error=1",
                "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1", "CCQ_LIBRARY": str(lib), "CCQ_ORACLE_LIBRARY": str(oracle)})
    tests = ["test_host_abi.py", "test_oracle_pins.py", "test_oracle_encoder.py", "test_oracle_scale_compression.py", "test_oracle_hybrid_word.py"]
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *[os.path.join(ROOT, "tests", t) for t in tests]],
                         capture_output=True, text=True, env=env, cwd=ROOT)
    tail = (res.stdout + res.stderr)[-4000:]
    assert res.returncode == 0, tail
    assert "AddressSanitizer" not in tail and "runtime error" not in tail, tail
    assert re.search(r"\b\d+ passed", res.stdout), tail
