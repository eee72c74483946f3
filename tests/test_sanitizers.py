"""The CPU side under AddressSanitizer and UndefinedBehaviorSanitizer.

The oracle (plain C) and the host code of the C-ABI library (argument validation, index polynomials,
grid sizing -- everything that runs before a kernel is launched) are rebuilt with
``-fsanitize=address,undefined`` by the clang that hipcc drives (device code is left alone), and the oracle's
pins and the host-side ABI tests run against those builds in a child interpreter that has the sanitizer
runtime preloaded.  Any report (heap overflow, signed overflow, misaligned access, ...) aborts the child
and fails this test.  No GPU is involved: the host tests make no compute calls.
"""
import glob
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2407_13726_amd", "csrc")
CLANG = "/opt/rocm/llvm/bin/clang"
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-shared-libasan", "-g", "-O1", "-fPIC"]

CHILD = r"""
import sys
sys.path.insert(0, {root!r})
import oracle
from paper_2407_13726_amd import dastac
oracle._LIB = {olib!r}
dastac.LIB_PATH = {hlib!r}
import pytest
sys.exit(pytest.main(["-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu",
                      {root!r} + "/tests/test_oracle_pins.py", {root!r} + "/tests/test_index_host.py"]))
"""


@pytest.mark.skipif(shutil.which("hipcc") is None or not os.path.exists(CLANG), reason="needs the ROCm compilers")
def test_oracle_pins_and_host_abi_under_asan_and_ubsan(tmp_path):
    runtime = subprocess.check_output([CLANG, "-print-file-name=libclang_rt.asan-x86_64.so"], text=True).strip()
    assert os.path.exists(runtime), runtime
    olib = str(tmp_path / "liboracle_san.so")
    subprocess.check_call([CLANG, "-std=c11", *SAN, "-shared", "-Wall", "-o", olib,
                           os.path.join(ROOT, "oracle", "dastac_oracle.c"), "-lm"])

    def compile_host_sanitized(src):
        obj = str(tmp_path / (os.path.basename(src)[:-4] + ".o"))
        subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-std=c++17", "-Wno-unused-function", "-w",
                               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                               "-fno-gpu-sanitize", *SAN, "-c", src, "-o", obj])
        return obj

    with ThreadPoolExecutor(8) as pool:
        objs = list(pool.map(compile_host_sanitized, sorted(glob.glob(os.path.join(CSRC, "*.hip")))))
    hlib = str(tmp_path / "libdastac_hip_san.so")
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-sanitize",
                           "-fsanitize=address,undefined", "-shared-libasan", "-o", hlib, *objs])

    env = dict(os.environ)
    # the sanitizer runtime has to be the first library of the process; whatever is preloaded already stays
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # the interpreter itself is not instrumented: its allocations are not this test's business
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    child = subprocess.run([sys.executable, "-c", CHILD.format(root=ROOT, olib=olib, hlib=hlib)], env=env,
                           capture_output=True, text=True, timeout=900)
    tail = (child.stdout + child.stderr)[-4000:]
    assert child.returncode == 0, tail
    assert "passed" in child.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
