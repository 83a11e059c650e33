"""Host side of the library under AddressSanitizer and UndefinedBehaviorSanitizer (device code is not instrumented:
sanitizers for the GPU are not available here).  Every translation unit is compiled with the sanitizers on the host
pass only, linked with a small C++ driver (tests/host/abi_host_check.cpp) that walks the argument validation and the
launch planners of the C ABI over a grid of shapes without touching a GPU, and run.  Any report makes the run fail."""
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2510_11696_amd", "csrc")
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]


@pytest.mark.timeout(900)
def test_abi_validation_and_planners_are_clean_under_asan_and_ubsan(tmp_path):
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc not found")
    clangxx = "/opt/rocm/lib/llvm/bin/clang++"
    if not os.path.exists(clangxx):
        pytest.skip("ROCm clang++ not found")
    out = str(tmp_path)
    srcs = sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))

    def compile_one(src):
        extra = ["-ffp-contract=off"] if src in ("quantize.hip", "mx.hip") else []
        obj = os.path.join(out, src.replace(".hip", ".o"))
        cmd = ["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-fPIC", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-Wno-unused-command-line-argument", *SAN, *extra, "-I" + os.path.join(ROOT, "include"),
               "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-3000:]
        return obj

    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(compile_one, srcs))
    main_o = os.path.join(out, "abi_host_check.o")
    r = subprocess.run([clangxx, "-std=c++17", "-O1", "-g", "-fsanitize=address", "-fsanitize=undefined",
                        "-fno-sanitize-recover=undefined", "-I" + os.path.join(ROOT, "include"), "-c",
                        os.path.join(ROOT, "tests", "host", "abi_host_check.cpp"), "-o", main_o], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    exe = os.path.join(out, "abi_host_check")
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                        *objs, main_o, "-o", exe], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "0 unexpected results" in r.stdout
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr
