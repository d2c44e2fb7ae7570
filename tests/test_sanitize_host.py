"""The host side of the library (layout builder, CSR import, union, window search, table packing, the
argument checks of the C ABI) compiled with AddressSanitizer and UndefinedBehaviorSanitizer and run
through tests/sanitize/host_abi_check.cpp.  Host code only: the kernels are replaced by stubs, no GPU
is touched, and the sanitizers are given to hipcc's host pass alone."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2508_12969_amd", "csrc")


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    sanitize = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                "-Xarch_host", "-fno-sanitize-recover=undefined"]
    common = [hipcc, "-x", "hip", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
              "-I", os.path.join(ROOT, "include"), "-I", CSRC, *sanitize]
    objs = []
    for src in (os.path.join(CSRC, "layout.cpp"), os.path.join(CSRC, "search.cpp"), os.path.join(CSRC, "api.cpp"),
                os.path.join(ROOT, "tests", "sanitize", "host_abi_check.cpp")):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        res = subprocess.run(common + ["-c", src, "-o", obj], capture_output=True, text=True)
        assert res.returncode == 0, res.stderr[-3000:]
        objs.append(obj)
    exe = str(tmp_path / "host_abi_check")
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                          *objs, "-o", exe], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert res.returncode == 0, (res.stdout[-3000:], res.stderr[-3000:])
    assert "host ABI checks passed" in res.stdout
