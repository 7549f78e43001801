"""Host code of the library under AddressSanitizer + UndefinedBehaviorSanitizer
(CPU only; device code is compiled as usual and never runs here).  The library
is rebuilt into a temporary directory with the sanitizers switched on for the
host pass, and two C programs drive it through the C ABI on a host-only device:
the worked placement example and a longer workout of the planner, the region
sub-allocator, the graph analyzer and the tracer's bookkeeping."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1805_08430_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANG = "/opt/rocm/llvm/bin/clang"


@pytest.mark.skipif(not (os.path.exists(HIPCC) and os.path.exists(CLANG)), reason="needs the ROCm compilers")
def test_host_code_under_address_and_ub_sanitizers(tmp_path):
    lib = tmp_path / "librdev_san.so"
    cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-shared",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", str(lib)] + \
          [os.path.join(CSRC, f) for f in ("rdev.hip", "planner.cpp", "graph.cpp")]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    for src, want in (("c_abi_check.c", "c abi ok"), ("san_host_check.c", "san host ok")):
        exe = tmp_path / src.replace(".c", "")
        r = subprocess.run([CLANG, "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-g", "-std=c99",
                            "-I", os.path.join(ROOT, "include"), "-o", str(exe), os.path.join(ROOT, "tests", src),
                            "-L", str(tmp_path), "-lrdev_san", "-Wl,-rpath," + str(tmp_path)],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-3000:]
        r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
        assert r.returncode == 0 and want in r.stdout, (r.stdout[-2000:], r.stderr[-4000:])
        assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    shutil.rmtree(tmp_path, ignore_errors=True)
