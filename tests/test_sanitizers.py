"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the CPU oracle and of the host side of the C ABI
(host code only; the GPU code objects are not instrumented).  Each driver exercises its subject with exactly-sized
buffers and exits non-zero -- or is stopped by the sanitizer -- on any finding."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests")
SAN_ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def _run(exe):
    p = subprocess.run([exe], capture_output=True, text=True, env=SAN_ENV, timeout=300)
    assert p.returncode == 0, f"{exe} failed ({p.returncode}):\n{p.stdout}\n{p.stderr}"
    return p.stdout


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_oracle")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                           "-static-libasan", "-fopenmp", "-ffp-contract=off", "-o", exe,
                           os.path.join(HERE, "sanitize_oracle_main.c"), "-lm"])
    assert "sanitize-oracle ok" in _run(exe)


@pytest.mark.skipif(shutil.which("hipcc") is None or not os.path.exists("/opt/rocm/lib/llvm/bin/clang++"), reason="needs the ROCm compilers")
def test_c_abi_host_side_under_asan_ubsan(tmp_path):
    # api.hip's host pass instrumented (every -fsanitize directly after -Xarch_host); the kernels' objects are the
    # ordinary ones of the in-tree build
    from paper_2505_19115_amd import build as hip_build
    objs = [os.path.join(hip_build.OBJ, s.replace(".hip", ".o")) for s in hip_build.SOURCES if s != "api.hip"]
    if not all(os.path.exists(o) for o in objs):
        hip_build.build()
    api_o, exe = str(tmp_path / "api_san.o"), str(tmp_path / "sanitize_api")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]
    subprocess.check_call(["hipcc", *hip_build.FLAGS, "-g", *san, "-c", os.path.join(hip_build.CSRC, "api.hip"), "-o", api_o],
                          stderr=subprocess.DEVNULL)
    # the driver is plain C++ (host compiler, no HIP); the link line holds objects only
    main_o = str(tmp_path / "main.o")
    subprocess.check_call(["/opt/rocm/lib/llvm/bin/clang++", "-std=c++17", "-g", "-fsanitize=address", "-fsanitize=undefined",
                           "-fno-sanitize-recover=undefined", "-c", os.path.join(HERE, "sanitize_api_main.cpp"), "-o", main_o])
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                           "-o", exe, main_o, api_o, *objs], stderr=subprocess.DEVNULL)
    assert "sanitize-api ok" in _run(exe)
