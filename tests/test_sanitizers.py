"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer: the CPU oracle (C) and the
library's host side (key generation, import / export, encryption, every lowering, argument
checks) are built as small instrumented programs and run at a toy parameter set.  GPU code is not
instrumented (the device launchers are stubs in that build)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1806_03461_amd", "csrc")
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]


def run(cmd, **kw):
    return subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600, **kw)


def test_oracle_under_sanitizers(tmp_path):
    if not shutil.which("gcc"):
        pytest.skip("no gcc")
    exe = str(tmp_path / "oracle_san")
    b = run(["gcc", *SAN, "-fopenmp", os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), "-o", exe, "-lm"])
    assert b.returncode == 0, b.stdout
    r = run([exe])
    assert r.returncode == 0 and "oracle sanitizer run: ok" in r.stdout, r.stdout


def test_library_host_code_under_sanitizers(tmp_path):
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    if not shutil.which("g++") or not os.path.exists(os.path.join(rocm, "lib", "libamdhip64.so")):
        pytest.skip("no g++ or no HIP runtime to link against")
    exe = str(tmp_path / "host_san")
    src = [os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp")] + \
          [os.path.join(CSRC, f) for f in ("host_keys.cpp", "bnn_lower.cpp", "executor.cpp")]
    b = run(["g++", "-std=c++17", *SAN, "-D__HIP_PLATFORM_AMD__", f"-I{rocm}/include", "-pthread", *src,
             f"-L{rocm}/lib", "-lamdhip64", f"-Wl,-rpath,{rocm}/lib", "-o", exe])
    assert b.returncode == 0, b.stdout
    r = run([exe], env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1"))
    assert r.returncode == 0 and "host-code sanitizer run: ok" in r.stdout, r.stdout
