"""CPU run of the transform header the blind-rotation kernel is built from (csrc/fft512.h): the
host program tests/host/fft512_exactness.cpp drives the 256 lanes of a workgroup one after the other
through the kernel's own per-lane steps and compares the rounded products with exact 64-bit integer
negacyclic convolutions, on random operands and on operands at the ends of their ranges arranged so
that the 4,096 terms of one coefficient add coherently (|sum| = 2^36)."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_four_wave_transform_products_are_exact_on_the_host(tmp_path):
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    if not shutil.which("g++") or not os.path.exists(os.path.join(rocm, "include", "hip", "hip_runtime.h")):
        pytest.skip("no g++ or no HIP headers")
    exe = str(tmp_path / "fft512_exactness")
    b = subprocess.run(["g++", "-O2", "-std=c++17", "-D__HIP_PLATFORM_AMD__", f"-I{rocm}/include",
                        os.path.join(ROOT, "tests", "host", "fft512_exactness.cpp"), "-o", exe],
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert b.returncode == 0, b.stdout
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert r.returncode == 0, r.stdout
    m = re.search(r"fft512 exactness: ok \(largest distance from an integer ([0-9.e+-]+)\)", r.stdout)
    assert m, r.stdout
    # the bound derived for the worst case is about 2^-10.5; a wrong rounding needs 0.5
    assert float(m.group(1)) < 1e-3
    assert r.stdout.count("wrong 0 ") == 15, r.stdout
