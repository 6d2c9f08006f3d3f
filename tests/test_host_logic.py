"""Host-side logic of the library that needs no GPU: the bit gather / spread helpers with which
hdc_create packs the varying dimensions and expand_kernel's stage masks are made (a C++ check
program compiled with the host compiler against bit-by-bit definitions)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bit_gather_and_spread_helpers(tmp_path):
    exe = tmp_path / "bit_spread_check"
    src = os.path.join(ROOT, "tests", "host", "bit_spread_check.cpp")
    inc = os.path.join(ROOT, "paper_2206_04746_amd", "csrc")
    subprocess.run(["g++", "-O2", "-std=c++17", "-Wall", "-Werror", "-I", inc, src, "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    assert out.startswith("OK"), out
