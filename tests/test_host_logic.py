"""Host-side logic of the library that needs no GPU: the table builders of the contraction encoders
(a C++ check program built with the sanitizers) and the bit gather / spread helpers with which
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


def test_contraction_table_builders_under_the_sanitizers(tmp_path):
    """The tables hdc_create builds for the two contraction encoders (thresholds, tiles, columns,
    operands, placement, the feature slots that carry the vote threshold): a host program builds
    them for several model shapes with AddressSanitizer and UndefinedBehaviorSanitizer on, encodes
    samples from the tables alone and compares every bit with Sec. III Eq. (1) written out."""
    exe = tmp_path / "contract_tables_check"
    src = os.path.join(ROOT, "tests", "host", "contract_tables_check.cpp")
    inc = os.path.join(ROOT, "paper_2206_04746_amd", "csrc")
    subprocess.run(["g++", "-O1", "-g", "-std=c++17", "-Wall", "-Werror", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-I", inc, src, "-o", str(exe)], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0 and r.stdout.startswith("OK"), r.stdout + r.stderr
