"""Builds libhdc.so (hand-written HIP for gfx950) in-tree with hipcc.

    python -m paper_2206_04746_amd.build          # compile every translation unit and link
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libhdc.so")
SOURCES = ["hdc_api.hip", "encode.hip", "encode_contract.hip", "encode_wide.hip", "encode_sparse.hip", "classical.hip", "online.hip", "online_batched.hip", "search.hip", "search_mfma.hip", "primitives.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    "-Wall", "-Wno-unused-command-line-argument",
    # encode.hip names M0 and its fixed landing VGPRs in inline-asm clobber lists on purpose
    "-Wno-inline-asm",
    # packed-fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _compile(src: str, defines=(), tag: str = "") -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + tag + ".o")
    cmd = [HIPCC, *FLAGS, *[f"-D{d}" for d in defines], "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines()
                    if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True, defines=(), out: str = LIB) -> str:
    """Compile every translation unit and link `out` (default: the in-tree libhdc.so).
    `defines` are extra -D macros, used to build experimental variants next to the default."""
    os.makedirs(OBJ, exist_ok=True)
    tag = "".join("_" + d.replace("=", "") for d in defines)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda src: _compile(src, defines, tag), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(f"built {out}")
    return out


if __name__ == "__main__":
    build()
