"""Builds libcqa.so (HIP, gfx950 only) in-tree with hipcc.

Run as `python -m paper_2605_20868_amd.build`.  Each source is compiled to an
object, then linked into paper_2605_20868_amd/libcqa.so.  Packed-FP32 code
generation is switched off for all device code, and floating-point contraction
is switched off for the quantizer so its binary32 operation sequence is exact.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libcqa.so")
BUILD = os.path.join(HERE, "_build")

SOURCES = ["quantize.hip", "decode.hip", "decode_mfma.hip", "adaptive.hip", "dense.hip", "api.hip"]
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
PER_FILE = {"quantize.hip": ["-ffp-contract=off"]}


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the HIP extension cannot be built")
    return exe


def build(verbose: bool = True) -> str:
    os.makedirs(BUILD, exist_ok=True)
    cc = hipcc()
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(BUILD, src.replace(".hip", ".o"))
        cmd = [cc, *COMMON, *PER_FILE.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        text = out.decode(errors="replace")
        # the host pass does not know the packed-fp32 feature name; that warning is harmless
        text = "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l)
        if text.strip() and verbose:
            print(text)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{text}")
    cmd = [cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return OUT


if __name__ == "__main__":
    build()
    print("built", OUT)
    sys.exit(0)
