"""Builds libkvs.so (the C-ABI library of HIP kernels for gfx950) in-tree with hipcc.

Run as ``python -m paper_2508_04257_amd.build``.  hipcc cross-compiles without a GPU.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libkvs.so")

# translation unit -> extra flags.  The quantiser's arithmetic must match a fixed fp32 operation
# sequence bit for bit: no fused multiply-add, IEEE division.
DECODE_FLAGS = []

SOURCES = {
    "kvs_api.hip": [],
    "predict.hip": [],
    "quantize.hip": ["-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt"],
    "quantize_fast.hip": ["-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt"],
    "sparse.hip": [],
    "decode.hip": [],
    "error_report.hip": ["-ffp-contract=off"],
    "probe.hip": [],
    "prefill.hip": [],
    "decode_mfma.hip": [],
    "decode_mfma_b2.hip": DECODE_FLAGS,
    "decode_mfma_b3.hip": DECODE_FLAGS,
    "decode_mfma_b4.hip": DECODE_FLAGS,
    "decode_mfma_b8.hip": DECODE_FLAGS,
    "decode_mfma_kpt_b2.hip": DECODE_FLAGS,
    "decode_mfma_kpt_b3.hip": DECODE_FLAGS,
    "decode_mfma_kpt_b4.hip": DECODE_FLAGS,
    "decode_mfma_kpt_b8.hip": DECODE_FLAGS,
}

COMMON = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 instructions are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _compile(name: str) -> str:
    obj = os.path.join(OBJ, name.replace(".hip", ".o"))
    cmd = ["hipcc", *COMMON, *SOURCES[name], "-c", os.path.join(CSRC, name), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed for {name}:\n{res.stdout}\n{res.stderr}")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(_compile, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stdout}\n{res.stderr}")
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
