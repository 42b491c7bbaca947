"""Builds libdfk.so (hand-written HIP for gfx950) in-tree with hipcc.

    python -m paper_2602_11808_amd.build

hipcc cross-compiles for gfx950 without a GPU present.  The library is
written for gfx950 only; there is no other target and no fallback.
"""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libdfk.so")
SOURCES = ["dfk_api.hip", "dfk_valu.hip", "dfk_mfma.hip", "dfk_mfma_km.hip", "dfk_mfma_fused.hip", "dfk_mfma_big.hip", "dfk_util.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-munsafe-fp-atomics",
    # packed-fp32 VALU forms are kept out of all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _compile(hipcc: str, s: str, verbose: bool) -> str:
    src = os.path.join(CSRC, s)
    obj = os.path.join(CSRC, s.replace(".hip", ".o"))
    cmd = [hipcc, *[f for f in FLAGS if f != "-shared"], "-c", src, "-o", obj]
    if verbose:
        print("[dfk build]", " ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if out.strip() and verbose:
        print(out)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {s}:\n{out}")
    return obj


def build(verbose: bool = True) -> str:
    """Compiles every source (a few at a time: the kernel files take about half a minute each) and links."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    jobs = max(1, min(4, len(os.sched_getaffinity(0))))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(lambda s: _compile(hipcc, s, verbose), SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print("[dfk build]", " ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build()
    print("built", LIB)
    sys.exit(0)
