"""Builds libcommvq.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
SRC = os.path.join(PKG, "csrc", "commvq.hip")
SOURCES = [SRC, os.path.join(PKG, "csrc", "commvq_encode.hip"), os.path.join(PKG, "csrc", "commvq_em.hip"),
           os.path.join(PKG, "csrc", "commvq_vbits.hip")]
LIB = os.path.join(PKG, "libcommvq.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# packed fp32 VALU forms (v_pk_*_f32) are kept off for every device compile: some of their forms have
# given wrong results on this hardware, and the kernels do not need them
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = False) -> str:
    """Compile csrc/*.hip for gfx950 into paper_2506_18879_amd/libcommvq.so."""
    cmd = [HIPCC, *FLAGS, "-I" + os.path.join(ROOT, "include"), "-o", LIB, *SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(" ".join(cmd))
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libcommvq.so")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
