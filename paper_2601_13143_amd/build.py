"""Builds libfastav.so (gfx950) from csrc/*.hip with hipcc, in-tree.

    python -m paper_2601_13143_amd.build            # compile everything, link
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libfastav.so")

SOURCES = ["api", "elementwise", "score", "select", "gemm_generic", "attn_generic", "gemm_mfma", "attn_mfma", "decode", "rollout", "profile"]

# packed fp32 VALU forms are switched off for every device compile
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wno-unused-command-line-argument"]


def _compile(name: str) -> str:
    src = os.path.join(CSRC, name + ".hip")
    obj = os.path.join(OBJ, name + ".o")
    p = subprocess.run(["hipcc", *HIPCC_FLAGS, "-c", src, "-o", obj], capture_output=True, text=True)
    msgs = "\n".join(l for l in (p.stdout + p.stderr).splitlines()
                     if "packed-fp32-ops" not in l and "warning generated" not in l and l.strip())
    if p.returncode != 0:
        raise RuntimeError(f"hipcc failed on {name}.hip:\n{msgs}")
    return msgs


def build(verbose: bool = True, jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        for name, msgs in zip(SOURCES, ex.map(_compile, SOURCES)):
            if verbose and msgs:
                print(f"[{name}]\n{msgs}")
    objs = [os.path.join(OBJ, n + ".o") for n in SOURCES]
    p = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if p.returncode != 0:
        raise RuntimeError("link failed:\n" + p.stdout + p.stderr)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
