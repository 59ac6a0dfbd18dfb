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


# ---- host-side sanitizer build: the same sources with AddressSanitizer + UndefinedBehaviorSanitizer on the HOST code
# only (argument validation, the token schedule, workspace carving, launch-shape logic, small-array uploads).  The
# device code is compiled as usual; nothing here runs on a GPU under a sanitizer.
ASAN_LIB = os.path.join(HERE, "libfastav_asan.so")
ASAN_OBJ = os.path.join(OBJ, "asan")
ASAN_HOST_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                   "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def asan_runtime() -> str:
    """Path of the shared AddressSanitizer runtime of the ROCm clang (it has to be preloaded into python)."""
    p = subprocess.run(["hipcc", "--offload-arch=gfx950", "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    cand = p.stdout.strip()
    if cand and os.path.isabs(cand) and os.path.exists(cand):
        return cand
    for root, _, files in os.walk("/opt/rocm/lib/llvm/lib/clang"):
        if "libclang_rt.asan-x86_64.so" in files:
            return os.path.join(root, "libclang_rt.asan-x86_64.so")
    raise FileNotFoundError("libclang_rt.asan-x86_64.so not found under /opt/rocm")


def build_asan(jobs: int = 8) -> str:
    os.makedirs(ASAN_OBJ, exist_ok=True)
    flags = [f for f in HIPCC_FLAGS if f != "-O3"] + ["-O1"] + ASAN_HOST_FLAGS

    def one(name):
        p = subprocess.run(["hipcc", *flags, "-c", os.path.join(CSRC, name + ".hip"), "-o", os.path.join(ASAN_OBJ, name + ".o")],
                           capture_output=True, text=True)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc (host sanitizers) failed on {name}.hip:\n{p.stderr[-2000:]}")

    with ThreadPoolExecutor(max_workers=jobs) as ex:
        list(ex.map(one, SOURCES))
    p = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
                        "-shared-libsan", "-Wno-option-ignored", "-o", ASAN_LIB, *[os.path.join(ASAN_OBJ, n + ".o") for n in SOURCES]],
                       capture_output=True, text=True)
    if p.returncode != 0:
        raise RuntimeError("link (host sanitizers) failed:\n" + p.stdout + p.stderr)
    return ASAN_LIB


if __name__ == "__main__":
    if len(sys.argv) > 1 and sys.argv[1] == "asan":
        print("built", build_asan())
    else:
        build()
    sys.exit(0)
