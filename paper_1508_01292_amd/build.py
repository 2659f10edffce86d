"""Compile the HIP library (libcnnc.so) for gfx950, in-tree."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libcnnc.so")
OBJ = os.path.join(HERE, "_build")

SOURCES = ["cnnc_host.hip", "k_pyramid.hip", "k_stage1.hip", "k_compact.hip", "k_eval.hip", "k_eval_mfma.hip", "k_merge.hip", "k_peaks.hip", "k_scan.hip", "k_select.hip", "cnnc_pipe.hip"]

# -packed-fp32-ops is switched off on purpose: the compiler must not form packed fp32 instructions.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument", "-I", INCLUDE, "-I", CSRC]


def _hipcc() -> str:
    for p in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if p and (os.path.sep not in p or os.path.exists(p)):
            return p
    return "hipcc"


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    subprocess.run([_hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj], check=True)
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
