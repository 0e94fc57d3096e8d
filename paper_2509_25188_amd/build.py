"""Builds libl2pd.so (the HIP kernels + C ABI) and the kernel_bench measurement tool in-tree with
hipcc for gfx950."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libl2pd.so")
BENCH = os.path.join(HERE, "kernel_bench")
SOURCES = ["kernels_misc.hip", "kernels_f32.hip", "gemm_bf16.hip", "attn_bf16.hip", "l2pd_api.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: cannot build libl2pd.so")
    return exe


def build_library(verbose: bool = False) -> str:
    """Compiles every translation unit and links the shared library.  Always recompiles."""
    objs = []
    procs = []
    for src in SOURCES + ["kernel_bench.hip"]:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if src in SOURCES:
            objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out)
    tmp = LIB + ".tmp"
    r = subprocess.run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp],
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}")
    os.replace(tmp, LIB)
    # stand-alone kernel timing tool: links the same kernel objects
    kobjs = [os.path.join(CSRC, n) for n in ("kernel_bench.o", "kernels_misc.o", "gemm_bf16.o", "attn_bf16.o")]
    r = subprocess.run([hipcc(), "--offload-arch=gfx950", *kobjs, "-o", BENCH + ".tmp"],
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"kernel_bench link failed:\n{r.stdout}")
    os.replace(BENCH + ".tmp", BENCH)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
