"""Builds libspcfg.so (HIP kernels + C ABI, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libspcfg.so")
CLIENT = os.path.join(HERE, "abi_client.bin")  # plain C program that uses the library through its C ABI only
CEILING_SRC = os.path.join(os.path.dirname(HERE), "bench_mfma_ceiling.hip")  # measurement aid of bench.py
CEILING = os.path.join(HERE, "mfma_ceiling.bin")
SOURCES = ["spcfg_api.hip", "kernels_elem.hip", "gemm_nt.hip", "gemm_nt16.hip", "gemm_nt3.hip", "gemm_tn.hip", "gemm_tn3.hip", "rules_frontend.hip", "decode.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wno-unused-function",
         # packed fp32 ops are kept off for all device code on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def find_hipcc():
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: the HIP library cannot be built")


def build(verbose=True):
    import concurrent.futures as cf
    hipcc = find_hipcc()
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in FLAGS if f != "-shared"]

    def compile_one(src):
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc] + compile_flags + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        return obj

    # one translation unit per source file, compiled side by side, then linked into the shared library
    with cf.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    # the C client: compiled as C (host only), linked against the library and the HIP runtime
    rocm = os.path.dirname(os.path.dirname(find_hipcc()))
    cc = ["gcc", "-std=c99", "-O2", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"),
          os.path.join(CSRC, "abi_client.c"), "-o", CLIENT, "-L", HERE, "-lspcfg", "-L", os.path.join(rocm, "lib"),
          "-lamdhip64", "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cc), flush=True)
    subprocess.check_call(cc)
    # bench.py's probe of the matrix pipes' sustained rate (a standalone program, not linked against the library)
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", CEILING_SRC, "-o", CEILING]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build()
    print("built", LIB)
    sys.exit(0)
