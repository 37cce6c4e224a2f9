"""Compiles the HIP sources in csrc/ into libmkv.so next to this file (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB_PATH = os.path.join(HERE, "libmkv.so")
SOURCES = ["mkv_api.hip", "mkv_attn.hip", "mkv_attn_mq.hip", "mkv_evict.hip", "mkv_project.hip"]

# packed-fp32 instructions are switched off on purpose; hipcc's host pass warns that it does not
# know the feature, which is harmless
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def build_library(verbose: bool = False, extra_flags: list[str] | None = None) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    build_dir = os.path.join(HERE, "_build")
    os.makedirs(build_dir, exist_ok=True)
    procs = []
    for src in SOURCES:
        obj = os.path.join(build_dir, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *(extra_flags or []), "-I", os.path.join(ROOT, "include"),
               "-c", os.path.join(HERE, "csrc", src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        text = out.decode(errors="replace")
        if p.returncode != 0:
            sys.stderr.write(text)
            raise RuntimeError(f"hipcc failed on {src}")
        if verbose and text.strip():
            print(text)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH]
    subprocess.run(cmd, check=True)
    build_c_driver(verbose)
    return LIB_PATH


# A caller of the C ABI written in plain C99 (tests/abi_gpu_driver.c): device memory from hipMalloc,
# no Python in the process.  Built here, next to the library, so that it travels with it; a GPU
# test runs it.
C_DRIVER_PATH = os.path.join(HERE, "abi_gpu_driver.bin")


def build_c_driver(verbose: bool = False) -> str:
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = [os.path.join(rocm, "llvm", "bin", "clang"), "-std=c99", "-O1", "-Wall", "-Werror",
           "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"), "-I", os.path.join(rocm, "include"),
           os.path.join(ROOT, "tests", "abi_gpu_driver.c"), "-o", C_DRIVER_PATH,
           "-L", HERE, "-lmkv", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return C_DRIVER_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
