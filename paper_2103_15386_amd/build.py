"""Build step of the HIP library (hipcc cross-compiles for gfx950; no GPU needed)."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgnnd_hip.so")
SOURCES = ["graph_kernels.hip", "wide_lists.hip", "long_samples.hip", "segmented_lists.hip", "join_valu.hip",
           "join_mfma.hip", "join_gram.hip", "sample_buckets.hip", "gnnd_api.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-result",
         # packed FP32 instructions are kept off on purpose
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _headers():
    inc = os.path.join(os.path.dirname(HERE), "include", "gnnd.h")
    return [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hpp")] + [inc]


def build_library(force=False, verbose=False):
    """Compile every HIP source for gfx950 and link libgnnd_hip.so in-tree."""
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    objs = [s[:-4] + ".o" for s in srcs]
    newest_hdr = max(os.path.getmtime(h) for h in _headers())

    def compile_one(pair):
        src, obj = pair
        if (not force and os.path.exists(obj)
                and os.path.getmtime(obj) >= max(os.path.getmtime(src), newest_hdr)):
            return False
        cmd = [HIPCC, *FLAGS, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return True

    with ThreadPoolExecutor(max_workers=4) as ex:
        rebuilt = list(ex.map(compile_one, zip(srcs, objs)))
    if force or any(rebuilt) or not os.path.exists(LIB):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
    build_abi_demo(force or any(rebuilt), verbose)
    return LIB


DEMO = os.path.join(HERE, "abi_demo")


def build_abi_demo(force=False, verbose=False):
    """The plain-C caller of the library (csrc/abi_demo.c), compiled by gcc as C11:
    proof that the boundary needs neither C++ nor Python."""
    src = os.path.join(CSRC, "abi_demo.c")
    if not force and os.path.exists(DEMO) and os.path.getmtime(DEMO) >= os.path.getmtime(src):
        return DEMO
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c11", "-O2", "-Wall", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(os.path.dirname(HERE), "include"), "-I", os.path.join(rocm, "include"),
           src, "-o", DEMO, "-L", HERE, "-lgnnd_hip", "-L", os.path.join(rocm, "lib"),
           "-lamdhip64", "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return DEMO


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
