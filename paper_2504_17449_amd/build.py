"""Builds libhmi.so (the C-ABI library: HIP kernels + pool) in-tree for gfx950.

    python paper_2504_17449_amd/build.py
    python paper_2504_17449_amd/build.py --lib /tmp/libhmi_x.so --obj-suffix _x -DHMI_ABLATE_MFMA=1

The second form writes another library (load it with HMI_LIB_PATH=...) from the same sources with extra
compiler flags: the timing-only ablation builds of the persistent GEMM are made this way.
hipcc cross-compiles without a GPU.  Packed-fp32 code generation is switched off for the
device pass, as required on the target machines.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhmi.so")
SOURCES = ["pool.hip", "queue.hip", "router.hip", "gemm_bf16.hip", "gemm_bf16_p256.hip", "gemm_bf16_skinny.hip", "adapter_bf16.hip", "gemm_f32.hip",
           "layernorm.hip", "attention.hip", "head.hip", "kv_cache.hip", "plot.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


def build(verbose: bool = True, lib: str = LIB, extra_flags=(), obj_suffix: str = "") -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", obj_suffix + ".o"))
        cmd = ([hipcc] + [f for f in FLAGS if f != "-shared"] + list(extra_flags)
               + ["-c", os.path.join(CSRC, src), "-o", obj])
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd)))
        objs.append(obj)
    for src, pr in procs:
        if pr.wait() != 0:
            raise RuntimeError(f"hipcc failed on {src}")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return lib


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("--lib", default=LIB)
    ap.add_argument("--obj-suffix", default="")
    ns, extra = ap.parse_known_args()
    build(lib=ns.lib, extra_flags=extra, obj_suffix=ns.obj_suffix)
    sys.exit(0)
