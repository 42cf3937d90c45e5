"""Build libsgmv.so (HIP, gfx950) in-tree with hipcc.

    python -m paper_2310_18547_amd.build
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsgmv.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the first 16 dwords of kernel arguments arrive in SGPRs at wave launch instead of
    # through a scalar load (one memory round trip less before the first weight load)
    "-mllvm", "-amdgpu-kernarg-preload-count=16",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = True, extra=(), trace: bool = False) -> str:
    """Compile every csrc/*.hip to an object (in parallel) and link libsgmv.so.

    ``trace=True`` builds the tuning variant libsgmv_trace.so instead: the same sources with
    -DSGMV_TRACE, whose single-launch kernels record an in-kernel timeline (csrc/trace.h)."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build_trace" if trace else "_build")
    lib = os.path.join(HERE, "libsgmv_trace.so") if trace else LIB
    if trace:
        extra = tuple(extra) + ("-DSGMV_TRACE",)
    os.makedirs(objdir, exist_ok=True)
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]

    def compile_one(src):
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        cmd = [hipcc, *flags, *extra, "-c", "-o", obj, src]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(sources()))) as pool:
        objs = list(pool.map(compile_one, sources()))
    tmp = lib + f".tmp{os.getpid()}"
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.check_call(link)
    os.replace(tmp, lib)
    return lib


if __name__ == "__main__":
    args = sys.argv[1:]
    build(extra=[a for a in args if a != "--trace"], trace="--trace" in args)
