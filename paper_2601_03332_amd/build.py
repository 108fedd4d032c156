"""Builds liblutkan.so (host LUT compiler + gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.environ.get("LUTKAN_LIBRARY", os.path.join(HERE, "liblutkan.so"))
SOURCES = [os.path.join(CSRC, "lutkan_compile.cpp"), os.path.join(CSRC, "lutkan_kernels.hip"),
           os.path.join(CSRC, "bspline_kernels.hip"), os.path.join(CSRC, "lutkan_probes.hip"),
           os.path.join(CSRC, "lutkan_stats.hip"), os.path.join(CSRC, "lutkan_base_gemm.hip")]
HEADERS = [os.path.join(CSRC, "lutkan_internal.h"), os.path.join(CSRC, "lutkan_device.h"), os.path.join(CSRC, "lutkan_pieces.h"),
           os.path.join(ROOT, "include", "lutkan.h")]

# -ffp-contract=off: the index arithmetic of the locate kernel and the host quantiser must round once per
#   operation; fused multiply-adds in the edge kernels are written explicitly.
# -packed-fp32-ops is switched off: the packed fp32 VALU forms are not used by this library.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-fno-fast-math",
    "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-Wno-inline-asm",      # the LDS-DMA helper names M0 in its clobber list on purpose (see lutkan_device.h)
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

    def compile_one(src: str) -> str:
        obj = os.path.splitext(src)[0] + ".o"
        cmd = [hipcc] + HIPCC_FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
        if src.endswith(".hip"):
            cmd += ["-x", "hip"]
        cmd += ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return obj

    # the translation units are independent: one compiler process each (lutkan_kernels.hip is the long one)
    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1, 8)) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs + ["-lpthread"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
