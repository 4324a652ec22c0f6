"""Builds libspanattn.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

Besides the product library, named measurement variants of the same sources can be built
(libspanattn_<variant>.so): they exist so that the design decisions recorded under profiles/ can be
re-measured, and are loaded only when SPAN_ATTN_VARIANT names one (bench.py --variant)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libspanattn.so")
SOURCES = [os.path.join(CSRC, "span_kernels.hip"), os.path.join(CSRC, "span_host.cpp")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
         # keep the compiler from forming packed-fp32 instructions
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
VARIANTS = {
    # thread 0 of every workgroup records a clock value at each phase boundary (bench.py --phase-trace)
    "trace": ["-DSPAN_PHASE_TRACE"],
    # K / V rows fetched with the default cache policy instead of the non-temporal one
    "no_nt": ["-DSPAN_ROW_LOAD_POLICY=0"],
    # K / V tiles staged through LDS with direct-to-LDS loads before the lanes read their pieces
    "lds": ["-DSPAN_STAGE_LDS"],
}


def variant_path(variant: str) -> str:
    return os.path.join(HERE, f"libspanattn_{variant}.so")


def build_library(verbose: bool = False, variant: str = None) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    lib = LIB if variant is None else variant_path(variant)
    extra = [] if variant is None else VARIANTS[variant]
    tmp = lib + f".tmp{os.getpid()}"
    cmd = [hipcc] + FLAGS + extra + ["-o", tmp] + SOURCES
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    os.replace(tmp, lib)
    return lib


if __name__ == "__main__":
    names = sys.argv[1:] or [None]
    for name in names:
        print(build_library(verbose=True, variant=None if name in (None, "product") else name))
