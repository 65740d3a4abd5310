"""Compile the HIP library for gfx950 into paper_2601_09212_amd/libcool_sd.so (in-tree)."""
import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libcool_sd.so")
SOURCES = ["api.hip", "verify_kernels.hip"]
HEADERS = ["device_utils.h", "kernels.h", "topk.h", "stats_kernels.h", "topk_kernels.h", "sequence_common.h",
           "sequence_whole.h", "early_exit_kernels.h", "sequence_long.h", "diagnostics_kernels.h"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # a*b followed by +-c stays two roundings unless the source says fma: the kernels rely on
         # p - min(q, omega p) being exactly zero where the two are equal
         "-ffp-contract=off",
         "-Wall", "-Wno-unused-function"]


def sources():
    return ([os.path.join(CSRC, s) for s in SOURCES] + [os.path.join(CSRC, h) for h in HEADERS]
            + [os.path.join(ROOT, "include", "cool_sd.h")])


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(s) > t for s in sources())


def build(verbose: bool = False, extra_flags=()) -> str:
    cmd = ([HIPCC] + FLAGS + list(extra_flags) + ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
           + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB])
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


EXAMPLE_SRC = os.path.join(PKG, "examples", "verify_example.c")
EXAMPLE_BIN = os.path.join(PKG, "examples", "verify_example")


def build_example(verbose: bool = False) -> str:
    """Compile examples/verify_example.c, a plain-C user of the C ABI, with gcc against the built
    library and the HIP runtime (the macro is the one HIP's own headers ask a host compiler for)."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-O2", "-Wall", "-std=c11", EXAMPLE_SRC, "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"),
           "-I", os.path.join(ROOT, "include"), "-L", PKG, "-lcool_sd", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
           "-lm", "-Wl,-rpath,$ORIGIN/..", "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", EXAMPLE_BIN]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return EXAMPLE_BIN


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_example(verbose=True))
