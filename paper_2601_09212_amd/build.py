"""Compile the HIP libraries for gfx950, in-tree:

  libcool_sd.so          the product (include/cool_sd.h)
  libcool_sd_checked.so  its debug build: every verify call checks the draft tokens on the device
  libcool_sd_bench.so    the benchmark companion (include/cool_sd_bench.h)

The kernels are compiled once, one object per translation unit and in parallel; the three
libraries differ only in the small host-side objects they are linked with.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libcool_sd.so")
LIB_CHECKED = os.path.join(PKG, "libcool_sd_checked.so")
LIB_BENCH = os.path.join(PKG, "libcool_sd_bench.so")
KERNEL_UNITS = ["stats_bf16_xf.hip", "stats_f32_xf.hip", "stats_bf16_plain.hip", "stats_f32_plain.hip", "stats_launch.hip",
                "sequence_launch.hip", "diagnostics_launch.hip", "verify_kernels.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # a*b followed by +-c stays two roundings unless the source says fma: the kernels rely on
         # p - min(q, omega p) being exactly zero where the two are equal
         "-ffp-contract=off",
         "-Wall", "-Wno-unused-function"]
INCLUDES = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]


def sources():
    names = [f for f in os.listdir(CSRC) if f.endswith((".hip", ".h"))]
    return [os.path.join(CSRC, f) for f in sorted(names)] + [os.path.join(ROOT, "include", h)
                                                            for h in ("cool_sd.h", "cool_sd_bench.h")]


def is_stale() -> bool:
    libs = (LIB, LIB_CHECKED, LIB_BENCH)
    if not all(os.path.exists(p) for p in libs):
        return True
    t = min(os.path.getmtime(p) for p in libs)
    return any(os.path.getmtime(s) > t for s in sources())


def _run(cmd, verbose):
    """Run a build command; hipcc's host pass says once per file that it does not know the
    packed-fp32 target feature (it only exists on the device side): that line is dropped."""
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    noise = "'-packed-fp32-ops' is not a recognized feature for this target"
    err = "\n".join(ln for ln in r.stderr.splitlines() if noise not in ln)
    if err:
        print(err, file=sys.stderr, flush=True)
    if r.returncode != 0:
        raise subprocess.CalledProcessError(r.returncode, cmd)


def build(verbose: bool = False, extra_flags=(), jobs: int = 6) -> str:
    os.makedirs(OBJ, exist_ok=True)
    units = [(u, os.path.join(OBJ, u.replace(".hip", ".o")), ()) for u in KERNEL_UNITS]
    units += [("api.hip", os.path.join(OBJ, "api.o"), ()),
              ("api.hip", os.path.join(OBJ, "api_checked.o"), ("-DCOOL_SD_CHECKED_BUILD",)),
              ("bench_api.hip", os.path.join(OBJ, "bench_api.o"), ())]

    def compile_one(u):
        src, obj, defs = u
        _run([HIPCC] + FLAGS + list(extra_flags) + list(defs) + INCLUDES + ["-c", os.path.join(CSRC, src), "-o", obj],
             verbose)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        list(ex.map(compile_one, units))
    kernels = [o for _, o, _ in units[:len(KERNEL_UNITS)]]
    # only the C entry points leave a library (kernel handles and runtime bookkeeping stay local)
    vers = os.path.join(OBJ, "exports.map")
    with open(vers, "w") as f:
        f.write("{ global: cool_sd_*; local: *; };\n")
    link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-Wl,--version-script=" + vers]
    _run(link + [os.path.join(OBJ, "api.o")] + kernels + ["-o", LIB], verbose)
    _run(link + [os.path.join(OBJ, "api_checked.o")] + kernels + ["-o", LIB_CHECKED], verbose)
    _run(link + [os.path.join(OBJ, "bench_api.o"), os.path.join(OBJ, "api.o")] + kernels + ["-o", LIB_BENCH], verbose)
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
    _run(cmd, verbose)
    return EXAMPLE_BIN


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_example(verbose=True))
