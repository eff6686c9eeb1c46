"""Compile libgsgd.so (hand-written HIP for gfx950) in-tree with hipcc."""
import os
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgsgd.so")
SOURCES = ["gsgd_api.hip", "host_perm.hip", "kernels_step.hip", "kernels_sweep.hip", "kernels_async.hip", "kernels_gen.hip",
           "kernels_stats.hip"]

# FP contraction is off: every fused multiply-add in the kernels is written out,
# so results do not depend on what the optimiser decides to fuse.  Packed fp32
# instructions are disabled as a precaution taken for the test machines.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: libgsgd needs the ROCm toolchain")
    return exe


DEMO_SRC = os.path.join(HERE, "examples", "abi_demo.c")
DEMO = os.path.join(HERE, "abi_demo")


def build(verbose: bool = False, extra_flags=()) -> str:
    """Every source to an object of its own, side by side, then one link; the objects live in a temporary folder."""
    common = [hipcc(), *FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    with tempfile.TemporaryDirectory(prefix="gsgd_build_") as tmp:
        def compile_one(name):
            obj = os.path.join(tmp, os.path.splitext(name)[0] + ".o")
            cmd = [*common, "-c", os.path.join(CSRC, name), "-o", obj]
            if verbose:
                print(" ".join(cmd))
            subprocess.run(cmd, check=True)
            return obj
        with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as pool:
            objects = list(pool.map(compile_one, SOURCES))
        cmd = [*common, "-shared", *objects, "-o", LIB]
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True)
    build_demo(verbose)
    return LIB


def build_demo(verbose: bool = False) -> str:
    """The plain-C user of the ABI (no Python, no PyTorch): host code only, linked against libgsgd.so."""
    rocm = os.path.dirname(os.path.dirname(os.path.realpath(hipcc())))
    cc = shutil.which("gcc") or shutil.which("cc")
    if not cc:
        raise RuntimeError("no C compiler for the ABI demo")
    cmd = [cc, "-std=c99", "-O2", "-Wall", DEMO_SRC, "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(rocm, "include"), "-L", HERE, "-L", os.path.join(rocm, "lib"), "-lgsgd", "-lamdhip64",
           "-lm", "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", DEMO]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return DEMO


if __name__ == "__main__":
    print(build(verbose=True))
