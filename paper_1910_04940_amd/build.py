"""Compile the HIP library in-tree: csrc/* -> libblink.so (gfx950 only).

The objects are linked WITHOUT a dependency on a particular libamdhip64: a
process must hold exactly one HIP runtime, and a PyTorch wheel brings its own.
The HIP entry points are therefore left undefined and bind, at load time, to
the runtime the process has already loaded (binding.py sees to that; a C or
C++ program simply links its own libamdhip64)."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libblink.so")
SOURCES = ["kernel_f32_stream.hip", "kernel_i32_stream.hip", "kernel_f32_many.hip", "kernel_i32_many.hip", "exec.hip",
           "api.cpp", "pack.cpp", "schedule.cpp", "miad.cpp"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-c",
    "-fno-gpu-flush-denormals-to-zero",      # fp32 subnormals are ordinary addends
    "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # A ticket is drawn by lane 0 alone.  The compiler's wave-level rewriting of
    # atomics (one lane adds for all, the others derive their values) gains
    # nothing there and reads the counter's answer, hence waits for it, right
    # after the atomic; without it the answer travels while loads are issued.
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
    "-Wall", "-Wno-unused-command-line-argument",
]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    def compile_one(src: str) -> str:
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc] + FLAGS + [os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True, stderr=None if verbose else subprocess.DEVNULL)
        return obj

    # the kernel instantiation units take about half a minute each: side by side
    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    link = [os.environ.get("CXX", "g++"), "-shared", "-o", LIB] + objs
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
