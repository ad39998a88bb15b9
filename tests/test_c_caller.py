"""The C ABI used from plain C: C99 programs are compiled against
include/blink.h, linked with the built library and run: one makes host-side
calls only (no GPU needed), one runs collectives on the GPU."""
import importlib.util
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_1910_04940_amd", "libblink.so")


def hip_runtime():
    """A libamdhip64.so to satisfy the library's HIP references (it is linked
    without one so that a process can bring its own)."""
    candidates = ["/opt/rocm/lib/libamdhip64.so"]
    spec = importlib.util.find_spec("torch")
    if spec is not None and spec.origin:
        candidates.append(os.path.join(os.path.dirname(spec.origin), "lib", "libamdhip64.so"))
    return next((p for p in candidates if os.path.exists(p)), None)


def test_header_is_valid_c99_and_cxx11():
    header = os.path.join(ROOT, "include", "blink.h")
    for cmd in (["gcc", "-std=c99", "-x", "c"], ["g++", "-std=c++11", "-x", "c++"]):
        subprocess.run(cmd + ["-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", header], check=True)


def test_c_program_calls_the_host_side_entry_points(tmp_path):
    hip = hip_runtime()
    if not os.path.exists(LIB) or hip is None or shutil.which("gcc") is None:
        pytest.skip("library, HIP runtime or gcc missing")
    exe = tmp_path / "abi_smoke"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "c", "abi_smoke.c"), "-o", str(exe), LIB, hip,
                    "-Wl,-rpath," + os.path.dirname(hip) + ",-rpath," + os.path.dirname(LIB)], check=True)
    got = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert got[:6] == ["trees", "3", "rate", "3.0", "steps", "108"]
    # shares of 349,524 / 349,524 / 349,528 elements; every element is copied into rank 3 once
    assert got[6:11] == ["bounds", "0", "349524", "699048", "1048576"]
    assert got[11:13] == ["copied_into_rank3", "1048576"]
    assert got[13:16] == ["split", "200.0", "500.0"]
    assert got[16:] == ["bad", "1"]          # chunk 0 -> BLINK_EINVAL


@pytest.mark.gpu
def test_c_program_runs_collectives_on_the_gpu(tmp_path):
    """tests/c/abi_gpu.c: hipMalloc'ed buffers, pack -> schedule -> allreduce /
    allreduce_noalloc / broadcast -> copy back, compared in C with the closed
    form of an integer sum.  A fresh child process with the system HIP runtime."""
    hip = "/opt/rocm/lib/libamdhip64.so"
    assert os.path.exists(LIB) and os.path.exists(hip) and shutil.which("gcc")
    exe = tmp_path / "abi_gpu"
    subprocess.run(["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "c", "abi_gpu.c"), "-o", str(exe), LIB, hip,
                    "-Wl,-rpath," + os.path.dirname(hip) + ",-rpath," + os.path.dirname(LIB)], check=True)
    done = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert done.returncode == 0, done.stderr
    assert done.stdout.split() == ["ok", str(5 * 4 * 1000003)]
