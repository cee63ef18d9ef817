"""Compile libiso.so (the HIP kernels and the C ABI) in-tree for gfx950."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB_PATH = os.path.join(HERE, "libiso.so")
SOURCES = [os.path.join(HERE, "csrc", "iso_api.hip"), os.path.join(HERE, "csrc", "iso_plan.cpp")]
HEADERS = [os.path.join(HERE, "csrc", h) for h in ("iso_kernels.hpp", "iso_plan.hpp", "iso_fastdiv.hpp", "iso_bind.hpp")]
HEADERS.append(os.path.join(ROOT, "include", "iso.h"))


def hipcc_command(out=LIB_PATH):
    return ["hipcc", "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wall", "-Wextra",
            "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
            *SOURCES, "-o", out]


def build(verbose=False):
    """Always recompiles; returns the library path."""
    cmd = hipcc_command()
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = [l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l]
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + "\n".join(lines))
    if verbose and lines:
        print("\n".join(lines))
    return LIB_PATH


SANITIZER_DRIVER_SRC = os.path.join(ROOT, "tests", "abi_sanitizer_driver.cpp")
SANITIZER_DRIVER = os.path.join(ROOT, "tests", "abi_sanitizer_driver")


def build_abi_sanitizer_driver(verbose=False):
    """The C ABI test driver with the library's host code under ASan + UBSan (sanitizers on
    the host pass only; the device code is the normal gfx950 build).  Returns its path."""
    cmd = ["hipcc", "-O1", "-g", "-std=c++17", "--offload-arch=gfx950",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-static-libsan",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
           SANITIZER_DRIVER_SRC, *SOURCES, "-o", SANITIZER_DRIVER]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = [l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l]
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + "\n".join(lines))
    return SANITIZER_DRIVER


def is_stale():
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
