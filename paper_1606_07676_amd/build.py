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


def is_stale():
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
