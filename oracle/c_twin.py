"""Build and call the C twin of the oracle (oracle/iso_oracle.c) through ctypes.

TEST INFRASTRUCTURE ONLY, like everything under oracle/.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "iso_oracle.c")
_LIB = os.path.join(_HERE, "libiso_oracle.so")
_lib = None


def build(force=False):
    """Compile the C oracle with gcc + OpenMP; returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        sig = [ctypes.c_int, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p,
               ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        for f in (lib.iso_oracle_alltoall, lib.iso_oracle_allgather):
            f.argtypes = sig
            f.restype = ctypes.c_int
        _lib = lib
    return _lib


def _call(fn, dims, offsets, m, send, recv, threads):
    dims_a = np.ascontiguousarray(dims, dtype=np.int32)
    offs_a = np.ascontiguousarray(offsets, dtype=np.int32).reshape(-1)
    used = fn(len(dims_a), dims_a.ctypes.data, len(offsets), offs_a.ctypes.data,
              m, send.ctypes.data, recv.ctypes.data, threads)
    if used < 0:
        raise ValueError("bad arguments to C oracle")
    return used


def alltoall(dims, offsets, send, out=None, threads=0):
    """send: C-contiguous uint8 (p, s, m).  Returns (recv, threads_used)."""
    send = np.ascontiguousarray(send)
    p, s, m = send.shape
    recv = np.empty_like(send) if out is None else out
    used = _call(_load().iso_oracle_alltoall, dims, offsets, m * send.itemsize, send, recv, threads)
    return recv, used


def allgather(dims, offsets, send, out=None, threads=0):
    """send: C-contiguous uint8 (p, m).  Returns (recv (p, s, m), threads_used)."""
    send = np.ascontiguousarray(send)
    p, m = send.shape
    s = len(offsets)
    recv = np.empty((p, s, m), dtype=send.dtype) if out is None else out
    used = _call(_load().iso_oracle_allgather, dims, offsets, m * send.itemsize, send, recv, threads)
    return recv, used
