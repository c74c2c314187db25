"""CPU oracle for the hierarchical recursive-doubling all-reduce (Algorithm 1, Section 4.1).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py; the product package never imports it and it never imports the
product package.

Three independent pieces:

* ``allreduce`` / ``step_combine``  - the schedule-ordered oracle in plain C
  (nvrar_oracle.c), rank by rank and phase by phase as in Algorithm 1;
* ``tree_allreduce`` (tree.py)      - the same result written as a balanced binary tree
  over node index, in numpy, used to pin the order of the inter-node phase;
* ``naive_sum_f64`` (naive.py)      - sequential fp64 sum over ranks 0..P-1, the yardstick
  for the error-bound check only.

bf16 data travels as numpy uint16 bit patterns, fp32 as numpy float32.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

from .naive import naive_sum_f64  # noqa: F401
from .tree import tree_allreduce  # noqa: F401

BF16 = 0
F32 = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nvrar_oracle.c")
_LIB = os.path.join(_HERE, "libnvrar_oracle.so")

_ERRORS = {-1: "bad argument", -3: "out of memory"}


def build(force: bool = False) -> str:
    """Compile nvrar_oracle.c with gcc (no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.nvrar_oracle_allreduce.restype = ctypes.c_int
        lib.nvrar_oracle_allreduce.argtypes = [
            ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_void_p), ctypes.c_int,
            ctypes.c_int, ctypes.c_size_t, ctypes.c_int, ctypes.c_int]
        lib.nvrar_oracle_step_combine.restype = ctypes.c_int
        lib.nvrar_oracle_step_combine.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int]
        lib.nvrar_oracle_threads_used.restype = ctypes.c_int
        lib.nvrar_oracle_threads_used.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def dtype_code(arr: np.ndarray) -> int:
    if arr.dtype == np.uint16:
        return BF16
    if arr.dtype == np.float32:
        return F32
    raise TypeError(f"oracle takes uint16 (bf16 bits) or float32 arrays, got {arr.dtype}")


def allreduce(x: np.ndarray, G: int, threads: int = 1) -> np.ndarray:
    """Schedule-ordered all-reduce of x[P, n] (rank p = r_n*G + r_g).  Returns out[P, n]."""
    x = np.ascontiguousarray(x)
    if x.ndim != 2:
        raise ValueError("x must be [P, n]")
    P, n = x.shape
    if G < 1 or P % G:
        raise ValueError("G must divide P")
    code = dtype_code(x)
    out = np.empty_like(x)
    ins = (ctypes.c_void_p * P)(*[x[p].ctypes.data for p in range(P)])
    outs = (ctypes.c_void_p * P)(*[out[p].ctypes.data for p in range(P)])
    rc = _load().nvrar_oracle_allreduce(ins, outs, G, P // G, n, code, threads)
    if rc != 0:
        raise ValueError(f"oracle: {_ERRORS.get(rc, rc)}")
    return out


def step_combine(dst: np.ndarray, src: np.ndarray, chunk: int, n: int) -> None:
    """In place: dst[chunk*n : chunk*n+n] <- narrow(widen(dst) + widen(src)) over that range."""
    if dst.dtype != src.dtype or not dst.flags.c_contiguous or not src.flags.c_contiguous:
        raise ValueError("dst and src must be contiguous and of one dtype")
    if (chunk + 1) * n > dst.size or (chunk + 1) * n > src.size:
        raise ValueError("range past the end of dst or src")
    rc = _load().nvrar_oracle_step_combine(dst.ctypes.data, src.ctypes.data, chunk, n,
                                           dtype_code(dst))
    if rc != 0:
        raise ValueError(f"oracle: {_ERRORS.get(rc, rc)}")


def threads_used(threads: int) -> int:
    return int(_load().nvrar_oracle_threads_used(threads))
