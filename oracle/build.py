"""Compile the plain-C oracle with gcc (test infrastructure, not the product)."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "treelstm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_treelstm.so")


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        lib.oracle_treelstm_forward.restype = ctypes.c_int
        lib.oracle_treelstm_forward.argtypes = [
            ctypes.c_int64, ctypes.POINTER(ctypes.c_int32), ctypes.c_int, ctypes.c_int,
            dp, dp, dp, dp, dp, dp, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
        _lib = lib
    return _lib


def forward_c(parent, x, W, U, b, n_threads: int = 0):
    """C oracle: returns (h, c, threads_used); fp64 arrays [N, H]."""
    lib = _load()
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    x = np.ascontiguousarray(x, dtype=np.float64)
    W = np.ascontiguousarray(W, dtype=np.float64)
    U = np.ascontiguousarray(U, dtype=np.float64)
    b = np.ascontiguousarray(b, dtype=np.float64)
    n, D = x.shape if x.ndim == 2 else (0, W.shape[1])
    H = U.shape[1]
    h = np.zeros((n, H))
    c = np.zeros((n, H))
    used = ctypes.c_int(0)
    dp = ctypes.POINTER(ctypes.c_double)
    rc = lib.oracle_treelstm_forward(
        n, parent.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), D, H,
        x.ctypes.data_as(dp), W.ctypes.data_as(dp), U.ctypes.data_as(dp), b.ctypes.data_as(dp),
        h.ctypes.data_as(dp), c.ctypes.data_as(dp), int(n_threads), ctypes.byref(used))
    if rc != 0:
        raise ValueError(f"oracle_treelstm_forward failed: {rc}")
    return h, c, used.value


if __name__ == "__main__":
    print(build(force=True))
