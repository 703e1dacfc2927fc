"""Compile the plain-C oracle with gcc (test infrastructure, not the product)."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "treelstm_oracle.c")
# fp64: the parity reference.  fp32: the same source with `real` = float, only ever timed
# (the CPU-baseline leg of the benchmark), never compared with anything.
_LIBS = {"f64": os.path.join(_HERE, "liboracle_treelstm.so"),
         "f32": os.path.join(_HERE, "liboracle_treelstm_f32.so")}
_LIB = _LIBS["f64"]
# -ffp-contract=off: no fused multiply-add, so the arithmetic is the source's, operation by operation
_FLAGS = ["-O3", "-march=native", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC"]


def build(force: bool = False) -> str:
    for prec, lib in _LIBS.items():
        if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(_SRC):
            cmd = ["gcc", *_FLAGS, *(["-DORACLE_REAL=float"] if prec == "f32" else []), "-o", lib, _SRC, "-lm"]
            subprocess.run(cmd, check=True)
    return _LIB


_lib = {}


def _load(precision: str = "f64"):
    if precision not in _lib:
        build()
        lib = ctypes.CDLL(_LIBS[precision])
        rp = ctypes.POINTER(ctypes.c_double if precision == "f64" else ctypes.c_float)
        lib.oracle_treelstm_forward.restype = ctypes.c_int
        lib.oracle_treelstm_forward.argtypes = [
            ctypes.c_int64, ctypes.POINTER(ctypes.c_int32), ctypes.c_int, ctypes.c_int,
            rp, rp, rp, rp, rp, rp, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
        _lib[precision] = lib
    return _lib[precision]


def forward_c(parent, x, W, U, b, n_threads: int = 0, precision: str = "f64"):
    """C oracle: returns (h, c, threads_used); arrays [N, H] in fp64 (the parity reference) or,
    with precision="f32", in fp32 (for timing only)."""
    lib = _load(precision)
    real = np.float64 if precision == "f64" else np.float32
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    x = np.ascontiguousarray(x, dtype=real)
    W = np.ascontiguousarray(W, dtype=real)
    U = np.ascontiguousarray(U, dtype=real)
    b = np.ascontiguousarray(b, dtype=real)
    n, D = x.shape if x.ndim == 2 else (0, W.shape[1])
    H = U.shape[1]
    h = np.zeros((n, H), dtype=real)
    c = np.zeros((n, H), dtype=real)
    used = ctypes.c_int(0)
    dp = ctypes.POINTER(ctypes.c_double if precision == "f64" else ctypes.c_float)
    rc = lib.oracle_treelstm_forward(
        n, parent.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), D, H,
        x.ctypes.data_as(dp), W.ctypes.data_as(dp), U.ctypes.data_as(dp), b.ctypes.data_as(dp),
        h.ctypes.data_as(dp), c.ctypes.data_as(dp), int(n_threads), ctypes.byref(used))
    if rc != 0:
        raise ValueError(f"oracle_treelstm_forward failed: {rc}")
    return h, c, used.value


if __name__ == "__main__":
    print(build(force=True))
