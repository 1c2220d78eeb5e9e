"""ctypes access to cr_native.c.  TEST INFRASTRUCTURE ONLY.

`build()` compiles the C file with gcc (-O2 -fopenmp, nothing tuned);
the functions below mirror `cr_tree.partial_gradient` / `cr_tree.full_gradient`
for inputs too large to widen to fp64 with numpy temporaries.  X is a C-contiguous
float32 array, or a uint16 array holding bf16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cr_native.c")
_LIB = os.path.join(_HERE, "libcr_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, vp = ctypes.c_int64, ctypes.c_void_p
        lib.cro_num_threads.restype = ctypes.c_int
        lib.cro_segment_gradient.restype = ctypes.c_int
        lib.cro_segment_gradient.argtypes = [vp, ctypes.c_int, vp, vp, i64, ctypes.c_int, i64, i64, vp]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().cro_num_threads())


def _dtype_code(X: np.ndarray) -> int:
    if X.dtype == np.float32:
        return 0
    if X.dtype == np.uint16:
        return 1
    raise TypeError("X must be float32, or uint16 holding bf16 bits")


def segment_gradient(X, y, w, b: int, e: int, model: int = 0) -> np.ndarray:
    lib = _load()
    assert X.flags.c_contiguous and X.ndim == 2
    y = np.ascontiguousarray(y, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    m, d = X.shape
    assert 0 <= b <= e <= m and y.shape == (m,) and w.shape == (d,)
    g = np.empty(d, dtype=np.float64)
    rc = lib.cro_segment_gradient(X.ctypes.data, _dtype_code(X), y.ctypes.data, w.ctypes.data,
                                  d, int(model), int(b), int(e), g.ctypes.data)
    if rc != 0:
        raise RuntimeError("cro_segment_gradient failed")
    return g


def full_gradient(X, y, w, model: int = 0) -> np.ndarray:
    return segment_gradient(X, y, w, 0, X.shape[0], model)


def local_coded_gradient(X, y, w, segments, model: int = 0) -> np.ndarray:
    g = np.zeros(X.shape[1])
    for b, e, c in segments:
        g += float(c) * segment_gradient(X, y, w, b, e, model)
    return g
