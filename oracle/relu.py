"""CPU oracle for the ReLU block: thin ctypes wrapper over relu_oracle.c.

TEST INFRASTRUCTURE ONLY (see the header of relu_oracle.c).  Arrays of any
shape; results have the shape of x, in fp64.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from ._cbuild import compile_shared

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "relu_oracle.c")
_LIB = os.path.join(_HERE, "librelu_oracle.so")


def build(force: bool = False) -> str:
    return compile_shared(_SRC, _LIB, force)


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        P, I64 = ctypes.c_void_p, ctypes.c_int64
        lib.orr_forward.argtypes = [P, P, I64]
        lib.orr_backward.argtypes = [P, P, P, I64]
        _lib = lib
    return _lib


def forward(x):
    """y = max(0, x)  (Sec. 4.4)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.empty_like(x)
    if _load().orr_forward(x.ctypes.data, y.ctypes.data, x.size):
        raise ValueError("bad argument")
    return y


def backward(x, dzdy):
    """dzdx = [x > 0] * dzdy  (Sec. 6.4.1).  x may equally be the block's output y: y > 0 iff x > 0."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    dzdy = np.ascontiguousarray(dzdy, dtype=np.float64)
    if dzdy.shape != x.shape:
        raise ValueError("dzdy has shape %r, expected %r" % (dzdy.shape, x.shape))
    dzdx = np.empty_like(x)
    if _load().orr_backward(x.ctypes.data, dzdy.ctypes.data, dzdx.ctypes.data, x.size):
        raise ValueError("bad argument")
    return dzdx
