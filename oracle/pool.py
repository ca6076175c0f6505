"""CPU oracle for the spatial pooling block: thin ctypes wrapper over pool_oracle.c.

TEST INFRASTRUCTURE ONLY (see the header of pool_oracle.c).  Arrays are numpy
arrays of shape (N, D, W, H) (H x W x D x N stored first index fastest); results
in fp64.  method: "max" or "avg".
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from ._cbuild import compile_shared

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pool_oracle.c")
_LIB = os.path.join(_HERE, "libpool_oracle.so")

OK, BAD_ARG, PAD_TOO_LARGE, WINDOW_TOO_LARGE = 0, 1, 2, 3
METHODS = {"max": 0, "avg": 1}


class OracleError(ValueError):
    def __init__(self, code):
        super().__init__({1: "bad argument", 2: "pad larger than window - 1", 3: "window larger than padded input"}.get(code, str(code)))
        self.code = code


class _Geom(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("H", "W", "D", "N", "Hp", "Wp", "Sh", "Sw", "Pt", "Pb", "Pl", "Pr", "method")]


def build(force: bool = False) -> str:
    return compile_shared(_SRC, _LIB, force)


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        P, G = ctypes.c_void_p, ctypes.POINTER(_Geom)
        lib.orp_output_size.argtypes = [G, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
        lib.orp_forward.argtypes = [G, P, P]
        lib.orp_backward.argtypes = [G, P, P, P]
        _lib = lib
    return _lib


def _geom(xshape, window, stride, pad, method):
    N, D, W, H = (int(v) for v in xshape)
    m = METHODS[method] if isinstance(method, str) else int(method)
    return _Geom(H, W, D, N, int(window[0]), int(window[1]), int(stride[0]), int(stride[1]),
                 int(pad[0]), int(pad[1]), int(pad[2]), int(pad[3]), m)


def _check(st):
    if st:
        raise OracleError(st)


def output_size(xshape, window, stride=(1, 1), pad=(0, 0, 0, 0), method="max"):
    g = _geom(xshape, window, stride, pad, method)
    ho, wo = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(_load().orp_output_size(ctypes.byref(g), ctypes.byref(ho), ctypes.byref(wo)))
    return ho.value, wo.value


def forward(x, window, stride=(1, 1), pad=(0, 0, 0, 0), method="max"):
    x = np.ascontiguousarray(x, dtype=np.float64)
    g = _geom(x.shape, window, stride, pad, method)
    ho, wo = output_size(x.shape, window, stride, pad, method)
    y = np.empty((x.shape[0], x.shape[1], wo, ho), dtype=np.float64)
    _check(_load().orp_forward(ctypes.byref(g), x.ctypes.data, y.ctypes.data))
    return y


def backward(x, dzdy, window, stride=(1, 1), pad=(0, 0, 0, 0), method="max"):
    x = np.ascontiguousarray(x, dtype=np.float64)
    g = _geom(x.shape, window, stride, pad, method)
    ho, wo = output_size(x.shape, window, stride, pad, method)
    dzdy = np.ascontiguousarray(dzdy, dtype=np.float64)
    if dzdy.shape != (x.shape[0], x.shape[1], wo, ho):
        raise ValueError("dzdy has shape %r, expected %r" % (dzdy.shape, (x.shape[0], x.shape[1], wo, ho)))
    dzdx = np.empty_like(x)
    _check(_load().orp_backward(ctypes.byref(g), x.ctypes.data, dzdy.ctypes.data, dzdx.ctypes.data))
    return dzdx
