"""CPU oracle for the convolution block: thin ctypes wrapper over conv_oracle.c.

TEST INFRASTRUCTURE ONLY.  Tests, the smoke check and the benchmark's CPU
baseline may import this; the product package never does, and this module
imports nothing from the product package.  All arithmetic lives in
conv_oracle.c (plain C, fp64); this file only marshals numpy arrays.

Array convention: the manual's H x W x D x N arrays are stored first index
fastest (Sec. 2.3.1, the vec() order).  A numpy array of shape (N, D, W, H)
in C order has exactly that memory order, so that is the shape used here:
x (N,D,W,H), f (K,Df,Wf,Hf), y (N,K,Wo,Ho), b (K,).
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from ._cbuild import compile_shared

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_LIB = os.path.join(_HERE, "libconv_oracle.so")

OK, BAD_ARG, BAD_GROUPS, FILTER_TOO_LARGE = 0, 1, 2, 3


class OracleError(ValueError):
    def __init__(self, code):
        super().__init__({1: "bad argument", 2: "bad groups", 3: "filter larger than padded input"}.get(code, str(code)))
        self.code = code


class _Geom(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("H", "W", "D", "N", "Hf", "Wf", "Df", "K", "Sh", "Sw", "Pt", "Pb", "Pl", "Pr")]


def build(force: bool = False) -> str:
    """Compile every C file of the oracle (this block's and those of the convolution transpose, ReLU and pooling blocks)."""
    from . import convt, pool, relu
    convt.build(force)
    relu.build(force)
    pool.build(force)
    return compile_shared(_SRC, _LIB, force)


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        P = ctypes.c_void_p
        G = ctypes.POINTER(_Geom)
        I64 = ctypes.c_int64
        lib.orc_output_size.argtypes = [G, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
        lib.orc_forward.argtypes = [G, P, P, P, P]
        lib.orc_forward_at.argtypes = [G, P, P, P, P, I64, P]
        lib.orc_backward_data.argtypes = [G, P, P, P]
        lib.orc_backward_data_at.argtypes = [G, P, P, P, I64, P]
        lib.orc_backward_filter.argtypes = [G, P, P, P]
        lib.orc_backward_filter_at.argtypes = [G, P, P, P, I64, P]
        lib.orc_backward_bias.argtypes = [G, P, P]
        lib.orc_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().orc_num_threads())


def _geom(xshape, fshape, stride, pad):
    N, D, W, H = (int(v) for v in xshape)
    K, Df, Wf, Hf = (int(v) for v in fshape)
    Sh, Sw = (int(v) for v in stride)
    Pt, Pb, Pl, Pr = (int(v) for v in pad)
    return _Geom(H, W, D, N, Hf, Wf, Df, K, Sh, Sw, Pt, Pb, Pl, Pr)


def _f64(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError("array has shape %r, expected %r" % (a.shape, tuple(shape)))
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data


def output_size(xshape, fshape, stride=(1, 1), pad=(0, 0, 0, 0)):
    """(Ho, Wo) from Sec. 4.1 'Output size'; raises OracleError on bad geometry."""
    g = _geom(xshape, fshape, stride, pad)
    ho, wo = ctypes.c_int32(0), ctypes.c_int32(0)
    st = _load().orc_output_size(ctypes.byref(g), ctypes.byref(ho), ctypes.byref(wo))
    if st:
        raise OracleError(st)
    return ho.value, wo.value


def _yshape(x_shape, f_shape, stride, pad):
    ho, wo = output_size(x_shape, f_shape, stride, pad)
    return (int(x_shape[0]), int(f_shape[0]), wo, ho)


def forward(x, f, b=None, stride=(1, 1), pad=(0, 0, 0, 0)):
    x, f = _f64(x), _f64(f)
    g = _geom(x.shape, f.shape, stride, pad)
    ysh = _yshape(x.shape, f.shape, stride, pad)
    bb = None if b is None else _f64(b, (f.shape[0],))
    y = np.empty(ysh, dtype=np.float64)
    st = _load().orc_forward(ctypes.byref(g), _ptr(x), _ptr(f), _ptr(bb), _ptr(y))
    if st:
        raise OracleError(st)
    return y


def forward_at(x, f, b, idx, stride=(1, 1), pad=(0, 0, 0, 0)):
    """Forward at the linear addresses idx (into y's memory)."""
    x, f = _f64(x), _f64(f)
    g = _geom(x.shape, f.shape, stride, pad)
    bb = None if b is None else _f64(b, (f.shape[0],))
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.empty(idx.shape, dtype=np.float64)
    st = _load().orc_forward_at(ctypes.byref(g), _ptr(x), _ptr(f), _ptr(bb), _ptr(idx), idx.size, _ptr(out))
    if st:
        raise OracleError(st)
    return out


def backward_data(xshape, f, dzdy, stride=(1, 1), pad=(0, 0, 0, 0)):
    f = _f64(f)
    g = _geom(xshape, f.shape, stride, pad)
    dzdy = _f64(dzdy, _yshape(xshape, f.shape, stride, pad))
    dzdx = np.empty(tuple(int(v) for v in xshape), dtype=np.float64)
    st = _load().orc_backward_data(ctypes.byref(g), _ptr(f), _ptr(dzdy), _ptr(dzdx))
    if st:
        raise OracleError(st)
    return dzdx


def backward_data_at(xshape, f, dzdy, idx, stride=(1, 1), pad=(0, 0, 0, 0)):
    f = _f64(f)
    g = _geom(xshape, f.shape, stride, pad)
    dzdy = _f64(dzdy, _yshape(xshape, f.shape, stride, pad))
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.empty(idx.shape, dtype=np.float64)
    st = _load().orc_backward_data_at(ctypes.byref(g), _ptr(f), _ptr(dzdy), _ptr(idx), idx.size, _ptr(out))
    if st:
        raise OracleError(st)
    return out


def backward_filter(x, fshape, dzdy, stride=(1, 1), pad=(0, 0, 0, 0)):
    x = _f64(x)
    g = _geom(x.shape, fshape, stride, pad)
    dzdy = _f64(dzdy, _yshape(x.shape, fshape, stride, pad))
    dzdw = np.empty(tuple(int(v) for v in fshape), dtype=np.float64)
    st = _load().orc_backward_filter(ctypes.byref(g), _ptr(x), _ptr(dzdy), _ptr(dzdw))
    if st:
        raise OracleError(st)
    return dzdw


def backward_filter_at(x, fshape, dzdy, idx, stride=(1, 1), pad=(0, 0, 0, 0)):
    x = _f64(x)
    g = _geom(x.shape, fshape, stride, pad)
    dzdy = _f64(dzdy, _yshape(x.shape, fshape, stride, pad))
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.empty(idx.shape, dtype=np.float64)
    st = _load().orc_backward_filter_at(ctypes.byref(g), _ptr(x), _ptr(dzdy), _ptr(idx), idx.size, _ptr(out))
    if st:
        raise OracleError(st)
    return out


def backward_bias(xshape, fshape, dzdy, stride=(1, 1), pad=(0, 0, 0, 0)):
    g = _geom(xshape, fshape, stride, pad)
    dzdy = _f64(dzdy, _yshape(xshape, fshape, stride, pad))
    dzdb = np.empty((int(fshape[0]),), dtype=np.float64)
    st = _load().orc_backward_bias(ctypes.byref(g), _ptr(dzdy), _ptr(dzdb))
    if st:
        raise OracleError(st)
    return dzdb
