"""CPU oracle for the convolution transpose block: thin ctypes wrapper over
convt_oracle.c.

TEST INFRASTRUCTURE ONLY (see the header of convt_oracle.c).  All arithmetic
lives in the C file (fp64); this module only marshals numpy arrays.

Array convention: H x W x D x N arrays stored first index fastest are numpy
arrays of shape (N, D, W, H) in C order.  Hence
    x (N, D, W, H),  f (D, Kf, Wf, Hf),  y (N, G*Kf, Wo, Ho),  b (G*Kf,)
where the filter bank's THIRD axis (Kf) runs over output channels and its
FOURTH (D) over input channels (Sec. 4.2 of the manual).
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from ._cbuild import compile_shared

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "convt_oracle.c")
_LIB = os.path.join(_HERE, "libconvt_oracle.so")

OK, BAD_ARG, BAD_GROUPS, CROP_TOO_LARGE = 0, 1, 2, 3


class OracleError(ValueError):
    def __init__(self, code):
        super().__init__({1: "bad argument", 2: "bad groups", 3: "crops leave no output"}.get(code, str(code)))
        self.code = code


class _Geom(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("H", "W", "D", "N", "Hf", "Wf", "Kf", "G", "Uh", "Uw", "Ct", "Cb", "Cl", "Cr")]


def build(force: bool = False) -> str:
    return compile_shared(_SRC, _LIB, force)


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        P = ctypes.c_void_p
        G = ctypes.POINTER(_Geom)
        I64 = ctypes.c_int64
        lib.orct_output_size.argtypes = [G, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
        lib.orct_forward.argtypes = [G, P, P, P, P]
        lib.orct_forward_at.argtypes = [G, P, P, P, P, I64, P]
        lib.orct_backward_data.argtypes = [G, P, P, P]
        lib.orct_backward_data_at.argtypes = [G, P, P, P, I64, P]
        lib.orct_backward_filter.argtypes = [G, P, P, P]
        lib.orct_backward_filter_at.argtypes = [G, P, P, P, I64, P]
        lib.orct_backward_bias.argtypes = [G, P, P]
        lib.orct_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().orct_num_threads())


def _geom(xshape, fshape, upsample, crop, groups):
    N, D, W, H = (int(v) for v in xshape)
    Df, Kf, Wf, Hf = (int(v) for v in fshape)
    if Df != D:
        raise ValueError("the filter bank's last axis (%d) must equal the input depth (%d)" % (Df, D))
    Uh, Uw = (int(v) for v in upsample)
    Ct, Cb, Cl, Cr = (int(v) for v in crop)
    return _Geom(H, W, D, N, Hf, Wf, Kf, int(groups), Uh, Uw, Ct, Cb, Cl, Cr)


def _f64(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError("array has shape %r, expected %r" % (a.shape, tuple(shape)))
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data


def _check(st):
    if st:
        raise OracleError(st)


def output_size(xshape, fshape, upsample=(1, 1), crop=(0, 0, 0, 0), groups=1):
    """(Ho, Wo) = (U_h (H-1) + H' - crops, ...) of Sec. 4.2; raises OracleError on bad geometry."""
    g = _geom(xshape, fshape, upsample, crop, groups)
    ho, wo = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(_load().orct_output_size(ctypes.byref(g), ctypes.byref(ho), ctypes.byref(wo)))
    return ho.value, wo.value


def _yshape(xshape, fshape, upsample, crop, groups):
    ho, wo = output_size(xshape, fshape, upsample, crop, groups)
    return (int(xshape[0]), int(groups) * int(fshape[1]), wo, ho)


def forward(x, f, b=None, upsample=(1, 1), crop=(0, 0, 0, 0), groups=1):
    x, f = _f64(x), _f64(f)
    g = _geom(x.shape, f.shape, upsample, crop, groups)
    ysh = _yshape(x.shape, f.shape, upsample, crop, groups)
    bb = None if b is None else _f64(b, (ysh[1],))
    y = np.empty(ysh, dtype=np.float64)
    _check(_load().orct_forward(ctypes.byref(g), _ptr(x), _ptr(f), _ptr(bb), _ptr(y)))
    return y


def forward_at(x, f, b, idx, upsample=(1, 1), crop=(0, 0, 0, 0), groups=1):
    """Forward at the linear addresses idx (into y's memory)."""
    x, f = _f64(x), _f64(f)
    g = _geom(x.shape, f.shape, upsample, crop, groups)
    ysh = _yshape(x.shape, f.shape, upsample, crop, groups)
    bb = None if b is None else _f64(b, (ysh[1],))
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.empty(idx.shape, dtype=np.float64)
    _check(_load().orct_forward_at(ctypes.byref(g), _ptr(x), _ptr(f), _ptr(bb), _ptr(idx), idx.size, _ptr(out)))
    return out


def backward_data(xshape, f, dzdy, upsample=(1, 1), crop=(0, 0, 0, 0), groups=1):
    f = _f64(f)
    g = _geom(xshape, f.shape, upsample, crop, groups)
    dzdy = _f64(dzdy, _yshape(xshape, f.shape, upsample, crop, groups))
    dzdx = np.empty(tuple(int(v) for v in xshape), dtype=np.float64)
    _check(_load().orct_backward_data(ctypes.byref(g), _ptr(f), _ptr(dzdy), _ptr(dzdx)))
    return dzdx


def backward_data_at(xshape, f, dzdy, idx, upsample=(1, 1), crop=(0, 0, 0, 0), groups=1):
    f = _f64(f)
    g = _geom(xshape, f.shape, upsample, crop, groups)
    dzdy = _f64(dzdy, _yshape(xshape, f.shape, upsample, crop, groups))
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.empty(idx.shape, dtype=np.float64)
    _check(_load().orct_backward_data_at(ctypes.byref(g), _ptr(f), _ptr(dzdy), _ptr(idx), idx.size, _ptr(out)))
    return out


def backward_filter(x, fshape, dzdy, upsample=(1, 1), crop=(0, 0, 0, 0), groups=1):
    x = _f64(x)
    g = _geom(x.shape, fshape, upsample, crop, groups)
    dzdy = _f64(dzdy, _yshape(x.shape, fshape, upsample, crop, groups))
    dzdf = np.empty(tuple(int(v) for v in fshape), dtype=np.float64)
    _check(_load().orct_backward_filter(ctypes.byref(g), _ptr(x), _ptr(dzdy), _ptr(dzdf)))
    return dzdf


def backward_filter_at(x, fshape, dzdy, idx, upsample=(1, 1), crop=(0, 0, 0, 0), groups=1):
    x = _f64(x)
    g = _geom(x.shape, fshape, upsample, crop, groups)
    dzdy = _f64(dzdy, _yshape(x.shape, fshape, upsample, crop, groups))
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.empty(idx.shape, dtype=np.float64)
    _check(_load().orct_backward_filter_at(ctypes.byref(g), _ptr(x), _ptr(dzdy), _ptr(idx), idx.size, _ptr(out)))
    return out


def backward_bias(xshape, fshape, dzdy, upsample=(1, 1), crop=(0, 0, 0, 0), groups=1):
    g = _geom(xshape, fshape, upsample, crop, groups)
    ysh = _yshape(xshape, fshape, upsample, crop, groups)
    dzdy = _f64(dzdy, ysh)
    dzdb = np.empty((ysh[1],), dtype=np.float64)
    _check(_load().orct_backward_bias(ctypes.byref(g), _ptr(dzdy), _ptr(dzdb)))
    return dzdb
