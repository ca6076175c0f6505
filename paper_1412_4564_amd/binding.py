"""ctypes binding of libmcnconv.so: the same names as include/mcnconv.h.

Argument marshalling only -- every step of the convolution runs in the HIP
kernels behind the C ABI.  There is no CPU fallback: if the library is not
built, importing this module's functions raises.

Tensor convention: the manual's H x W x D x N arrays are first-index-fastest,
which is the memory order of a contiguous torch tensor of shape (N, D, W, H).
So x is (N,D,W,H), w is (K,Df,Wf,Hf), y and dzdy are (N,K,Wo,Ho), b is (K,).
For the convolution transpose the filter bank H' x W' x K' x D is (D,Kf,Wf,Hf) and y has
groups*Kf channels.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmcnconv.so")

MCN_OK, MCN_BAD_ARG, MCN_BAD_GROUPS, MCN_FILTER_TOO_LARGE = 0, 1, 2, 3
MCN_WORKSPACE_TOO_SMALL, MCN_UNSUPPORTED, MCN_HIP_ERROR, MCN_CROP_TOO_LARGE, MCN_PAD_TOO_LARGE = 4, 5, 6, 7, 8
MCN_STATIC_SCRATCH_EXCEEDED = 9
MCN_STATIC_SCRATCH_BYTES = 1 << 20
MCN_POOL_MAX, MCN_POOL_AVG = 0, 1
MCN_OP_FORWARD, MCN_OP_BACKWARD_DATA, MCN_OP_BACKWARD_FILTER, MCN_OP_BACKWARD_BIAS = 0, 1, 2, 3
MCN_OP_BACKWARD_FILTER_BIAS = 4
MCN_PREC_FP32, MCN_PREC_BF16, MCN_PREC_FP32_PLAIN, MCN_PREC_FP32_BF16X3 = 0, 1, 2, 3

EXPORTS = (
    "mcn_conv_output_size", "mcn_conv_workspace_size", "mcn_conv_forward", "mcn_conv_backward_data",
    "mcn_conv_backward_filter", "mcn_conv_backward_bias", "mcn_conv_backward_filter_bias", "mcn_status_string",
    "mcn_last_hip_error",
    "mcn_conv_kernel_name", "mcn_conv_relu_forward", "mcn_conv_relu_backward_bias",
    "mcn_convt_output_size", "mcn_convt_workspace_size", "mcn_convt_forward", "mcn_convt_backward_data",
    "mcn_convt_backward_filter", "mcn_convt_backward_bias", "mcn_convt_kernel_name",
    "mcn_pool_output_size", "mcn_pool_workspace_size", "mcn_pool_forward", "mcn_pool_backward",
    "mcn_probe_mfma", "mcn_probe_copy", "mcn_conv_backward_bias_static",
)
MCN_PROBE_SINK_FLOATS = 2048 * 256


class mcn_conv_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "H", "W", "D", "N", "Hf", "Wf", "Df", "K", "stride_h", "stride_w",
        "pad_top", "pad_bottom", "pad_left", "pad_right", "precision")]


class mcn_convt_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "H", "W", "D", "N", "Hf", "Wf", "Kf", "groups", "up_h", "up_w",
        "crop_top", "crop_bottom", "crop_left", "crop_right", "precision")]


class mcn_pool_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "H", "W", "D", "N", "Hp", "Wp", "stride_h", "stride_w",
        "pad_top", "pad_bottom", "pad_left", "pad_right", "method")]


class McnError(RuntimeError):
    def __init__(self, status, where=""):
        self.status = int(status)
        msg = lib().mcn_status_string(self.status).decode()
        if self.status == MCN_HIP_ERROR:
            msg += " (hipError %d)" % lib().mcn_last_hip_error()
        super().__init__("%s: %s" % (where, msg) if where else msg)


_lib = None


def lib():
    """Load libmcnconv.so (built by paper_1412_4564_amd.build); fails loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is not built: run `python -m paper_1412_4564_amd.build`" % LIB_PATH)
        # PyTorch bundles its own HIP runtime under the same soname.  Import it first so that
        # this library binds to the runtime that owns the tensors and streams it is handed;
        # the other order leaves two runtimes in the process and launches fail with "no device".
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        D = ctypes.POINTER(mcn_conv_desc)
        P, SZ, I32P = ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_int32)
        L.mcn_conv_output_size.argtypes = [D, I32P, I32P]
        L.mcn_conv_workspace_size.argtypes = [D, ctypes.c_int, ctypes.POINTER(SZ)]
        L.mcn_conv_forward.argtypes = [D, P, P, P, P, P, SZ, P]
        L.mcn_conv_backward_data.argtypes = [D, P, P, P, P, SZ, P]
        L.mcn_conv_backward_filter.argtypes = [D, P, P, P, P, SZ, P]
        L.mcn_conv_backward_bias.argtypes = [D, P, P, P, SZ, P]
        L.mcn_conv_backward_filter_bias.argtypes = [D, P, P, P, P, P, SZ, P]
        L.mcn_conv_backward_filter_bias.restype = ctypes.c_int
        L.mcn_conv_backward_bias_static.argtypes = [D, P, P, P]
        L.mcn_conv_backward_bias_static.restype = ctypes.c_int
        L.mcn_status_string.argtypes = [ctypes.c_int]
        L.mcn_status_string.restype = ctypes.c_char_p
        L.mcn_last_hip_error.restype = ctypes.c_int
        L.mcn_conv_kernel_name.argtypes = [D, ctypes.c_int]
        L.mcn_conv_kernel_name.restype = ctypes.c_char_p
        L.mcn_conv_relu_forward.argtypes = [D, P, P, P, P, P, SZ, P]
        L.mcn_conv_relu_backward_bias.argtypes = [D, P, P, P, P, P, SZ, P]
        L.mcn_conv_relu_forward.restype = ctypes.c_int
        L.mcn_conv_relu_backward_bias.restype = ctypes.c_int
        PD = ctypes.POINTER(mcn_pool_desc)
        L.mcn_pool_output_size.argtypes = [PD, I32P, I32P]
        L.mcn_pool_forward.argtypes = [PD, P, P, P]
        L.mcn_pool_backward.argtypes = [PD, P, P, P, P, SZ, P]
        L.mcn_pool_workspace_size.argtypes = [PD, ctypes.POINTER(SZ)]
        for f in ("mcn_pool_output_size", "mcn_pool_workspace_size", "mcn_pool_forward", "mcn_pool_backward"):
            getattr(L, f).restype = ctypes.c_int
        L.mcn_probe_mfma.argtypes = [ctypes.c_int, ctypes.c_int32, P, SZ, ctypes.POINTER(ctypes.c_double), P]
        L.mcn_probe_copy.argtypes = [P, P, SZ, P]
        L.mcn_probe_mfma.restype = L.mcn_probe_copy.restype = ctypes.c_int
        T = ctypes.POINTER(mcn_convt_desc)
        L.mcn_convt_output_size.argtypes = [T, I32P, I32P]
        L.mcn_convt_workspace_size.argtypes = [T, ctypes.c_int, ctypes.POINTER(SZ)]
        L.mcn_convt_forward.argtypes = [T, P, P, P, P, P, SZ, P]
        L.mcn_convt_backward_data.argtypes = [T, P, P, P, P, SZ, P]
        L.mcn_convt_backward_filter.argtypes = [T, P, P, P, P, SZ, P]
        L.mcn_convt_backward_bias.argtypes = [T, P, P, P, SZ, P]
        L.mcn_convt_kernel_name.argtypes = [T, ctypes.c_int]
        L.mcn_convt_kernel_name.restype = ctypes.c_char_p
        for f in ("mcn_conv_output_size", "mcn_conv_workspace_size", "mcn_conv_forward",
                  "mcn_conv_backward_data", "mcn_conv_backward_filter", "mcn_conv_backward_bias",
                  "mcn_convt_output_size", "mcn_convt_workspace_size", "mcn_convt_forward",
                  "mcn_convt_backward_data", "mcn_convt_backward_filter", "mcn_convt_backward_bias"):
            getattr(L, f).restype = ctypes.c_int
        _lib = L
    return _lib


def make_desc(xshape, wshape, stride=(1, 1), pad=(0, 0, 0, 0), precision=MCN_PREC_FP32):
    """Descriptor from tensor shapes x (N,D,W,H), w (K,Df,Wf,Hf), stride (Sh,Sw), pad (t,b,l,r)."""
    N, D, W, H = (int(v) for v in xshape)
    K, Df, Wf, Hf = (int(v) for v in wshape)
    return mcn_conv_desc(H, W, D, N, Hf, Wf, Df, K, int(stride[0]), int(stride[1]),
                         int(pad[0]), int(pad[1]), int(pad[2]), int(pad[3]), int(precision))


# ---- raw calls: same names and argument order as the C header; pointers are ints ----
def mcn_conv_output_size(desc):
    ho, wo = ctypes.c_int32(0), ctypes.c_int32(0)
    st = lib().mcn_conv_output_size(ctypes.byref(desc), ctypes.byref(ho), ctypes.byref(wo))
    if st:
        raise McnError(st, "mcn_conv_output_size")
    return ho.value, wo.value


def mcn_conv_workspace_size(desc, op):
    n = ctypes.c_size_t(0)
    st = lib().mcn_conv_workspace_size(ctypes.byref(desc), int(op), ctypes.byref(n))
    if st:
        raise McnError(st, "mcn_conv_workspace_size")
    return int(n.value)


def mcn_conv_kernel_name(desc, op):
    s = lib().mcn_conv_kernel_name(ctypes.byref(desc), int(op))
    return None if s is None else s.decode()


def mcn_conv_forward(desc, x, w, b, y, ws, ws_bytes, stream):
    return lib().mcn_conv_forward(ctypes.byref(desc), x, w, b, y, ws, ws_bytes, stream)


def mcn_conv_backward_data(desc, w, dzdy, dzdx, ws, ws_bytes, stream):
    return lib().mcn_conv_backward_data(ctypes.byref(desc), w, dzdy, dzdx, ws, ws_bytes, stream)


def mcn_conv_backward_filter(desc, x, dzdy, dzdw, ws, ws_bytes, stream):
    return lib().mcn_conv_backward_filter(ctypes.byref(desc), x, dzdy, dzdw, ws, ws_bytes, stream)


def mcn_conv_backward_filter_bias(desc, x, dzdy, dzdw, dzdb, ws, ws_bytes, stream):
    return lib().mcn_conv_backward_filter_bias(ctypes.byref(desc), x, dzdy, dzdw, dzdb, ws, ws_bytes, stream)


def mcn_conv_backward_bias(desc, dzdy, dzdb, ws, ws_bytes, stream):
    return lib().mcn_conv_backward_bias(ctypes.byref(desc), dzdy, dzdb, ws, ws_bytes, stream)


def mcn_conv_backward_bias_static(desc, dzdy, dzdb, stream):
    return lib().mcn_conv_backward_bias_static(ctypes.byref(desc), dzdy, dzdb, stream)


def mcn_conv_relu_forward(desc, x, w, b, y, ws, ws_bytes, stream):
    return lib().mcn_conv_relu_forward(ctypes.byref(desc), x, w, b, y, ws, ws_bytes, stream)


def mcn_conv_relu_backward_bias(desc, y, dzdy, dzdp, dzdb, ws, ws_bytes, stream):
    return lib().mcn_conv_relu_backward_bias(ctypes.byref(desc), y, dzdy, dzdp, dzdb, ws, ws_bytes, stream)


def make_pool_desc(xshape, window, stride=(1, 1), pad=(0, 0, 0, 0), method=MCN_POOL_MAX):
    """Descriptor from x's shape (N,D,W,H), window (Hp,Wp), stride (Sh,Sw), pad (t,b,l,r)."""
    N, D, W, H = (int(v) for v in xshape)
    return mcn_pool_desc(H, W, D, N, int(window[0]), int(window[1]), int(stride[0]), int(stride[1]),
                         int(pad[0]), int(pad[1]), int(pad[2]), int(pad[3]), int(method))


def mcn_pool_output_size(desc):
    ho, wo = ctypes.c_int32(0), ctypes.c_int32(0)
    st = lib().mcn_pool_output_size(ctypes.byref(desc), ctypes.byref(ho), ctypes.byref(wo))
    if st:
        raise McnError(st, "mcn_pool_output_size")
    return ho.value, wo.value


def mcn_pool_forward(desc, x, y, stream):
    return lib().mcn_pool_forward(ctypes.byref(desc), x, y, stream)


def mcn_pool_workspace_size(desc):
    n = ctypes.c_size_t(0)
    st = lib().mcn_pool_workspace_size(ctypes.byref(desc), ctypes.byref(n))
    if st:
        raise McnError(st, "mcn_pool_workspace_size")
    return int(n.value)


def mcn_pool_backward(desc, x, dzdy, dzdx, ws, ws_bytes, stream):
    return lib().mcn_pool_backward(ctypes.byref(desc), x, dzdy, dzdx, ws, ws_bytes, stream)


def mcn_probe_mfma(precision, iters, sink, sink_floats, stream):
    """Launches the register-only MFMA loop; returns (status, flops of the launch)."""
    flops = ctypes.c_double(0.0)
    st = lib().mcn_probe_mfma(int(precision), int(iters), sink, sink_floats, ctypes.byref(flops), stream)
    return st, flops.value


def mcn_probe_copy(src, dst, n, stream):
    return lib().mcn_probe_copy(src, dst, n, stream)


def make_convt_desc(xshape, fshape, upsample=(1, 1), crop=(0, 0, 0, 0), groups=1, precision=MCN_PREC_FP32):
    """Descriptor from tensor shapes x (N,D,W,H), f (D,Kf,Wf,Hf), upsample (Sh,Sw), crop (t,b,l,r)."""
    N, D, W, H = (int(v) for v in xshape)
    Df, Kf, Wf, Hf = (int(v) for v in fshape)
    if Df != D:
        raise ValueError("the filter bank's last axis (%d) must equal the input depth (%d)" % (Df, D))
    return mcn_convt_desc(H, W, D, N, Hf, Wf, Kf, int(groups), int(upsample[0]), int(upsample[1]),
                          int(crop[0]), int(crop[1]), int(crop[2]), int(crop[3]), int(precision))


def mcn_convt_output_size(desc):
    ho, wo = ctypes.c_int32(0), ctypes.c_int32(0)
    st = lib().mcn_convt_output_size(ctypes.byref(desc), ctypes.byref(ho), ctypes.byref(wo))
    if st:
        raise McnError(st, "mcn_convt_output_size")
    return ho.value, wo.value


def mcn_convt_workspace_size(desc, op):
    n = ctypes.c_size_t(0)
    st = lib().mcn_convt_workspace_size(ctypes.byref(desc), int(op), ctypes.byref(n))
    if st:
        raise McnError(st, "mcn_convt_workspace_size")
    return int(n.value)


def mcn_convt_kernel_name(desc, op):
    s = lib().mcn_convt_kernel_name(ctypes.byref(desc), int(op))
    return None if s is None else s.decode()


def mcn_convt_forward(desc, x, f, b, y, ws, ws_bytes, stream):
    return lib().mcn_convt_forward(ctypes.byref(desc), x, f, b, y, ws, ws_bytes, stream)


def mcn_convt_backward_data(desc, f, dzdy, dzdx, ws, ws_bytes, stream):
    return lib().mcn_convt_backward_data(ctypes.byref(desc), f, dzdy, dzdx, ws, ws_bytes, stream)


def mcn_convt_backward_filter(desc, x, dzdy, dzdf, ws, ws_bytes, stream):
    return lib().mcn_convt_backward_filter(ctypes.byref(desc), x, dzdy, dzdf, ws, ws_bytes, stream)


def mcn_convt_backward_bias(desc, dzdy, dzdb, ws, ws_bytes, stream):
    return lib().mcn_convt_backward_bias(ctypes.byref(desc), dzdy, dzdb, ws, ws_bytes, stream)


# ---- tensor-level helpers: allocate outputs / workspace with torch, pass pointers ----
def _check(t, shape, name):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise TypeError("%s must be a contiguous fp32 CUDA tensor" % name)
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s has shape %r, expected %r" % (name, tuple(t.shape), tuple(shape)))


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


class Workspace:
    """A reusable device scratch buffer (grown on demand, never shrunk)."""

    def __init__(self):
        self.buf = None

    def get(self, nbytes, device):
        import torch
        if nbytes == 0:
            return None, 0
        if self.buf is None or self.buf.numel() < nbytes or self.buf.device != device:
            self.buf = torch.empty(nbytes, dtype=torch.uint8, device=device)
        return self.buf.data_ptr(), self.buf.numel()


_default_ws = Workspace()


def conv_forward(x, w, b=None, stride=(1, 1), pad=(0, 0, 0, 0), precision=MCN_PREC_FP32, out=None, workspace=None):
    import torch
    _check(x, None, "x"); _check(w, None, "w")
    desc = make_desc(x.shape, w.shape, stride, pad, precision)
    ho, wo = mcn_conv_output_size(desc)
    if b is not None:
        _check(b, (w.shape[0],), "b")
    ysh = (x.shape[0], w.shape[0], wo, ho)
    y = out if out is not None else torch.empty(ysh, dtype=torch.float32, device=x.device)
    _check(y, ysh, "out")
    wsp, wsn = (workspace or _default_ws).get(mcn_conv_workspace_size(desc, MCN_OP_FORWARD), x.device)
    st = mcn_conv_forward(desc, x.data_ptr(), w.data_ptr(), None if b is None else b.data_ptr(), y.data_ptr(),
                          wsp, wsn, _stream())
    if st:
        raise McnError(st, "mcn_conv_forward")
    return y


def conv_backward_data(xshape, w, dzdy, stride=(1, 1), pad=(0, 0, 0, 0), precision=MCN_PREC_FP32, out=None, workspace=None):
    import torch
    _check(w, None, "w")
    desc = make_desc(xshape, w.shape, stride, pad, precision)
    ho, wo = mcn_conv_output_size(desc)
    _check(dzdy, (xshape[0], w.shape[0], wo, ho), "dzdy")
    dzdx = out if out is not None else torch.empty(tuple(xshape), dtype=torch.float32, device=w.device)
    _check(dzdx, tuple(xshape), "out")
    wsp, wsn = (workspace or _default_ws).get(mcn_conv_workspace_size(desc, MCN_OP_BACKWARD_DATA), w.device)
    st = mcn_conv_backward_data(desc, w.data_ptr(), dzdy.data_ptr(), dzdx.data_ptr(), wsp, wsn, _stream())
    if st:
        raise McnError(st, "mcn_conv_backward_data")
    return dzdx


def conv_backward_filter(x, wshape, dzdy, stride=(1, 1), pad=(0, 0, 0, 0), precision=MCN_PREC_FP32, out=None, workspace=None):
    import torch
    _check(x, None, "x")
    desc = make_desc(x.shape, wshape, stride, pad, precision)
    ho, wo = mcn_conv_output_size(desc)
    _check(dzdy, (x.shape[0], wshape[0], wo, ho), "dzdy")
    dzdw = out if out is not None else torch.empty(tuple(wshape), dtype=torch.float32, device=x.device)
    _check(dzdw, tuple(wshape), "out")
    wsp, wsn = (workspace or _default_ws).get(mcn_conv_workspace_size(desc, MCN_OP_BACKWARD_FILTER), x.device)
    st = mcn_conv_backward_filter(desc, x.data_ptr(), dzdy.data_ptr(), dzdw.data_ptr(), wsp, wsn, _stream())
    if st:
        raise McnError(st, "mcn_conv_backward_filter")
    return dzdw


def conv_backward_filter_bias(x, wshape, dzdy, stride=(1, 1), pad=(0, 0, 0, 0), precision=MCN_PREC_FP32, out=None, workspace=None):
    """(dzdw, dzdb) in one call; out = (dzdw, dzdb) to write into existing tensors."""
    import torch
    _check(x, None, "x")
    desc = make_desc(x.shape, wshape, stride, pad, precision)
    ho, wo = mcn_conv_output_size(desc)
    _check(dzdy, (x.shape[0], wshape[0], wo, ho), "dzdy")
    dzdw = out[0] if out is not None else torch.empty(tuple(wshape), dtype=torch.float32, device=x.device)
    dzdb = out[1] if out is not None else torch.empty((wshape[0],), dtype=torch.float32, device=x.device)
    _check(dzdw, tuple(wshape), "out[0]")
    _check(dzdb, (wshape[0],), "out[1]")
    wsp, wsn = (workspace or _default_ws).get(mcn_conv_workspace_size(desc, MCN_OP_BACKWARD_FILTER_BIAS), x.device)
    st = mcn_conv_backward_filter_bias(desc, x.data_ptr(), dzdy.data_ptr(), dzdw.data_ptr(), dzdb.data_ptr(), wsp, wsn, _stream())
    if st:
        raise McnError(st, "mcn_conv_backward_filter_bias")
    return dzdw, dzdb


def conv_backward_bias(xshape, wshape, dzdy, stride=(1, 1), pad=(0, 0, 0, 0), out=None, workspace=None):
    import torch
    desc = make_desc(xshape, wshape, stride, pad)
    ho, wo = mcn_conv_output_size(desc)
    _check(dzdy, (xshape[0], wshape[0], wo, ho), "dzdy")
    dzdb = out if out is not None else torch.empty((wshape[0],), dtype=torch.float32, device=dzdy.device)
    _check(dzdb, (wshape[0],), "out")
    wsp, wsn = (workspace or _default_ws).get(mcn_conv_workspace_size(desc, MCN_OP_BACKWARD_BIAS), dzdy.device)
    st = mcn_conv_backward_bias(desc, dzdy.data_ptr(), dzdb.data_ptr(), wsp, wsn, _stream())
    if st:
        raise McnError(st, "mcn_conv_backward_bias")
    return dzdb


# ---- convolution + ReLU ----
def conv_relu_forward(x, w, b=None, stride=(1, 1), pad=(0, 0, 0, 0), precision=MCN_PREC_FP32, out=None, workspace=None):
    import torch
    _check(x, None, "x"); _check(w, None, "w")
    desc = make_desc(x.shape, w.shape, stride, pad, precision)
    ho, wo = mcn_conv_output_size(desc)
    if b is not None:
        _check(b, (w.shape[0],), "b")
    ysh = (x.shape[0], w.shape[0], wo, ho)
    y = out if out is not None else torch.empty(ysh, dtype=torch.float32, device=x.device)
    _check(y, ysh, "out")
    wsp, wsn = (workspace or _default_ws).get(mcn_conv_workspace_size(desc, MCN_OP_FORWARD), x.device)
    st = mcn_conv_relu_forward(desc, x.data_ptr(), w.data_ptr(), None if b is None else b.data_ptr(), y.data_ptr(),
                               wsp, wsn, _stream())
    if st:
        raise McnError(st, "mcn_conv_relu_forward")
    return y


def conv_relu_backward_bias(xshape, wshape, y, dzdy, stride=(1, 1), pad=(0, 0, 0, 0), out=None, inplace=False,
                            workspace=None):
    """Returns (dzdp, dzdb); with inplace=True dzdp overwrites dzdy."""
    import torch
    desc = make_desc(xshape, wshape, stride, pad)
    ho, wo = mcn_conv_output_size(desc)
    ysh = (xshape[0], wshape[0], wo, ho)
    _check(y, ysh, "y"); _check(dzdy, ysh, "dzdy")
    dzdp = dzdy if inplace else (out if out is not None else torch.empty_like(dzdy))
    _check(dzdp, ysh, "out")
    dzdb = torch.empty((wshape[0],), dtype=torch.float32, device=dzdy.device)
    wsp, wsn = (workspace or _default_ws).get(mcn_conv_workspace_size(desc, MCN_OP_BACKWARD_BIAS), dzdy.device)
    st = mcn_conv_relu_backward_bias(desc, y.data_ptr(), dzdy.data_ptr(), dzdp.data_ptr(), dzdb.data_ptr(), wsp, wsn,
                                     _stream())
    if st:
        raise McnError(st, "mcn_conv_relu_backward_bias")
    return dzdp, dzdb


# ---- convolution transpose ----
def _convt_shapes(xshape, fshape, upsample, crop, groups, precision=MCN_PREC_FP32):
    desc = make_convt_desc(xshape, fshape, upsample, crop, groups, precision)
    ho, wo = mcn_convt_output_size(desc)
    return desc, (int(xshape[0]), int(groups) * int(fshape[1]), wo, ho)


def convt_forward(x, f, b=None, upsample=(1, 1), crop=(0, 0, 0, 0), groups=1, precision=MCN_PREC_FP32, out=None,
                  workspace=None):
    import torch
    _check(x, None, "x"); _check(f, None, "f")
    desc, ysh = _convt_shapes(x.shape, f.shape, upsample, crop, groups, precision)
    if b is not None:
        _check(b, (ysh[1],), "b")
    y = out if out is not None else torch.empty(ysh, dtype=torch.float32, device=x.device)
    _check(y, ysh, "out")
    wsp, wsn = (workspace or _default_ws).get(mcn_convt_workspace_size(desc, MCN_OP_FORWARD), x.device)
    st = mcn_convt_forward(desc, x.data_ptr(), f.data_ptr(), None if b is None else b.data_ptr(), y.data_ptr(),
                           wsp, wsn, _stream())
    if st:
        raise McnError(st, "mcn_convt_forward")
    return y


def convt_backward_data(xshape, f, dzdy, upsample=(1, 1), crop=(0, 0, 0, 0), groups=1, precision=MCN_PREC_FP32,
                        out=None, workspace=None):
    import torch
    _check(f, None, "f")
    desc, ysh = _convt_shapes(xshape, f.shape, upsample, crop, groups, precision)
    _check(dzdy, ysh, "dzdy")
    dzdx = out if out is not None else torch.empty(tuple(xshape), dtype=torch.float32, device=f.device)
    _check(dzdx, tuple(xshape), "out")
    wsp, wsn = (workspace or _default_ws).get(mcn_convt_workspace_size(desc, MCN_OP_BACKWARD_DATA), f.device)
    st = mcn_convt_backward_data(desc, f.data_ptr(), dzdy.data_ptr(), dzdx.data_ptr(), wsp, wsn, _stream())
    if st:
        raise McnError(st, "mcn_convt_backward_data")
    return dzdx


def convt_backward_filter(x, fshape, dzdy, upsample=(1, 1), crop=(0, 0, 0, 0), groups=1, precision=MCN_PREC_FP32,
                          out=None, workspace=None):
    import torch
    _check(x, None, "x")
    desc, ysh = _convt_shapes(x.shape, fshape, upsample, crop, groups, precision)
    _check(dzdy, ysh, "dzdy")
    dzdf = out if out is not None else torch.empty(tuple(fshape), dtype=torch.float32, device=x.device)
    _check(dzdf, tuple(fshape), "out")
    wsp, wsn = (workspace or _default_ws).get(mcn_convt_workspace_size(desc, MCN_OP_BACKWARD_FILTER), x.device)
    st = mcn_convt_backward_filter(desc, x.data_ptr(), dzdy.data_ptr(), dzdf.data_ptr(), wsp, wsn, _stream())
    if st:
        raise McnError(st, "mcn_convt_backward_filter")
    return dzdf


def convt_backward_bias(xshape, fshape, dzdy, upsample=(1, 1), crop=(0, 0, 0, 0), groups=1, out=None, workspace=None):
    import torch
    desc, ysh = _convt_shapes(xshape, fshape, upsample, crop, groups)
    _check(dzdy, ysh, "dzdy")
    dzdb = out if out is not None else torch.empty((ysh[1],), dtype=torch.float32, device=dzdy.device)
    _check(dzdb, (ysh[1],), "out")
    wsp, wsn = (workspace or _default_ws).get(mcn_convt_workspace_size(desc, MCN_OP_BACKWARD_BIAS), dzdy.device)
    st = mcn_convt_backward_bias(desc, dzdy.data_ptr(), dzdb.data_ptr(), wsp, wsn, _stream())
    if st:
        raise McnError(st, "mcn_convt_backward_bias")
    return dzdb


# ---- spatial pooling ----
def pool_forward(x, window, stride=(1, 1), pad=(0, 0, 0, 0), method=MCN_POOL_MAX, out=None):
    import torch
    _check(x, None, "x")
    desc = make_pool_desc(x.shape, window, stride, pad, method)
    ho, wo = mcn_pool_output_size(desc)
    ysh = (x.shape[0], x.shape[1], wo, ho)
    y = out if out is not None else torch.empty(ysh, dtype=torch.float32, device=x.device)
    _check(y, ysh, "out")
    st = mcn_pool_forward(desc, x.data_ptr(), y.data_ptr(), _stream())
    if st:
        raise McnError(st, "mcn_pool_forward")
    return y


def pool_backward(x, dzdy, window, stride=(1, 1), pad=(0, 0, 0, 0), method=MCN_POOL_MAX, out=None, workspace=None):
    import torch
    _check(x, None, "x")
    desc = make_pool_desc(x.shape, window, stride, pad, method)
    ho, wo = mcn_pool_output_size(desc)
    _check(dzdy, (x.shape[0], x.shape[1], wo, ho), "dzdy")
    dzdx = out if out is not None else torch.empty_like(x)
    _check(dzdx, tuple(x.shape), "out")
    wsp, wsn = (workspace or _default_ws).get(mcn_pool_workspace_size(desc), x.device)
    st = mcn_pool_backward(desc, x.data_ptr(), dzdy.data_ptr(), dzdx.data_ptr(), wsp, wsn, _stream())
    if st:
        raise McnError(st, "mcn_pool_backward")
    return dzdx
