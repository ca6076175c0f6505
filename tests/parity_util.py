"""Shared helpers for the GPU-vs-oracle parity tests (test code only)."""
import numpy as np
import torch

import oracle
from paper_1412_4564_amd import binding as B
from paper_1412_4564_amd import synth

TOL_FWD = 1e-4      # fp32 forward
TOL_BWD = 1e-3      # fp32 backward passes
TOL_BF16 = 1e-2     # bf16-operand variant


def norm_err(got, ref, den):
    """max |got-ref| / den, where den is the same operator applied to absolute
    values (the sum of |w||x| over each result's receptive field).  Where den is 0 the
    result is structurally zero and must match exactly."""
    got = np.asarray(got, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    den = np.asarray(den, dtype=np.float64).ravel()
    assert got.shape == ref.shape == den.shape
    assert np.all(np.isfinite(got)), "non-finite values in GPU result"
    zero = den == 0
    if zero.any():
        assert np.all(got[zero] == 0.0), "structurally-zero results must be exactly 0"
    nz = ~zero
    if not nz.any():
        return 0.0
    return float(np.max(np.abs(got[nz] - ref[nz]) / den[nz]))


def layer_args(L):
    return dict(stride=L["stride"], pad=L["pad"])


def gpu(t, misalign=0):
    """Copy to the GPU; with misalign = 1..3 the copy starts that many floats past a 16-byte
    boundary (torch allocations are aligned to 256 bytes or more)."""
    if not misalign:
        return t.cuda()
    flat = torch.empty(t.numel() + 4, dtype=t.dtype, device="cuda")
    out = flat[misalign:misalign + t.numel()].view(t.shape)
    out.copy_(t)
    assert out.data_ptr() % 16 == 4 * misalign and out.is_contiguous()
    return out


def np64(t):
    return t.numpy().astype(np.float64)


def sample_idx(total, count, seed):
    rng = np.random.default_rng(seed)
    if total <= count:
        return np.arange(total, dtype=np.int64)
    idx = rng.choice(total, size=count, replace=False).astype(np.int64)
    # always include the very first and last elements (tile corners / ragged tails)
    idx[0], idx[1] = 0, total - 1
    return idx


def run_layer_full(L, precision=B.MCN_PREC_FP32, with_bias=True, seed=0, misalign=0):
    """All four operations on layer L, every element compared.  Returns dict of errors.
    misalign: the input arrays start that many floats past a 16-byte boundary."""
    st, pad = L["stride"], L["pad"]
    x, w, b = synth.make_x(L, seed), synth.make_w(L, seed), synth.make_b(L, seed)
    ho, wo = oracle.output_size(x.shape, w.shape, st, pad)
    p = synth.make_dzdy(L, ho, wo, seed)
    xd, wd, bd, pd = np64(x), np64(w), np64(b), np64(p)
    bb = bd if with_bias else None
    out = {}
    xg, wg, bg, pg = gpu(x, misalign), gpu(w, misalign), gpu(b), gpu(p, misalign)
    y = B.conv_forward(xg, wg, bg if with_bias else None, st, pad, precision)
    dx = B.conv_backward_data(x.shape, wg, pg, st, pad, precision)
    dw = B.conv_backward_filter(xg, w.shape, pg, st, pad, precision)
    db = B.conv_backward_bias(x.shape, w.shape, pg, st, pad)
    torch.cuda.synchronize()
    assert tuple(y.shape) == (L["N"], L["K"], wo, ho)
    out["forward"] = norm_err(y.cpu().numpy(), oracle.forward(xd, wd, bb, st, pad),
                              oracle.forward(np.abs(xd), np.abs(wd), None if bb is None else np.abs(bb), st, pad))
    out["backward_data"] = norm_err(dx.cpu().numpy(), oracle.backward_data(x.shape, wd, pd, st, pad),
                                    oracle.backward_data(x.shape, np.abs(wd), np.abs(pd), st, pad))
    out["backward_filter"] = norm_err(dw.cpu().numpy(), oracle.backward_filter(xd, w.shape, pd, st, pad),
                                      oracle.backward_filter(np.abs(xd), w.shape, np.abs(pd), st, pad))
    out["backward_bias"] = norm_err(db.cpu().numpy(), oracle.backward_bias(x.shape, w.shape, pd, st, pad),
                                    oracle.backward_bias(x.shape, w.shape, np.abs(pd), st, pad))
    return out


def run_layer_sampled(L, n_out=4000, n_filt=96, precision=B.MCN_PREC_FP32, seed=0):
    """All four operations at full size; y and dzdx compared at sampled places that the oracle computes one by
    one, dzdw at n_filt sampled places or (n_filt=None) everywhere, the bias derivative everywhere."""
    st, pad = L["stride"], L["pad"]
    x, w, b = synth.make_x(L, seed), synth.make_w(L, seed), synth.make_b(L, seed)
    ho, wo = oracle.output_size(x.shape, w.shape, st, pad)
    p = synth.make_dzdy(L, ho, wo, seed)
    xg, wg, bg, pg = gpu(x), gpu(w), gpu(b), gpu(p)
    y = B.conv_forward(xg, wg, bg, st, pad, precision)
    dx = B.conv_backward_data(x.shape, wg, pg, st, pad, precision)
    dw = B.conv_backward_filter(xg, w.shape, pg, st, pad, precision)
    db = B.conv_backward_bias(x.shape, w.shape, pg, st, pad)
    torch.cuda.synchronize()
    y, dx, dw, db = (t.cpu().numpy().ravel() for t in (y, dx, dw, db))
    del xg, wg, pg
    xd, wd, bd, pd = np64(x), np64(w), np64(b), np64(p)
    out = {}
    iy = sample_idx(y.size, n_out, 1)
    out["forward"] = norm_err(y[iy], oracle.forward_at(xd, wd, bd, iy, st, pad),
                              oracle.forward_at(np.abs(xd), np.abs(wd), np.abs(bd), iy, st, pad))
    ix = sample_idx(dx.size, n_out, 2)
    out["backward_data"] = norm_err(dx[ix], oracle.backward_data_at(x.shape, wd, pd, ix, st, pad),
                                    oracle.backward_data_at(x.shape, np.abs(wd), np.abs(pd), ix, st, pad))
    if n_filt is None:      # every filter coefficient
        out["backward_filter"] = norm_err(dw, oracle.backward_filter(xd, w.shape, pd, st, pad),
                                          oracle.backward_filter(np.abs(xd), w.shape, np.abs(pd), st, pad))
    else:
        iw = sample_idx(dw.size, n_filt, 3)
        out["backward_filter"] = norm_err(dw[iw], oracle.backward_filter_at(xd, w.shape, pd, iw, st, pad),
                                          oracle.backward_filter_at(np.abs(xd), w.shape, np.abs(pd), iw, st, pad))
    out["backward_bias"] = norm_err(db, oracle.backward_bias(x.shape, w.shape, pd, st, pad),
                                    oracle.backward_bias(x.shape, w.shape, np.abs(pd), st, pad))
    return out


class OracleResults:
    """The four results of the oracle for layer L and their normalisers (the same operators on absolute values), every
    element, computed once so that several GPU runs (summation orders, entry points) can be compared with them."""

    def __init__(self, L, seed=0, filter_only=False):
        self.L, self.st, self.pad = L, L["stride"], L["pad"]
        st, pad = self.st, self.pad
        self.x, self.w, self.b = synth.make_x(L, seed), synth.make_w(L, seed), synth.make_b(L, seed)
        self.ho, self.wo = oracle.output_size(self.x.shape, self.w.shape, st, pad)
        self.p = synth.make_dzdy(L, self.ho, self.wo, seed)
        xd, wd, bd, pd = np64(self.x), np64(self.w), np64(self.b), np64(self.p)
        xs, ws = self.x.shape, self.w.shape
        if not filter_only:
            self.y, self.y_den = oracle.forward(xd, wd, bd, st, pad), oracle.forward(np.abs(xd), np.abs(wd), np.abs(bd), st, pad)
            self.dx, self.dx_den = oracle.backward_data(xs, wd, pd, st, pad), oracle.backward_data(xs, np.abs(wd), np.abs(pd), st, pad)
        self.dw, self.dw_den = oracle.backward_filter(xd, ws, pd, st, pad), oracle.backward_filter(np.abs(xd), ws, np.abs(pd), st, pad)
        self.db, self.db_den = oracle.backward_bias(xs, ws, pd, st, pad), oracle.backward_bias(xs, ws, np.abs(pd), st, pad)


def assert_errors(errs, precision=B.MCN_PREC_FP32, label=""):
    tol_f = TOL_BF16 if precision == B.MCN_PREC_BF16 else TOL_FWD
    tol_b = TOL_BF16 if precision == B.MCN_PREC_BF16 else TOL_BWD
    print(label, {k: "%.2e" % v for k, v in errs.items()}, flush=True)
    assert errs["forward"] <= tol_f, (label, errs)
    assert errs["backward_data"] <= tol_b, (label, errs)
    assert errs["backward_filter"] <= tol_b, (label, errs)
    assert errs["backward_bias"] <= TOL_BWD, (label, errs)


# ---- convolution transpose ----
from oracle import convt as oracle_t  # noqa: E402


def _targs(L):
    return L["up"], L["crop"], L["groups"]


def run_convt_full(L, with_bias=True, seed=0, precision=B.MCN_PREC_FP32):
    """All four operations of the transpose block on layer L, every element compared."""
    up, crop, G = _targs(L)
    x, f, b = synth.make_tx(L, seed), synth.make_tf(L, seed), synth.make_tb(L, seed)
    ho, wo = oracle_t.output_size(x.shape, f.shape, up, crop, G)
    p = synth.make_tdzdy(L, ho, wo, seed)
    xd, fd, bd, pd = np64(x), np64(f), np64(b), np64(p)
    bb = bd if with_bias else None
    xg, fg, bg, pg = gpu(x), gpu(f), gpu(b), gpu(p)
    y = B.convt_forward(xg, fg, bg if with_bias else None, up, crop, G, precision)
    dx = B.convt_backward_data(x.shape, fg, pg, up, crop, G, precision)
    df = B.convt_backward_filter(xg, f.shape, pg, up, crop, G, precision)
    db = B.convt_backward_bias(x.shape, f.shape, pg, up, crop, G)
    torch.cuda.synchronize()
    assert tuple(y.shape) == (L["N"], G * L["Kf"], wo, ho)
    out = {}
    out["forward"] = norm_err(y.cpu().numpy(), oracle_t.forward(xd, fd, bb, up, crop, G),
                              oracle_t.forward(np.abs(xd), np.abs(fd), None if bb is None else np.abs(bb), up, crop, G))
    out["backward_data"] = norm_err(dx.cpu().numpy(), oracle_t.backward_data(x.shape, fd, pd, up, crop, G),
                                    oracle_t.backward_data(x.shape, np.abs(fd), np.abs(pd), up, crop, G))
    out["backward_filter"] = norm_err(df.cpu().numpy(), oracle_t.backward_filter(xd, f.shape, pd, up, crop, G),
                                      oracle_t.backward_filter(np.abs(xd), f.shape, np.abs(pd), up, crop, G))
    out["backward_bias"] = norm_err(db.cpu().numpy(), oracle_t.backward_bias(x.shape, f.shape, pd, up, crop, G),
                                    oracle_t.backward_bias(x.shape, f.shape, np.abs(pd), up, crop, G))
    return out


def run_convt_sampled(L, n_out=4000, n_filt=96, seed=0):
    """The transpose block at full size, compared at sampled places (bias derivative: all channels)."""
    up, crop, G = _targs(L)
    x, f, b = synth.make_tx(L, seed), synth.make_tf(L, seed), synth.make_tb(L, seed)
    ho, wo = oracle_t.output_size(x.shape, f.shape, up, crop, G)
    p = synth.make_tdzdy(L, ho, wo, seed)
    xg, fg, bg, pg = gpu(x), gpu(f), gpu(b), gpu(p)
    y = B.convt_forward(xg, fg, bg, up, crop, G)
    dx = B.convt_backward_data(x.shape, fg, pg, up, crop, G)
    df = B.convt_backward_filter(xg, f.shape, pg, up, crop, G)
    db = B.convt_backward_bias(x.shape, f.shape, pg, up, crop, G)
    torch.cuda.synchronize()
    y, dx, df, db = (t.cpu().numpy().ravel() for t in (y, dx, df, db))
    del xg, fg, pg
    xd, fd, bd, pd = np64(x), np64(f), np64(b), np64(p)
    out = {}
    iy = sample_idx(y.size, n_out, 1)
    out["forward"] = norm_err(y[iy], oracle_t.forward_at(xd, fd, bd, iy, up, crop, G),
                              oracle_t.forward_at(np.abs(xd), np.abs(fd), np.abs(bd), iy, up, crop, G))
    ix = sample_idx(dx.size, n_out, 2)
    out["backward_data"] = norm_err(dx[ix], oracle_t.backward_data_at(x.shape, fd, pd, ix, up, crop, G),
                                    oracle_t.backward_data_at(x.shape, np.abs(fd), np.abs(pd), ix, up, crop, G))
    iw = sample_idx(df.size, n_filt, 3)
    out["backward_filter"] = norm_err(df[iw], oracle_t.backward_filter_at(xd, f.shape, pd, iw, up, crop, G),
                                      oracle_t.backward_filter_at(np.abs(xd), f.shape, np.abs(pd), iw, up, crop, G))
    out["backward_bias"] = norm_err(db, oracle_t.backward_bias(x.shape, f.shape, pd, up, crop, G),
                                    oracle_t.backward_bias(x.shape, f.shape, np.abs(pd), up, crop, G))
    return out
