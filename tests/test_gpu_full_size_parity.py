"""Every element of every result at the sizes and on the kernels that the benchmark times.

The deep 3x3 layers (224x224x64->64, 56x56x256->256, 14x14x512->512 at N=32) run through the four entry points and
through the call that returns dzdw and dzdb together; all of y, dzdx, dzdw and dzdb are compared with the oracle's
full passes (the sum of Sec. 4.1 and its adjoints, Sec. 6.1), in the default summation order and in the plain one.
Layers just above the size at which the filter derivative switches to its chunked schedule get every coefficient
compared in both tile shapes of both kernels.  Bars: 1e-4 forward, 1e-3 backward, normalised by the same operator
on absolute values; structurally-zero results exactly zero."""
import time

import numpy as np
import pytest
import torch

from paper_1412_4564_amd import binding as B
from paper_1412_4564_amd import synth

import parity_util as U

pytestmark = pytest.mark.gpu

MODES = ((B.MCN_PREC_FP32, "default order"), (B.MCN_PREC_FP32_PLAIN, "plain order"))


def custom_layer(H, W, D, N, Hf, Wf, Df, K, stride=(1, 1), pad=(0, 0, 0, 0), idx=0):
    return dict(H=H, W=W, D=D, N=N, Hf=Hf, Wf=Wf, Df=Df, K=K, stride=tuple(stride), pad=tuple(pad),
                config=10, index=idx)


def names(L, precision):
    d = B.make_desc(synth.x_shape(L), synth.w_shape(L), L["stride"], L["pad"], precision)
    return [B.mcn_conv_kernel_name(d, op) for op in range(5)]


@pytest.mark.parametrize("name", ["4a", "4b", "4c"])
def test_deep_3x3_layers_full_size_every_element(name):
    L = synth.LAYERS[name]
    st, pad = L["stride"], L["pad"]
    t0 = time.time()
    R = U.OracleResults(L)
    print("layer %s: oracle passes %.1f s" % (name, time.time() - t0), flush=True)
    # what the benchmark's step runs on these layers
    expect = {"4a": ["igemm_f23", "igemm_f23", "wgrad_f23_chunked", "reduce2", "wgrad_f23+bias"],
              "4b": ["igemm_f23", "igemm_f23", "wgrad_f23_chunked", "reduce2", "wgrad_f23+bias"],
              "4c": ["igemm_f23", "igemm_f23", "wgrad_f23", "reduce2", "two passes"]}[name]
    assert names(L, B.MCN_PREC_FP32) == expect
    assert names(L, B.MCN_PREC_FP32_PLAIN)[:3] == ["igemm", "igemm", "wgrad_igemm_chunked" if name != "4c" else "wgrad_igemm"]
    xg, wg, bg, pg = U.gpu(R.x), U.gpu(R.w), U.gpu(R.b), U.gpu(R.p)
    for prec, label in MODES:
        y = B.conv_forward(xg, wg, bg, st, pad, prec)
        dx = B.conv_backward_data(R.x.shape, wg, pg, st, pad, prec)
        dw = B.conv_backward_filter(xg, R.w.shape, pg, st, pad, prec)
        db = B.conv_backward_bias(R.x.shape, R.w.shape, pg, st, pad)
        dw2, db2 = B.conv_backward_filter_bias(xg, R.w.shape, pg, st, pad, prec)
        torch.cuda.synchronize()
        errs = {"forward": U.norm_err(y.cpu().numpy(), R.y, R.y_den),
                "backward_data": U.norm_err(dx.cpu().numpy(), R.dx, R.dx_den),
                "backward_filter": U.norm_err(dw.cpu().numpy(), R.dw, R.dw_den),
                "backward_bias": U.norm_err(db.cpu().numpy(), R.db, R.db_den)}
        del y, dx
        U.assert_errors(errs, label="layer %s full size, %s" % (name, label))
        both = {"forward": 0.0, "backward_data": 0.0,
                "backward_filter": U.norm_err(dw2.cpu().numpy(), R.dw, R.dw_den),
                "backward_bias": U.norm_err(db2.cpu().numpy(), R.db, R.db_den)}
        U.assert_errors(both, label="layer %s full size, dzdw and dzdb in one call, %s" % (name, label))


CHUNKED = [
    # Arrays that stream from memory, with enough units per block: the filter derivative cuts every tile's reduction
    # into chunks, and the row-pair kernel sums dzdy on the way.
    # H    W    D   N   Hf Wf Df  K    stride  pad            kernel in the default order
    (200, 180, 24, 40, 3, 3, 24, 48, (1, 1), (1, 1, 1, 1), "wgrad_f23_chunked"),      # tiles of 64 filters on 12 waves
    (75, 61, 96, 56, 3, 3, 48, 200, (1, 1), (1, 0, 0, 1), "wgrad_f23_chunked"),       # two groups of 100 filters: tiles of 128
    (199, 181, 32, 48, 3, 3, 16, 80, (1, 1), (0, 1, 2, 1), "wgrad_f23_chunked"),      # odd planes, two groups of 40 filters
    (60, 64, 64, 48, 5, 5, 64, 112, (1, 1), (2, 2, 2, 2), "wgrad_igemm_chunked"),     # 5x5: the one-row kernel only
    (100, 80, 64, 48, 5, 5, 64, 96, (1, 1), (2, 2, 2, 2), "wgrad_igemm_chunked"),     # 5x5 on tiles of 96 filters
    (120, 90, 16, 512, 4, 3, 16, 24, (2, 1), (1, 0, 1, 1), "wgrad_igemm_chunked"),    # vertical stride, 32-filter tiles
]


@pytest.mark.parametrize("case", range(len(CHUNKED)))
def test_chunked_filter_derivative_every_coefficient(case):
    H, W, D, N, Hf, Wf, Df, K, st, pad, kernel = CHUNKED[case]
    L = custom_layer(H, W, D, N, Hf, Wf, Df, K, st, pad, idx=case)
    assert names(L, B.MCN_PREC_FP32)[2] == kernel
    assert names(L, B.MCN_PREC_FP32)[4] == ("wgrad_f23+bias" if "f23" in kernel else "two passes")
    assert names(L, B.MCN_PREC_FP32_PLAIN)[2] == "wgrad_igemm_chunked"
    R = U.OracleResults(L, filter_only=True)
    xg, pg = U.gpu(R.x), U.gpu(R.p)
    for prec, label in MODES:
        dw = B.conv_backward_filter(xg, R.w.shape, pg, st, pad, prec)
        dw2, db2 = B.conv_backward_filter_bias(xg, R.w.shape, pg, st, pad, prec)
        torch.cuda.synchronize()
        e = (U.norm_err(dw.cpu().numpy(), R.dw, R.dw_den), U.norm_err(dw2.cpu().numpy(), R.dw, R.dw_den),
             U.norm_err(db2.cpu().numpy(), R.db, R.db_den))
        print("chunked case %d, %s: dzdw %.2e, in one call %.2e, dzdb %.2e" % ((case, label) + e), flush=True)
        assert max(e) <= U.TOL_BWD


@pytest.mark.parametrize("name", ["2a", "2b", "3a", "3b", "5a", "5b"])
def test_other_layers_full_size_all_of_dzdw(name):
    """The remaining workload layers at full size: every filter coefficient and all of dzdb; y and dzdx at sampled places."""
    U.assert_errors(U.run_layer_sampled(synth.LAYERS[name], n_filt=None), label="layer %s full size, all of dzdw" % name)
