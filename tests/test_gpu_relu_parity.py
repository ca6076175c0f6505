"""Convolution + ReLU, fused: GPU-vs-oracle parity through the C ABI.

Forward: max(0, .) of the convolution oracle (ReLU is continuous, so the convolution's forward bar
applies unchanged).  Backward: the mask is decided by the array y that the caller passes in, and both
sides are given the same y, so dzdp must match the ReLU oracle bit for bit; dzdb is a sum of up to
Ho*Wo*N terms and gets the backward bar."""
import numpy as np
import pytest
import torch

import oracle
from oracle import relu as oracle_relu
from paper_1412_4564_amd import binding as B
from paper_1412_4564_amd import synth

import parity_util as U

pytestmark = pytest.mark.gpu


def custom_layer(H, W, D, N, Hf, Wf, Df, K, stride=(1, 1), pad=(0, 0, 0, 0), idx=0):
    return dict(H=H, W=W, D=D, N=N, Hf=Hf, Wf=Wf, Df=Df, K=K, stride=tuple(stride), pad=tuple(pad),
                config=10, index=idx)


def run_fused(L, precision=B.MCN_PREC_FP32, with_bias=True, sample=None):
    st, pad = L["stride"], L["pad"]
    x, w, b = synth.make_x(L), synth.make_w(L), synth.make_b(L)
    ho, wo = oracle.output_size(x.shape, w.shape, st, pad)
    p = synth.make_dzdy(L, ho, wo)
    xg, wg, bg, pg = x.cuda(), w.cuda(), b.cuda(), p.cuda()
    y = B.conv_relu_forward(xg, wg, bg if with_bias else None, st, pad, precision)
    plain = B.conv_forward(xg, wg, bg if with_bias else None, st, pad, precision)
    dzdp, dzdb = B.conv_relu_backward_bias(x.shape, w.shape, y, pg, st, pad)
    torch.cuda.synchronize()
    # fused forward = max(0, unfused forward), bit for bit
    assert torch.equal(y, torch.clamp_min(plain, 0.0))
    assert float((y == 0).float().mean()) > 0.05 and float((y > 0).float().mean()) > 0.05
    yh, ph = y.cpu().numpy(), U.np64(p)
    # backward: exact mask, summed bias
    ref_p = oracle_relu.backward(yh.astype(np.float64), ph)
    assert np.array_equal(dzdp.cpu().numpy().astype(np.float64), ref_p)
    ref_b = oracle.backward_bias(x.shape, w.shape, ref_p, st, pad)
    den_b = oracle.backward_bias(x.shape, w.shape, np.abs(ref_p), st, pad)
    e_bias = U.norm_err(dzdb.cpu().numpy(), ref_b, den_b)
    # in place
    pg2 = pg.clone()
    dzdp2, dzdb2 = B.conv_relu_backward_bias(x.shape, w.shape, y, pg2, st, pad, inplace=True)
    torch.cuda.synchronize()
    assert dzdp2.data_ptr() == pg2.data_ptr() and torch.equal(dzdp2, dzdp) and torch.equal(dzdb2, dzdb)
    # forward against the oracle
    xd, wd, bd = U.np64(x), U.np64(w), U.np64(b)
    bb = bd if with_bias else None
    ab = None if bb is None else np.abs(bb)
    if sample is None:
        ref_y = oracle_relu.forward(oracle.forward(xd, wd, bb, st, pad))
        den_y = oracle.forward(np.abs(xd), np.abs(wd), ab, st, pad)
        e_fwd = U.norm_err(yh, ref_y, den_y)
    else:
        iy = U.sample_idx(yh.size, sample, 21)
        ref_y = oracle_relu.forward(oracle.forward_at(xd, wd, bb, iy, st, pad))
        den_y = oracle.forward_at(np.abs(xd), np.abs(wd), ab, iy, st, pad)
        e_fwd = U.norm_err(yh.ravel()[iy], ref_y, den_y)
    return e_fwd, e_bias


@pytest.mark.parametrize("name,nb", [("1", 8), ("2b", 5), ("3a", 2), ("3b", 3), ("4b", 2), ("4c", 5), ("5a", 9), ("5b", 3),
                                     ("5c", 4)])
def test_fused_relu_workload_layers_reduced_batch(name, nb):
    L = synth.with_batch(synth.LAYERS[name], nb)
    e_fwd, e_bias = run_fused(L)
    print("conv+relu layer %s at N=%d" % (name, nb), "%.2e %.2e" % (e_fwd, e_bias), flush=True)
    assert e_fwd <= U.TOL_FWD and e_bias <= U.TOL_BWD


@pytest.mark.parametrize("name", ["4a", "4b", "5a"])
def test_fused_relu_full_size_sampled(name):
    e_fwd, e_bias = run_fused(synth.LAYERS[name], sample=4000)
    print("conv+relu layer %s full size" % name, "%.2e %.2e" % (e_fwd, e_bias), flush=True)
    assert e_fwd <= U.TOL_FWD and e_bias <= U.TOL_BWD


def test_fused_relu_without_bias_and_odd_shapes():
    for idx, (H, W, D, N, Hf, Wf, Df, K, st, pad) in enumerate([
            (13, 9, 4, 3, 3, 2, 2, 6, (2, 1), (1, 2, 0, 1)),
            (70, 40, 8, 2, 3, 3, 8, 40, (1, 1), (1, 1, 1, 1)),
            (4, 5, 3, 4, 4, 5, 3, 10, (1, 1), (0, 0, 0, 0)),          # fully connected
            (1, 1, 1, 1, 1, 1, 1, 1, (1, 1), (0, 0, 0, 0))]):
        L = custom_layer(H, W, D, N, Hf, Wf, Df, K, st, pad, idx)
        if L["N"] * L["K"] < 4:
            continue                      # too few values for the "both signs occur" check
        e_fwd, e_bias = run_fused(L, with_bias=(idx % 2 == 1))
        assert e_fwd <= U.TOL_FWD and e_bias <= U.TOL_BWD


def test_fused_relu_bf16_operands():
    L = synth.with_batch(synth.LAYERS["4b"], 2)
    e_fwd, e_bias = run_fused(L, precision=B.MCN_PREC_BF16)
    assert e_fwd <= U.TOL_BF16 and e_bias <= U.TOL_BWD


def test_fused_relu_chain_equals_unfused_chain():
    """dzdx and dzdw computed from the fused calls equal those of the unfused sequence
    conv -> relu -> (backward) relu -> conv, with the ReLU steps done by torch."""
    L = synth.with_batch(synth.LAYERS["2b"], 6)
    st, pad = L["stride"], L["pad"]
    x, w, b = synth.make_x(L).cuda(), synth.make_w(L).cuda(), synth.make_b(L).cuda()
    y = B.conv_relu_forward(x, w, b, st, pad)
    p = torch.randn_like(y)
    dzdp, dzdb = B.conv_relu_backward_bias(x.shape, w.shape, y, p, st, pad)
    dx = B.conv_backward_data(x.shape, w, dzdp, st, pad)
    dw = B.conv_backward_filter(x, w.shape, dzdp, st, pad)
    pre = B.conv_forward(x, w, b, st, pad)
    masked = torch.where(pre > 0, p, torch.zeros_like(p))
    assert torch.equal(dzdp, masked)
    assert torch.equal(dx, B.conv_backward_data(x.shape, w, masked, st, pad))
    assert torch.equal(dw, B.conv_backward_filter(x, w.shape, masked, st, pad))
    assert torch.equal(dzdb, B.conv_backward_bias(x.shape, w.shape, masked, st, pad))
