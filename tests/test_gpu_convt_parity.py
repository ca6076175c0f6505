"""Convolution transpose: GPU-vs-oracle parity, through the C ABI.  Same error bar
as the convolution block: normalised error <= 1e-4 forward, <= 1e-3 backward in fp32;
structurally-zero results exactly zero."""
import numpy as np
import pytest
import torch

from paper_1412_4564_amd import binding as B
from paper_1412_4564_amd import synth

import parity_util as U

pytestmark = pytest.mark.gpu


def tlayer(H, W, D, N, Hf, Wf, Kf, G, up=(1, 1), crop=(0, 0, 0, 0), idx=0):
    return dict(H=H, W=W, D=D, N=N, Hf=Hf, Wf=Wf, Kf=Kf, groups=G, up=tuple(up), crop=tuple(crop), config=8, index=idx)


def with_batch(L, n):
    out = dict(L)
    out["N"] = int(n)
    return out


@pytest.mark.parametrize("name,nb", [("t1", 2), ("t2", 3), ("t3", 8), ("t4", 1), ("t5", 3)])
def test_convt_workload_layers_reduced_batch_full(name, nb):
    L = with_batch(synth.CONVT_LAYERS[name], nb)
    U.assert_errors(U.run_convt_full(L), label="convt layer %s at N=%d" % (name, nb))
    if name in ("t3", "t5"):
        U.assert_errors(U.run_convt_full(L, with_bias=False, seed=1), label="convt layer %s, no bias" % name)


@pytest.mark.parametrize("name", ["t1", "t2", "t4"])
def test_convt_workload_layers_full_size_sampled(name):
    L = synth.CONVT_LAYERS[name]
    U.assert_errors(U.run_convt_sampled(L), label="convt layer %s full size" % name)


@pytest.mark.parametrize("name,nb", [("t1", 2), ("t2", 3), ("t3", 4)])
def test_convt_bf16_operands(name, nb):
    """The transpose block under the bf16-operand flag: its three MFMA passes run on the bf16 kernels where
    those apply (error bar 1e-2 against the oracle on the fp32 inputs)."""
    L = with_batch(synth.CONVT_LAYERS[name], nb)
    d = B.make_convt_desc(synth.tx_shape(L), synth.tf_shape(L), L["up"], L["crop"], L["groups"], B.MCN_PREC_BF16)
    names = [B.mcn_convt_kernel_name(d, op) for op in range(3)]
    errs = U.run_convt_full(L, precision=B.MCN_PREC_BF16)
    print("convt bf16", name, names, errs, flush=True)
    U.assert_errors(errs, precision=B.MCN_PREC_BF16, label="convt bf16 %s" % name)
    if name in ("t1", "t2"):
        assert "bf16" in names[0] and "bf16" in names[1], names
        assert errs["forward"] > 2e-5      # the operands really were rounded


TSWEEP = [
    # H  W  D  N  Hf Wf Kf G   up      crop
    (5, 7, 4, 2, 3, 3, 5, 1, (1, 1), (0, 0, 0, 0)),          # plain full correlation
    (5, 7, 4, 2, 3, 3, 5, 2, (2, 2), (1, 1, 1, 1)),
    (9, 4, 6, 3, 2, 5, 3, 3, (3, 1), (0, 2, 1, 0)),
    (6, 6, 2, 2, 2, 2, 2, 1, (4, 5), (0, 0, 0, 0)),          # upsampling > filter: samples no tap reaches hold the bias
    (6, 6, 2, 2, 2, 2, 2, 1, (4, 5), (3, 1, 2, 6)),
    (1, 1, 8, 5, 6, 4, 7, 1, (1, 1), (0, 0, 0, 0)),          # 1x1 input: a matrix product (transpose of a fully-connected layer)
    (1, 1, 1, 1, 1, 1, 1, 1, (1, 1), (0, 0, 0, 0)),          # the smallest problem
    (40, 3, 64, 1, 3, 2, 64, 1, (1, 1), (1, 1, 0, 0)),       # deep reduction
    (20, 20, 24, 2, 3, 3, 70, 2, (2, 2), (0, 1, 1, 0)),      # 140 output channels: ragged tiles
    (11, 13, 3, 2, 7, 7, 2, 3, (2, 3), (5, 4, 6, 6)),
    (33, 2, 5, 4, 1, 1, 9, 1, (1, 1), (0, 0, 0, 0)),         # 1x1 filter
    (33, 2, 5, 4, 1, 1, 9, 1, (2, 2), (0, 0, 0, 0)),         # 1x1 filter with upsampling: mostly bias
]


@pytest.mark.parametrize("case", range(len(TSWEEP)))
def test_convt_geometry_sweep(case):
    H, W, D, N, Hf, Wf, Kf, G, up, crop = TSWEEP[case]
    L = tlayer(H, W, D, N, Hf, Wf, Kf, G, up, crop, idx=case)
    U.assert_errors(U.run_convt_full(L, with_bias=(case % 3 != 2)), label="convt sweep %d" % case)


def test_convt_random_geometries():
    rng = np.random.default_rng(27182)
    for t in range(30):
        G = int(rng.choice([1, 1, 2, 3]))
        Dg, Kf = int(rng.integers(1, 20)), int(rng.integers(1, 20))
        Hf, Wf = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        H, W = int(rng.integers(1, 20)), int(rng.integers(1, 20))
        up = (int(rng.integers(1, 4)), int(rng.integers(1, 4)))
        fh, fw = up[0] * (H - 1) + Hf, up[1] * (W - 1) + Wf
        ct = int(rng.integers(0, min(fh, 4))); cb = int(rng.integers(0, min(fh - ct, 4)))
        cl = int(rng.integers(0, min(fw, 4))); cr = int(rng.integers(0, min(fw - cl, 4)))
        L = tlayer(H, W, G * Dg, int(rng.integers(1, 5)), Hf, Wf, Kf, G, up, (ct, cb, cl, cr), idx=100 + t)
        print("random convt case", t, L, flush=True)
        U.assert_errors(U.run_convt_full(L, with_bias=bool(t % 2)), label="random convt %d" % t)


def test_convt_interpolation_closed_form():
    # per-class 2x interpolation with a triangle filter: even places keep x, odd places average
    x = torch.randn(3, 5, 9, 11, device="cuda")
    tri = torch.tensor([0.5, 1.0, 0.5], device="cuda")
    f = torch.outer(tri, tri).expand(5, 1, 3, 3).contiguous()
    y = B.convt_forward(x, f, None, (2, 2), (1, 1, 1, 1), groups=5)
    torch.cuda.synchronize()
    assert tuple(y.shape) == (3, 5, 17, 21)
    assert torch.equal(y[:, :, 0::2, 0::2], x)
    mid = 0.25 * (x[:, :, :-1, :-1] + x[:, :, 1:, :-1] + x[:, :, :-1, 1:] + x[:, :, 1:, 1:])
    assert torch.allclose(y[:, :, 1::2, 1::2], mid, rtol=0, atol=1e-6)


def test_convt_is_the_transpose_of_conv_on_the_gpu():
    # <convt(x), p> = <x, conv(p)> with both sides computed by the library
    L = synth.CONVT_LAYERS["t5"]
    x, f = synth.make_tx(L).cuda(), synth.make_tf(L).cuda()
    y = B.convt_forward(x, f, None, L["up"], L["crop"], L["groups"])
    p = torch.randn_like(y)
    back = B.conv_forward(p, f, None, L["up"], L["crop"])
    torch.cuda.synchronize()
    lhs, rhs = float((y.double() * p.double()).sum()), float((x.double() * back.double()).sum())
    scale = float((y.double().abs() * p.double().abs()).sum())
    assert abs(lhs - rhs) <= 1e-5 * scale


def test_convt_kernel_choice():
    for name in ("t1", "t2", "t3"):
        L = synth.CONVT_LAYERS[name]
        d = B.make_convt_desc(synth.tx_shape(L), synth.tf_shape(L), L["up"], L["crop"], L["groups"])
        names = [B.mcn_convt_kernel_name(d, op) for op in range(4)]
        print(name, names, flush=True)
        # t1 is a 3x3 filter without upsampling: both passes run on the kernel that computes pairs of rows
        expect = "igemm_f23" if name == "t1" else "igemm"
        assert names[0] == expect and names[1] == expect, (name, names)
        assert names[2].startswith("wgrad_f23" if name == "t1" else "wgrad_igemm"), (name, names)
