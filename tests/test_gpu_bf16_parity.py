"""The bf16-operand variant (operands rounded to bf16 on chip, fp32 accumulation), through the
C ABI.  Two bars: (1) against the oracle on the fp32 inputs, normalised error <= 1e-2 (rounding two
operands to 8 significant bits costs at most 2^-8 + 2^-16 of the sum of |w||x|); (2) against the
oracle on inputs rounded to bf16 beforehand (round to nearest even), the fp32 bars (1e-4 forward,
1e-3 backward) -- this pins the rounding model itself: what the kernel computes is the exact sum
over rounded operands, accumulated in fp32."""
import numpy as np
import pytest
import torch

import oracle
from paper_1412_4564_amd import binding as B
from paper_1412_4564_amd import synth

import parity_util as U

pytestmark = pytest.mark.gpu
BF = B.MCN_PREC_BF16


def rne_bf16(t):
    return t.to(torch.bfloat16).to(torch.float32)


def custom_layer(H, W, D, N, Hf, Wf, Df, K, stride=(1, 1), pad=(0, 0, 0, 0), idx=0):
    return dict(H=H, W=W, D=D, N=N, Hf=Hf, Wf=Wf, Df=Df, K=K, stride=tuple(stride), pad=tuple(pad),
                config=7, index=idx)


def run_bf16(L, with_bias=True, seed=0):
    st, pad = L["stride"], L["pad"]
    x, w, b = synth.make_x(L, seed), synth.make_w(L, seed), synth.make_b(L, seed)
    ho, wo = oracle.output_size(x.shape, w.shape, st, pad)
    p = synth.make_dzdy(L, ho, wo, seed)
    xg, wg, bg, pg = x.cuda(), w.cuda(), b.cuda(), p.cuda()
    y = B.conv_forward(xg, wg, bg if with_bias else None, st, pad, BF)
    dx = B.conv_backward_data(x.shape, wg, pg, st, pad, BF)
    dw = B.conv_backward_filter(xg, w.shape, pg, st, pad, BF)
    torch.cuda.synchronize()
    y, dx, dw = y.cpu().numpy(), dx.cpu().numpy(), dw.cpu().numpy()
    xd, wd, bd, pd = (U.np64(t) for t in (x, w, b, p))
    xr, wr, pr = (U.np64(rne_bf16(t)) for t in (x, w, p))
    bb = bd if with_bias else None
    ab = None if bb is None else np.abs(bb)
    den_y = oracle.forward(np.abs(xd), np.abs(wd), ab, st, pad)
    den_x = oracle.backward_data(x.shape, np.abs(wd), np.abs(pd), st, pad)
    den_w = oracle.backward_filter(np.abs(xd), w.shape, np.abs(pd), st, pad)
    vs_fp32 = {"forward": U.norm_err(y, oracle.forward(xd, wd, bb, st, pad), den_y),
               "backward_data": U.norm_err(dx, oracle.backward_data(x.shape, wd, pd, st, pad), den_x),
               "backward_filter": U.norm_err(dw, oracle.backward_filter(xd, w.shape, pd, st, pad), den_w)}
    vs_rounded = {"forward": U.norm_err(y, oracle.forward(xr, wr, bb, st, pad), den_y),
                  "backward_data": U.norm_err(dx, oracle.backward_data(x.shape, wr, pr, st, pad), den_x),
                  "backward_filter": U.norm_err(dw, oracle.backward_filter(xr, w.shape, pr, st, pad), den_w)}
    return vs_fp32, vs_rounded


def check_filter_derivative(names, vs_fp32, vs_rounded, label):
    """On the bf16 kernel the filter derivative is the exact sum over rounded x and dzdy."""
    if names[2] == "wgrad_bf16":
        assert vs_rounded["backward_filter"] <= U.TOL_BWD, (label, vs_rounded)
        assert vs_fp32["backward_filter"] > 1e-6, (label, vs_fp32)


def check(L, label, with_bias=True, expect_kernel="igemm_bf16"):
    d = B.make_desc(synth.x_shape(L), synth.w_shape(L), L["stride"], L["pad"], BF)
    names = [B.mcn_conv_kernel_name(d, op) for op in range(3)]
    vs_fp32, vs_rounded = run_bf16(L, with_bias)
    print(label, names, "vs fp32 inputs", {k: "%.2e" % v for k, v in vs_fp32.items()},
          "vs rounded inputs", {k: "%.2e" % v for k, v in vs_rounded.items()}, flush=True)
    for k, v in vs_fp32.items():
        assert v <= U.TOL_BF16, (label, k, v)
    if expect_kernel:
        assert names[0] == expect_kernel and names[1] == expect_kernel, names
        assert vs_rounded["forward"] <= U.TOL_FWD, (label, vs_rounded)
        assert vs_rounded["backward_data"] <= U.TOL_BWD, (label, vs_rounded)
        # the operands really were rounded: an fp32 computation would be two orders closer
        assert vs_fp32["forward"] > 2e-5, (label, vs_fp32)
    check_filter_derivative(names, vs_fp32, vs_rounded, label)


@pytest.mark.parametrize("name,nb", [("4a", 1), ("4b", 2), ("4c", 5), ("3b", 3), ("2b", 7), ("2c", 9), ("5b", 3)])
def test_bf16_workload_layers_reduced_batch(name, nb):
    check(synth.with_batch(synth.LAYERS[name], nb), "bf16 layer %s at N=%d" % (name, nb))


BF_SWEEP = [
    # H  W  D  N  Hf Wf Df K   stride   pad
    (23, 17, 16, 3, 3, 3, 16, 40, (1, 1), (1, 1, 1, 1)),     # exactly one MFMA depth of channels
    (23, 17, 40, 2, 3, 3, 40, 24, (1, 1), (1, 1, 1, 1)),     # 40 channels: a ragged last unit
    (30, 30, 48, 2, 5, 5, 24, 66, (2, 2), (2, 1, 0, 2)),     # 2 groups, stride 2: four phases in dzdx
    (19, 21, 32, 2, 7, 7, 32, 33, (3, 2), (3, 3, 3, 3)),     # 49 taps: several tap ranges
    (64, 9, 64, 2, 1, 1, 64, 130, (1, 1), (0, 0, 0, 0)),     # 1x1
    (12, 12, 17, 2, 2, 2, 17, 19, (1, 1), (0, 1, 1, 0)),     # odd channel counts
    (9, 9, 32, 40, 3, 3, 32, 32, (1, 1), (1, 1, 1, 1)),      # many small images per tile
]


@pytest.mark.parametrize("case", range(len(BF_SWEEP)))
def test_bf16_geometry_sweep(case):
    H, W, D, N, Hf, Wf, Df, K, st, pad = BF_SWEEP[case]
    L = custom_layer(H, W, D, N, Hf, Wf, Df, K, st, pad, idx=case)
    # the input derivative's reduction depth is K per group: below 16 it stays on the fp32 kernel
    d = B.make_desc(synth.x_shape(L), synth.w_shape(L), st, pad, BF)
    both = B.mcn_conv_kernel_name(d, 1) == "igemm_bf16"
    vs_fp32, vs_rounded = run_bf16(L, with_bias=(case % 2 == 0))
    print("bf16 sweep", case, [B.mcn_conv_kernel_name(d, op) for op in range(3)], vs_fp32, vs_rounded, flush=True)
    assert B.mcn_conv_kernel_name(d, 0) == "igemm_bf16"
    for k, v in vs_fp32.items():
        assert v <= U.TOL_BF16, (case, k, v)
    assert vs_rounded["forward"] <= U.TOL_FWD
    if both:
        assert vs_rounded["backward_data"] <= U.TOL_BWD
    check_filter_derivative([B.mcn_conv_kernel_name(d, op) for op in range(3)], vs_fp32, vs_rounded, "sweep %d" % case)


WG_SWEEP = [
    # H  W  D  N  Hf Wf Df K   stride   pad                     expected filter-derivative kernel
    (14, 14, 32, 5, 3, 3, 32, 64, (1, 1), (1, 1, 1, 1), "wgrad_bf16"),     # 14 rows: a partial octet in every patch
    (23, 9, 24, 3, 3, 3, 24, 40, (1, 1), (1, 1, 1, 1), "wgrad_bf16"),      # odd width: a patch with a missing column
    (30, 31, 16, 2, 5, 5, 8, 66, (1, 2), (2, 2, 1, 3), "wgrad_bf16"),      # two groups, horizontal stride 2
    (40, 12, 8, 3, 1, 1, 8, 130, (1, 1), (0, 0, 0, 0), "wgrad_bf16"),      # 1x1
    (17, 20, 6, 2, 2, 4, 6, 48, (1, 3), (0, 1, 2, 0), "wgrad_bf16"),       # even filter height, stride 3 across
    (19, 19, 12, 2, 4, 2, 12, 100, (1, 1), (3, 0, 0, 1), "wgrad_bf16"),
    (70, 6, 4, 2, 3, 3, 4, 36, (1, 1), (0, 0, 0, 0), "wgrad_bf16"),        # no padding, tall plane: several row blocks
    (9, 9, 16, 70, 3, 3, 16, 64, (1, 1), (1, 1, 1, 1), "wgrad_bf16"),      # many images: several chunks per tile
    (20, 20, 16, 2, 3, 3, 16, 24, (1, 1), (1, 1, 1, 1), "wgrad_igemm"),    # 24 filters: stays on the fp32 kernel
    (20, 20, 16, 2, 3, 3, 16, 64, (2, 1), (1, 1, 1, 1), "wgrad_igemm"),    # vertical stride: stays on the fp32 kernel
    (30, 30, 8, 2, 7, 7, 8, 64, (1, 1), (3, 3, 3, 3), "wgrad_igemm"),      # 7 filter rows: stays on the fp32 kernel
]


@pytest.mark.parametrize("case", range(len(WG_SWEEP)))
def test_bf16_filter_derivative_sweep(case):
    H, W, D, N, Hf, Wf, Df, K, st, pad, kernel = WG_SWEEP[case]
    L = custom_layer(H, W, D, N, Hf, Wf, Df, K, st, pad, idx=50 + case)
    d = B.make_desc(synth.x_shape(L), synth.w_shape(L), st, pad, BF)
    names = [B.mcn_conv_kernel_name(d, op) for op in range(3)]
    assert names[2] == kernel, names
    vs_fp32, vs_rounded = run_bf16(L)
    print("bf16 filter derivative", case, names, vs_fp32, vs_rounded, flush=True)
    for k, v in vs_fp32.items():
        assert v <= U.TOL_BF16, (case, k, v)
    check_filter_derivative(names, vs_fp32, vs_rounded, "filter derivative %d" % case)


def test_bf16_random_geometries():
    rng = np.random.default_rng(57721)
    for t in range(24):
        g = int(rng.choice([1, 1, 2]))
        Df, Kg = int(rng.integers(8, 70)), int(rng.integers(20, 150))
        Hf, Wf = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        H, W = int(rng.integers(Hf, 34)), int(rng.integers(Wf, 34))
        st = (int(rng.integers(1, 3)), int(rng.integers(1, 3)))
        pad = tuple(int(v) for v in rng.integers(0, 3, size=4))
        L = custom_layer(H, W, g * Df, int(rng.integers(1, 5)), Hf, Wf, Df, g * Kg, st, pad, idx=200 + t)
        d = B.make_desc(synth.x_shape(L), synth.w_shape(L), st, pad, BF)
        names = [B.mcn_conv_kernel_name(d, op) for op in range(3)]
        vs_fp32, vs_rounded = run_bf16(L, with_bias=bool(t % 2))
        print("random bf16 case", t, L, names, vs_fp32, vs_rounded, flush=True)
        for k, v in vs_fp32.items():
            assert v <= U.TOL_BF16, (t, k, v)
        if names[0] == "igemm_bf16":
            assert vs_rounded["forward"] <= U.TOL_FWD, (t, vs_rounded)
        if names[1] == "igemm_bf16":
            assert vs_rounded["backward_data"] <= U.TOL_BWD, (t, vs_rounded)
        check_filter_derivative(names, vs_fp32, vs_rounded, "random bf16 %d" % t)


def test_bf16_few_channels_stay_on_fp32_kernels():
    # 3 input channels: the bf16 kernel would waste 13 of its 16 reduction lanes; the fp32 kernel
    # meets the bf16 bound trivially
    L = synth.with_batch(synth.LAYERS["2a"], 4)
    check(L, "bf16 precision, 3 channels", expect_kernel=None)
    d = B.make_desc(synth.x_shape(L), synth.w_shape(L), L["stride"], L["pad"], BF)
    assert B.mcn_conv_kernel_name(d, 0) == "igemm"


@pytest.mark.parametrize("name", ["4a", "4b", "4c"])
def test_bf16_full_size_sampled(name):
    """Full benchmark size, sampled outputs against the oracle on the fp32 inputs."""
    L = synth.LAYERS[name]
    st, pad = L["stride"], L["pad"]
    x, w, b = synth.make_x(L), synth.make_w(L), synth.make_b(L)
    ho, wo = oracle.output_size(x.shape, w.shape, st, pad)
    p = synth.make_dzdy(L, ho, wo)
    xg, wg, bg, pg = x.cuda(), w.cuda(), b.cuda(), p.cuda()
    y = B.conv_forward(xg, wg, bg, st, pad, BF).cpu().numpy().ravel()
    dx = B.conv_backward_data(x.shape, wg, pg, st, pad, BF).cpu().numpy().ravel()
    dw = B.conv_backward_filter(xg, w.shape, pg, st, pad, BF).cpu().numpy().ravel()
    del xg, pg
    xd, wd, bd, pd = (U.np64(t) for t in (x, w, b, p))
    xr, wr, pr = (U.np64(rne_bf16(t)) for t in (x, w, p))
    iy, ix = U.sample_idx(y.size, 3000, 11), U.sample_idx(dx.size, 3000, 12)
    den_y = oracle.forward_at(np.abs(xd), np.abs(wd), np.abs(bd), iy, st, pad)
    den_x = oracle.backward_data_at(x.shape, np.abs(wd), np.abs(pd), ix, st, pad)
    e = {"forward": U.norm_err(y[iy], oracle.forward_at(xd, wd, bd, iy, st, pad), den_y),
         "backward_data": U.norm_err(dx[ix], oracle.backward_data_at(x.shape, wd, pd, ix, st, pad), den_x),
         "forward_rounded": U.norm_err(y[iy], oracle.forward_at(xr, wr, bd, iy, st, pad), den_y),
         "backward_data_rounded": U.norm_err(dx[ix], oracle.backward_data_at(x.shape, wr, pr, ix, st, pad), den_x)}
    iw = U.sample_idx(dw.size, 64, 13)
    den_w = oracle.backward_filter_at(np.abs(xd), w.shape, np.abs(pd), iw, st, pad)
    e["backward_filter"] = U.norm_err(dw[iw], oracle.backward_filter_at(xd, w.shape, pd, iw, st, pad), den_w)
    e["backward_filter_rounded"] = U.norm_err(dw[iw], oracle.backward_filter_at(xr, w.shape, pr, iw, st, pad), den_w)
    print("bf16 layer %s full size" % name, e, flush=True)
    assert e["backward_filter"] <= U.TOL_BF16 and e["backward_filter_rounded"] <= U.TOL_BWD
    assert e["forward"] <= U.TOL_BF16 and e["backward_data"] <= U.TOL_BF16
    assert e["forward_rounded"] <= U.TOL_FWD and e["backward_data_rounded"] <= U.TOL_BWD
