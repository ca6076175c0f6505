"""GPU-vs-oracle parity, through the C ABI.  Error bar: normalised error
(|gpu - oracle| / the same sum taken over absolute values) <= 1e-4 forward,
<= 1e-3 backward in fp32; structurally-zero results exactly zero."""
import numpy as np
import pytest
import torch

import oracle
from paper_1412_4564_amd import binding as B
from paper_1412_4564_amd import synth

import parity_util as U

pytestmark = pytest.mark.gpu


def custom_layer(H, W, D, N, Hf, Wf, Df, K, stride=(1, 1), pad=(0, 0, 0, 0), idx=0):
    return dict(H=H, W=W, D=D, N=N, Hf=Hf, Wf=Wf, Df=Df, K=K, stride=tuple(stride), pad=tuple(pad),
                config=9, index=idx)


# ---- small layers of the workloads: every element ---------------------------------
@pytest.mark.parametrize("name", ["1", "5c", "2c"])
def test_small_workload_layers_full(name):
    L = synth.LAYERS[name]
    U.assert_errors(U.run_layer_full(L), label="layer " + name)
    U.assert_errors(U.run_layer_full(L, with_bias=False, seed=1), label="layer %s, no bias" % name)


@pytest.mark.parametrize("name,nb", [("2a", 6), ("2b", 5), ("3a", 2), ("3b", 3), ("4a", 1), ("4b", 2), ("4c", 5),
                                     ("5a", 9), ("5b", 3)])
def test_workload_layers_reduced_batch_full(name, nb):
    """Real spatial/channel shape, small batch: every element compared."""
    L = synth.with_batch(synth.LAYERS[name], nb)
    U.assert_errors(U.run_layer_full(L), label="layer %s at N=%d" % (name, nb))


# ---- full-size workloads, in the configuration the benchmark times: sampled -------
# (full-size workloads, in the configuration the benchmark times: tests/test_gpu_full_size_parity.py)


# ---- irregular geometry sweep: strides, four pads, groups, non-square everything ---
SWEEP = [
    # H  W  D  N  Hf Wf Df K   stride   pad
    (13, 9, 4, 3, 3, 2, 2, 6, (1, 1), (0, 0, 0, 0)),
    (13, 9, 4, 3, 3, 2, 2, 6, (2, 1), (1, 2, 0, 1)),
    (9, 13, 6, 2, 2, 4, 2, 9, (1, 3), (3, 0, 1, 2)),
    (33, 35, 5, 2, 5, 3, 5, 7, (3, 2), (2, 1, 0, 2)),
    (70, 40, 8, 2, 3, 3, 8, 40, (1, 1), (1, 1, 1, 1)),      # several 32-pixel tiles + ragged tail
    (67, 5, 3, 3, 7, 5, 3, 33, (1, 1), (3, 3, 2, 2)),
    (16, 16, 12, 2, 1, 1, 4, 9, (1, 1), (0, 0, 0, 0)),       # 1x1, 3 groups
    (16, 16, 12, 2, 1, 1, 12, 5, (2, 2), (0, 0, 0, 0)),      # 1x1 with stride: unread samples
    (10, 11, 2, 2, 4, 4, 2, 3, (5, 6), (0, 0, 0, 0)),        # stride > filter: unread rows/cols
    (4, 5, 3, 4, 4, 5, 3, 10, (1, 1), (0, 0, 0, 0)),         # fully connected: 1x1 output
    (3, 3, 2, 2, 2, 2, 2, 2, (1, 1), (4, 4, 4, 4)),          # pad larger than the filter
    (1, 1, 1, 1, 1, 1, 1, 1, (1, 1), (0, 0, 0, 0)),          # the smallest problem
    (2, 40, 1, 1, 2, 3, 1, 1, (1, 1), (0, 0, 1, 1)),         # single channel, single filter
    (40, 2, 64, 1, 3, 2, 64, 64, (1, 1), (1, 1, 0, 0)),      # deep reduction
    (31, 29, 6, 5, 3, 3, 3, 130, (1, 1), (1, 1, 1, 1)),      # K = 2 groups x 65: ragged filter tiles
    (21, 17, 7, 2, 6, 6, 7, 3, (2, 2), (0, 5, 5, 0)),
]


@pytest.mark.parametrize("case", range(len(SWEEP)))
def test_geometry_sweep(case):
    H, W, D, N, Hf, Wf, Df, K, st, pad = SWEEP[case]
    L = custom_layer(H, W, D, N, Hf, Wf, Df, K, st, pad, idx=case)
    U.assert_errors(U.run_layer_full(L, with_bias=(case % 2 == 0)), label="sweep %d" % case)


def test_random_geometries():
    rng = np.random.default_rng(31415)
    for t in range(40):
        g = int(rng.choice([1, 1, 2, 3]))
        Df, Kg = int(rng.integers(1, 9)), int(rng.integers(1, 40))
        Hf, Wf = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        H, W = int(rng.integers(1, 40)), int(rng.integers(1, 40))
        pad = [int(v) for v in rng.integers(0, 4, size=4)]
        while H + pad[0] + pad[1] < Hf:
            pad[1] += 1
        while W + pad[2] + pad[3] < Wf:
            pad[3] += 1
        st = (int(rng.integers(1, 4)), int(rng.integers(1, 4)))
        L = custom_layer(H, W, g * Df, int(rng.integers(1, 5)), Hf, Wf, Df, g * Kg, st, pad, idx=100 + t)
        U.assert_errors(U.run_layer_full(L, with_bias=bool(t % 2), seed=t), label="random %d %r" % (t, L))


def test_random_geometries_many_channels():
    """Channel and filter counts large enough for the instantiations with a compile-time filter size (1x1, 3x3,
    5x5), the two-blocks-per-unit shapes and ragged filter tiles, at random sizes, strides and pads."""
    rng = np.random.default_rng(27182)
    for t in range(24):
        g = int(rng.choice([1, 1, 1, 2]))
        F = int(rng.choice([1, 3, 3, 5]))
        Df = int(rng.choice([8, 16, 24, 32, 64, 72])) if F > 1 else int(rng.choice([64, 96, 128]))
        Kg = int(rng.integers(33, 200))
        H, W = int(rng.integers(F, 31)), int(rng.integers(F, 31))
        pad = [int(v) for v in rng.integers(0, F, size=4)] if F > 1 else [0, 0, 0, 0]
        st = (int(rng.integers(1, 3)), int(rng.integers(1, 3)))
        L = custom_layer(H, W, g * Df, int(rng.integers(1, 7)), F, F, Df, g * Kg, st, pad, idx=300 + t)
        print("random wide case", t, L, flush=True)
        U.assert_errors(U.run_layer_full(L, with_bias=bool(t % 2), seed=t), label="random wide %d %r" % (t, L))


_FALLBACK_SCRIPT = r"""
import sys
sys.path.insert(0, sys.argv[1]); sys.path.insert(0, sys.argv[1] + "/tests")
import parity_util as U
from paper_1412_4564_amd import binding as B, synth
cases = [(13, 9, 4, 3, 3, 2, 2, 6, (2, 1), (1, 2, 0, 1)), (16, 16, 12, 2, 1, 1, 4, 9, (1, 1), (0, 0, 0, 0)),
         (10, 11, 2, 2, 4, 4, 2, 3, (5, 6), (0, 0, 0, 0)), (3, 3, 2, 2, 2, 2, 2, 2, (1, 1), (4, 4, 4, 4)),
         (31, 29, 6, 5, 3, 3, 3, 130, (1, 1), (1, 1, 1, 1)), (4, 5, 3, 4, 4, 5, 3, 10, (1, 1), (0, 0, 0, 0))]
for i, (H, W, D, N, Hf, Wf, Df, K, st, pad) in enumerate(cases):
    L = dict(H=H, W=W, D=D, N=N, Hf=Hf, Wf=Wf, Df=Df, K=K, stride=st, pad=pad, config=9, index=400 + i)
    d = B.make_desc(synth.x_shape(L), synth.w_shape(L), st, pad)
    names = [B.mcn_conv_kernel_name(d, op) for op in range(3)]
    assert names == ["direct"] * 3, names
    U.assert_errors(U.run_layer_full(L, with_bias=bool(i % 2)), label="fallback %d" % i)
print("FALLBACK-OK")
"""


def test_fallback_kernels_in_a_process_of_their_own():
    """The one-result-per-thread kernels serve geometries the planners reject; MCN_FORCE_DIRECT=1 (read once per
    process) routes everything to them, so they are checked against the oracle in a child process."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    env = dict(os.environ, MCN_FORCE_DIRECT="1")
    r = subprocess.run([sys.executable, "-c", _FALLBACK_SCRIPT, root], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "FALLBACK-OK" in r.stdout, (r.stdout[-2000:], r.stderr[-2000:])


# ---- 3x3 filters at stride 1: the kernel that computes pairs of output rows -------------
ROW_PAIRS = [
    # H   W   D   N  Df   K   pad
    (16, 12, 16, 3, 16, 48, (1, 1, 1, 1)),       # even number of output rows
    (15, 13, 16, 2, 16, 40, (1, 1, 1, 1)),       # odd: the last pair has one row
    (17, 9, 24, 2, 24, 64, (0, 0, 0, 0)),        # no padding
    (11, 14, 40, 3, 40, 72, (2, 0, 1, 2)),       # four different pads, filters ragged against the tile
    (20, 10, 48, 2, 16, 144, (1, 1, 1, 1)),      # three groups
    (14, 14, 64, 4, 64, 160, (1, 1, 1, 1)),      # two filter tiles of 128, the second ragged
    (150, 6, 16, 2, 16, 40, (1, 1, 1, 1)),       # tall planes: several row blocks
    (40, 40, 32, 8, 32, 64, (1, 1, 1, 1)),       # more tiles than compute units, some shared between blocks
    (28, 28, 64, 16, 64, 256, (1, 1, 1, 1)),
    (3, 3, 16, 1, 16, 40, (1, 1, 1, 1)),         # one pair and a single row
    (6, 7, 16, 2, 16, 36, (3, 2, 2, 3)),         # pads larger than the filter reach
    # more than 64 filters per group: wider tiles in the filter derivative
    (15, 13, 16, 2, 16, 80, (1, 1, 1, 1)),       # odd number of output rows
    (150, 6, 16, 2, 16, 72, (1, 1, 1, 1)),       # several row blocks
    (6, 7, 16, 2, 16, 68, (3, 2, 2, 3)),
    (3, 3, 16, 1, 16, 72, (1, 1, 1, 1)),
    (9, 10, 20, 3, 20, 96, (0, 1, 1, 0)),        # channels that do not fill units of 8
    (10, 9, 50, 2, 50, 75, (1, 1, 0, 0)),        # neither do the filters, which are the input derivative's channels
    (30, 30, 160, 6, 80, 400, (1, 1, 1, 1)),     # two groups, several tiles in both directions, shared between blocks
]


@pytest.mark.parametrize("case", range(len(ROW_PAIRS)))
def test_3x3_stride1_row_pair_kernel(case):
    H, W, D, N, Df, K, pad = ROW_PAIRS[case]
    L = custom_layer(H, W, D, N, 3, 3, Df, K, (1, 1), pad, idx=500 + case)
    d = B.make_desc(synth.x_shape(L), synth.w_shape(L), (1, 1), pad)
    # the input derivative is a 3x3 sum over dzdy with the layer's input channels as its filters: the row-pair
    # kernel takes it when those are more than 32
    Kg = K // (D // Df)
    fwd = "igemm_f23"
    bwd = "igemm_f23" if Df > 32 else "igemm"
    ho, wo = oracle.output_size(synth.x_shape(L), synth.w_shape(L), (1, 1), pad)
    wg = "wgrad_f23" if N * ho * wo >= 64 else "wgrad_igemm"      # not for reductions over a handful of pixels
    assert [B.mcn_conv_kernel_name(d, op) for op in range(3)] == [fwd, bwd, wg]
    for with_bias in (True, False):
        U.assert_errors(U.run_layer_full(L, with_bias=with_bias, misalign=case % 2), label="row pairs %d" % case)


def test_row_pair_kernels_random_geometries():
    """3x3 filters at stride 1 at random plane sizes (odd and even, down to a single row), pads up to 5 per side, one to
    three groups, ragged filter and channel counts: whichever of the three passes qualify run on the row-pair
    kernels, the rest on the others."""
    rng = np.random.default_rng(161803)
    for t in range(40):
        g = int(rng.choice([1, 1, 2, 3]))
        Df = int(rng.choice([8, 16, 20, 24, 40, 48, 72, 104]))
        Kg = int(rng.choice([33, 40, 56, 64, 65, 72, 96, 130, 136, 200]))
        pad = [int(v) for v in rng.integers(0, 6, size=4)]
        lo_h, lo_w = max(1, 3 - pad[0] - pad[1]), max(1, 3 - pad[2] - pad[3])
        H = int(rng.integers(lo_h, lo_h + int(rng.choice([4, 12, 45]))))       # a third of the planes are tiny
        W = int(rng.integers(lo_w, lo_w + int(rng.choice([4, 12, 30]))))
        L = custom_layer(H, W, g * Df, int(rng.integers(1, 6)), 3, 3, Df, g * Kg, (1, 1), pad, idx=560 + t)
        d = B.make_desc(synth.x_shape(L), synth.w_shape(L), (1, 1), pad)
        print("random row-pair case", t, L, [B.mcn_conv_kernel_name(d, op) for op in range(3)], flush=True)
        U.assert_errors(U.run_layer_full(L, with_bias=bool(t % 2), seed=t, misalign=t % 4), label="random row pairs %d %r" % (t, L))


# ---- dzdw and dzdb in one call (Sec. 2.3.2: the backward mode returns both) ---------------
def test_filter_and_bias_derivative_in_one_call_small():
    """Geometries where the call runs the two passes one after the other: results identical to the separate calls."""
    for i, (H, W, D, N, Hf, Wf, Df, K, st, pad) in enumerate((
            (13, 9, 4, 3, 3, 2, 2, 6, (2, 1), (1, 2, 0, 1)), (20, 20, 16, 2, 3, 3, 16, 48, (1, 1), (1, 1, 1, 1)),
            (6, 6, 8, 5, 6, 6, 8, 7, (1, 1), (0, 0, 0, 0)), (16, 16, 32, 4, 5, 5, 32, 32, (1, 1), (2, 2, 2, 2)))):
        L = custom_layer(H, W, D, N, Hf, Wf, Df, K, st, pad, idx=600 + i)
        x, p = U.gpu(synth.make_x(L)), None
        ho, wo = oracle.output_size(synth.x_shape(L), synth.w_shape(L), st, pad)
        p = U.gpu(synth.make_dzdy(L, ho, wo))
        d = B.make_desc(synth.x_shape(L), synth.w_shape(L), st, pad)
        assert B.mcn_conv_kernel_name(d, B.MCN_OP_BACKWARD_FILTER_BIAS) == "two passes"
        dw, db = B.conv_backward_filter_bias(x, synth.w_shape(L), p, st, pad)
        dw2 = B.conv_backward_filter(x, synth.w_shape(L), p, st, pad)
        db2 = B.conv_backward_bias(synth.x_shape(L), synth.w_shape(L), p, st, pad)
        torch.cuda.synchronize()
        assert torch.equal(dw, dw2) and torch.equal(db, db2), i


# (the one-kernel form of that call, on layers that stream from memory: tests/test_gpu_full_size_parity.py)


def test_filter_rows_that_meet_no_input_keep_exact_zeros():
    """Planes of one or two rows under large pads: some filter row never overlaps the input, its derivative is
    structurally zero and must come out as exactly 0 (norm_err checks that), which a difference of rounded sums
    would not give: the filter derivative of such layers stays on the kernel that sums the taps one by one."""
    for i, (H, W, D, N, Df, K, pad) in enumerate(((1, 20, 72, 1, 24, 387, (1, 3, 1, 0)), (1, 9, 16, 2, 16, 40, (2, 1, 1, 1)),
                                                  (2, 12, 32, 3, 32, 72, (3, 3, 0, 2)), (2, 7, 16, 2, 16, 96, (0, 1, 1, 1)))):
        L = custom_layer(H, W, D, N, 3, 3, Df, K, (1, 1), pad, idx=640 + i)
        d = B.make_desc(synth.x_shape(L), synth.w_shape(L), (1, 1), pad)
        names = [B.mcn_conv_kernel_name(d, op) for op in range(3)]
        print("case", i, L, names, flush=True)
        if i < 2:       # in the other two every filter row meets an input row
            assert names[2] == "wgrad_igemm", names
        U.assert_errors(U.run_layer_full(L, with_bias=bool(i % 2)), label="few rows %d" % i)


def test_row_pair_kernel_only_where_it_applies():
    """Other filter sizes, strides, few filters or few channels per group keep the kernels that compute one output
    row per pixel."""
    for (Hf, Wf, Df, K, st) in ((3, 3, 16, 32, (1, 1)), (3, 3, 12, 64, (1, 1)), (3, 3, 16, 64, (2, 1)), (3, 3, 16, 64, (1, 2)),
                                (4, 3, 16, 64, (1, 1)), (3, 5, 16, 64, (1, 1)), (3, 3, 8, 64, (1, 1))):      # 12, 8: under 16 channels
        L = custom_layer(12, 12, Df, 2, Hf, Wf, Df, K, st, (1, 1, 1, 1), idx=520)
        d = B.make_desc(synth.x_shape(L), synth.w_shape(L), st, (1, 1, 1, 1))
        assert B.mcn_conv_kernel_name(d, 0) == "igemm", (Hf, Wf, Df, K, st)
        # the filter derivative: 3x3 at stride 1 with more than 32 filters per group, whatever the channels
        expect = "wgrad_f23" if (Hf, Wf, st) == (3, 3, (1, 1)) and K > 32 else "wgrad_igemm"
        assert B.mcn_conv_kernel_name(d, 2) == expect, (Hf, Wf, Df, K, st)


ONE_ROW = [(16, 12, 16, 3, 16, 48, (1, 1, 1, 1)), (15, 13, 16, 2, 16, 40, (1, 1, 1, 1)), (11, 14, 32, 3, 32, 70, (2, 0, 1, 2)),
           (20, 10, 48, 2, 16, 144, (1, 1, 1, 1)), (40, 40, 32, 8, 32, 64, (1, 1, 1, 1)), (28, 28, 64, 16, 64, 256, (1, 1, 1, 1))]


@pytest.mark.parametrize("case", range(len(ONE_ROW)))
def test_3x3_stride1_plain_order_of_summation(case):
    """MCN_PREC_FP32_PLAIN, chosen per call: 3x3 stride-1 layers on the kernels that compute one output row per
    pixel and add the products of Sec. 4.1's sum one by one."""
    H, W, D, N, Df, K, pad = ONE_ROW[case]
    L = custom_layer(H, W, D, N, 3, 3, Df, K, (1, 1), pad, idx=540 + case)
    d = B.make_desc(synth.x_shape(L), synth.w_shape(L), (1, 1), pad, B.MCN_PREC_FP32_PLAIN)
    assert [B.mcn_conv_kernel_name(d, op) for op in range(3)] == ["igemm", "igemm", "wgrad_igemm"]
    U.assert_errors(U.run_layer_full(L, precision=B.MCN_PREC_FP32_PLAIN, with_bias=bool(case % 2)), label="one row per pixel %d" % case)


# ---- 65 to 96 filters per group: tiles of 96 filters -------------------------------------------
FILTERS_96 = [
    # H   W   D   N  Hf  Wf  Df  K    stride  pad
    (31, 29, 6, 5, 3, 3, 3, 130, (1, 1), (1, 1, 1, 1)),       # two groups of 65
    (20, 20, 16, 4, 3, 3, 16, 96, (1, 1), (1, 1, 1, 1)),      # exactly one tile
    (40, 33, 3, 6, 7, 7, 3, 80, (2, 2), (3, 3, 3, 3)),        # three channels, stride 2
    (16, 16, 64, 8, 1, 1, 64, 90, (1, 1), (0, 0, 0, 0)),      # 1x1
    (24, 24, 8, 5, 5, 5, 8, 192, (1, 1), (2, 2, 2, 2)),       # two tiles per group
    (55, 55, 3, 16, 11, 11, 3, 96, (4, 4), (0, 0, 0, 0)),     # first layer of the Krizhevsky-style network, small: 363 coefficients in one tile
    (30, 26, 12, 6, 5, 5, 12, 72, (1, 1), (2, 2, 2, 2)),      # 300 coefficients: the 96 x 384 tile, ragged both ways
]


@pytest.mark.parametrize("case", range(len(FILTERS_96)))
def test_layers_with_65_to_96_filters_per_group(case):
    H, W, D, N, Hf, Wf, Df, K, st, pad = FILTERS_96[case]
    L = custom_layer(H, W, D, N, Hf, Wf, Df, K, st, pad, idx=800 + case)
    for prec in (B.MCN_PREC_FP32, B.MCN_PREC_FP32_PLAIN):
        U.assert_errors(U.run_layer_full(L, precision=prec, with_bias=bool(case % 2)), label="96-filter tiles %d" % case)


# ---- which kernels the dispatcher picks ----------------------------------------------
def test_workload_layers_run_on_the_matrix_core_kernels():
    """No layer of the workloads may fall back to the one-result-per-thread kernels."""
    for name, L in synth.LAYERS.items():
        d = B.make_desc(synth.x_shape(L), synth.w_shape(L), L["stride"], L["pad"])
        names = [B.mcn_conv_kernel_name(d, op) for op in range(4)]
        assert "direct" not in names, (name, names)
    d = B.make_desc(synth.x_shape(synth.LAYERS["5a"]), synth.w_shape(synth.LAYERS["5a"]))
    assert [B.mcn_conv_kernel_name(d, op) for op in range(3)] == ["fc_gemm"] * 3


# ---- fully-connected case (Sec. 4.1): matrix-product path, ragged sizes --------------
FC_CASES = [
    # H  W  D   N   K
    (6, 6, 8, 5, 7),          # everything smaller than one tile
    (3, 5, 33, 130, 70),      # N and K ragged against 128-wide tiles, R = 495 not a multiple of anything
    (1, 1, 300, 40, 129),     # 1x1 input: a plain matrix product
    (7, 2, 16, 257, 33),
]


@pytest.mark.parametrize("case", range(len(FC_CASES)))
def test_fully_connected_layers(case):
    H, W, D, N, K = FC_CASES[case]
    L = custom_layer(H, W, D, N, H, W, D, K, idx=40 + case)
    d = B.make_desc(synth.x_shape(L), synth.w_shape(L))
    assert B.mcn_conv_kernel_name(d, 0) == "fc_gemm"
    U.assert_errors(U.run_layer_full(L, with_bias=(case % 2 == 0)), label="fc %d" % case)


# ---- strided input derivative: every stride phase, phases without taps ------------------
STRIDED = [
    # H  W  D  N  Hf Wf Df K   stride   pad
    (23, 19, 8, 3, 5, 4, 8, 12, (2, 3), (2, 1, 0, 3)),
    (31, 31, 3, 2, 11, 11, 3, 20, (4, 4), (0, 0, 0, 0)),     # first layer of the Krizhevsky-style network, small
    (20, 18, 4, 2, 2, 3, 4, 6, (4, 5), (1, 0, 2, 2)),        # stride larger than the filter: rows/columns no tap reaches
    (17, 9, 6, 2, 3, 3, 3, 8, (3, 1), (1, 1, 1, 1)),         # two groups
    (12, 40, 5, 3, 1, 7, 5, 9, (2, 2), (0, 0, 3, 3)),
]


@pytest.mark.parametrize("case", range(len(STRIDED)))
def test_strided_layers(case):
    H, W, D, N, Hf, Wf, Df, K, st, pad = STRIDED[case]
    L = custom_layer(H, W, D, N, Hf, Wf, Df, K, st, pad, idx=60 + case)
    d = B.make_desc(synth.x_shape(L), synth.w_shape(L), st, pad)
    assert B.mcn_conv_kernel_name(d, 1) == "igemm"
    U.assert_errors(U.run_layer_full(L, with_bias=(case % 2 == 1)), label="strided %d" % case)


# ---- work sharing between blocks: many tiles, few tiles, shared tiles -------------------
def test_tiles_shared_between_blocks_match_whole_tiles():
    """Same layer at batch sizes that give fewer tiles than compute units (every tile is
    shared), about as many, and many more; every element compared."""
    base = custom_layer(20, 20, 32, 1, 3, 3, 32, 160, (1, 1), (1, 1, 1, 1), idx=80)
    for nb in (1, 3, 40):
        U.assert_errors(U.run_layer_full(synth.with_batch(base, nb)), label="sharing N=%d" % nb)
    # enough pixels that most tiles are computed by one block alone (the direct store path)
    big = custom_layer(40, 40, 16, 200, 3, 3, 16, 64, (1, 1), (1, 1, 1, 1), idx=81)
    U.assert_errors(U.run_layer_full(big), label="whole tiles, 3x3")
    big5 = custom_layer(24, 24, 6, 150, 5, 5, 6, 20, (1, 1), (2, 2, 2, 2), idx=82)
    U.assert_errors(U.run_layer_full(big5), label="whole tiles, 5x5, ragged filters")


# ---- device pointers carry no alignment promise beyond that of a float ----------------------
ANY_ALIGNMENT = [
    custom_layer(16, 12, 16, 6, 3, 3, 16, 40, (1, 1), (1, 1, 1, 1), idx=90),      # 3x3 instantiation
    custom_layer(24, 10, 64, 5, 1, 1, 64, 48, (1, 1), (0, 0, 0, 0), idx=91),      # 1x1 instantiation
    custom_layer(8, 8, 8, 30, 5, 5, 8, 24, (1, 1), (2, 2, 2, 2), idx=92),         # 5x5 instantiation
    custom_layer(20, 9, 6, 4, 4, 2, 6, 20, (1, 2), (2, 1, 0, 1), idx=93),         # general kernel, pad 2
    custom_layer(28, 28, 12, 3, 3, 3, 6, 18, (2, 2), (0, 1, 1, 0), idx=94),       # stride 2, two groups
    custom_layer(40, 7, 5, 9, 7, 3, 5, 12, (3, 1), (1, 1, 1, 1), idx=95),         # stride 3
    custom_layer(4, 4, 40, 70, 4, 4, 40, 150, idx=96),                            # fully connected
]


@pytest.mark.parametrize("case", range(len(ANY_ALIGNMENT)))
def test_inputs_at_any_pointer_alignment(case):
    """x, w and dzdy 0, 4, 8 or 12 bytes past a 16-byte boundary (the kernels load some operands 16 bytes
    per lane; none of that may lean on the caller's allocation)."""
    for misalign in (0, 1, 2, 3):
        U.assert_errors(U.run_layer_full(ANY_ALIGNMENT[case], misalign=misalign),
                        label="case %d, %d floats past alignment" % (case, misalign))


def test_tall_input_many_row_blocks():
    # many row blocks per image (the planner cuts the 224 rows)
    L = custom_layer(224, 40, 16, 2, 3, 3, 16, 64, (1, 1), (1, 1, 1, 1), idx=97)
    U.assert_errors(U.run_layer_full(L), label="tall")
    U.assert_errors(U.run_layer_full(L, misalign=2), label="tall, 8 bytes past alignment")


# ---- semantics of the boundary ---------------------------------------------------
def test_outputs_are_overwritten_and_runs_are_bit_identical():
    L = synth.with_batch(synth.LAYERS["2b"], 4)
    st, pad = L["stride"], L["pad"]
    x, w, b = (U.gpu(t) for t in (synth.make_x(L), synth.make_w(L), synth.make_b(L)))
    ho, wo = B.mcn_conv_output_size(B.make_desc(x.shape, w.shape, st, pad))
    p = U.gpu(synth.make_dzdy(L, ho, wo))
    outs1 = [B.conv_forward(x, w, b, st, pad), B.conv_backward_data(x.shape, w, p, st, pad),
             B.conv_backward_filter(x, w.shape, p, st, pad), B.conv_backward_bias(x.shape, w.shape, p, st, pad)]
    # second run into buffers pre-filled with NaN / large values: nothing may leak through
    bufs = [torch.full_like(o, float("nan")) for o in outs1]
    bufs[2].fill_(1e30)
    B.conv_forward(x, w, b, st, pad, out=bufs[0])
    B.conv_backward_data(x.shape, w, p, st, pad, out=bufs[1])
    B.conv_backward_filter(x, w.shape, p, st, pad, out=bufs[2])
    B.conv_backward_bias(x.shape, w.shape, p, st, pad, out=bufs[3])
    torch.cuda.synchronize()
    for a, c in zip(outs1, bufs):
        assert torch.equal(a, c)


def test_null_bias_equals_zero_bias():
    L = synth.LAYERS["5c"]
    st, pad = L["stride"], L["pad"]
    x, w = U.gpu(synth.make_x(L)), U.gpu(synth.make_w(L))
    y0 = B.conv_forward(x, w, None, st, pad)
    y1 = B.conv_forward(x, w, torch.zeros(L["K"], device="cuda"), st, pad)
    assert torch.equal(y0, y1)


def test_runs_on_a_side_stream():
    L = synth.LAYERS["1"]
    st, pad = L["stride"], L["pad"]
    x, w, b = U.gpu(synth.make_x(L)), U.gpu(synth.make_w(L)), U.gpu(synth.make_b(L))
    ref = B.conv_forward(x, w, b, st, pad)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        y = B.conv_forward(x, w, b, st, pad)
    s.synchronize()
    assert torch.equal(ref, y)


# ---- the two orders of summation on inputs of graded magnitude -------------------------------------
def _graded_layer_tensors(L, seed):
    """Filter rows scaled 1e3, 1, 1e-3 and input rows scaled 1e-3, 1, 1e3 in turn: for every third output row the
    result's own products w[t] x[i+t] are all of size 1 while products of other pairings of the same rows
    (w[0] x[i+2]) are of size 1e6."""
    x, w, b = synth.make_x(L, seed), synth.make_w(L, seed), synth.make_b(L, seed)
    rows = torch.tensor([1e-3, 1.0, 1e3])[torch.arange(L["H"]) % 3]
    x = (x * rows).contiguous()                      # last axis = rows (first index of the manual's arrays)
    w = (w * torch.tensor([1e3, 1.0, 1e-3])).contiguous()
    return x, w, b


def test_summation_order_modes_on_graded_magnitudes():
    """3x3 stride-1 layer whose filter rows and input rows span six orders of magnitude.  MCN_PREC_FP32_PLAIN must
    meet the bars against each result's own sum of |w||x|.  The default order (pairs of output rows, four products per
    filter column) is bounded by the sum over ALL pairings of the three filter rows with the three input rows of
    the result's field (forward, dzdx) resp. by the sum of the normalisers of the three row taps of a filter
    column (dzdw); against the result's own normaliser its error is reported, and is expected to be much larger."""
    L = custom_layer(36, 20, 32, 4, 3, 3, 32, 64, (1, 1), (1, 1, 1, 1), idx=700)
    st, pad = L["stride"], L["pad"]
    x, w, b = _graded_layer_tensors(L, 0)
    ho, wo = oracle.output_size(x.shape, w.shape, st, pad)
    p = synth.make_dzdy(L, ho, wo)
    p = (p * torch.tensor([1e3, 1.0, 1e-3])[torch.arange(ho) % 3]).contiguous()
    xd, wd, bd, pd = U.np64(x), U.np64(w), U.np64(b), U.np64(p)
    ref = {"y": oracle.forward(xd, wd, bd, st, pad), "dx": oracle.backward_data(x.shape, wd, pd, st, pad),
           "dw": oracle.backward_filter(xd, w.shape, pd, st, pad)}
    own = {"y": oracle.forward(np.abs(xd), np.abs(wd), np.abs(bd), st, pad),
           "dx": oracle.backward_data(x.shape, np.abs(wd), np.abs(pd), st, pad),
           "dw": oracle.backward_filter(np.abs(xd), w.shape, np.abs(pd), st, pad)}
    # every filter row replaced by the sum of the three rows' absolute values: all pairings of rows
    wsum = np.broadcast_to(np.abs(wd).sum(axis=3, keepdims=True), wd.shape).copy()
    cross = {"y": oracle.forward(np.abs(xd), wsum, np.abs(bd), st, pad),
             "dx": oracle.backward_data(x.shape, wsum, np.abs(pd), st, pad),
             "dw": np.broadcast_to(own["dw"].sum(axis=3, keepdims=True), own["dw"].shape).copy()}
    xg, wg, bg, pg = U.gpu(x), U.gpu(w), U.gpu(b), U.gpu(p)
    report = {}
    for prec in (B.MCN_PREC_FP32, B.MCN_PREC_FP32_PLAIN):
        d = B.make_desc(x.shape, w.shape, st, pad, prec)
        names = [B.mcn_conv_kernel_name(d, op) for op in range(3)]
        assert names == (["igemm_f23", "igemm", "wgrad_f23"] if prec == B.MCN_PREC_FP32 else ["igemm", "igemm", "wgrad_igemm"])
        got = {"y": B.conv_forward(xg, wg, bg, st, pad, prec), "dx": B.conv_backward_data(x.shape, wg, pg, st, pad, prec),
               "dw": B.conv_backward_filter(xg, w.shape, pg, st, pad, prec)}
        torch.cuda.synchronize()
        for k in got:
            g = got[k].cpu().numpy()
            report[(prec, k)] = (U.norm_err(g, ref[k], own[k]), U.norm_err(g, ref[k], cross[k]))
    for (prec, k), (e_own, e_cross) in sorted(report.items()):
        print("graded magnitudes, precision %d, %s: error / own sum %.2e, / sum over all row pairings %.2e" % (prec, k, e_own, e_cross), flush=True)
    for k, tol in (("y", U.TOL_FWD), ("dx", U.TOL_BWD), ("dw", U.TOL_BWD)):
        assert report[(B.MCN_PREC_FP32_PLAIN, k)][0] <= tol, (k, report)
        assert report[(B.MCN_PREC_FP32, k)][1] <= tol, (k, report)
    # the input derivative of this layer (32 channels) runs on the one-row kernel in both modes
    assert report[(B.MCN_PREC_FP32, "dx")][0] <= U.TOL_BWD


def test_summation_order_modes_on_graded_magnitudes_wide():
    """The same with more than 32 channels per group, so that the input derivative takes the row-pair kernel too."""
    L = custom_layer(24, 16, 48, 3, 3, 3, 48, 64, (1, 1), (1, 1, 1, 1), idx=701)
    st, pad = L["stride"], L["pad"]
    x, w, b = _graded_layer_tensors(L, 1)
    ho, wo = oracle.output_size(x.shape, w.shape, st, pad)
    p = synth.make_dzdy(L, ho, wo)
    p = (p * torch.tensor([1e3, 1.0, 1e-3])[torch.arange(ho) % 3]).contiguous()
    wd, pd = U.np64(w), U.np64(p)
    ref = oracle.backward_data(x.shape, wd, pd, st, pad)
    own = oracle.backward_data(x.shape, np.abs(wd), np.abs(pd), st, pad)
    wsum = np.broadcast_to(np.abs(wd).sum(axis=3, keepdims=True), wd.shape).copy()
    cross = oracle.backward_data(x.shape, wsum, np.abs(pd), st, pad)
    wg, pg = U.gpu(w), U.gpu(p)
    d = B.make_desc(x.shape, w.shape, st, pad)
    assert B.mcn_conv_kernel_name(d, 1) == "igemm_f23"
    dx = B.conv_backward_data(x.shape, wg, pg, st, pad).cpu().numpy()
    dxp = B.conv_backward_data(x.shape, wg, pg, st, pad, B.MCN_PREC_FP32_PLAIN).cpu().numpy()
    e = (U.norm_err(dx, ref, own), U.norm_err(dx, ref, cross), U.norm_err(dxp, ref, own))
    print("graded magnitudes, dzdx: default order %.2e of own sum, %.2e of all pairings; plain order %.2e of own sum" % e, flush=True)
    assert e[1] <= U.TOL_BWD and e[2] <= U.TOL_BWD


def test_batches_of_more_than_two_gibibytes():
    """Arrays of 2^31 bytes or more (under 2^31 elements) run on the matrix-core kernels: offsets inside the kernels
    are relative to an image.  Results at sampled places, dzdw and dzdb everywhere."""
    L = custom_layer(64, 64, 16, 8400, 3, 3, 16, 16, (1, 1), (1, 1, 1, 1), idx=710)
    assert 4 * L["H"] * L["W"] * L["D"] * L["N"] > (1 << 31)
    d = B.make_desc(synth.x_shape(L), synth.w_shape(L), L["stride"], L["pad"])
    names = [B.mcn_conv_kernel_name(d, op) for op in range(4)]
    assert "direct" not in names, names
    U.assert_errors(U.run_layer_sampled(L, n_filt=None), label="2.2 GB arrays %r" % names)
