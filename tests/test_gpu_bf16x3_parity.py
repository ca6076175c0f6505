"""MCN_PREC_FP32_BF16X3: fp32 arrays, operands of the forward pass and of dzdx split on chip into two bf16 planes
(hi + lo, 16 bits of the significand), three products per pair on the bf16 matrix core, fp32 accumulation.
The sum is the one of Sec. 4.1 of the manual, so the results are held to the fp32 bars against the fp64 oracle on
the unrounded inputs: 1e-4 forward, 1e-3 backward.  The bound that follows from the arithmetic is 1.2e-5 of the
sum of |w||x| (each operand is represented to 2^-18, the dropped lo*lo product is below 2^-16, fp32 accumulation
adds its own ~1e-7); the tests also assert that tighter figure."""
import numpy as np
import pytest
import torch

import oracle
from paper_1412_4564_amd import binding as B
from paper_1412_4564_amd import synth

import parity_util as U

pytestmark = pytest.mark.gpu
X3 = B.MCN_PREC_FP32_BF16X3
SPLIT_BOUND = 1.2e-5      # worst case of the split-operand products, relative to the sum of |w||x|


def custom_layer(H, W, D, N, Hf, Wf, Df, K, stride=(1, 1), pad=(0, 0, 0, 0), idx=0):
    return dict(H=H, W=W, D=D, N=N, Hf=Hf, Wf=Wf, Df=Df, K=K, stride=tuple(stride), pad=tuple(pad),
                config=13, index=idx)


CASES = [
    # H   W   D    N  Hf Wf Df  K    stride  pad            kernels of forward and dzdx
    (16, 12, 16, 3, 3, 3, 16, 48, (1, 1), (1, 1, 1, 1), ("igemm_bf16x3", "igemm_bf16x3")),
    (15, 13, 32, 2, 3, 3, 32, 40, (1, 1), (1, 1, 1, 1), ("igemm_bf16x3", "igemm_bf16x3")),
    (11, 14, 40, 3, 5, 5, 40, 72, (1, 1), (2, 0, 1, 2), ("igemm_bf16x3", "igemm_bf16x3")),      # channels and filters ragged against 16 / the tiles
    (20, 10, 48, 2, 3, 3, 16, 144, (1, 1), (1, 1, 1, 1), ("igemm_bf16x3", "igemm_bf16x3")),     # three groups
    (14, 14, 64, 4, 3, 3, 64, 160, (2, 2), (1, 1, 1, 1), ("igemm_bf16x3", "igemm_bf16x3")),     # stride 2: four phases of dzdx
    (30, 30, 160, 6, 3, 3, 80, 400, (1, 1), (1, 1, 1, 1), ("igemm_bf16x3", "igemm_bf16x3")),    # tiles shared between blocks
    (28, 28, 64, 16, 1, 1, 64, 256, (1, 1), (0, 0, 0, 0), ("igemm_bf16x3", "igemm_bf16x3")),    # 1x1
    (40, 40, 32, 8, 7, 3, 32, 64, (1, 2), (3, 3, 1, 1), None),                                  # many taps: several tap ranges per group of channels
    (27, 27, 96, 8, 5, 5, 48, 256, (1, 1), (2, 2, 2, 2), ("igemm_bf16x3", "igemm_bf16x3")),     # two groups, 25 taps
    (13, 9, 4, 3, 3, 2, 2, 6, (2, 1), (1, 2, 0, 1), ("igemm", "igemm")),                        # under 16 channels: fp32 kernels
]


@pytest.mark.parametrize("case", range(len(CASES)))
def test_split_operand_layers_every_element(case):
    H, W, D, N, Hf, Wf, Df, K, st, pad, kernels = CASES[case]
    L = custom_layer(H, W, D, N, Hf, Wf, Df, K, st, pad, idx=case)
    d = B.make_desc(synth.x_shape(L), synth.w_shape(L), st, pad, X3)
    names = [B.mcn_conv_kernel_name(d, op) for op in range(3)]
    print("split operands, case", case, names, flush=True)
    if kernels:
        assert tuple(names[:2]) == kernels, names
    assert "bf16" not in names[2]        # dzdw computes as under MCN_PREC_FP32
    for with_bias in (True, False):
        e = U.run_layer_full(L, precision=X3, with_bias=with_bias, seed=case)
        U.assert_errors(e, label="split operands %d" % case)            # the fp32 bars
        assert e["forward"] <= SPLIT_BOUND and e["backward_data"] <= SPLIT_BOUND, e


@pytest.mark.parametrize("name", ["4a", "4b", "4c", "3b", "5b"])
def test_split_operand_workload_layers_full_size(name):
    """Full-size layers under the split-operand mode: y and dzdx at sampled places, dzdw at sampled places, dzdb everywhere."""
    e = U.run_layer_sampled(synth.LAYERS[name], precision=X3)
    U.assert_errors(e, label="layer %s full size, split operands" % name)
    assert e["forward"] <= SPLIT_BOUND and e["backward_data"] <= SPLIT_BOUND, e


def test_split_operands_are_closer_than_rounded_operands():
    """On one layer: error of MCN_PREC_BF16 (operands rounded to 8 significant bits), of the split operands (16) and of
    fp32, against the oracle: each step down must be a step in accuracy."""
    L = custom_layer(24, 24, 64, 4, 3, 3, 64, 96, (1, 1), (1, 1, 1, 1), idx=50)
    errs = {p: U.run_layer_full(L, precision=p)["forward"] for p in (B.MCN_PREC_BF16, X3, B.MCN_PREC_FP32)}
    print("forward error by precision:", {k: "%.2e" % v for k, v in errs.items()}, flush=True)
    assert errs[B.MCN_PREC_BF16] > 20 * errs[X3] > 20 * errs[B.MCN_PREC_FP32] / 20
    assert errs[X3] < 1e-5 and errs[B.MCN_PREC_FP32] < 1e-6
