"""mcn_conv_backward_bias_static: the bias derivative with its scratch in the library's own static device buffer
(for callers that cannot allocate), through the C ABI, against mcn_conv_backward_bias: two calls in a row, the
second on a smaller input, must each equal the existing entry point bit for bit (same kernels, same order of
additions) and meet the backward bar against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_1412_4564_amd import binding as B
from paper_1412_4564_amd import synth

import parity_util as U

pytestmark = pytest.mark.gpu


def _both(L, seed):
    st, pad = L["stride"], L["pad"]
    xs, ws = synth.x_shape(L), synth.w_shape(L)
    d = B.make_desc(xs, ws, st, pad)
    ho, wo = B.mcn_conv_output_size(d)
    p = synth.make_dzdy(L, ho, wo, seed)
    pg = p.cuda()
    stream = torch.cuda.current_stream().cuda_stream
    got = torch.full((L["K"],), float("nan"), device="cuda")
    status = B.mcn_conv_backward_bias_static(d, pg.data_ptr(), got.data_ptr(), stream)
    assert status == B.MCN_OK, status
    ref = B.conv_backward_bias(xs, ws, pg, st, pad)
    torch.cuda.synchronize()
    assert torch.equal(got, ref)
    pd = U.np64(p)
    e = U.norm_err(got.cpu().numpy(), oracle.backward_bias(xs, ws, pd, st, pad), oracle.backward_bias(xs, ws, np.abs(pd), st, pad))
    assert e <= U.TOL_BWD
    return e


def test_static_scratch_bias_derivative_two_calls_in_a_row():
    big = synth.with_batch(synth.LAYERS["4b"], 8)              # 56x56 planes, 256 filters: two-stage sum over chunks
    small = synth.LAYERS["5c"]                                 # 18x18 planes, 24 filters, 4 images
    rows = dict(H=6, W=6, D=8, N=70, Hf=6, Wf=6, Df=8, K=33, stride=(1, 1), pad=(0, 0, 0, 0), config=11, index=0)   # 1x1 planes
    errs = [_both(big, 0), _both(small, 1), _both(rows, 2), _both(small, 3), _both(big, 4)]
    print("static-scratch bias derivative, errors against the oracle:", ["%.2e" % e for e in errs], flush=True)
