"""The two measurement aids of the library, through the C ABI: the copy kernel copies, and
the register-only MFMA loop really issues the matrix instructions it is priced by (its
accumulators hold the products of the operands it feeds them)."""
import numpy as np
import pytest
import torch

from paper_1412_4564_amd import binding as B

pytestmark = pytest.mark.gpu


def stream():
    return torch.cuda.current_stream().cuda_stream


@pytest.mark.parametrize("n", [1, 3, 4, 1023, 4096 * 256 * 4 + 2, (1 << 24) + 1])
def test_copy_probe_copies(n):
    g = torch.Generator().manual_seed(n)
    src = torch.randn(n, generator=g).cuda()
    dst = torch.full((n + 8,), -7.0, device="cuda")
    assert B.mcn_probe_copy(src.data_ptr(), dst.data_ptr(), n, stream()) == B.MCN_OK
    torch.cuda.synchronize()
    assert torch.equal(dst[:n], src)
    assert bool((dst[n:] == -7.0).all())          # nothing past the end is touched


@pytest.mark.parametrize("precision,per_mfma,expect", [
    # A[i][k] = 1 + (i mod 8) (+ k within the lane's eight for bf16), B = 1/2 everywhere; a lane of the
    # lower / upper half-wave holds rows with (i mod 8) in 0..3 / 4..7, four times each, in each of
    # its four accumulators.
    (B.MCN_PREC_FP32, 2 * 32 * 32 * 2, (160.0, 416.0)),
    (B.MCN_PREC_BF16, 2 * 32 * 32 * 16, (3072.0, 5120.0)),
])
def test_mfma_probe_counts_its_work(precision, per_mfma, expect):
    iters = 3
    sink = torch.zeros(B.MCN_PROBE_SINK_FLOATS, device="cuda")
    st, flops = B.mcn_probe_mfma(precision, iters, sink.data_ptr(), sink.numel(), stream())
    assert st == B.MCN_OK
    torch.cuda.synchronize()
    assert flops == per_mfma * 4 * iters * 4 * 2048       # 4 accumulators, 4 waves, 2048 blocks
    got = sink.cpu().numpy().reshape(-1, 64)
    want = np.concatenate([np.full(32, expect[0] * iters), np.full(32, expect[1] * iters)])
    assert np.array_equal(got, np.broadcast_to(want, got.shape))
