"""Pins for the CPU oracle of the spatial pooling block (Sec. 4.3, 5.2, 6.3 of the MatConvNet
manual, arXiv 1412.4564): hand-worked numbers, brute force with an explicitly padded array,
library routines, the sum-pooling-as-grouped-convolution remark of Sec. 4.1, identities of the
selector matrix, and finite differences."""
import itertools
import json
import os

import numpy as np
import pytest

import oracle
from oracle import pool


def colmajor(values, dims):
    a, b, c, d = dims
    return np.asarray(values, dtype=np.float64).reshape(d, c, b, a)


def random_case(rng, max_hw=9):
    Hp, Wp = int(rng.integers(1, 5)), int(rng.integers(1, 5))
    H, W = int(rng.integers(1, max_hw + 1)), int(rng.integers(1, max_hw + 1))
    pad = [int(rng.integers(0, Hp)), int(rng.integers(0, Hp)), int(rng.integers(0, Wp)), int(rng.integers(0, Wp))]
    while H + pad[0] + pad[1] < Hp:
        H += 1
    while W + pad[2] + pad[3] < Wp:
        W += 1
    stride = (int(rng.integers(1, 4)), int(rng.integers(1, 4)))
    x = rng.standard_normal((int(rng.integers(1, 4)), int(rng.integers(1, 4)), W, H))
    ho, wo = pool.output_size(x.shape, (Hp, Wp), stride, pad)
    p = rng.standard_normal((x.shape[0], x.shape[1], wo, ho))
    return x, p, (Hp, Wp), stride, tuple(pad)


def test_hand_worked_examples(golden_dir):
    with open(os.path.join(golden_dir, "pool_hand_examples.json")) as fh:
        examples = json.load(fh)["examples"]
    assert len(examples) >= 2
    for ex in examples:
        x = colmajor(ex["x"], ex["x_hwdn"])
        Ho, Wo, D, N = ex["y_hwdn"]
        p = colmajor(ex["dzdy"], ex["y_hwdn"])
        for m in ("max", "avg"):
            y = pool.forward(x, ex["window"], ex["stride"], ex["pad"], m)
            assert y.shape == (N, D, Wo, Ho)
            np.testing.assert_allclose(y.ravel(), ex["y_" + m], rtol=0, atol=1e-15, err_msg=ex["name"])
            dx = pool.backward(x, p, ex["window"], ex["stride"], ex["pad"], m)
            np.testing.assert_allclose(dx.ravel(), ex["dzdx_" + m], rtol=0, atol=1e-13, err_msg=ex["name"])


def test_output_size_and_errors():
    # the size rule is the convolution block's (Sec. 5.2); that one is pinned by brute force elsewhere
    for H, Hp, S in itertools.product(range(1, 9), range(1, 5), range(1, 4)):
        for pt, pb in itertools.product(range(0, Hp), range(0, Hp)):
            if H + pt + pb < Hp:
                with pytest.raises(pool.OracleError) as e:
                    pool.output_size((1, 1, 1, H), (Hp, 1), (S, 1), (pt, pb, 0, 0))
                assert e.value.code == pool.WINDOW_TOO_LARGE
                continue
            expect = oracle.output_size((1, 1, 1, H), (1, 1, 1, Hp), (S, 1), (pt, pb, 0, 0))[0]
            assert pool.output_size((1, 1, 1, H), (Hp, 1), (S, 1), (pt, pb, 0, 0)) == (expect, 1)
            assert pool.output_size((1, 1, H, 1), (1, Hp), (1, S), (0, 0, pt, pb)) == (1, expect)
    # Sec. 5.2.1: pads are at most window - 1
    for pad in [(3, 0, 0, 0), (0, 3, 0, 0), (0, 0, 2, 0), (0, 0, 0, 2)]:
        with pytest.raises(pool.OracleError) as e:
            pool.output_size((1, 1, 8, 8), (3, 2), (1, 1), pad)
        assert e.value.code == pool.PAD_TOO_LARGE
    for bad in [dict(window=(0, 1)), dict(stride=(1, 0)), dict(pad=(-1, 0, 0, 0)), dict(method=2)]:
        kw = dict(xshape=(1, 1, 8, 8), window=(2, 2), stride=(1, 1), pad=(0, 0, 0, 0), method="max")
        kw.update(bad)
        with pytest.raises(pool.OracleError) as e:
            pool.output_size(**kw)
        assert e.value.code == pool.BAD_ARG


def brute(x, window, stride, pad, method):
    """Pad explicitly (with -inf, or with NaN that the mean skips) and slide the window."""
    N, D, W, H = x.shape
    Hp, Wp = window
    fill = -np.inf if method == "max" else np.nan
    xp = np.full((N, D, W + pad[2] + pad[3], H + pad[0] + pad[1]), fill)
    xp[:, :, pad[2]:pad[2] + W, pad[0]:pad[0] + H] = x
    Ho = (H + pad[0] + pad[1] - Hp) // stride[0] + 1
    Wo = (W + pad[2] + pad[3] - Wp) // stride[1] + 1
    y = np.empty((N, D, Wo, Ho))
    for jo in range(Wo):
        for io in range(Ho):
            win = xp[:, :, jo * stride[1]:jo * stride[1] + Wp, io * stride[0]:io * stride[0] + Hp].reshape(N, D, -1)
            y[:, :, jo, io] = win.max(axis=2) if method == "max" else np.nanmean(win, axis=2)
    return y


def test_forward_matches_brute_force_on_padded_array():
    rng = np.random.default_rng(301)
    for _ in range(80):
        x, p, window, stride, pad = random_case(rng)
        for m in ("max", "avg"):
            np.testing.assert_allclose(pool.forward(x, window, stride, pad, m), brute(x, window, stride, pad, m),
                                       rtol=0, atol=1e-13)


def test_matches_torch_pooling_for_symmetric_pads():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    rng = np.random.default_rng(302)
    done = 0
    while done < 30:
        x, p, window, stride, pad = random_case(rng)
        if pad[0] != pad[1] or pad[2] != pad[3] or 2 * pad[0] > window[0] or 2 * pad[2] > window[1]:
            continue      # torch takes one pad per direction, at most half the window
        done += 1
        t = torch.from_numpy(x).requires_grad_(True)
        # arrays are (N, C, W, H): torch's first spatial axis is our W
        k, s, pd = (window[1], window[0]), (stride[1], stride[0]), (pad[2], pad[0])
        for m, y in (("max", F.max_pool2d(t, k, s, pd)), ("avg", F.avg_pool2d(t, k, s, pd, count_include_pad=False))):
            np.testing.assert_allclose(pool.forward(x, window, stride, pad, m), y.detach().numpy(), rtol=0, atol=1e-13)
            (g,) = torch.autograd.grad(y, t, torch.from_numpy(p))
            np.testing.assert_allclose(pool.backward(x, p, window, stride, pad, m), g.numpy(), rtol=0, atol=1e-13)


def test_sum_pooling_is_a_grouped_convolution_with_ones():
    # Sec. 4.1 "Filter groups": D groups of one-channel all-ones filters sum each window; dividing by
    # the same convolution of an all-ones array (the count of samples inside) gives the average
    rng = np.random.default_rng(303)
    for _ in range(40):
        x, p, window, stride, pad = random_case(rng)
        D = x.shape[1]
        ones = np.ones((D, 1, window[1], window[0]))
        s = oracle.forward(x, ones, None, stride, pad)
        cnt = oracle.forward(np.ones_like(x), ones, None, stride, pad)
        np.testing.assert_allclose(pool.forward(x, window, stride, pad, "avg"), s / cnt, rtol=0, atol=1e-13)
        # and its derivative is that convolution's input derivative of dzdy / count
        np.testing.assert_allclose(pool.backward(x, p, window, stride, pad, "avg"),
                                   oracle.backward_data(x.shape, ones, p / cnt, stride, pad), rtol=0, atol=1e-13)


def test_selector_identities():
    rng = np.random.default_rng(304)
    for _ in range(60):
        x, p, window, stride, pad = random_case(rng)
        for m in ("max", "avg"):
            y = pool.forward(x, window, stride, pad, m)
            dx = pool.backward(x, p, window, stride, pad, m)
            # y = S x and dzdx = S^T dzdy  =>  <dzdx, x> = <dzdy, y>
            assert abs(float((dx * x).sum()) - float((p * y).sum())) <= 1e-11 * (1 + float(np.abs(p * y).sum()))
            # every row of S sums to one: all of dzdy is handed on
            assert abs(float(dx.sum()) - float(p.sum())) <= 1e-11 * (1 + float(np.abs(p).sum()))
        ymax, yavg = pool.forward(x, window, stride, pad, "max"), pool.forward(x, window, stride, pad, "avg")
        assert np.all(ymax >= yavg - 1e-15)
        # max pooling commutes with increasing maps, average pooling is linear
        np.testing.assert_array_equal(pool.forward(np.exp(x), window, stride, pad, "max"), np.exp(ymax))
        np.testing.assert_allclose(pool.forward(3 * x - 1, window, stride, pad, "avg"), 3 * yavg - 1, rtol=0, atol=1e-13)


def test_one_by_one_window_subsamples():
    rng = np.random.default_rng(305)
    x = rng.standard_normal((2, 3, 7, 9))
    for m in ("max", "avg"):
        np.testing.assert_array_equal(pool.forward(x, (1, 1), (2, 3), (0, 0, 0, 0), m), x[:, :, ::3, ::2])
    whole = pool.forward(x, (9, 7), (1, 1), (0, 0, 0, 0), "max")
    np.testing.assert_array_equal(whole.reshape(2, 3), x.max(axis=(2, 3)))
    np.testing.assert_allclose(pool.forward(x, (9, 7), (1, 1), (0, 0, 0, 0), "avg").reshape(2, 3), x.mean(axis=(2, 3)),
                               rtol=0, atol=1e-14)


def test_finite_differences():
    rng = np.random.default_rng(306)
    for _ in range(8):
        x, p, window, stride, pad = random_case(rng, max_hw=5)
        for m in ("max", "avg"):
            dx = pool.backward(x, p, window, stride, pad, m)
            h = 1e-6       # distinct Gaussian samples differ by far more: the selection does not change
            flat = x.reshape(-1)
            for e in range(flat.size):
                old = flat[e]
                flat[e] = old + h
                zp = float((pool.forward(x, window, stride, pad, m) * p).sum())
                flat[e] = old - h
                zm = float((pool.forward(x, window, stride, pad, m) * p).sum())
                flat[e] = old
                assert abs((zp - zm) / (2 * h) - dx.reshape(-1)[e]) <= 1e-7 * (1 + np.abs(p).max())


def test_ties_go_to_the_first_maximum_in_memory_order():
    x = np.zeros((1, 1, 3, 3))           # every window is all ties
    p = np.arange(1.0, 5.0).reshape(1, 1, 2, 2)
    dx = pool.backward(x, p, (2, 2), (1, 1), (0, 0, 0, 0), "max")
    # window (io, jo) selects its top-left sample (io, jo)
    expect = np.zeros((3, 3))
    expect[:2, :2] = p[0, 0]
    np.testing.assert_array_equal(dx[0, 0], expect)
