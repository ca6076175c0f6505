"""Pins for the CPU oracle: every check here compares oracle/ with something
that is NOT the oracle's own code path -- hand-worked numbers, closed forms,
textbook special cases, a structurally different matrix formulation, the
manual's 1-D transpose formula, finite differences and adjoint identities.

Citations are to the MatConvNet manual (arXiv 1412.4564).
"""
import itertools
import json
import os

import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(20141220)


def colmajor(values, hwdn):
    """Memory-order list + (H,W,D,N) -> array of shape (N,D,W,H)."""
    H, W, D, N = hwdn
    return np.asarray(values, dtype=np.float64).reshape(N, D, W, H)


# --------------------------------------------------------------------------
# P1  output size: Sec. 4.1 "Output size" vs. the inequality of Sec. 5.2
# --------------------------------------------------------------------------
def test_output_size_is_largest_window_count_that_fits():
    # Sec. 5.2: H'' is the largest i'' with  H' + S(i''-1) - P^-  <=  H + P^+.
    for H, Hf, Pt, Pb, S in itertools.product(range(1, 11), range(1, 8), range(0, 4), range(0, 4), range(1, 5)):
        if H + Pt + Pb < Hf:
            with pytest.raises(oracle.OracleError) as e:
                oracle.output_size((1, 1, 1, H), (1, 1, 1, Hf), (S, 1), (Pt, Pb, 0, 0))
            assert e.value.code == oracle.FILTER_TOO_LARGE
            continue
        brute = 0
        while Hf + S * (brute + 1 - 1) - Pt <= H + Pb:
            brute += 1
        ho, wo = oracle.output_size((1, 1, 1, H), (1, 1, 1, Hf), (S, 1), (Pt, Pb, 0, 0))
        assert (ho, wo) == (brute, 1)
        # the same rule must be applied to the horizontal direction with (left, right, S_w)
        ho, wo = oracle.output_size((1, 1, H, 1), (1, 1, Hf, 1), (1, S), (0, 0, Pt, Pb))
        assert (ho, wo) == (1, brute)


WORKLOAD_SHAPES = [  # x HWDN, w HWDK, stride, pad, expected (Ho, Wo): arithmetic done by hand from Sec. 4.1
    ((32, 32, 3, 8), (5, 5, 3, 32), (1, 1), (2, 2, 2, 2), (32, 32)),
    ((16, 16, 32, 100), (5, 5, 32, 32), (1, 1), (2, 2, 2, 2), (16, 16)),
    ((8, 8, 32, 100), (5, 5, 32, 64), (1, 1), (2, 2, 2, 2), (8, 8)),
    ((227, 227, 3, 128), (11, 11, 3, 96), (4, 4), (0, 0, 0, 0), (55, 55)),
    ((27, 27, 96, 128), (5, 5, 48, 256), (1, 1), (2, 2, 2, 2), (27, 27)),
    ((224, 224, 64, 32), (3, 3, 64, 64), (1, 1), (1, 1, 1, 1), (224, 224)),
    ((56, 56, 256, 32), (3, 3, 256, 256), (1, 1), (1, 1, 1, 1), (56, 56)),
    ((14, 14, 512, 32), (3, 3, 512, 512), (1, 1), (1, 1, 1, 1), (14, 14)),
    ((6, 6, 256, 256), (6, 6, 256, 4096), (1, 1), (0, 0, 0, 0), (1, 1)),
    ((28, 28, 512, 64), (1, 1, 512, 128), (1, 1), (0, 0, 0, 0), (28, 28)),
    ((37, 53, 16, 4), (3, 5, 16, 24), (2, 3), (1, 0, 2, 1), (18, 18)),
]


@pytest.mark.parametrize("x,w,stride,pad,expect", WORKLOAD_SHAPES)
def test_output_size_of_workload_shapes(x, w, stride, pad, expect):
    H, W, D, N = x
    Hf, Wf, Df, K = w
    assert oracle.output_size((N, D, W, H), (K, Df, Wf, Hf), stride, pad) == expect


def test_geometry_errors():
    ok = dict(xshape=(1, 4, 5, 5), fshape=(6, 2, 3, 3), stride=(1, 1), pad=(0, 0, 0, 0))
    assert oracle.output_size(**ok) == (3, 3)
    # D' must divide D (Sec. 4.1 "Filter groups")
    with pytest.raises(oracle.OracleError) as e:
        oracle.output_size((1, 4, 5, 5), (6, 3, 3, 3))
    assert e.value.code == oracle.BAD_GROUPS
    # the number of filters must split evenly over the groups
    with pytest.raises(oracle.OracleError) as e:
        oracle.output_size((1, 4, 5, 5), (5, 2, 3, 3))
    assert e.value.code == oracle.BAD_GROUPS
    for bad in [dict(stride=(0, 1)), dict(stride=(1, 0)), dict(pad=(-1, 0, 0, 0)), dict(pad=(0, 0, 0, -1)),
                dict(xshape=(0, 4, 5, 5)), dict(fshape=(6, 2, 0, 3))]:
        with pytest.raises(oracle.OracleError) as e:
            oracle.output_size(**{**ok, **bad})
        assert e.value.code == oracle.BAD_ARG
    # Sec. 4.1: padded input smaller than the filter is an error, in either direction
    with pytest.raises(oracle.OracleError) as e:
        oracle.output_size((1, 1, 5, 2), (1, 1, 3, 4), (1, 1), (1, 0, 0, 0))
    assert e.value.code == oracle.FILTER_TOO_LARGE
    assert oracle.output_size((1, 1, 5, 2), (1, 1, 3, 4), (1, 1), (1, 1, 0, 0)) == (1, 3)
    with pytest.raises(oracle.OracleError) as e:
        oracle.output_size((1, 1, 2, 5), (1, 1, 4, 3), (1, 1), (0, 0, 0, 1))
    assert e.value.code == oracle.FILTER_TOO_LARGE


# --------------------------------------------------------------------------
# P2-P4  hand-worked examples
# --------------------------------------------------------------------------
def _load_examples(golden_dir):
    with open(os.path.join(golden_dir, "hand_examples.json")) as fh:
        return json.load(fh)["examples"]


def test_hand_worked_examples(golden_dir):
    examples = _load_examples(golden_dir)
    assert len(examples) >= 3
    for ex in examples:
        x = colmajor(ex["x"], ex["x_hwdn"])
        w = colmajor(ex["w"], ex["w_hwdk"])
        b = None if ex["b"] is None else np.asarray(ex["b"], dtype=np.float64)
        st, pad = ex["stride"], ex["pad"]
        y = oracle.forward(x, w, b, st, pad)
        Ho, Wo, K, N = ex["y_hwkn"]
        assert y.shape == (N, K, Wo, Ho), ex["name"]
        np.testing.assert_array_equal(y.ravel(), np.asarray(ex["y"], dtype=np.float64), err_msg=ex["name"])
        p = np.asarray(ex["dzdy"], dtype=np.float64).reshape(y.shape)
        np.testing.assert_array_equal(oracle.backward_data(x.shape, w, p, st, pad).ravel(), ex["dzdx"], err_msg=ex["name"])
        np.testing.assert_array_equal(oracle.backward_filter(x, w.shape, p, st, pad).ravel(), ex["dzdw"], err_msg=ex["name"])
        np.testing.assert_array_equal(oracle.backward_bias(x.shape, w.shape, p, st, pad).ravel(), ex["dzdb"], err_msg=ex["name"])
        # the three inner products of the hand computation agree with each other
        y0 = oracle.forward(x, w, None, st, pad)
        assert float((y0 * p).sum()) == ex["inner"]
        assert float((x.ravel() * np.asarray(ex["dzdx"])).sum()) == ex["inner"]
        assert float((w.ravel() * np.asarray(ex["dzdw"])).sum()) == ex["inner"]


# --------------------------------------------------------------------------
# random geometry helper
# --------------------------------------------------------------------------
def random_case(rng, max_hw=9, groups=(1, 2, 3), allow_big_pad=True):
    g = int(rng.choice(groups))
    Df = int(rng.integers(1, 4))
    Kg = int(rng.integers(1, 4))
    D, K = g * Df, g * Kg
    Hf, Wf = int(rng.integers(1, 5)), int(rng.integers(1, 5))
    H, W = int(rng.integers(1, max_hw + 1)), int(rng.integers(1, max_hw + 1))
    pmax = 5 if allow_big_pad else 2
    pad = [int(v) for v in rng.integers(0, pmax, size=4)]
    while H + pad[0] + pad[1] < Hf:
        pad[1] += 1
    while W + pad[2] + pad[3] < Wf:
        pad[3] += 1
    stride = (int(rng.integers(1, 4)), int(rng.integers(1, 4)))
    N = int(rng.integers(1, 4))
    x = rng.standard_normal((N, D, W, H))
    w = rng.standard_normal((K, Df, Wf, Hf))
    b = rng.standard_normal((K,))
    Ho, Wo = oracle.output_size(x.shape, w.shape, stride, pad)
    p = rng.standard_normal((N, K, Wo, Ho))
    return x, w, b, p, stride, tuple(pad)


# --------------------------------------------------------------------------
# P8  matrix form of Sec. 6.1: y = phi(x) F, dF = phi(x)^T dY, dX = phi*(dY F^T)
#     (im2row map of Sec. 6.1 with the padded/strided index of Sec. 4.1)
# --------------------------------------------------------------------------
def im2row(xn, Hf, Wf, stride, pad, Ho, Wo):
    """phi(x) for one image and one group: rows p = io + Ho*jo, cols q = fi + Hf*(fj + Wf*d)."""
    Dg, W, H = xn.shape
    phi = np.zeros((Ho * Wo, Hf * Wf * Dg))
    for jo in range(Wo):
        for io in range(Ho):
            for d in range(Dg):
                for fj in range(Wf):
                    for fi in range(Hf):
                        i = stride[0] * io + fi - pad[0]
                        j = stride[1] * jo + fj - pad[2]
                        if 0 <= i < H and 0 <= j < W:
                            phi[io + Ho * jo, fi + Hf * (fj + Wf * d)] = xn[d, j, i]
    return phi


def row2im(M, Dg, W, H, Hf, Wf, stride, pad, Ho, Wo):
    """phi*(M): scatter-add every entry of M back to the sample it was read from."""
    out = np.zeros((Dg, W, H))
    for jo in range(Wo):
        for io in range(Ho):
            for d in range(Dg):
                for fj in range(Wf):
                    for fi in range(Hf):
                        i = stride[0] * io + fi - pad[0]
                        j = stride[1] * jo + fj - pad[2]
                        if 0 <= i < H and 0 <= j < W:
                            out[d, j, i] += M[io + Ho * jo, fi + Hf * (fj + Wf * d)]
    return out


def matrix_form(x, w, b, p, stride, pad):
    N, D, W, H = x.shape
    K, Df, Wf, Hf = w.shape
    g = D // Df
    Kg = K // g
    Ho = (H - Hf + pad[0] + pad[1]) // stride[0] + 1
    Wo = (W - Wf + pad[2] + pad[3]) // stride[1] + 1
    y = np.zeros((N, K, Wo, Ho))
    dx = np.zeros_like(x)
    dw = np.zeros_like(w)
    for m in range(g):
        # F: (Hf Wf Df) x Kg, column k is filter k flattened in memory order
        F = w[m * Kg:(m + 1) * Kg].reshape(Kg, -1).T
        for n in range(N):
            phi = im2row(x[n, m * Df:(m + 1) * Df], Hf, Wf, stride, pad, Ho, Wo)
            Y = phi @ F                                   # (Ho Wo) x Kg
            y[n, m * Kg:(m + 1) * Kg] = Y.T.reshape(Kg, Wo, Ho)
            dY = p[n, m * Kg:(m + 1) * Kg].reshape(Kg, -1).T
            dw[m * Kg:(m + 1) * Kg] += (phi.T @ dY).T.reshape(Kg, Df, Wf, Hf)
            dx[n, m * Df:(m + 1) * Df] = row2im(dY @ F.T, Df, W, H, Hf, Wf, stride, pad, Ho, Wo)
    y += b[None, :, None, None]
    return y, dx, dw


def test_matches_matrix_form_of_sec_6_1():
    rng = np.random.default_rng(61)
    for _ in range(40):
        x, w, b, p, stride, pad = random_case(rng)
        y, dx, dw = matrix_form(x, w, b, p, stride, pad)
        np.testing.assert_allclose(oracle.forward(x, w, b, stride, pad), y, rtol=0, atol=1e-12)
        np.testing.assert_allclose(oracle.backward_data(x.shape, w, p, stride, pad), dx, rtol=0, atol=1e-12)
        np.testing.assert_allclose(oracle.backward_filter(x, w.shape, p, stride, pad), dw, rtol=0, atol=1e-12)


# --------------------------------------------------------------------------
# P5  delta filters shift the input; 1x1 identity bank reproduces it
# --------------------------------------------------------------------------
def test_delta_filter_is_a_shift():
    rng = np.random.default_rng(5)
    N, D, W, H = 2, 3, 7, 6
    Hf, Wf = 3, 4
    x = rng.standard_normal((N, D, W, H))
    for (a, bb, c) in [(0, 0, 0), (2, 3, 1), (1, 2, 2), (2, 0, 0)]:
        for pad in [(0, 0, 0, 0), (1, 2, 3, 1), (2, 2, 0, 3)]:
            w = np.zeros((1, D, Wf, Hf))
            w[0, c, bb, a] = 1.0
            y = oracle.forward(x, w, None, (1, 1), pad)
            Ho, Wo = y.shape[3], y.shape[2]
            expect = np.zeros_like(y)
            for jo in range(Wo):
                for io in range(Ho):
                    i, j = io + a - pad[0], jo + bb - pad[2]
                    if 0 <= i < H and 0 <= j < W:
                        expect[:, 0, jo, io] = x[:, c, j, i]
            np.testing.assert_array_equal(y, expect)


def test_identity_bank_reproduces_input():
    rng = np.random.default_rng(55)
    x = rng.standard_normal((3, 4, 5, 6))
    w = np.zeros((4, 4, 1, 1))
    for c in range(4):
        w[c, c, 0, 0] = 1.0
    np.testing.assert_array_equal(oracle.forward(x, w), x)
    # stride subsamples: y[io,jo] = x[2 io, 3 jo]
    y = oracle.forward(x, w, None, (2, 3))
    np.testing.assert_array_equal(y, x[:, :, ::3, ::2])


# --------------------------------------------------------------------------
# P6  adjoint identities (Sec. 2.3.2 eq. (projected); Sec. 6.2 transpose identity)
# --------------------------------------------------------------------------
def test_adjoint_identities():
    rng = np.random.default_rng(6)
    for _ in range(60):
        x, w, b, p, stride, pad = random_case(rng)
        y0 = oracle.forward(x, w, None, stride, pad)
        lhs = float((y0 * p).sum())
        dx = oracle.backward_data(x.shape, w, p, stride, pad)
        dw = oracle.backward_filter(x, w.shape, p, stride, pad)
        db = oracle.backward_bias(x.shape, w.shape, p, stride, pad)
        scale = float((np.abs(y0) * np.abs(p)).sum()) + 1.0
        assert abs(lhs - float((x * dx).sum())) <= 1e-12 * scale
        assert abs(lhs - float((w * dw).sum())) <= 1e-12 * scale
        yb = oracle.forward(x, w, b, stride, pad)
        assert abs(float(((yb - y0) * p).sum()) - float((b * db).sum())) <= 1e-12 * scale


# --------------------------------------------------------------------------
# P7  finite differences of z = <p, y>; z is bilinear so central differences are exact
# --------------------------------------------------------------------------
def test_finite_differences():
    rng = np.random.default_rng(7)
    for _ in range(6):
        x, w, b, p, stride, pad = random_case(rng, max_hw=5, groups=(1, 2))
        z = lambda xx, ww, bb: float((oracle.forward(xx, ww, bb, stride, pad) * p).sum())
        dx = oracle.backward_data(x.shape, w, p, stride, pad)
        dw = oracle.backward_filter(x, w.shape, p, stride, pad)
        db = oracle.backward_bias(x.shape, w.shape, p, stride, pad)
        h = 0.5
        for arr, grad, which in [(x, dx, 0), (w, dw, 1), (b, db, 2)]:
            flat = arr.reshape(-1)
            for e in range(flat.size):
                old = flat[e]
                flat[e] = old + h
                zp = z(x, w, b)
                flat[e] = old - h
                zm = z(x, w, b)
                flat[e] = old
                fd = (zp - zm) / (2 * h)
                assert abs(fd - grad.reshape(-1)[e]) <= 1e-9 * (1.0 + abs(fd)), (which, e)


# --------------------------------------------------------------------------
# P9  Sec. 6.2 eq. (convt-step): the 1-D gather form of the transpose
# --------------------------------------------------------------------------
def test_backward_data_matches_1d_transpose_formula():
    rng = np.random.default_rng(9)
    for _ in range(200):
        H = int(rng.integers(1, 14))
        Hf = int(rng.integers(1, 7))
        S = int(rng.integers(1, 5))
        Pt, Pb = int(rng.integers(0, 4)), int(rng.integers(0, 4))
        while H + Pt + Pb < Hf:
            Pb += 1
        Ho = (H - Hf + Pt + Pb) // S + 1
        f = rng.standard_normal(Hf)
        y = rng.standard_normal(Ho)
        # x_k = sum_{q>=1} y[floor((k-1+Pt)/S) + 2 - q] * f[(k-1+Pt) mod S + S(q-1) + 1], 1-based,
        # terms with an index outside y or f are zero.
        expect = np.zeros(H)
        for k in range(1, H + 1):
            acc = 0.0
            for q in range(1, 2 + (Hf - 1) // S):
                iy = (k - 1 + Pt) // S + 2 - q
                jf = (k - 1 + Pt) % S + S * (q - 1) + 1
                if 1 <= iy <= Ho and 1 <= jf <= Hf:
                    acc += y[iy - 1] * f[jf - 1]
            expect[k - 1] = acc
        got = oracle.backward_data((1, 1, 1, H), f.reshape(1, 1, 1, Hf), y.reshape(1, 1, 1, Ho), (S, 1), (Pt, Pb, 0, 0))
        np.testing.assert_allclose(got.ravel(), expect, rtol=0, atol=1e-13)
        # and the same along the width with (left, right, S_w)
        got = oracle.backward_data((1, 1, H, 1), f.reshape(1, 1, Hf, 1), y.reshape(1, 1, Ho, 1), (1, S), (0, 0, Pt, Pb))
        np.testing.assert_allclose(got.ravel(), expect, rtol=0, atol=1e-13)


# --------------------------------------------------------------------------
# P10  special cases that are textbook matrix products
# --------------------------------------------------------------------------
def test_fully_connected_case_is_a_matrix_product():
    # Sec. 4.1 "Fully connected layers": H''=W''=1 -> Y = F^T X with X = (HWD) x N
    rng = np.random.default_rng(10)
    N, D, W, H, K = 5, 3, 4, 2, 7
    x = rng.standard_normal((N, D, W, H))
    w = rng.standard_normal((K, D, W, H))
    b = rng.standard_normal(K)
    p = rng.standard_normal((N, K, 1, 1))
    X = x.reshape(N, -1).T
    F = w.reshape(K, -1).T
    np.testing.assert_allclose(oracle.forward(x, w, b).reshape(N, K).T, F.T @ X + b[:, None], rtol=0, atol=1e-12)
    P = p.reshape(N, K).T
    np.testing.assert_allclose(oracle.backward_data(x.shape, w, p).reshape(N, -1).T, F @ P, rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.backward_filter(x, w.shape, p).reshape(K, -1).T, X @ P.T, rtol=0, atol=1e-12)


def test_1x1_case_is_a_per_pixel_matrix_product():
    rng = np.random.default_rng(11)
    N, D, W, H, K = 2, 5, 3, 4, 6
    x = rng.standard_normal((N, D, W, H))
    w = rng.standard_normal((K, D, 1, 1))
    p = rng.standard_normal((N, K, W, H))
    Wm = w.reshape(K, D)
    np.testing.assert_allclose(oracle.forward(x, w), np.einsum("kd,ndwh->nkwh", Wm, x), rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.backward_data(x.shape, w, p), np.einsum("kd,nkwh->ndwh", Wm, p), rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.backward_filter(x, w.shape, p).reshape(K, D), np.einsum("nkwh,ndwh->kd", p, x), rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.backward_bias(x.shape, w.shape, p), p.sum(axis=(0, 2, 3)), rtol=0, atol=1e-12)


# --------------------------------------------------------------------------
# P11  Sec. 4.1 "Filter groups": D groups of all-ones 1-channel filters = sum pooling
# --------------------------------------------------------------------------
def test_ones_filters_in_d_groups_are_sum_pooling():
    rng = np.random.default_rng(12)
    N, D, W, H = 2, 4, 7, 6
    x = rng.standard_normal((N, D, W, H))
    w = np.ones((D, 1, 3, 2))            # Hf=2, Wf=3
    y = oracle.forward(x, w, None, (2, 1), (0, 0, 1, 1))
    xp = np.pad(x, ((0, 0), (0, 0), (1, 1), (0, 0)))
    expect = np.zeros_like(y)
    for jo in range(y.shape[2]):
        for io in range(y.shape[3]):
            expect[:, :, jo, io] = xp[:, :, jo:jo + 3, 2 * io:2 * io + 2].sum(axis=(2, 3))
    np.testing.assert_allclose(y, expect, rtol=0, atol=1e-13)


def test_groups_are_independent_convolutions():
    # group m = plain convolution of channel block m with filter block m
    rng = np.random.default_rng(13)
    x, w, b, p, stride, pad = random_case(rng, groups=(3,))
    g = x.shape[1] // w.shape[1]
    Kg = w.shape[0] // g
    Df = w.shape[1]
    y = oracle.forward(x, w, b, stride, pad)
    dx = oracle.backward_data(x.shape, w, p, stride, pad)
    dw = oracle.backward_filter(x, w.shape, p, stride, pad)
    for m in range(g):
        xs, ws, bs, ps = x[:, m * Df:(m + 1) * Df], w[m * Kg:(m + 1) * Kg], b[m * Kg:(m + 1) * Kg], p[:, m * Kg:(m + 1) * Kg]
        np.testing.assert_array_equal(y[:, m * Kg:(m + 1) * Kg], oracle.forward(xs, ws, bs, stride, pad))
        np.testing.assert_array_equal(dx[:, m * Df:(m + 1) * Df], oracle.backward_data(xs.shape, ws, ps, stride, pad))
        np.testing.assert_array_equal(dw[m * Kg:(m + 1) * Kg], oracle.backward_filter(xs, ws.shape, ps, stride, pad))


# --------------------------------------------------------------------------
# P12  structure: linearity, batch independence, batch-summed parameter derivatives
# --------------------------------------------------------------------------
def test_linearity_and_batch_structure():
    rng = np.random.default_rng(14)
    for _ in range(10):
        x, w, b, p, stride, pad = random_case(rng)
        x2 = rng.standard_normal(x.shape)
        a = 1.75
        lhs = oracle.forward(a * x + x2, w, None, stride, pad)
        rhs = a * oracle.forward(x, w, None, stride, pad) + oracle.forward(x2, w, None, stride, pad)
        np.testing.assert_allclose(lhs, rhs, rtol=0, atol=1e-12)
        y = oracle.forward(x, w, b, stride, pad)
        dw = oracle.backward_filter(x, w.shape, p, stride, pad)
        db = oracle.backward_bias(x.shape, w.shape, p, stride, pad)
        dx = oracle.backward_data(x.shape, w, p, stride, pad)
        dw_sum = np.zeros_like(dw)
        db_sum = np.zeros_like(db)
        for n in range(x.shape[0]):
            np.testing.assert_array_equal(oracle.forward(x[n:n + 1], w, b, stride, pad), y[n:n + 1])
            np.testing.assert_array_equal(oracle.backward_data(x[n:n + 1].shape, w, p[n:n + 1], stride, pad), dx[n:n + 1])
            dw_sum += oracle.backward_filter(x[n:n + 1], w.shape, p[n:n + 1], stride, pad)
            db_sum += oracle.backward_bias(x[n:n + 1].shape, w.shape, p[n:n + 1], stride, pad)
        np.testing.assert_allclose(dw_sum, dw, rtol=0, atol=1e-12)
        np.testing.assert_allclose(db_sum, db, rtol=0, atol=1e-12)


# --------------------------------------------------------------------------
# P13  empty bias == zero bias; windows wholly in padding give the bias;
#      samples no window reaches have exactly zero derivative
# --------------------------------------------------------------------------
def test_null_bias_equals_zero_bias_and_padding_only_windows():
    rng = np.random.default_rng(15)
    x, w, b, p, stride, pad = random_case(rng)
    np.testing.assert_array_equal(oracle.forward(x, w, None, stride, pad),
                                  oracle.forward(x, w, np.zeros_like(b), stride, pad))
    # pad far larger than the filter: corner outputs see only zeros
    x = rng.standard_normal((1, 2, 3, 3))
    w = rng.standard_normal((2, 2, 2, 2))
    b = np.array([0.25, -4.0])
    y = oracle.forward(x, w, b, (1, 1), (4, 4, 4, 4))
    assert y.shape == (1, 2, 10, 10)
    np.testing.assert_array_equal(y[0, :, 0, 0], b)
    np.testing.assert_array_equal(y[0, :, 9, 9], b)
    np.testing.assert_array_equal(y[0, :, 2, 7], b)
    assert np.all(y[0, :, 3, 3] != b)


def test_unreached_samples_have_zero_derivative():
    # Sec. 4.1, caption of the convolution figure: with a stride the last samples may never be read
    x = RNG.standard_normal((1, 1, 1, 8))
    w = RNG.standard_normal((1, 1, 1, 2))
    p = RNG.standard_normal((1, 1, 1, 3))      # Ho = floor((8-2)/3)+1 = 3, reads rows 0,1,3,4,6,7
    dx = oracle.backward_data(x.shape, w, p, (3, 1), (0, 0, 0, 0))
    assert dx[0, 0, 0, 2] == 0.0 and dx[0, 0, 0, 5] == 0.0
    assert np.all(dx[0, 0, 0, [0, 1, 3, 4, 6, 7]] != 0.0)
    w4 = RNG.standard_normal((1, 1, 1, 4))
    p2 = RNG.standard_normal((1, 1, 1, 2))     # H=9, Hf=4, S=4: Ho=2, rows 0..7 read, row 8 never
    dx = oracle.backward_data((1, 1, 1, 9), w4, p2, (4, 1), (0, 0, 0, 0))
    assert dx[0, 0, 0, 8] == 0.0


# --------------------------------------------------------------------------
# the "at chosen places" entry points agree with the full ones (the gather form
# of dzdx is separate code from the scatter form)
# --------------------------------------------------------------------------
def test_sampled_entry_points_agree_with_full_ones():
    rng = np.random.default_rng(16)
    for _ in range(30):
        x, w, b, p, stride, pad = random_case(rng)
        y = oracle.forward(x, w, b, stride, pad)
        dx = oracle.backward_data(x.shape, w, p, stride, pad)
        dw = oracle.backward_filter(x, w.shape, p, stride, pad)
        iy = np.arange(y.size)
        np.testing.assert_array_equal(oracle.forward_at(x, w, b, iy, stride, pad), y.ravel())
        np.testing.assert_allclose(oracle.backward_data_at(x.shape, w, p, np.arange(x.size), stride, pad), dx.ravel(), rtol=0, atol=1e-12)
        np.testing.assert_array_equal(oracle.backward_filter_at(x, w.shape, p, np.arange(w.size), stride, pad), dw.ravel())
        sub = rng.permutation(y.size)[: max(1, y.size // 3)]
        np.testing.assert_array_equal(oracle.forward_at(x, w, None, sub, stride, pad),
                                      oracle.forward(x, w, None, stride, pad).ravel()[sub])
    with pytest.raises(oracle.OracleError):
        oracle.forward_at(x, w, b, np.array([y.size]), stride, pad)
    with pytest.raises(oracle.OracleError):
        oracle.backward_data_at(x.shape, w, p, np.array([-1]), stride, pad)
