"""Pins for the CPU oracle of the convolution transpose block: every check
compares oracle/convt with something that is NOT its own code path -- numbers
worked by hand, the manual's closed-form sum, the transposed matrix of the
(separately written and separately pinned) convolution oracle, a library
routine, interpolation closed forms, finite differences and adjoint identities.

Citations are to the MatConvNet manual (arXiv 1412.4564).
"""
import itertools
import json
import os

import numpy as np
import pytest

import oracle
from oracle import convt


def colmajor(values, dims):
    """Memory-order list + 4 dims (first fastest) -> array of the reversed shape."""
    a, b, c, d = dims
    return np.asarray(values, dtype=np.float64).reshape(d, c, b, a)


def random_case(rng, max_hw=6, groups=(1, 2, 3), max_up=3):
    G = int(rng.choice(groups))
    Dg, Kf = int(rng.integers(1, 4)), int(rng.integers(1, 4))
    D = G * Dg
    N = int(rng.integers(1, 4))
    H, W = int(rng.integers(1, max_hw + 1)), int(rng.integers(1, max_hw + 1))
    Hf, Wf = int(rng.integers(1, 6)), int(rng.integers(1, 6))
    up = (int(rng.integers(1, max_up + 1)), int(rng.integers(1, max_up + 1)))
    full_h, full_w = up[0] * (H - 1) + Hf, up[1] * (W - 1) + Wf
    ct = int(rng.integers(0, full_h)); cb = int(rng.integers(0, full_h - ct))
    cl = int(rng.integers(0, full_w)); cr = int(rng.integers(0, full_w - cl))
    crop = (ct, cb, cl, cr)
    x = rng.standard_normal((N, D, W, H))
    f = rng.standard_normal((D, Kf, Wf, Hf))
    b = rng.standard_normal(G * Kf)
    ho, wo = full_h - ct - cb, full_w - cl - cr
    p = rng.standard_normal((N, G * Kf, wo, ho))
    return x, f, b, p, up, crop, G


# --------------------------------------------------------------------------
# T1  output size (Sec. 4.2, derived in Sec. 5.3)
# --------------------------------------------------------------------------
def test_output_size_is_the_smallest_height_whose_convolution_has_height_H():
    # Sec. 5.3: of the S_h heights H'' for which the convolution (filter H', stride S_h, pads = crops)
    # has output height H, the block takes the smallest.  The convolution's size rule comes from the
    # convolution oracle, pinned by brute force elsewhere.
    for H, Hf, S, ct, cb in itertools.product(range(1, 7), range(1, 6), range(1, 4), range(0, 3), range(0, 3)):
        expect = S * (H - 1) + Hf - ct - cb
        if expect < 1:
            with pytest.raises(convt.OracleError) as e:
                convt.output_size((1, 1, 1, H), (1, 1, 1, Hf), (S, 1), (ct, cb, 0, 0))
            assert e.value.code == convt.CROP_TOO_LARGE
            continue
        ho, wo = convt.output_size((1, 1, 1, H), (1, 1, 1, Hf), (S, 1), (ct, cb, 0, 0))
        assert (ho, wo) == (expect, 1)
        assert oracle.output_size((1, 1, 1, ho), (1, 1, 1, Hf), (S, 1), (ct, cb, 0, 0))[0] == H
        if ho > 1:
            try:
                smaller = oracle.output_size((1, 1, 1, ho - 1), (1, 1, 1, Hf), (S, 1), (ct, cb, 0, 0))[0]
            except oracle.OracleError:
                smaller = 0
            assert smaller < H
        # the same rule horizontally, with (left, right, S_w)
        assert convt.output_size((1, 1, H, 1), (1, 1, Hf, 1), (1, S), (0, 0, ct, cb)) == (1, expect)


def test_geometry_errors():
    ok = dict(xshape=(1, 4, 3, 3), fshape=(4, 2, 3, 3), upsample=(2, 2), crop=(1, 1, 1, 1), groups=2)
    assert convt.output_size(**ok) == (5, 5)
    with pytest.raises(convt.OracleError) as e:          # the groups must divide the input depth
        convt.output_size(**dict(ok, groups=3))
    assert e.value.code == convt.BAD_GROUPS
    for bad in [dict(upsample=(0, 1)), dict(upsample=(1, 0)), dict(crop=(-1, 0, 0, 0)), dict(crop=(0, 0, 0, -1)),
                dict(groups=0)]:
        with pytest.raises(convt.OracleError) as e:
            convt.output_size(**dict(ok, **bad))
        assert e.value.code == convt.BAD_ARG
    with pytest.raises(convt.OracleError) as e:          # crops that eat the whole output
        convt.output_size(**dict(ok, crop=(4, 3, 0, 0)))
    assert e.value.code == convt.CROP_TOO_LARGE
    with pytest.raises(ValueError):                      # f's fourth axis is the input depth
        convt.output_size((1, 4, 3, 3), (3, 2, 3, 3))


# --------------------------------------------------------------------------
# T2  numbers worked by hand
# --------------------------------------------------------------------------
def test_hand_worked_examples(golden_dir):
    with open(os.path.join(golden_dir, "convt_hand_examples.json")) as fh:
        examples = json.load(fh)["examples"]
    assert len(examples) >= 2
    for ex in examples:
        x = colmajor(ex["x"], ex["x_hwdn"])
        f = colmajor(ex["f"], ex["f_hwkd"])
        b = None if ex["b"] is None else np.asarray(ex["b"], dtype=np.float64)
        up, crop, G = ex["upsample"], ex["crop"], ex["groups"]
        y = convt.forward(x, f, b, up, crop, G)
        Ho, Wo, K, N = ex["y_hwkn"]
        assert y.shape == (N, K, Wo, Ho), ex["name"]
        np.testing.assert_array_equal(y.ravel(), np.asarray(ex["y"], dtype=np.float64), err_msg=ex["name"])
        p = np.asarray(ex["dzdy"], dtype=np.float64).reshape(y.shape)
        np.testing.assert_array_equal(convt.backward_data(x.shape, f, p, up, crop, G).ravel(), ex["dzdx"], err_msg=ex["name"])
        np.testing.assert_array_equal(convt.backward_filter(x, f.shape, p, up, crop, G).ravel(), ex["dzdf"], err_msg=ex["name"])
        np.testing.assert_array_equal(convt.backward_bias(x.shape, f.shape, p, up, crop, G).ravel(), ex["dzdb"], err_msg=ex["name"])
        y0 = convt.forward(x, f, None, up, crop, G)
        assert float((y0 * p).sum()) == ex["inner"]
        assert float((x.ravel() * np.asarray(ex["dzdx"])).sum()) == ex["inner"]
        assert float((f.ravel() * np.asarray(ex["dzdf"])).sum()) == ex["inner"]


# --------------------------------------------------------------------------
# T3  the closed form of Sec. 4.2 eq. (convt), in the manual's 1-based notation
# --------------------------------------------------------------------------
def closed_form(x, f, up, crop):
    """y_{i''j''d''} = sum_{d'} sum_{i'=0}^{q(H',S_h)} sum_{j'=0}^{q(W',S_w)}
         f[1 + S_h i' + m(i''+P_h^-, S_h), 1 + S_w j' + m(j''+P_w^-, S_w), d'', d']
       * x[1 - i' + q(i''+P_h^-, S_h), 1 - j' + q(j''+P_w^-, S_w), d']
    with m(k,S) = (k-1) mod S, q(k,S) = floor((k-1)/S), x and f zero outside their support."""
    N, D, W, H = x.shape
    _, Kf, Wf, Hf = f.shape
    Sh, Sw = up
    Pt, Pb, Pl, Pr = crop
    Ho, Wo = Sh * (H - 1) + Hf - Pt - Pb, Sw * (W - 1) + Wf - Pl - Pr
    m = lambda k, S: (k - 1) % S
    q = lambda k, S: (k - 1) // S
    X = lambda i, j, d, n: x[n - 1, d - 1, j - 1, i - 1] if 1 <= i <= H and 1 <= j <= W else 0.0
    F = lambda i, j, k, d: f[d - 1, k - 1, j - 1, i - 1] if 1 <= i <= Hf and 1 <= j <= Wf else 0.0
    y = np.zeros((N, Kf, Wo, Ho))
    for n, k, jj, ii in itertools.product(range(1, N + 1), range(1, Kf + 1), range(1, Wo + 1), range(1, Ho + 1)):
        acc = 0.0
        for d in range(1, D + 1):
            for ip in range(0, q(Hf, Sh) + 1):
                for jp in range(0, q(Wf, Sw) + 1):
                    acc += F(1 + Sh * ip + m(ii + Pt, Sh), 1 + Sw * jp + m(jj + Pl, Sw), k, d) * \
                           X(1 - ip + q(ii + Pt, Sh), 1 - jp + q(jj + Pl, Sw), d, n)
        y[n - 1, k - 1, jj - 1, ii - 1] = acc
    return y


def test_forward_matches_closed_form_of_sec_4_2():
    rng = np.random.default_rng(42)
    for _ in range(40):
        x, f, b, p, up, crop, G = random_case(rng, max_hw=5, groups=(1,))
        got = convt.forward(x, f, None, up, crop, 1)
        np.testing.assert_allclose(got, closed_form(x, f, up, crop), rtol=0, atol=1e-12)


# --------------------------------------------------------------------------
# T4  the definition itself: y = M^T x with M the matrix of the convolution block
# --------------------------------------------------------------------------
def conv_matrix(yshape, xshape, f, up, crop, G):
    """Matrix of the convolution of Sec. 4.1 (via the convolution oracle) that takes an array of y's
    shape to one of x's shape, column by column from unit impulses."""
    D, Kf = f.shape[0], f.shape[1]
    # the convolution's bank: D filters of depth Kf; as an (K, Df, Wf, Hf) array that is f's own memory
    bank = f.reshape(D, Kf, f.shape[2], f.shape[3])
    ny, nx = int(np.prod(yshape)), int(np.prod(xshape))
    M = np.zeros((nx, ny))
    for c in range(ny):
        e = np.zeros(ny)
        e[c] = 1.0
        M[:, c] = oracle.forward(e.reshape(yshape), bank, None, up, crop).ravel()
    return M


def test_forward_is_the_transposed_convolution_matrix():
    rng = np.random.default_rng(43)
    for _ in range(25):
        x, f, b, p, up, crop, G = random_case(rng, max_hw=4)
        y = convt.forward(x, f, b, up, crop, G)
        M = conv_matrix(p.shape, x.shape, f, up, crop, G)
        expect = (M.T @ x.ravel()).reshape(y.shape) + b[None, :, None, None]
        np.testing.assert_allclose(y, expect, rtol=0, atol=1e-12)
        # and the input derivative is the convolution itself: dzdx = M dzdy
        dx = convt.backward_data(x.shape, f, p, up, crop, G)
        np.testing.assert_allclose(dx.ravel(), M @ p.ravel(), rtol=0, atol=1e-12)


def test_transposition_identity_against_the_convolution_oracle():
    # <convt(x), p> = <x, conv(p)> for every x, p (Sec. 4.2: the two blocks are transposes of each other)
    rng = np.random.default_rng(44)
    for _ in range(60):
        x, f, b, p, up, crop, G = random_case(rng, max_hw=7)
        lhs = float((convt.forward(x, f, None, up, crop, G) * p).sum())
        rhs = float((x * oracle.forward(p, f, None, up, crop)).sum())
        assert abs(lhs - rhs) <= 1e-11 * (1.0 + abs(lhs))


# --------------------------------------------------------------------------
# T5  a library routine: torch's conv_transpose2d, cropped afterwards
# --------------------------------------------------------------------------
def test_forward_matches_torch_conv_transpose2d():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(45)
    for _ in range(30):
        x, f, b, p, up, crop, G = random_case(rng, max_hw=6)
        # arrays are (N, C, W, H): torch's "height" axis is our W; strides and crops swap accordingly
        full = torch.nn.functional.conv_transpose2d(torch.from_numpy(x), torch.from_numpy(f), torch.from_numpy(b),
                                                    stride=(up[1], up[0]), groups=G).numpy()
        ct, cb, cl, cr = crop
        expect = full[:, :, cl:full.shape[2] - cr, ct:full.shape[3] - cb]
        np.testing.assert_allclose(convt.forward(x, f, b, up, crop, G), expect, rtol=0, atol=1e-12)


# --------------------------------------------------------------------------
# T6  interpolation closed forms (Sec. 4.2: the block acts as an interpolating filter)
# --------------------------------------------------------------------------
def test_box_filter_replicates_samples():
    rng = np.random.default_rng(46)
    for S in (1, 2, 3, 4):
        x = rng.standard_normal((2, 1, 1, 6))
        y = convt.forward(x, np.ones((1, 1, 1, S)), None, (S, 1))
        np.testing.assert_array_equal(y, np.repeat(x, S, axis=3))
        xt = x.transpose(0, 1, 3, 2).copy()
        y = convt.forward(xt, np.ones((1, 1, S, 1)), None, (1, S))
        np.testing.assert_array_equal(y, np.repeat(xt, S, axis=2))


def test_triangle_filter_interpolates_linearly():
    # upsampling 2 with taps (1/2, 1, 1/2) and one sample cropped at each end keeps x at the even
    # places and puts the mean of the two neighbours between them
    rng = np.random.default_rng(47)
    x = rng.standard_normal((1, 1, 1, 9))
    y = convt.forward(x, np.array([0.5, 1.0, 0.5]).reshape(1, 1, 1, 3), None, (2, 1), (1, 1, 0, 0))
    assert y.shape == (1, 1, 1, 17)
    v, xv = y.ravel(), x.ravel()
    np.testing.assert_array_equal(v[0::2], xv)
    np.testing.assert_allclose(v[1::2], 0.5 * (xv[:-1] + xv[1:]), rtol=0, atol=1e-15)
    # one group per channel keeps the channels apart (per-channel interpolation)
    x = rng.standard_normal((2, 3, 4, 5))
    tri = np.array([0.5, 1.0, 0.5])
    f = np.broadcast_to(np.outer(tri, tri), (3, 1, 3, 3)).copy()
    y = convt.forward(x, f, None, (2, 2), (1, 1, 1, 1), groups=3)
    assert y.shape == (2, 3, 7, 9)
    np.testing.assert_array_equal(y[:, :, 0::2, 0::2], x)
    np.testing.assert_allclose(y[:, :, 1::2, 1::2],
                               0.25 * (x[:, :, :-1, :-1] + x[:, :, 1:, :-1] + x[:, :, :-1, 1:] + x[:, :, 1:, 1:]),
                               rtol=0, atol=1e-15)


def test_no_upsampling_is_a_full_correlation_with_the_flipped_filter():
    # with S = 1 and no crop the block is the textbook full convolution of x with f
    rng = np.random.default_rng(48)
    x, f = rng.standard_normal(11), rng.standard_normal(4)
    y = convt.forward(x.reshape(1, 1, 1, 11), f.reshape(1, 1, 1, 4))
    np.testing.assert_allclose(y.ravel(), np.convolve(x, f), rtol=0, atol=1e-13)


# --------------------------------------------------------------------------
# T7  derivatives: adjoint identities and finite differences of z = <p, y> (Sec. 2.3.2)
# --------------------------------------------------------------------------
def test_adjoint_identities():
    rng = np.random.default_rng(49)
    for _ in range(60):
        x, f, b, p, up, crop, G = random_case(rng)
        y0 = convt.forward(x, f, None, up, crop, G)
        lhs = float((y0 * p).sum())
        dx = convt.backward_data(x.shape, f, p, up, crop, G)
        df = convt.backward_filter(x, f.shape, p, up, crop, G)
        db = convt.backward_bias(x.shape, f.shape, p, up, crop, G)
        scale = float((np.abs(y0) * np.abs(p)).sum()) + 1.0
        assert abs(lhs - float((x * dx).sum())) <= 1e-12 * scale
        assert abs(lhs - float((f * df).sum())) <= 1e-12 * scale
        yb = convt.forward(x, f, b, up, crop, G)
        assert abs(float(((yb - y0) * p).sum()) - float((b * db).sum())) <= 1e-12 * scale
        np.testing.assert_allclose(db, p.sum(axis=(0, 2, 3)), rtol=0, atol=1e-12)


def test_finite_differences():
    rng = np.random.default_rng(50)
    for _ in range(6):
        x, f, b, p, up, crop, G = random_case(rng, max_hw=4, groups=(1, 2))
        z = lambda xx, ff, bb: float((convt.forward(xx, ff, bb, up, crop, G) * p).sum())
        grads = [convt.backward_data(x.shape, f, p, up, crop, G), convt.backward_filter(x, f.shape, p, up, crop, G),
                 convt.backward_bias(x.shape, f.shape, p, up, crop, G)]
        h = 0.5
        for arr, grad in zip((x, f, b), grads):
            flat = arr.reshape(-1)
            for e in range(flat.size):
                old = flat[e]
                flat[e] = old + h
                zp = z(x, f, b)
                flat[e] = old - h
                zm = z(x, f, b)
                flat[e] = old
                fd = (zp - zm) / (2 * h)   # z is affine in each argument: central differences are exact
                assert abs(fd - grad.reshape(-1)[e]) <= 1e-9 * (1.0 + abs(fd))


def test_filter_derivative_is_the_convolution_filter_derivative_with_roles_swapped():
    # dzdf of the transpose block = filter derivative of the convolution that maps dzdy's shape to
    # x's shape, fed dzdy as its input and x as its output derivative
    rng = np.random.default_rng(51)
    for _ in range(40):
        x, f, b, p, up, crop, G = random_case(rng, max_hw=6)
        got = convt.backward_filter(x, f.shape, p, up, crop, G)
        expect = oracle.backward_filter(p, f.shape, x, up, crop)
        np.testing.assert_allclose(got, expect, rtol=0, atol=1e-11)


# --------------------------------------------------------------------------
# T8  structure: groups, batch, sampled entry points
# --------------------------------------------------------------------------
def test_groups_are_independent_blocks():
    rng = np.random.default_rng(52)
    for _ in range(20):
        x, f, b, p, up, crop, G = random_case(rng, groups=(2, 3))
        y = convt.forward(x, f, b, up, crop, G)
        Dg, Kf = x.shape[1] // G, f.shape[1]
        for m in range(G):
            part = convt.forward(x[:, m * Dg:(m + 1) * Dg], f[m * Dg:(m + 1) * Dg], b[m * Kf:(m + 1) * Kf], up, crop, 1)
            np.testing.assert_allclose(y[:, m * Kf:(m + 1) * Kf], part, rtol=0, atol=1e-13)


def test_images_of_a_batch_are_independent():
    rng = np.random.default_rng(53)
    x, f, b, p, up, crop, G = random_case(rng)
    y = convt.forward(x, f, b, up, crop, G)
    for n in range(x.shape[0]):
        np.testing.assert_array_equal(y[n:n + 1], convt.forward(x[n:n + 1], f, b, up, crop, G))


def test_null_bias_equals_zero_bias():
    rng = np.random.default_rng(54)
    x, f, b, p, up, crop, G = random_case(rng)
    np.testing.assert_array_equal(convt.forward(x, f, None, up, crop, G), convt.forward(x, f, 0 * b, up, crop, G))


def test_sampled_entry_points_agree_with_full_ones():
    rng = np.random.default_rng(55)
    for _ in range(10):
        x, f, b, p, up, crop, G = random_case(rng)
        y = convt.forward(x, f, b, up, crop, G)
        idx = rng.integers(0, y.size, size=50)
        np.testing.assert_array_equal(convt.forward_at(x, f, b, idx, up, crop, G), y.ravel()[idx])
        dx = convt.backward_data(x.shape, f, p, up, crop, G)
        idx = rng.integers(0, dx.size, size=50)
        np.testing.assert_array_equal(convt.backward_data_at(x.shape, f, p, idx, up, crop, G), dx.ravel()[idx])
        df = convt.backward_filter(x, f.shape, p, up, crop, G)
        idx = rng.integers(0, df.size, size=50)
        np.testing.assert_array_equal(convt.backward_filter_at(x, f.shape, p, idx, up, crop, G), df.ravel()[idx])
        with pytest.raises(convt.OracleError):
            convt.forward_at(x, f, b, np.array([y.size]), up, crop, G)
