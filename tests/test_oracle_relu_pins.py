"""Pins for the CPU oracle of the ReLU block (Sec. 4.4 and 6.4.1 of the MatConvNet manual,
arXiv 1412.4564): values written out by hand, a library routine, and the identities that
characterise the block."""
import numpy as np

from oracle import relu


def test_values_written_out_by_hand():
    x = np.array([-2.0, -0.0, 0.0, 1e-300, 3.5, -1e-300, 7.0])
    np.testing.assert_array_equal(relu.forward(x), [0.0, 0.0, 0.0, 1e-300, 3.5, 0.0, 7.0])
    p = np.array([1.0, 2.0, 3.0, 4.0, 5.0, 6.0, -7.0])
    # the indicator is [x > 0]: nothing passes at x = 0 or below
    np.testing.assert_array_equal(relu.backward(x, p), [0.0, 0.0, 0.0, 4.0, 5.0, 0.0, -7.0])


def test_matches_library_maximum_and_indicator():
    rng = np.random.default_rng(441)
    x = rng.standard_normal((3, 4, 5, 6))
    x[rng.random(x.shape) < 0.1] = 0.0
    p = rng.standard_normal(x.shape)
    y = relu.forward(x)
    np.testing.assert_array_equal(y, np.maximum(x, 0.0))
    np.testing.assert_array_equal(relu.backward(x, p), np.where(x > 0, p, 0.0))
    # the output carries the same indicator as the input
    np.testing.assert_array_equal(relu.backward(y, p), relu.backward(x, p))
    assert y.shape == x.shape


def test_identities():
    rng = np.random.default_rng(442)
    x = rng.standard_normal(1000)
    p = rng.standard_normal(1000)
    y = relu.forward(x)
    np.testing.assert_array_equal(relu.forward(y), y)                        # idempotent
    np.testing.assert_array_equal(relu.forward(3.0 * x), 3.0 * y)            # positively homogeneous
    np.testing.assert_allclose(y - relu.forward(-x), x, rtol=0, atol=0)      # x = x+ - x-
    dx = relu.backward(x, p)
    assert float((dx * x).sum()) == float((p * y).sum())                      # <dzdx, x> = <dzdy, y>
    # finite differences of z = <p, y> away from the kink
    h = 1e-6
    far = np.abs(x) > 1e-3
    fd = (p * (relu.forward(x + h) - relu.forward(x - h))).ravel() / (2 * h)
    np.testing.assert_allclose(fd[far], dx[far], rtol=1e-8, atol=1e-8)
