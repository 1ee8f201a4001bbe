"""Pins of the point-wise tail's definition: closed forms and textbook properties."""
import numpy as np


def test_zero_filter_leaves_the_tail_alone(oracle):
    rng = np.random.default_rng(0)
    x = rng.standard_normal((2, 3, 6, 6)).astype(np.float32)
    w = np.zeros((4, 3, 3, 3), dtype=np.float32)
    b = np.array([1.0, -2.0, 0.5, 0.0])
    r = rng.standard_normal((2, 4, 6, 6))
    got = oracle.conv_forward_fused(x, w, 1, 1, bias=b, residual=r, relu=True)
    assert np.array_equal(got, np.maximum(r + b[None, :, None, None], 0.0))


def test_each_part_is_optional_and_relu_comes_last(oracle):
    rng = np.random.default_rng(1)
    x = rng.integers(-3, 4, (1, 2, 5, 5)).astype(np.float32)
    w = rng.integers(-3, 4, (3, 2, 3, 3)).astype(np.float32)
    y = oracle.conv_forward(x, w, 1, 1)
    b = np.array([100.0, -100.0, 0.0])
    assert np.array_equal(oracle.conv_forward_fused(x, w, 1, 1), y)
    assert np.array_equal(oracle.conv_forward_fused(x, w, 1, 1, bias=b)[:, 0], y[:, 0] + 100.0)
    out = oracle.conv_forward_fused(x, w, 1, 1, bias=b, relu=True)
    assert (out >= 0).all() and np.array_equal(out, np.maximum(y + b[None, :, None, None], 0.0))
    # a residual equal to minus the convolution cancels it exactly
    assert (oracle.conv_forward_fused(x, w, 1, 1, residual=-y) == 0).all()
