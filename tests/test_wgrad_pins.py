"""Pins of the oracle's weight gradient: the adjoint of the (pinned) forward definition
in its filter argument."""
import numpy as np
import pytest
import torch

SHAPES = [
    # N, C, H, W, K, R, S, stride, pad
    (2, 3, 7, 9, 4, 3, 3, 1, 1),
    (1, 2, 8, 8, 3, 3, 3, 2, 1),
    (2, 4, 9, 6, 5, 2, 4, 1, 0),
    (1, 3, 11, 11, 2, 5, 5, 3, 2),
    (3, 1, 5, 5, 1, 1, 1, 1, 0),
    (2, 2, 6, 7, 3, 3, 2, 2, 2),
]


def _ints(rng, shape):
    return rng.integers(-3, 4, size=shape).astype(np.float32)


@pytest.mark.parametrize("shape", SHAPES)
def test_adjoint_identity_exact_on_integers(oracle, shape):
    """<dy, forward(x, w)> == <wgrad(x, dy), w> for every w, dy."""
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(sum(shape))
    x, w = _ints(rng, (N, C, H, W)), _ints(rng, (K, C, R, S))
    y = oracle.conv_forward(x, w, st, pd)
    dy = _ints(rng, y.shape)
    dw = oracle.conv_wgrad(x, dy, R, S, st, pd)
    assert dw.shape == w.shape and dw.dtype == np.float64
    assert float((dy.astype(np.float64) * y).sum()) == float((dw * w).sum())


@pytest.mark.parametrize("shape", SHAPES)
def test_gradient_of_each_filter_element(oracle, shape):
    """dw[e] is the forward response to a filter that is 1 at e and 0 elsewhere, weighted by dy."""
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(1 + sum(shape))
    x = _ints(rng, (N, C, H, W))
    P, Q = oracle.out_dim(H, R, st, pd), oracle.out_dim(W, S, st, pd)
    dy = _ints(rng, (N, K, P, Q))
    dw = oracle.conv_wgrad(x, dy, R, S, st, pd)
    for _ in range(12):
        k, c, r, s = (int(rng.integers(0, d)) for d in (K, C, R, S))
        e = np.zeros((K, C, R, S), dtype=np.float32)
        e[k, c, r, s] = 1.0
        assert dw[k, c, r, s] == float((oracle.conv_forward(x, e, st, pd) * dy).sum())


def test_pointwise_is_a_matrix_product(oracle):
    rng = np.random.default_rng(2)
    x, dy = _ints(rng, (3, 5, 4, 6)), _ints(rng, (3, 7, 4, 6))
    want = np.einsum("nkpq,ncpq->kc", dy.astype(np.float64), x.astype(np.float64))
    assert np.array_equal(oracle.conv_wgrad(x, dy, 1, 1, 1, 0)[:, :, 0, 0], want)


@pytest.mark.parametrize("shape", SHAPES)
def test_agrees_with_autograd_in_float64(oracle, shape):
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(7 + sum(shape))
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w = rng.standard_normal((K, C, R, S)).astype(np.float32)
    wt = torch.from_numpy(w).double().requires_grad_(True)
    y = torch.nn.functional.conv2d(torch.from_numpy(x).double(), wt, stride=st, padding=pd)
    dy = rng.standard_normal(tuple(y.shape)).astype(np.float32)
    y.backward(torch.from_numpy(dy).double())
    assert np.abs(oracle.conv_wgrad(x, dy, R, S, st, pd) - wt.grad.numpy()).max() <= 1e-10
