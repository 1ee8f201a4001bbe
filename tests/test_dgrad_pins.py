"""Pins of the oracle's data gradient against what the mathematics fixes: it is the
adjoint of the forward definition (already pinned) in its input argument."""
import numpy as np
import pytest
import torch

SHAPES = [
    # N, C, H, W, K, R, S, stride, pad
    (2, 3, 7, 9, 4, 3, 3, 1, 1),
    (1, 2, 8, 8, 3, 3, 3, 2, 1),
    (2, 4, 9, 6, 5, 2, 4, 1, 0),
    (1, 3, 11, 11, 2, 5, 5, 3, 2),
    (1, 1, 5, 5, 1, 1, 1, 1, 0),
    (2, 2, 6, 7, 3, 3, 2, 2, 2),
]


def _ints(rng, shape):
    return rng.integers(-3, 4, size=shape).astype(np.float32)


@pytest.mark.parametrize("shape", SHAPES)
def test_adjoint_identity_exact_on_integers(oracle, shape):
    """<dy, forward(x, w)> == <dgrad(dy, w), x> for every x, dy: both sides are the same
    triple sum of dy*w*x products, exact in float64 on small integers."""
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(sum(shape))
    x, w = _ints(rng, (N, C, H, W)), _ints(rng, (K, C, R, S))
    y = oracle.conv_forward(x, w, st, pd)
    dy = _ints(rng, y.shape)
    dx = oracle.conv_dgrad(dy, w, H, W, st, pd)
    assert dx.shape == x.shape and dx.dtype == np.float64
    assert float((dy.astype(np.float64) * y).sum()) == float((dx * x).sum())


@pytest.mark.parametrize("shape", SHAPES)
def test_gradient_of_each_input_element(oracle, shape):
    """dx[e] is the forward response to a unit impulse at e, weighted by dy (the forward map
    is linear in x): checked element by element on a sample."""
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(1 + sum(shape))
    w = _ints(rng, (K, C, R, S))
    P, Q = oracle.out_dim(H, R, st, pd), oracle.out_dim(W, S, st, pd)
    dy = _ints(rng, (N, K, P, Q))
    dx = oracle.conv_dgrad(dy, w, H, W, st, pd)
    for _ in range(12):
        n, c, h, x_ = (int(rng.integers(0, d)) for d in (N, C, H, W))
        e = np.zeros((N, C, H, W), dtype=np.float32)
        e[n, c, h, x_] = 1.0
        assert dx[n, c, h, x_] == float((oracle.conv_forward(e, w, st, pd) * dy).sum())


def test_delta_filter_scatters_dy_back(oracle):
    N, C, H, W, K, R, S, st, pd = 1, 2, 9, 8, 3, 3, 3, 2, 1
    rng = np.random.default_rng(3)
    P, Q = oracle.out_dim(H, R, st, pd), oracle.out_dim(W, S, st, pd)
    dy = _ints(rng, (N, K, P, Q))
    k0, c0, r0, s0 = 1, 1, 2, 0
    w = np.zeros((K, C, R, S), dtype=np.float32)
    w[k0, c0, r0, s0] = 1.0
    dx = oracle.conv_dgrad(dy, w, H, W, st, pd)
    want = np.zeros((N, C, H, W))
    for p in range(P):
        for q in range(Q):
            h, x_ = p * st + r0 - pd, q * st + s0 - pd
            if 0 <= h < H and 0 <= x_ < W:
                want[0, c0, h, x_] += dy[0, k0, p, q]
    assert np.array_equal(dx, want)


@pytest.mark.parametrize("shape", [s for s in SHAPES if s[7] == 1 and s[5] == s[6] and s[8] <= s[5] - 1])
def test_stride_one_is_a_forward_pass_over_the_flipped_transposed_filter(oracle, shape):
    """For stride 1: dgrad(dy, w) == forward(dy, w~, pad' = R-1-pad) with
    w~[c][k][r][s] = w[k][c][R-1-r][S-1-s] (the identity the GPU path rests on)."""
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(5 + sum(shape))
    w = _ints(rng, (K, C, R, S))
    dy = _ints(rng, (N, K, oracle.out_dim(H, R, 1, pd), oracle.out_dim(W, S, 1, pd)))
    wt = np.ascontiguousarray(w[:, :, ::-1, ::-1].transpose(1, 0, 2, 3))
    assert np.array_equal(oracle.conv_dgrad(dy, w, H, W, 1, pd), oracle.conv_forward(dy, wt, 1, R - 1 - pd))


@pytest.mark.parametrize("shape", SHAPES)
def test_agrees_with_autograd_in_float64(oracle, shape):
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(7 + sum(shape))
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w = rng.standard_normal((K, C, R, S)).astype(np.float32)
    xt = torch.from_numpy(x).double().requires_grad_(True)
    y = torch.nn.functional.conv2d(xt, torch.from_numpy(w).double(), stride=st, padding=pd)
    dy = rng.standard_normal(tuple(y.shape)).astype(np.float32)
    y.backward(torch.from_numpy(dy).double())
    got = oracle.conv_dgrad(dy, w, H, W, st, pd)
    assert np.abs(got - xt.grad.numpy()).max() <= 1e-10


@pytest.mark.parametrize("shape", [(2, 3, 11, 12, 4, 3, 3, 2, 1), (1, 2, 13, 10, 3, 5, 5, 3, 2), (2, 2, 9, 9, 3, 4, 4, 2, 1),
                                   (1, 3, 12, 11, 2, 3, 3, 2, 0), (1, 2, 10, 10, 2, 3, 3, 3, 1), (1, 2, 9, 8, 3, 1, 1, 2, 0)])
def test_strided_layer_is_one_small_convolution_per_phase(oracle, shape):
    """The identity the GPU path for strided layers rests on, on the oracle alone: with h + pad = st*u + a, dx at the
    rows of phase a is the stride-1 convolution of dy with the taps a, a+st, ... (flipped, zero where past the
    filter), padding RT-1, result u stored at h = st*u + a - pad; rows no window reaches stay zero."""
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(77 + sum(shape))
    w = rng.integers(-3, 4, (K, C, R, S)).astype(np.float64)
    P, Q = oracle.out_dim(H, R, st, pd), oracle.out_dim(W, S, st, pd)
    dy = rng.integers(-3, 4, (N, K, P, Q)).astype(np.float64)
    RT = -(-R // st)
    dx = np.zeros((N, C, H, W))
    for a in range(min(st, R)):            # (phases a >= R have no tap: their rows of dx stay zero)
        for b in range(min(st, S)):
            wf = np.zeros((C, K, RT, RT))
            for j in range(RT):
                for l in range(RT):
                    r, s = a + st * (RT - 1 - j), b + st * (RT - 1 - l)
                    if r < R and s < S:
                        wf[:, :, j, l] = w[:, :, r, s].T
            sub = oracle.conv_forward(dy.astype(np.float32), wf.astype(np.float32), 1, RT - 1)   # [N][C][P+RT-1][Q+RT-1]
            for u in range(sub.shape[2]):
                for v in range(sub.shape[3]):
                    h, x = st * u + a - pd, st * v + b - pd
                    if 0 <= h < H and 0 <= x < W:
                        dx[:, :, h, x] = sub[:, :, u, v]
    want = oracle.conv_dgrad(dy.astype(np.float32), w.astype(np.float32), H, W, st, pd)
    assert np.array_equal(dx, want)
