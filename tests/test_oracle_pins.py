"""Pins for the CPU oracle: every check compares it with something fixed by the paper
or by mathematics, never with itself.  No GPU needed.

Paper passages: Section 3 / Algorithm 1 (the definition), Section 3.1.2 / Algorithm 2
(a second loop order, "any permutation of the loops is correct"), Section 2.2 (im2col
matrix shape, Figure 2 caption shape example).
"""
import os

import numpy as np
import pytest
import torch

from paper_1809_10170_amd import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [[int(t) for t in ln.split()] for ln in f if ln.strip() and not ln.startswith("#")]


def _ints(rng, shape, amp=3):
    return rng.integers(-amp, amp + 1, size=shape).astype(np.float32)


SMALL_SHAPES = [
    # N, C, H, W, K, R, S, stride, pad
    (1, 1, 1, 1, 1, 1, 1, 1, 0),
    (1, 3, 5, 5, 2, 3, 3, 1, 0),
    (2, 3, 7, 6, 4, 3, 3, 1, 1),
    (2, 4, 9, 11, 5, 3, 2, 2, 1),
    (1, 2, 12, 13, 3, 5, 5, 1, 2),
    (3, 5, 8, 8, 7, 1, 1, 1, 0),
    (1, 3, 23, 19, 6, 11, 11, 4, 0),
    (2, 3, 16, 15, 4, 7, 7, 2, 3),
    (1, 2, 6, 9, 3, 2, 4, 3, 2),
    (1, 1, 4, 4, 1, 3, 3, 1, 3),      # pad as large as the filter: all-zero border outputs
]


# ---- an independent lowering: im2col matrix, then a matrix product (Section 2.2) ----
def im2col_matmul(x, w, stride, pad):
    x = x.astype(np.float64)
    w = w.astype(np.float64)
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    xp = np.zeros((N, C, H + 2 * pad, W + 2 * pad))
    xp[:, :, pad:pad + H, pad:pad + W] = x
    out = np.empty((N, K, P, Q))
    for n in range(N):
        cols = np.empty((C * R * S, P * Q))
        row = 0
        for c in range(C):
            for r in range(R):
                for s in range(S):
                    patch = xp[n, c, r:r + (P - 1) * stride + 1:stride, s:s + (Q - 1) * stride + 1:stride]
                    cols[row] = patch.reshape(-1)
                    row += 1
        assert cols.shape == (C * R * S, P * Q)
        out[n] = (w.reshape(K, -1) @ cols).reshape(K, P, Q)
    return out


def test_shape_example_from_paper(oracle):
    for H, W, C, K, R, S, st, pd, P, Q, mrows, mcols in _rows("fig2_shapes.txt"):
        assert oracle.out_dim(H, R, st, pd) == P
        assert oracle.out_dim(W, S, st, pd) == Q
        x = np.ones((1, C, H, W), np.float32)
        w = np.ones((K, C, R, S), np.float32)
        out = oracle.conv_forward(x, w, st, pd)
        assert out.shape == (1, K, P, Q)
        assert (C * R * S, P * Q) == (mrows, mcols)
        # all-ones, no padding: every output is the number of taps
        assert np.array_equal(out, np.full((1, K, P, Q), float(C * R * S)))


def test_config_output_sizes(oracle):
    for H, R, st, pd, P in _rows("config_shapes.txt"):
        assert oracle.out_dim(H, R, st, pd) == P
    for l in workloads.ALL_LAYERS:
        assert oracle.out_dim(l.H, l.R, l.stride, l.pad) == l.P
        assert oracle.out_dim(l.W, l.S, l.stride, l.pad) == l.Q


def test_out_dim_floor_and_reject(oracle):
    # floor when the span is not a multiple of the stride: 7x7 s2 p3 on 224 -> 112
    assert oracle.out_dim(224, 7, 2, 3) == 112
    assert oracle.out_dim(10, 3, 4, 0) == 2          # taps at 0 and 4; row 9 unused
    assert oracle.out_dim(2, 3, 1, 0) == 0           # filter does not fit
    assert oracle.out_dim(2, 3, 1, 1) == 2
    assert oracle.out_dim(5, 3, 0, 0) == 0
    # brute force: count window starts that fit
    for H in range(1, 12):
        for R in range(1, 6):
            for st in range(1, 4):
                for pd in range(0, 3):
                    starts = [t for t in range(0, H + 2 * pd) if t % st == 0 and t + R <= H + 2 * pd]
                    assert oracle.out_dim(H, R, st, pd) == len(starts)


@pytest.mark.parametrize("shape", SMALL_SHAPES)
def test_equals_im2col_matmul_bit_exact_on_integers(oracle, shape):
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(11)
    x, w = _ints(rng, (N, C, H, W)), _ints(rng, (K, C, R, S))
    assert np.array_equal(oracle.conv_forward(x, w, st, pd), im2col_matmul(x, w, st, pd))


@pytest.mark.parametrize("shape", SMALL_SHAPES)
def test_algorithm2_loop_order_bit_exact_on_integers(oracle, shape):
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(12)
    x, w = _ints(rng, (N, C, H, W)), _ints(rng, (K, C, R, S))
    assert np.array_equal(oracle.conv_forward(x, w, st, pd),
                          oracle.conv_forward_reordered(x, w, st, pd))


@pytest.mark.parametrize("shape", SMALL_SHAPES)
def test_random_fp32_inputs_match_im2col_and_torch_fp64(oracle, shape):
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(13)
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    w = rng.uniform(-1, 1, (K, C, R, S)).astype(np.float32)
    got = oracle.conv_forward(x, w, st, pd)
    assert np.allclose(got, im2col_matmul(x, w, st, pd), rtol=0, atol=1e-12 * C * R * S)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                     stride=st, padding=pd).numpy()
    assert np.allclose(got, ref, rtol=0, atol=1e-12 * C * R * S)


def test_pointwise_is_matrix_product(oracle):
    rng = np.random.default_rng(14)
    N, C, H, W, K = 3, 6, 5, 7, 4
    x, w = _ints(rng, (N, C, H, W)), _ints(rng, (K, C, 1, 1))
    out = oracle.conv_forward(x, w, 1, 0)
    for n in range(N):
        want = w.reshape(K, C).astype(np.float64) @ x[n].reshape(C, H * W).astype(np.float64)
        assert np.array_equal(out[n].reshape(K, H * W), want)


@pytest.mark.parametrize("stride,pad", [(1, 0), (1, 2), (2, 1), (3, 2)])
def test_delta_filter_is_shifted_crop(oracle, stride, pad):
    rng = np.random.default_rng(15)
    N, C, H, W, K, R, S = 2, 3, 9, 10, 4, 3, 4
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    P, Q = oracle.out_dim(H, R, stride, pad), oracle.out_dim(W, S, stride, pad)
    for k, (c0, r0, s0) in enumerate([(0, 0, 0), (2, 2, 3), (1, 1, 2), (2, 0, 3)]):
        w = np.zeros((K, C, R, S), np.float32)
        w[k, c0, r0, s0] = 1.0
        out = oracle.conv_forward(x, w, stride, pad)
        want = np.zeros((N, K, P, Q))
        for p in range(P):
            for q in range(Q):
                ih, iw = p * stride + r0 - pad, q * stride + s0 - pad
                if 0 <= ih < H and 0 <= iw < W:
                    want[:, k, p, q] = x[:, c0, ih, iw]
        assert np.array_equal(out, want)   # other channels stay exactly zero


@pytest.mark.parametrize("shape", SMALL_SHAPES)
def test_all_ones_counts_valid_taps(oracle, shape):
    N, C, H, W, K, R, S, st, pd = shape
    out = oracle.conv_forward(np.ones((N, C, H, W), np.float32), np.ones((K, C, R, S), np.float32), st, pd)
    P, Q = out.shape[2:]

    def valid(o, extent, f):
        lo = o * st - pd
        return max(0, min(f, extent - lo) - max(0, -lo))

    want = np.array([[C * valid(p, H, R) * valid(q, W, S) for q in range(Q)] for p in range(P)], float)
    assert np.array_equal(out, np.broadcast_to(want, out.shape))


@pytest.mark.parametrize("shape", [s for s in SMALL_SHAPES if s[8] > 0])
def test_padding_equals_explicit_zero_border(oracle, shape):
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(16)
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    w = rng.uniform(-1, 1, (K, C, R, S)).astype(np.float32)
    xp = np.zeros((N, C, H + 2 * pd, W + 2 * pd), np.float32)
    xp[:, :, pd:pd + H, pd:pd + W] = x
    assert np.array_equal(oracle.conv_forward(x, w, st, pd), oracle.conv_forward(xp, w, st, 0))


@pytest.mark.parametrize("t", [2, 3, 4])
def test_stride_is_subsampling_of_stride_one(oracle, t):
    rng = np.random.default_rng(17)
    x = rng.uniform(-1, 1, (2, 3, 14, 13)).astype(np.float32)
    w = rng.uniform(-1, 1, (4, 3, 3, 5)).astype(np.float32)
    full = oracle.conv_forward(x, w, 1, 2)
    assert np.array_equal(oracle.conv_forward(x, w, t, 2), full[:, :, ::t, ::t])


def test_linearity_exact_on_integers(oracle):
    rng = np.random.default_rng(18)
    x1, x2 = _ints(rng, (2, 3, 8, 9)), _ints(rng, (2, 3, 8, 9))
    w1, w2 = _ints(rng, (4, 3, 3, 3)), _ints(rng, (4, 3, 3, 3))
    a, b = 2.0, -3.0
    f = lambda x, w: oracle.conv_forward(x, w, 2, 1)
    assert np.array_equal(f(a * x1 + b * x2, w1), a * f(x1, w1) + b * f(x2, w1))
    assert np.array_equal(f(x1, a * w1 + b * w2), a * f(x1, w1) + b * f(x1, w2))
    assert np.array_equal(f(np.zeros_like(x1), w1), np.zeros_like(f(x1, w1)))


def test_batch_and_output_channel_independence(oracle):
    rng = np.random.default_rng(19)
    x = rng.uniform(-1, 1, (4, 3, 7, 8)).astype(np.float32)
    w = rng.uniform(-1, 1, (5, 3, 3, 3)).astype(np.float32)
    out = oracle.conv_forward(x, w, 1, 1)
    nperm, kperm = np.array([2, 0, 3, 1]), np.array([4, 1, 0, 3, 2])
    assert np.array_equal(oracle.conv_forward(x[nperm], w, 1, 1), out[nperm])
    assert np.array_equal(oracle.conv_forward(x, w[kperm], 1, 1), out[:, kperm])
    assert np.array_equal(oracle.conv_forward(x[1:2], w[3:4], 1, 1), out[1:2, 3:4])


def test_not_a_flipped_filter(oracle):
    # cross-correlation: out[p,q] = sum in[p+r, q+s] * w[r,s]; an asymmetric filter tells
    x = np.arange(16, dtype=np.float32).reshape(1, 1, 4, 4)
    w = np.array([[[[1.0, 2.0], [3.0, 4.0]]]], np.float32)
    out = oracle.conv_forward(x, w, 1, 0)
    assert out[0, 0, 0, 0] == 0 * 1 + 1 * 2 + 4 * 3 + 5 * 4
    assert out[0, 0, 2, 1] == 9 * 1 + 10 * 2 + 13 * 3 + 14 * 4


def test_rectangular_axes_not_transposed(oracle):
    # H != W and R != S: a tall filter on a wide image
    x = np.zeros((1, 1, 3, 6), np.float32)
    x[0, 0, 2, 5] = 1.0
    w = np.zeros((1, 1, 3, 2), np.float32)
    w[0, 0, 2, 1] = 7.0
    out = oracle.conv_forward(x, w, 1, 0)
    assert out.shape == (1, 1, 1, 5)
    want = np.zeros((1, 1, 1, 5))
    want[0, 0, 0, 4] = 7.0
    assert np.array_equal(out, want)


def test_points_match_full(oracle):
    l = workloads.TOY
    x, w = workloads.make_inputs(l)
    full = oracle.conv_forward(x, w, l.stride, l.pad)
    pts = workloads.sample_points(l, 200)
    got = oracle.conv_forward_points(x, w, pts, l.stride, l.pad)
    assert np.array_equal(got, full[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]])
    with pytest.raises(ValueError):
        oracle.conv_forward_points(x, w, np.array([[0, l.K, 0, 0]], np.int32), l.stride, l.pad)


def test_rejects_bad_dims(oracle):
    with pytest.raises(ValueError):
        oracle.conv_forward(np.ones((1, 1, 2, 2), np.float32), np.ones((1, 1, 3, 3), np.float32), 1, 0)
    with pytest.raises(ValueError):
        oracle.conv_forward(np.ones((1, 2, 4, 4), np.float32), np.ones((1, 1, 3, 3), np.float32), 1, 0)


def test_tolerance_formula(oracle):
    assert oracle.tolerance(3, 3, 3) == pytest.approx(1e-4 * 27 ** 0.5)
    assert oracle.tolerance(512, 3, 3) == pytest.approx(6.788e-3, rel=1e-3)


def test_seeded_inputs_are_reproducible_and_distributed():
    l = workloads.BY_NAME["alex_conv3_n64"]
    x1, w1 = workloads.make_inputs(l, N=2)
    x2, w2 = workloads.make_inputs(l, N=3)
    assert np.array_equal(x1, x2[:2]) and np.array_equal(w1, w2)
    assert x1.min() >= -1 and x1.max() <= 1 and x1.min() < -0.9
    assert abs(w1.std() * np.sqrt(l.crs) - 1.0) < 0.02
    xa, _ = workloads.make_inputs(workloads.BY_NAME["alex_conv1_n1"])
    assert xa.min() >= 0 and xa.max() <= 1
    assert workloads.TOY.seed == 0
    xi, wi = workloads.make_integer_inputs(l, N=1)
    assert np.array_equal(xi, np.round(xi)) and np.abs(xi).max() <= 4 and l.crs * 16 < 2 ** 24
