"""Pins of the layout oracle (oracle/layout_ref.py) against what the paper's Section 4
fixes: the storage order written out by hand for tiny cases, the order enumerated by
loops from slowest to fastest index, inverses, zero fill, a direct loop nest on the
blocked arrays, the same-layout property that lets layers chain, and the gradients on
blocked arrays (scatter form, direct sums, adjoint identities)."""
import os

import numpy as np
import pytest

from oracle import conv_ref, layout_ref as L

GOLD = os.path.join(os.path.dirname(__file__), "golden", "layout_tiny.txt")


def _gold(tag):
    for ln in open(GOLD):
        if ln.startswith(tag + " "):
            return np.array([float(t) for t in ln.split()[1:]], dtype=np.float32)
    raise KeyError(tag)


def test_activation_layout_matches_hand_written_case():
    x = np.zeros((1, 5, 1, 2), dtype=np.float32)
    for c in range(5):
        for w in range(2):
            x[0, c, 0, w] = 10 * c + w
    assert np.array_equal(L.pack_activations(x, 4).ravel(), _gold("act"))


def test_weight_layout_matches_hand_written_case():
    w = np.zeros((3, 2, 1, 2), dtype=np.float32)
    for k in range(3):
        for c in range(2):
            for s in range(2):
                w[k, c, 0, s] = 100 * k + 10 * c + s
    assert np.array_equal(L.pack_weights(w, 2, 2).ravel(), _gold("wgt"))


@pytest.mark.parametrize("N,C,H,W,cb", [(2, 6, 3, 5, 4), (1, 4, 2, 2, 4), (3, 9, 1, 7, 8), (1, 3, 4, 4, 4)])
def test_activation_storage_order_enumerated(N, C, H, W, cb):
    rng = np.random.default_rng(1)
    x = rng.integers(-9, 10, size=(N, C, H, W)).astype(np.float32)
    seq = []
    for n in range(N):                       # slowest
        for blk in range(-(-C // cb)):
            for h in range(H):
                for w in range(W):
                    for ci in range(cb):     # fastest: the pencil
                        c = blk * cb + ci
                        seq.append(x[n, c, h, w] if c < C else 0.0)
    assert np.array_equal(L.pack_activations(x, cb).ravel(), np.array(seq, dtype=np.float32))


@pytest.mark.parametrize("K,C,R,S,cb,kb", [(5, 6, 3, 2, 4, 4), (40, 5, 1, 3, 4, 32), (3, 3, 2, 2, 2, 8)])
def test_weight_storage_order_enumerated(K, C, R, S, cb, kb):
    rng = np.random.default_rng(2)
    w = rng.integers(-9, 10, size=(K, C, R, S)).astype(np.float32)
    seq = []
    for kblk in range(-(-K // kb)):          # slowest: output-channel block
        for cblk in range(-(-C // cb)):      # input-channel block
            for r in range(R):               # filter row
                for s in range(S):           # filter column
                    for ci in range(cb):     # input channel in its block
                        for ki in range(kb): # fastest: output channel in its block
                            k, c = kblk * kb + ki, cblk * cb + ci
                            seq.append(w[k, c, r, s] if (k < K and c < C) else 0.0)
    assert np.array_equal(L.pack_weights(w, cb, kb).ravel(), np.array(seq, dtype=np.float32))


def test_pack_and_unpack_are_inverse_and_pad_is_zero():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 7, 3, 4)).astype(np.float32)
    xb = L.pack_activations(x, 4)
    assert xb.shape == (2, 2, 3, 4, 4)
    assert np.array_equal(L.unpack_activations(xb, 7), x)
    assert np.all(xb[:, 1, :, :, 3] == 0)
    w = rng.standard_normal((37, 7, 3, 3)).astype(np.float32)
    wb = L.pack_weights(w, 4, 32)
    assert wb.shape == (2, 2, 3, 3, 4, 32)
    assert np.array_equal(L.unpack_weights(wb, 37, 7), w)
    assert np.all(wb[1, :, :, :, :, 5:] == 0) and np.all(wb[:, 1, :, :, 3, :] == 0)
    assert xb.size * 4 == 2 * 8 * 3 * 4 * 4      # same bytes as the plain tensor rounded up to whole blocks


def test_direct_loops_on_blocked_arrays_bit_exact_on_integers():
    """The sum written directly on the blocked arrays (every index taken apart into block
    and position in block) equals the oracle's unpack / plain definition / pack."""
    rng = np.random.default_rng(4)
    N, C, H, W, K, R, S, stride, pad, cb, kb = 2, 6, 5, 6, 10, 3, 2, 2, 1, 4, 8
    x = rng.integers(-3, 4, size=(N, C, H, W)).astype(np.float32)
    w = rng.integers(-3, 4, size=(K, C, R, S)).astype(np.float32)
    xb, wb = L.pack_activations(x, cb), L.pack_weights(w, cb, kb)
    P, Q = conv_ref.out_dim(H, R, stride, pad), conv_ref.out_dim(W, S, stride, pad)
    ob = np.zeros((N, -(-K // cb), P, Q, cb), dtype=np.float64)
    for n in range(N):
        for k in range(K):
            for p in range(P):
                for q in range(Q):
                    acc = 0.0
                    for c in range(C):
                        for r in range(R):
                            for s in range(S):
                                ih, iw = p * stride + r - pad, q * stride + s - pad
                                if 0 <= ih < H and 0 <= iw < W:
                                    acc += float(xb[n, c // cb, ih, iw, c % cb]) * float(wb[k // kb, c // cb, r, s, c % cb, k % kb])
                    ob[n, k // cb, p, q, k % cb] = acc
    got = L.conv_forward_blocked(xb, wb, C, K, stride, pad)
    assert got.dtype == np.float64 and np.array_equal(got, ob)


def test_output_layout_is_the_next_layers_input_layout():
    rng = np.random.default_rng(5)
    x = rng.integers(-2, 3, size=(1, 5, 6, 6)).astype(np.float32)
    w1 = rng.integers(-2, 3, size=(7, 5, 3, 3)).astype(np.float32)
    w2 = rng.integers(-2, 3, size=(6, 7, 3, 3)).astype(np.float32)
    plain = conv_ref.conv_forward(conv_ref.conv_forward(x, w1, 1, 1).astype(np.float32), w2, 1, 1)
    y1 = L.conv_forward_blocked(L.pack_activations(x, 4), L.pack_weights(w1, 4, 32), 5, 7, 1, 1).astype(np.float32)
    y2 = L.conv_forward_blocked(y1, L.pack_weights(w2, 4, 32), 7, 6, 1, 1)
    assert np.array_equal(L.unpack_activations(y2, 6), plain)


GRAD_CASES = [  # N, C, H, W, K, R, S, stride, pad
    (2, 6, 5, 6, 10, 3, 3, 1, 1),
    (1, 5, 7, 6, 7, 3, 2, 2, 1),
    (2, 3, 9, 8, 5, 5, 5, 3, 2),
    (1, 9, 6, 6, 4, 1, 1, 2, 0),
]


@pytest.mark.parametrize("N,C,H,W,K,R,S,stride,pad", GRAD_CASES)
def test_data_gradient_on_blocked_arrays_scatter_form_bit_exact_on_integers(N, C, H, W, K, R, S, stride, pad):
    """The adjoint written as a scatter directly on the blocked arrays (every dy element adds
    dy*w to the input positions its window covered) equals the oracle's unpack / gather
    definition / pack, and the pencils' spare channels are zero."""
    rng = np.random.default_rng(11)
    cb = 4
    dy = rng.integers(-3, 4, size=(N, K, conv_ref.out_dim(H, R, stride, pad), conv_ref.out_dim(W, S, stride, pad))).astype(np.float32)
    w = rng.integers(-3, 4, size=(K, C, R, S)).astype(np.float32)
    dyb = L.pack_activations(dy, cb)
    P, Q = dy.shape[2:]
    dxb = np.zeros((N, -(-C // cb), H, W, cb), dtype=np.float64)
    for n in range(N):
        for k in range(K):
            for p in range(P):
                for q in range(Q):
                    g = float(dyb[n, k // cb, p, q, k % cb])
                    for c in range(C):
                        for r in range(R):
                            for s in range(S):
                                ih, iw = p * stride + r - pad, q * stride + s - pad
                                if 0 <= ih < H and 0 <= iw < W:
                                    dxb[n, c // cb, ih, iw, c % cb] += g * float(w[k, c, r, s])
    got = L.conv_dgrad_blocked(dyb, w, H, W, stride, pad)
    assert got.dtype == np.float64 and got.shape == dxb.shape and np.array_equal(got, dxb)
    if C % cb:
        assert np.all(got[:, -1, :, :, C % cb:] == 0)


@pytest.mark.parametrize("N,C,H,W,K,R,S,stride,pad", GRAD_CASES)
def test_weight_gradient_on_blocked_arrays_bit_exact_on_integers(N, C, H, W, K, R, S, stride, pad):
    """dw[k][c][r][s] summed directly over the blocked x and dy arrays, against the oracle, in the
    plain and in the blocked weight layout."""
    rng = np.random.default_rng(12)
    cb, kb = 4, 8
    P, Q = conv_ref.out_dim(H, R, stride, pad), conv_ref.out_dim(W, S, stride, pad)
    x = rng.integers(-3, 4, size=(N, C, H, W)).astype(np.float32)
    dy = rng.integers(-3, 4, size=(N, K, P, Q)).astype(np.float32)
    xb, dyb = L.pack_activations(x, cb), L.pack_activations(dy, cb)
    dw = np.zeros((K, C, R, S), dtype=np.float64)
    for k in range(K):
        for c in range(C):
            for r in range(R):
                for s in range(S):
                    acc = 0.0
                    for n in range(N):
                        for p in range(P):
                            for q in range(Q):
                                ih, iw = p * stride + r - pad, q * stride + s - pad
                                if 0 <= ih < H and 0 <= iw < W:
                                    acc += float(dyb[n, k // cb, p, q, k % cb]) * float(xb[n, c // cb, ih, iw, c % cb])
                    dw[k, c, r, s] = acc
    got = L.conv_wgrad_blocked(xb, dyb, C, K, R, S, stride, pad)
    assert got.dtype == np.float64 and np.array_equal(got, dw)
    gotb = L.conv_wgrad_blocked(xb, dyb, C, K, R, S, stride, pad, cb=cb, kb=kb)
    assert np.array_equal(L.unpack_weights(gotb, K, C), dw) and gotb.shape == (-(-K // kb), -(-C // cb), R, S, cb, kb)


def test_blocked_gradients_are_the_adjoints_of_the_blocked_forward_map():
    """<dy, forward(x, w)> = <dgrad(dy, w), x> = <wgrad(x, dy), w>, every term computed on blocked
    arrays (spare channels are zero on both sides of each product); exact on integers."""
    rng = np.random.default_rng(13)
    N, C, H, W, K, R, S, stride, pad = 2, 6, 7, 7, 9, 3, 3, 2, 1
    x = rng.integers(-3, 4, size=(N, C, H, W)).astype(np.float32)
    w = rng.integers(-3, 4, size=(K, C, R, S)).astype(np.float32)
    P, Q = conv_ref.out_dim(H, R, stride, pad), conv_ref.out_dim(W, S, stride, pad)
    dy = rng.integers(-3, 4, size=(N, K, P, Q)).astype(np.float32)
    xb, dyb, wb = L.pack_activations(x, 4), L.pack_activations(dy, 4), L.pack_weights(w, 4, 32)
    yb = L.conv_forward_blocked(xb, wb, C, K, stride, pad)
    lhs = float(np.sum(dyb.astype(np.float64) * yb))
    mid = float(np.sum(L.conv_dgrad_blocked(dyb, w, H, W, stride, pad) * xb.astype(np.float64)))
    rhs = float(np.sum(L.conv_wgrad_blocked(xb, dyb, C, K, R, S, stride, pad, cb=4, kb=32) * wb.astype(np.float64)))
    assert lhs == mid == rhs and lhs != 0.0
