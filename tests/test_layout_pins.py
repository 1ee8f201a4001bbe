"""Pins of the layout oracle (oracle/layout_ref.py) against what the paper's Section 4
fixes: the storage order written out by hand for tiny cases, the order enumerated by
loops from slowest to fastest index, inverses, zero fill, a direct loop nest on the
blocked arrays, and the same-layout property that lets layers chain."""
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
