"""Plain definitions of the paper's convolution-friendly layouts (Section 4).

TEST INFRASTRUCTURE ONLY: the GPU package never imports this module.

Activations (Section 4.1, Figure 3 left): channels are cut into blocks of `cb`; a tensor
is a sequence of blocks, each an H x W row-major matrix of pencils of `cb` channels, so
the channel inside the block is the fastest index, then the column, then the row, then
the channel block (then the image: the batch dimension is this build's addition):
    blocked[n][c // cb][h][w][c % cb] = plain[n][c][h][w]
Input and output use the same layout, so that a layer's output is the next layer's
input without a reshape.

Weights (Section 4.2, Figure 3 right): fastest to slowest the output channel inside
its block of `kb`, the input channel inside its block of `cb`, the filter column, the
filter row, the input-channel block, the output-channel block:
    blocked[k // kb][c // cb][r][s][c % cb][k % kb] = plain[k][c][r][s]

Channels that complete the last block hold zeros.  The paper leaves the block sizes to
the implementation (Section 3.1.2 derives them per machine); callers pass them in.

The convolution on blocked tensors is the same function of the same numbers: unpack,
apply the plain definition (conv_ref), pack.
"""
from __future__ import annotations

import numpy as np

from . import conv_ref


def _blocks(n: int, b: int) -> int:
    return -(-n // b)


def pack_activations(x: np.ndarray, cb: int) -> np.ndarray:
    """[N][C][H][W] -> [N][ceil(C/cb)][H][W][cb], zero-filled past C."""
    N, C, H, W = x.shape
    out = np.zeros((N, _blocks(C, cb), H, W, cb), dtype=x.dtype)
    for c in range(C):
        out[:, c // cb, :, :, c % cb] = x[:, c, :, :]
    return out


def unpack_activations(xb: np.ndarray, C: int) -> np.ndarray:
    """[N][ceil(C/cb)][H][W][cb] -> [N][C][H][W]."""
    N, nb, H, W, cb = xb.shape
    if nb != _blocks(C, cb):
        raise ValueError("block count does not match C")
    out = np.empty((N, C, H, W), dtype=xb.dtype)
    for c in range(C):
        out[:, c, :, :] = xb[:, c // cb, :, :, c % cb]
    return out


def pack_weights(w: np.ndarray, cb: int, kb: int) -> np.ndarray:
    """[K][C][R][S] -> [ceil(K/kb)][ceil(C/cb)][R][S][cb][kb], zero-filled past K and C."""
    K, C, R, S = w.shape
    out = np.zeros((_blocks(K, kb), _blocks(C, cb), R, S, cb, kb), dtype=w.dtype)
    for k in range(K):
        for c in range(C):
            out[k // kb, c // cb, :, :, c % cb, k % kb] = w[k, c, :, :]
    return out


def unpack_weights(wb: np.ndarray, K: int, C: int) -> np.ndarray:
    """Inverse of pack_weights."""
    nkb, ncb, R, S, cb, kb = wb.shape
    if nkb != _blocks(K, kb) or ncb != _blocks(C, cb):
        raise ValueError("block counts do not match K, C")
    out = np.empty((K, C, R, S), dtype=wb.dtype)
    for k in range(K):
        for c in range(C):
            out[k, c, :, :] = wb[k // kb, c // cb, :, :, c % cb, k % kb]
    return out


def conv_forward_blocked(xb: np.ndarray, wb: np.ndarray, C: int, K: int, stride: int = 1, pad: int = 0,
                         out_cb: int | None = None) -> np.ndarray:
    """Forward convolution of blocked fp32 tensors; float64 result in the activation
    layout with pencils of out_cb channels (default: the input's pencil length)."""
    cb = xb.shape[-1]
    out = conv_ref.conv_forward(unpack_activations(xb, C), unpack_weights(wb, K, C), stride, pad)
    return pack_activations(out, out_cb or cb)


def conv_dgrad_blocked(dyb: np.ndarray, w: np.ndarray, H: int, W: int, stride: int = 1, pad: int = 0,
                       out_cb: int | None = None) -> np.ndarray:
    """Data gradient (the adjoint of the forward map in its input; the paper's closing
    section names the backward pass without an algorithm) with the activations in the
    blocked layout of Section 4.1: dy [N][ceil(K/cb)][P][Q][cb], weights plain
    [K][C][R][S]; float64 dx [N][ceil(C/out_cb)][H][W][out_cb].  Same function of the
    same numbers: unpack, plain definition (conv_ref.conv_dgrad), pack."""
    K = w.shape[0]
    cb = dyb.shape[-1]
    dx = conv_ref.conv_dgrad(unpack_activations(dyb, K), w, H, W, stride, pad)
    return pack_activations(dx, out_cb or cb)


def conv_wgrad_blocked(xb: np.ndarray, dyb: np.ndarray, C: int, K: int, R: int, S: int, stride: int = 1,
                       pad: int = 0, cb: int | None = None, kb: int | None = None) -> np.ndarray:
    """Weight gradient (the adjoint in the filter) of blocked activations x
    [N][ceil(C/.)][H][W][.] and dy [N][ceil(K/.)][P][Q][.]; float64 dw, plain [K][C][R][S],
    or in the blocked weight layout of Section 4.2 when both cb and kb are given."""
    dw = conv_ref.conv_wgrad(unpack_activations(xb, C), unpack_activations(dyb, K), R, S, stride, pad)
    if cb is None and kb is None:
        return dw
    if cb is None or kb is None:
        raise ValueError("give both block sizes, or neither")
    return pack_weights(dw, cb, kb)
