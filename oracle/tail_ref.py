"""Plain definition of the point-wise layers folded into the convolution's store
(paper, Section 4.3 names skip and activation layers as point-wise operations).

TEST INFRASTRUCTURE ONLY: the GPU package never imports this module.

    out[n][k][p][q] = relu?( conv[n][k][p][q] + bias[k] + residual[n][k][p][q] )

in float64, on the float64 result of the convolution oracle; relu(v) = max(v, 0).
"""
from __future__ import annotations

import numpy as np

from . import conv_ref


def apply_tail(y: np.ndarray, bias=None, residual=None, relu: bool = False) -> np.ndarray:
    out = np.array(y, dtype=np.float64, copy=True)
    if bias is not None:
        b = np.asarray(bias, dtype=np.float64)
        if b.shape != (y.shape[1],):
            raise ValueError("bias must have one value per output channel")
        for k in range(y.shape[1]):
            out[:, k, :, :] += b[k]
    if residual is not None:
        r = np.asarray(residual, dtype=np.float64)
        if r.shape != y.shape:
            raise ValueError("residual must have the output's shape")
        out += r
    if relu:
        out[out < 0.0] = 0.0
    return out


def conv_forward_fused(x, w, stride=1, pad=0, bias=None, residual=None, relu=False) -> np.ndarray:
    return apply_tail(conv_ref.conv_forward(x, w, stride, pad), bias, residual, relu)
