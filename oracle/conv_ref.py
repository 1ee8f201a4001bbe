"""ctypes loader for the C oracle in conv_ref.c.

TEST INFRASTRUCTURE ONLY.  This wraps the plain CPU definition of the forward
convolution (paper: Section 3, Algorithm 1, with batch and zero padding added) so
that tests, the smoke check and the benchmark's cpu_baseline leg can call it with
numpy arrays.  It holds no arithmetic of its own beyond the tolerance formula and
does not import the GPU package.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_ref.c")
_LIB = os.path.join(_HERE, "libconv_ref.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile conv_ref.c with gcc (-O2, OpenMP, no fast-math) into libconv_ref.so."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i = ctypes.c_int
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        dims = [i] * 9
        lib.conv_ref_out_dim.argtypes = [i, i, i, i]
        lib.conv_ref_out_dim.restype = i
        lib.conv_ref_forward.argtypes = [fp, fp, dp] + dims
        lib.conv_ref_forward.restype = i
        lib.conv_ref_forward_reordered.argtypes = [fp, fp, dp] + dims
        lib.conv_ref_forward_reordered.restype = i
        lib.conv_ref_forward_points.argtypes = [fp, fp, ip, dp, ctypes.c_size_t] + dims
        lib.conv_ref_forward_points.restype = i
        lib.conv_ref_wgrad.argtypes = [fp, fp, dp] + dims
        lib.conv_ref_wgrad.restype = i
        lib.conv_ref_dgrad.argtypes = [fp, fp, dp] + dims
        lib.conv_ref_dgrad.restype = i
        lib.conv_ref_threads.argtypes = []
        lib.conv_ref_threads.restype = i
        _lib = lib
    return _lib


def out_dim(in_extent: int, filter_extent: int, stride: int, pad: int) -> int:
    """Output extent along one dimension (0 if the filter does not fit)."""
    return int(_load().conv_ref_out_dim(in_extent, filter_extent, stride, pad))


def threads() -> int:
    """Threads the full forward pass uses."""
    return int(_load().conv_ref_threads())


def tolerance(C: int, R: int, S: int) -> float:
    """Pass bound on max |gpu - oracle| for inputs of magnitude <= 1: 1e-4 * sqrt(C*R*S)."""
    return 1e-4 * math.sqrt(C * R * S)


def _prep(x, w):
    x = np.ascontiguousarray(x, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    if x.ndim != 4 or w.ndim != 4 or x.shape[1] != w.shape[1]:
        raise ValueError("expected in [N,C,H,W] and w [K,C,R,S] with equal C")
    return x, w


def _as(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _full(fn, x, w, stride, pad):
    x, w = _prep(x, w)
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    P, Q = out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)
    if P <= 0 or Q <= 0:
        raise ValueError("filter does not fit the padded input")
    out = np.empty((N, K, P, Q), dtype=np.float64)
    rc = fn(_as(x, ctypes.c_float), _as(w, ctypes.c_float), _as(out, ctypes.c_double),
            N, C, H, W, K, R, S, stride, pad)
    if rc != 0:
        raise ValueError(f"oracle rejected the dimensions (rc={rc})")
    return out


def conv_forward(x, w, stride: int = 1, pad: int = 0) -> np.ndarray:
    """out[n,k,p,q] in float64 for fp32 in [N,C,H,W] and w [K,C,R,S]."""
    return _full(_load().conv_ref_forward, x, w, stride, pad)


def conv_forward_reordered(x, w, stride: int = 1, pad: int = 0) -> np.ndarray:
    """Same result through the loop order of the paper's Algorithm 2 (self-check)."""
    return _full(_load().conv_ref_forward_reordered, x, w, stride, pad)


def conv_forward_points(x, w, idx, stride: int = 1, pad: int = 0) -> np.ndarray:
    """Oracle values at the listed (n,k,p,q) rows of idx (int32 [npts,4])."""
    x, w = _prep(x, w)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    if idx.ndim != 2 or idx.shape[1] != 4:
        raise ValueError("idx must be [npts,4]")
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    out = np.empty((idx.shape[0],), dtype=np.float64)
    rc = _load().conv_ref_forward_points(
        _as(x, ctypes.c_float), _as(w, ctypes.c_float), _as(idx, ctypes.c_int32),
        _as(out, ctypes.c_double), idx.shape[0], N, C, H, W, K, R, S, stride, pad)
    if rc != 0:
        raise ValueError(f"oracle rejected the request (rc={rc})")
    return out


def conv_dgrad(dy, w, H: int, W: int, stride: int = 1, pad: int = 0) -> np.ndarray:
    """Data gradient dx[n,c,h,w] in float64 for fp32 dy [N,K,P,Q] and w [K,C,R,S] of the
    layer whose input is H x W (the adjoint of conv_forward in its input)."""
    dy = np.ascontiguousarray(dy, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    if dy.ndim != 4 or w.ndim != 4 or dy.shape[1] != w.shape[0]:
        raise ValueError("expected dy [N,K,P,Q] and w [K,C,R,S] with equal K")
    N, K, P, Q = dy.shape
    _, C, R, S = w.shape
    if (P, Q) != (out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)):
        raise ValueError("dy does not have the layer's output size")
    dx = np.empty((N, C, H, W), dtype=np.float64)
    rc = _load().conv_ref_dgrad(_as(dy, ctypes.c_float), _as(w, ctypes.c_float), _as(dx, ctypes.c_double),
                                N, C, H, W, K, R, S, stride, pad)
    if rc != 0:
        raise ValueError(f"oracle rejected the dimensions (rc={rc})")
    return dx


def conv_wgrad(x, dy, R: int, S: int, stride: int = 1, pad: int = 0) -> np.ndarray:
    """Weight gradient dw[k,c,r,s] in float64 for fp32 x [N,C,H,W] and dy [N,K,P,Q] of the
    layer with an R x S filter (the adjoint of conv_forward in its filter)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    dy = np.ascontiguousarray(dy, dtype=np.float32)
    if x.ndim != 4 or dy.ndim != 4 or x.shape[0] != dy.shape[0]:
        raise ValueError("expected x [N,C,H,W] and dy [N,K,P,Q] with equal N")
    N, C, H, W = x.shape
    _, K, P, Q = dy.shape
    if (P, Q) != (out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)):
        raise ValueError("dy does not have the layer's output size")
    dw = np.empty((K, C, R, S), dtype=np.float64)
    rc = _load().conv_ref_wgrad(_as(x, ctypes.c_float), _as(dy, ctypes.c_float), _as(dw, ctypes.c_double),
                                N, C, H, W, K, R, S, stride, pad)
    if rc != 0:
        raise ValueError(f"oracle rejected the dimensions (rc={rc})")
    return dw
