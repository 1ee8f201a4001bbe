"""Thin ctypes binding of the C ABI in include/conv_direct.h.

Argument marshalling only: every step of the convolution runs in the HIP kernels of
libconv_direct.so.  There is no CPU fallback: if the library is missing, loading
raises.  PyTorch appears only as the owner of device memory and streams.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
# CONV_DIRECT_LIB overrides the library path (e.g. an experimental build of the same ABI)
LIB_PATH = os.environ.get("CONV_DIRECT_LIB") or os.path.join(_HERE, "libconv_direct.so")

OK, EINVAL, EUNSUPPORTED, EALIGN, EHIP, ENOMEM = 0, -1, -2, -3, -4, -5

_lib = None


class ConvDirectError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} (code {code})")


def lib():
    """Load libconv_direct.so (built by build.py / __graft_entry__.build); raise if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_1809_10170_amd.build` "
                "(hipcc, gfx950).  There is no fallback path.")
        l = ctypes.CDLL(LIB_PATH)
        i, vp, cp = ctypes.c_int, ctypes.c_void_p, ctypes.c_char_p
        pp = ctypes.POINTER(vp)
        l.conv_direct_create.argtypes = [pp] + [i] * 9
        l.conv_direct_create.restype = i
        l.conv_direct_create_with_variant.argtypes = [pp, cp] + [i] * 9
        l.conv_direct_create_with_variant.restype = i
        l.conv_direct_variant_name.argtypes = [i]
        l.conv_direct_variant_name.restype = cp
        l.conv_direct_run.argtypes = [vp, vp, vp, vp, vp]
        l.conv_direct_run.restype = i
        l.conv_direct_destroy.argtypes = [vp]
        l.conv_direct_destroy.restype = i
        l.conv_direct_output_dims.argtypes = [vp, ctypes.POINTER(i), ctypes.POINTER(i)]
        l.conv_direct_output_dims.restype = i
        l.conv_direct_workspace_bytes.argtypes = [vp]
        l.conv_direct_workspace_bytes.restype = ctypes.c_size_t
        l.conv_direct_plan_info.argtypes = [vp, ctypes.c_char_p, ctypes.c_size_t]
        l.conv_direct_plan_info.restype = i
        l.conv_direct_strerror.argtypes = [i]
        l.conv_direct_strerror.restype = cp
        l.conv_direct_last_hip_error.argtypes = []
        l.conv_direct_last_hip_error.restype = i
        _lib = l
    return _lib


def strerror(code: int) -> str:
    return lib().conv_direct_strerror(code).decode()


def variant_names():
    out, i = [], 0
    while True:
        nm = lib().conv_direct_variant_name(i)
        if nm is None:
            return out
        out.append(nm.decode())
        i += 1


class Plan:
    """conv_direct_create / run / destroy around one opaque plan pointer."""

    def __init__(self, N, C, H, W, K, R, S, stride, pad, variant: str | None = None):
        self._p = ctypes.c_void_p()
        dims = [int(v) for v in (N, C, H, W, K, R, S, stride, pad)]
        if variant is None:
            rc = lib().conv_direct_create(ctypes.byref(self._p), *dims)
        else:
            rc = lib().conv_direct_create_with_variant(ctypes.byref(self._p), variant.encode(), *dims)
        if rc != OK:
            self._p = ctypes.c_void_p()
            raise ConvDirectError(rc, "conv_direct_create")
        self.dims = tuple(dims)

    def output_dims(self):
        P, Q = ctypes.c_int(), ctypes.c_int()
        rc = lib().conv_direct_output_dims(self._p, ctypes.byref(P), ctypes.byref(Q))
        if rc != OK:
            raise ConvDirectError(rc, "conv_direct_output_dims")
        return P.value, Q.value

    def workspace_bytes(self) -> int:
        return int(lib().conv_direct_workspace_bytes(self._p))

    def info(self) -> dict:
        buf = ctypes.create_string_buffer(1024)
        n = lib().conv_direct_plan_info(self._p, buf, len(buf))
        if n < 0:
            raise ConvDirectError(n, "conv_direct_plan_info")
        out = {}
        for tok in buf.value.decode().split():
            k, v = tok.split("=", 1)
            try:
                out[k] = int(v)
            except ValueError:
                try:
                    out[k] = float(v)
                except ValueError:
                    out[k] = v
        return out

    def run_ptr(self, in_ptr: int, w_ptr: int, out_ptr: int, stream: int = 0) -> None:
        """Raw device addresses (ints) and a hipStream_t handle (0 = default stream)."""
        rc = lib().conv_direct_run(self._p, in_ptr, w_ptr, out_ptr, stream)
        if rc != OK:
            raise ConvDirectError(rc, "conv_direct_run")

    def run(self, x, w, out, stream: int | None = None) -> None:
        """Device tensors (contiguous fp32); asynchronous on torch's current stream by default."""
        import torch
        N, C, H, W, K, R, S, _, _ = self.dims
        P, Q = self.output_dims()
        for t, shape, nm in ((x, (N, C, H, W), "in"), (w, (K, C, R, S), "w"), (out, (N, K, P, Q), "out")):
            if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and tuple(t.shape) == shape):
                raise ValueError(f"{nm}: need a contiguous fp32 device tensor of shape {shape}")
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        self.run_ptr(x.data_ptr(), w.data_ptr(), out.data_ptr(), stream)

    def destroy(self) -> None:
        if self._p:
            lib().conv_direct_destroy(self._p)
            self._p = ctypes.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def conv_forward(x, w, stride: int = 1, pad: int = 0, variant: str | None = None):
    """One-shot helper: plan, allocate the output tensor (caller-side memory), run."""
    import torch
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    plan = Plan(N, C, H, W, K, R, S, stride, pad, variant)
    P, Q = plan.output_dims()
    out = torch.empty((N, K, P, Q), device=x.device, dtype=torch.float32)
    plan.run(x, w, out)
    plan.destroy()
    return out
