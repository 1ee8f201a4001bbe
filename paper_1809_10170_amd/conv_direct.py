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

OK, EINVAL, EUNSUPPORTED, EALIGN, EHIP, ENOMEM, ETOOBIG = 0, -1, -2, -3, -4, -5, -6
STATIC_WT_ELEMS = 4 << 20      # CONV_DIRECT_STATIC_WT_ELEMS
PLAIN, BLOCKED = 0, 1          # CONV_DIRECT_LAYOUT_*
ACT_BLOCK, W_KBLOCK = 4, 32    # CONV_DIRECT_ACT_BLOCK, CONV_DIRECT_W_KBLOCK

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
        l.conv_direct_run_fused.argtypes = [vp, vp, vp, vp, vp, i, vp, vp]
        l.conv_direct_run_fused.restype = i
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
        l.conv_direct_create_layout.argtypes = [pp] + [i] * 11
        l.conv_direct_create_layout.restype = i
        l.conv_direct_create_ex.argtypes = [pp, cp] + [i] * 11
        l.conv_direct_create_ex.restype = i
        l.conv_direct_blocked_act_elems.argtypes = [i] * 4
        l.conv_direct_blocked_act_elems.restype = ctypes.c_size_t
        l.conv_direct_blocked_w_elems.argtypes = [i] * 4
        l.conv_direct_blocked_w_elems.restype = ctypes.c_size_t
        l.conv_direct_create_tuned.argtypes = [pp] + [i] * 11 + [vp, vp, vp, vp, i]
        l.conv_direct_create_tuned.restype = i
        for nm in ("conv_direct_tuning_save", "conv_direct_tuning_load"):
            getattr(l, nm).argtypes = [cp]
            getattr(l, nm).restype = i
        for nm in ("conv_direct_tuning_clear", "conv_direct_tuning_size"):
            getattr(l, nm).argtypes = []
            getattr(l, nm).restype = i
        l.conv_direct_create_wgrad.argtypes = [pp] + [i] * 9
        l.conv_direct_create_wgrad.restype = i
        l.conv_direct_create_wgrad_ex.argtypes = [pp, cp] + [i] * 9
        l.conv_direct_create_wgrad_ex.restype = i
        l.conv_direct_create_wgrad_deterministic.argtypes = [pp] + [i] * 9
        l.conv_direct_create_wgrad_deterministic.restype = i
        l.conv_direct_create_wgrad_layout.argtypes = [pp, cp, i] + [i] * 12
        l.conv_direct_create_wgrad_layout.restype = i
        l.conv_direct_wgrad_variant_name.argtypes = [i]
        l.conv_direct_wgrad_variant_name.restype = cp
        l.conv_direct_run_wgrad.argtypes = [vp, vp, vp, vp, vp]
        l.conv_direct_run_wgrad.restype = i
        l.conv_direct_create_dgrad.argtypes = [pp] + [i] * 9
        l.conv_direct_create_dgrad.restype = i
        l.conv_direct_create_dgrad_layout.argtypes = [pp] + [i] * 11
        l.conv_direct_create_dgrad_layout.restype = i
        l.conv_direct_create_dgrad_ex.argtypes = [pp, cp] + [i] * 11
        l.conv_direct_create_dgrad_ex.restype = i
        l.conv_direct_dgrad_wt_elems.argtypes = [vp]
        l.conv_direct_dgrad_wt_elems.restype = ctypes.c_size_t
        l.conv_direct_dgrad_prepare.argtypes = [vp, vp, vp, vp]
        l.conv_direct_dgrad_prepare.restype = i
        l.conv_direct_mfma_probe.argtypes = [vp, i, vp]
        l.conv_direct_mfma_probe.restype = i
        l.conv_direct_run_dgrad_static.argtypes = [vp, vp, vp, vp, vp]
        l.conv_direct_run_dgrad_static.restype = i
        for nm in ("conv_direct_pack_act", "conv_direct_unpack_act", "conv_direct_pack_w", "conv_direct_dgrad_filter"):
            getattr(l, nm).argtypes = [vp, vp] + [i] * 4 + [vp]
            getattr(l, nm).restype = i
        _lib = l
    return _lib


def strerror(code: int) -> str:
    return lib().conv_direct_strerror(code).decode()


def wgrad_variant_names():
    out, i = [], 0
    while True:
        nm = lib().conv_direct_wgrad_variant_name(i)
        if nm is None:
            return out
        out.append(nm.decode())
        i += 1


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

    def __init__(self, N, C, H, W, K, R, S, stride, pad, variant: str | None = None,
                 in_layout: int = PLAIN, out_layout: int = PLAIN):
        self._p = ctypes.c_void_p()
        dims = [int(v) for v in (N, C, H, W, K, R, S, stride, pad)]
        self.in_layout, self.out_layout = int(in_layout), int(out_layout)
        if self.in_layout != PLAIN or self.out_layout != PLAIN:
            rc = lib().conv_direct_create_ex(ctypes.byref(self._p), variant.encode() if variant else None, *dims,
                                             self.in_layout, self.out_layout)
        elif variant is None:
            rc = lib().conv_direct_create(ctypes.byref(self._p), *dims)
        else:
            rc = lib().conv_direct_create_with_variant(ctypes.byref(self._p), variant.encode(), *dims)
        if rc != OK:
            self._p = ctypes.c_void_p()
            raise ConvDirectError(rc, "conv_direct_create")
        self.dims = tuple(dims)

    @classmethod
    def tuned(cls, x, w, out, N, C, H, W, K, R, S, stride, pad, in_layout: int = PLAIN, out_layout: int = PLAIN,
              reps: int = 5, stream: int | None = None):
        """Time every variant that serves the shape on the given device tensors (out is overwritten, the
        stream synchronised) and return a plan for the fastest; the choice is remembered for later plans."""
        self = cls.__new__(cls)
        self._p = ctypes.c_void_p()
        self.in_layout, self.out_layout = int(in_layout), int(out_layout)
        dims = [int(v) for v in (N, C, H, W, K, R, S, stride, pad)]
        rc = lib().conv_direct_create_tuned(ctypes.byref(self._p), *dims, self.in_layout, self.out_layout,
                                            x.data_ptr(), w.data_ptr(), out.data_ptr(), _stream(stream), int(reps))
        if rc != OK:
            self._p = ctypes.c_void_p()
            raise ConvDirectError(rc, "conv_direct_create_tuned")
        self.dims = tuple(dims)
        return self

    @classmethod
    def dgrad(cls, N, C, H, W, K, R, S, stride, pad, dy_layout: int = PLAIN, dx_layout: int = PLAIN, variant: str | None = None):
        """Plan of the data gradient of the forward layer (N, C, H, W, K, R, S, stride, pad):
        run(dy [N,K,P,Q], wt from dgrad_prepare (dgrad_wt_elems() floats), dx [N,C,H,W]); dy and dx plain or in
        the blocked activation layout ([N, ceil(K/4), P, Q, 4], [N, ceil(C/4), H, W, 4])."""
        self = cls.__new__(cls)
        self._p = ctypes.c_void_p()
        self.in_layout, self.out_layout = int(dy_layout), int(dx_layout)
        rc = lib().conv_direct_create_dgrad_ex(ctypes.byref(self._p), variant.encode() if variant else None,
                                               *[int(v) for v in (N, C, H, W, K, R, S, stride, pad)], int(dy_layout), int(dx_layout))
        if rc != OK:
            self._p = ctypes.c_void_p()
            raise ConvDirectError(rc, "conv_direct_create_dgrad")
        self._dgrad = True
        self.fwd_dims = tuple(int(v) for v in (N, C, H, W, K, R, S, stride, pad))
        i = self.info()   # the problem the plan runs is a forward pass over dy [N][K][P][Q]: its "input" size is P x Q
        self.dims = (int(N), int(K), i["H"], i["W"], int(C), int(R), int(S), 1, R - 1 - pad)
        return self

    def dgrad_wt_elems(self) -> int:
        """Floats of the transformed filter a data-gradient plan takes (see dgrad_prepare)."""
        return int(lib().conv_direct_dgrad_wt_elems(self._p))

    def dgrad_prepare(self, w, wt, stream: int | None = None) -> None:
        """w [K,C,R,S] -> wt (a flat or shaped device tensor of dgrad_wt_elems() floats): the filter(s) this
        data-gradient plan runs with; once per weight update."""
        import torch
        for t, n, nm in ((w, None, "w"), (wt, self.dgrad_wt_elems(), "wt")):
            if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and (n is None or t.numel() == n)):
                raise ValueError(f"{nm}: need a contiguous fp32 device tensor" + (f" of {n} elements" if n else ""))
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        rc = lib().conv_direct_dgrad_prepare(self._p, w.data_ptr(), wt.data_ptr(), stream)
        if rc != OK:
            raise ConvDirectError(rc, "conv_direct_dgrad_prepare")

    def run_dgrad_static(self, dy, w, dx, stream: int | None = None) -> None:
        """conv_direct_run_dgrad_static: the data gradient from the layer's weights w [K,C,R,S] as they are,
        the transformed filter held in the library's static device array (nothing is allocated)."""
        import torch
        N, C, H, W, K, R, S, _, _ = self.fwd_dims
        n_, k_, p_, q_ = self.dims[:4]
        dys = (n_, k_, p_, q_) if self.in_layout == PLAIN else (n_, -(-k_ // ACT_BLOCK), p_, q_, ACT_BLOCK)
        dxs = (N, C, H, W) if self.out_layout == PLAIN else (N, -(-C // ACT_BLOCK), H, W, ACT_BLOCK)
        for t, shape, nm in ((dy, dys, "dy"), (w, (K, C, R, S), "w"), (dx, dxs, "dx")):
            if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and tuple(t.shape) == tuple(shape)):
                raise ValueError(f"{nm}: need a contiguous fp32 device tensor of shape {tuple(shape)}")
        rc = lib().conv_direct_run_dgrad_static(self._p, dy.data_ptr(), w.data_ptr(), dx.data_ptr(), _stream(stream))
        if rc != OK:
            raise ConvDirectError(rc, "conv_direct_run_dgrad_static")

    @classmethod
    def wgrad(cls, N, C, H, W, K, R, S, stride, pad, variant: str | None = None, deterministic: bool = False,
              x_layout: int = PLAIN, dy_layout: int = PLAIN, dw_layout: int = PLAIN):
        """Plan of the weight gradient of the forward layer: run_wgrad(x [N,C,H,W], dy [N,K,P,Q], dw [K,C,R,S]), each
        tensor plain or in its blocked layout.  deterministic: one workgroup per tile of dw (plain stores, the same
        bits every run)."""
        self = cls.__new__(cls)
        self._p = ctypes.c_void_p()
        self.in_layout, self.dy_layout, self.out_layout = int(x_layout), int(dy_layout), int(dw_layout)
        dims = [int(v) for v in (N, C, H, W, K, R, S, stride, pad)]
        if (self.in_layout, self.dy_layout, self.out_layout) != (PLAIN, PLAIN, PLAIN):
            rc = lib().conv_direct_create_wgrad_layout(ctypes.byref(self._p), variant.encode() if variant else None,
                                                       1 if deterministic else 0, *dims, self.in_layout, self.dy_layout, self.out_layout)
        elif deterministic:
            rc = lib().conv_direct_create_wgrad_deterministic(ctypes.byref(self._p), *dims)
        else:
            rc = lib().conv_direct_create_wgrad_ex(ctypes.byref(self._p), variant.encode() if variant else None, *dims)
        if rc != OK:
            self._p = ctypes.c_void_p()
            raise ConvDirectError(rc, "conv_direct_create_wgrad")
        self.dims = tuple(dims)
        return self

    def run_wgrad(self, x, dy, dw, stream: int | None = None) -> None:
        import torch
        N, C, H, W, K, R, S, st, pd = self.dims
        i = self.info()
        P, Q = i["P"], i["Q"]
        cb, kb = ACT_BLOCK, W_KBLOCK
        xs = (N, C, H, W) if self.in_layout == PLAIN else (N, -(-C // cb), H, W, cb)
        ys = (N, K, P, Q) if self.dy_layout == PLAIN else (N, -(-K // cb), P, Q, cb)
        ws = (K, C, R, S) if self.out_layout == PLAIN else (-(-K // kb), -(-C // cb), R, S, cb, kb)
        for t, shape, nm in ((x, xs, "x"), (dy, ys, "dy"), (dw, ws, "dw")):
            if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and tuple(t.shape) == shape):
                raise ValueError(f"{nm}: need a contiguous fp32 device tensor of shape {shape}")
        rc = lib().conv_direct_run_wgrad(self._p, x.data_ptr(), dy.data_ptr(), dw.data_ptr(), _stream(stream))
        if rc != OK:
            raise ConvDirectError(rc, "conv_direct_run_wgrad")

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

    def run(self, x, w, out, stream: int | None = None, bias=None, residual=None, relu: bool = False) -> None:
        """Device tensors (contiguous fp32); asynchronous on torch's current stream by default.
        bias [K], residual (out's shape and layout) and relu fold the point-wise tail into the store."""
        import torch
        N, C, H, W, K, R, S, _, _ = self.dims
        P, Q = self.output_dims()
        cb, kb = ACT_BLOCK, W_KBLOCK
        xs, ws = ((N, C, H, W), (K, C, R, S)) if self.in_layout == PLAIN else \
                 ((N, -(-C // cb), H, W, cb), (-(-K // kb), -(-C // cb), R, S, cb, kb))
        os_ = (N, K, P, Q) if self.out_layout == PLAIN else (N, -(-K // cb), P, Q, cb)
        for t, shape, nm in ((x, xs, "in"), (w, ws, "w"), (out, os_, "out")):
            if nm == "w" and getattr(self, "_dgrad", False):   # the transformed filter(s): size by the plan, any shape
                ok = t.numel() == self.dgrad_wt_elems()
                shape = (self.dgrad_wt_elems(),)
            else:
                ok = tuple(t.shape) == shape
            if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and ok):
                raise ValueError(f"{nm}: need a contiguous fp32 device tensor of shape {shape}")
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        if bias is None and residual is None and not relu:
            return self.run_ptr(x.data_ptr(), w.data_ptr(), out.data_ptr(), stream)
        for t, shape, nm in ((bias, (K,), "bias"), (residual, os_, "residual")):
            if t is not None and not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and tuple(t.shape) == shape):
                raise ValueError(f"{nm}: need a contiguous fp32 device tensor of shape {shape}")
        rc = lib().conv_direct_run_fused(self._p, x.data_ptr(), w.data_ptr(), bias.data_ptr() if bias is not None else None,
                                         residual.data_ptr() if residual is not None else None, 1 if relu else 0,
                                         out.data_ptr(), stream)
        if rc != OK:
            raise ConvDirectError(rc, "conv_direct_run_fused")

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


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    return stream


def _rearrange(fn, what, src, dst, dims, stream):
    rc = fn(src.data_ptr(), dst.data_ptr(), *[int(d) for d in dims], _stream(stream))
    if rc != OK:
        raise ConvDirectError(rc, what)
    return dst


def blocked_act_elems(N, C, H, W) -> int:
    return int(lib().conv_direct_blocked_act_elems(N, C, H, W))


def blocked_w_elems(K, C, R, S) -> int:
    return int(lib().conv_direct_blocked_w_elems(K, C, R, S))


def pack_act(plain, blocked, stream=None):
    """plain [N][C][H][W] -> blocked [N][ceil(C/4)][H][W][4] (device tensors, both the caller's)."""
    return _rearrange(lib().conv_direct_pack_act, "conv_direct_pack_act", plain, blocked, plain.shape, stream)


def unpack_act(blocked, plain, stream=None):
    """blocked [N][ceil(C/4)][H][W][4] -> plain [N][C][H][W]."""
    return _rearrange(lib().conv_direct_unpack_act, "conv_direct_unpack_act", blocked, plain, plain.shape, stream)


def pack_w(plain, blocked, stream=None):
    """plain [K][C][R][S] -> blocked [ceil(K/32)][ceil(C/4)][R][S][4][32]."""
    return _rearrange(lib().conv_direct_pack_w, "conv_direct_pack_w", plain, blocked, plain.shape, stream)


def dgrad_filter(w, wt, stream=None):
    """w [K][C][R][S] -> wt [C][K][R][S] with wt[c][k][r][s] = w[k][c][R-1-r][S-1-s] (device tensors)."""
    return _rearrange(lib().conv_direct_dgrad_filter, "conv_direct_dgrad_filter", w, wt, w.shape, stream)


PROBE_BYTES = 512 * 256 * 4 + 512 * 2 * 8          # CONV_DIRECT_PROBE_BYTES
PROBE_FLOP_PER_ITER = 512.0 * 4 * 8 * 7 * 4096      # CONV_DIRECT_PROBE_FLOP_PER_ITER


def mfma_probe(buf, iters: int, stream=None) -> None:
    """Enqueue the bare-MFMA measurement kernel (buf: a device tensor of at least PROBE_BYTES bytes)."""
    if buf.numel() * buf.element_size() < PROBE_BYTES:
        raise ValueError(f"buf: need {PROBE_BYTES} bytes")
    rc = lib().conv_direct_mfma_probe(buf.data_ptr(), int(iters), _stream(stream))
    if rc != OK:
        raise ConvDirectError(rc, "conv_direct_mfma_probe")


def tuning_save(path: str) -> None:
    rc = lib().conv_direct_tuning_save(os.fsencode(path))
    if rc != OK:
        raise ConvDirectError(rc, "conv_direct_tuning_save")


def tuning_load(path: str) -> None:
    rc = lib().conv_direct_tuning_load(os.fsencode(path))
    if rc != OK:
        raise ConvDirectError(rc, "conv_direct_tuning_load")


def tuning_clear() -> None:
    lib().conv_direct_tuning_clear()


def tuning_size() -> int:
    return int(lib().conv_direct_tuning_size())
