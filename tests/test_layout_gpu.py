"""GPU parity of the blocked-layout path (paper, Section 4) against the layout oracle:
the re-arrangers bit for bit, the convolution on blocked tensors bit for bit on integer
inputs and within 1e-4*sqrt(C*R*S) on random ones, in every mix of layouts the library
serves, and a chain of layers that never leaves the blocked layout."""
import re

import numpy as np
import pytest
import torch

from oracle import layout_ref as L
from paper_1809_10170_amd import conv_direct as cd
from paper_1809_10170_amd import workloads

pytestmark = pytest.mark.gpu
CB, KB = cd.ACT_BLOCK, cd.W_KBLOCK


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _nan(shape):
    return torch.full(shape, float("nan"), device="cuda", dtype=torch.float32)


def _conv(x, w, stride, pad, in_layout, out_layout, variant=None):
    """x, w plain host arrays; runs the library in the given layouts, returns a plain host array."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    plan = cd.Plan(N, C, H, W, K, R, S, stride, pad, variant, in_layout=in_layout, out_layout=out_layout)
    P, Q = plan.output_dims()
    xd = _dev(L.pack_activations(x, CB)) if in_layout == cd.BLOCKED else _dev(x)
    wd = _dev(L.pack_weights(w, CB, KB)) if in_layout == cd.BLOCKED else _dev(w)
    out = _nan((N, -(-K // CB), P, Q, CB)) if out_layout == cd.BLOCKED else _nan((N, K, P, Q))
    plan.run(xd, wd, out)
    torch.cuda.synchronize()
    info = plan.info()
    plan.destroy()
    got = out.cpu().numpy()
    assert not np.isnan(got).any(), f"{info['variant']}: an output element was never written"
    if out_layout == cd.BLOCKED:
        if K % CB:
            assert np.all(got[:, -1, :, :, K % CB:] == 0), "channels completing the last pencil must be zero"
        got = L.unpack_activations(got, K)
    return got, info


@pytest.mark.parametrize("N,C,H,W", [(2, 5, 7, 9), (1, 4, 1, 1), (3, 64, 13, 13), (2, 3, 31, 33)])
def test_activation_rearrangers_bit_exact(N, C, H, W):
    rng = np.random.default_rng(N * 1000 + C)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    assert cd.blocked_act_elems(N, C, H, W) == L.pack_activations(x, CB).size
    b = cd.pack_act(_dev(x), _nan((N, -(-C // CB), H, W, CB)))
    torch.cuda.synchronize()
    assert np.array_equal(b.cpu().numpy(), L.pack_activations(x, CB))
    back = cd.unpack_act(b, _nan((N, C, H, W)))
    torch.cuda.synchronize()
    assert np.array_equal(back.cpu().numpy(), x)


@pytest.mark.parametrize("K,C,R,S", [(37, 5, 3, 3), (32, 4, 1, 1), (96, 3, 11, 11), (70, 6, 5, 5)])
def test_weight_rearranger_bit_exact(K, C, R, S):
    rng = np.random.default_rng(K * 100 + C)
    w = rng.standard_normal((K, C, R, S)).astype(np.float32)
    want = L.pack_weights(w, CB, KB)
    assert cd.blocked_w_elems(K, C, R, S) == want.size
    b = cd.pack_w(_dev(w), _nan(want.shape))
    torch.cuda.synchronize()
    assert np.array_equal(b.cpu().numpy(), want)


def _blocked_variants():
    # (merged-phase variants, ...k64m..., serve only the data gradient of stride-2 layers: tests/test_dgrad_gpu.py; the walk
    # over all output channels, ..._kall, takes one channel count only: tests/test_pointwise_forms_gpu.py)
    return [n for n in cd.variant_names() if n.startswith("b") and "k64m" not in n and "_kall" not in n]


def _shape_for(nm, C):
    m = re.match(r"[a-z](\d+)s(\d+)_", nm)
    R, st = int(m.group(1)), int(m.group(2))
    fl = re.search(r"_flat(\d+)_", nm)
    H, W = (int(fl.group(1)),) * 2 if fl else (37, 41)
    if R == 1:
        C = {8: 40, 6: 37, 21: 70}[C]      # pointwise: enough channels for whole groups of steps and a tail
    return (3 if not fl else 9, C, H, W, 70, R, R, st, R // 2)


@pytest.mark.parametrize("C", [8, 6, 21])
@pytest.mark.parametrize("out_layout", [cd.BLOCKED, cd.PLAIN])
def test_every_blocked_variant_integer_inputs_bit_exact(oracle, C, out_layout):
    """Every compiled blocked variant, forced: whole and ragged channel blocks (C = 6, 21; K = 70),
    several tiles and a ragged tail, both output layouts."""
    names = _blocked_variants()
    assert names
    for nm in names:
        N, C_, H, W, K, R, S, st, pd = _shape_for(nm, C)
        rng = np.random.default_rng(300 + C + len(nm))
        x = rng.integers(-4, 5, (N, C_, H, W)).astype(np.float32)
        w = rng.integers(-4, 5, (K, C_, R, S)).astype(np.float32)
        assert C_ * R * S * 16 < 2 ** 24
        got, info = _conv(x, w, st, pd, cd.BLOCKED, out_layout, variant=nm)
        assert info["variant"] == nm
        want = oracle.conv_forward(x, w, st, pd)
        assert np.array_equal(got.astype(np.float64), want), f"{nm} C={C} out_layout={out_layout}"


@pytest.mark.parametrize("shape", [
    (2, 3, 99, 227, 96, 11, 11, 4, 0),    # first layer, row-pair family
    (2, 3, 75, 230, 64, 7, 7, 2, 3),
    (2, 7, 30, 61, 70, 3, 3, 1, 1),       # channel-pair family, ragged K
    (2, 37, 19, 23, 65, 1, 1, 1, 0),      # pointwise family
    (1, 64, 57, 59, 96, 1, 1, 1, 0),
])
def test_plain_input_blocked_output_bit_exact(oracle, shape):
    """The layout mix of a network's first layer (the paper keeps its input plain)."""
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(400 + sum(shape))
    x = rng.integers(-4, 5, (N, C, H, W)).astype(np.float32)
    w = rng.integers(-4, 5, (K, C, R, S)).astype(np.float32)
    assert C * R * S * 16 < 2 ** 24
    got, info = _conv(x, w, st, pd, cd.PLAIN, cd.BLOCKED)
    assert not info["variant"].startswith("generic")
    assert np.array_equal(got.astype(np.float64), oracle.conv_forward(x, w, st, pd)), info["variant"]


def test_chain_of_layers_stays_blocked(oracle):
    """conv1 (plain in, blocked out) -> 3x3 (blocked, blocked) -> 3x3 stride 2 (blocked in, plain out),
    each layer's blocked output handed to the next as it is."""
    rng = np.random.default_rng(7)
    x = rng.uniform(0, 1, (2, 3, 67, 67)).astype(np.float32)
    ws = [(rng.standard_normal(s) / np.sqrt(s[1] * s[2] * s[3])).astype(np.float32)
          for s in ((70, 3, 7, 7), (40, 70, 3, 3), (33, 40, 3, 3))]
    cfg = [(2, 3, cd.PLAIN, cd.BLOCKED), (1, 1, cd.BLOCKED, cd.BLOCKED), (2, 1, cd.BLOCKED, cd.PLAIN)]
    cur = _dev(x)
    shape = x.shape
    ref = x
    for w, (st, pd, li, lo) in zip(ws, cfg):
        N, C, H, W = shape
        K, _, R, S = w.shape
        plan = cd.Plan(N, C, H, W, K, R, S, st, pd, in_layout=li, out_layout=lo)
        P, Q = plan.output_dims()
        wd = _dev(L.pack_weights(w, CB, KB)) if li == cd.BLOCKED else _dev(w)
        out = _nan((N, -(-K // CB), P, Q, CB)) if lo == cd.BLOCKED else _nan((N, K, P, Q))
        plan.run(cur, wd, out)
        plan.destroy()
        cur, shape = out, (N, K, P, Q)
        ref = oracle.conv_forward(ref, w, st, pd).astype(np.float32)   # fp32 between layers, as on the GPU
    torch.cuda.synchronize()
    got = cur.cpu().numpy()
    # error of the last layer plus what the earlier layers' rounding differences grow to
    tol = 3 * oracle.tolerance(40, 3, 3)
    err = np.abs(got.astype(np.float64) - ref).max()
    assert not np.isnan(got).any() and err <= tol, err


BLOCKED_LAYERS = [l for l in workloads.ALL_LAYERS if l.N >= 32 and l.C >= 4]


@pytest.mark.parametrize("layer", BLOCKED_LAYERS, ids=lambda l: l.name)
def test_benchmark_layers_blocked_full_size(oracle, layer):
    """Full-size layers, blocked in and out, in the configuration the benchmark's blocked
    suite times: 10^5 seeded sampled outputs and three whole images against the oracle."""
    l = layer
    x, w = workloads.make_inputs(l)
    plan = cd.Plan(*l.dims(), in_layout=cd.BLOCKED, out_layout=cd.BLOCKED)
    assert plan.info()["variant"].startswith("b")
    xd, wd = _nan((l.N, -(-l.C // CB), l.H, l.W, CB)), _nan((-(-l.K // KB), -(-l.C // CB), l.R, l.S, CB, KB))
    cd.pack_act(_dev(x), xd)
    cd.pack_w(_dev(w), wd)
    out = _nan((l.N, -(-l.K // CB), l.P, l.Q, CB))
    plan.run(xd, wd, out)
    plain = cd.unpack_act(out, _nan((l.N, l.K, l.P, l.Q)))
    torch.cuda.synchronize()
    plan.destroy()
    got = plain.cpu().numpy()
    assert not np.isnan(got).any(), "an output element was never written"
    pts = workloads.sample_points(l, 100000)
    want = oracle.conv_forward_points(x, w, pts, l.stride, l.pad)
    err = np.abs(got[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]].astype(np.float64) - want).max()
    assert err <= oracle.tolerance(l.C, l.R, l.S), err
    for n in sorted({0, l.N // 2, l.N - 1}):   # the first, the middle and the last image in full
        want = oracle.conv_forward(x[n:n + 1], w, l.stride, l.pad)
        err = np.abs(got[n:n + 1].astype(np.float64) - want).max()
        assert err <= oracle.tolerance(l.C, l.R, l.S), (n, err)


@pytest.mark.parametrize("shape", [(2, 21, 30, 28, 40, 3, 3, 1, 1), (3, 8, 13, 13, 70, 3, 3, 1, 1), (2, 37, 20, 23, 33, 1, 1, 1, 0)])
def test_data_gradient_in_blocked_layouts(oracle, shape):
    """The stride-1 data gradient with dy, the filter and dx in the blocked layouts: it is the forward problem over
    dy (C output channels, padding R-1-pad), so the layout-aware forward entry points serve it; the transformed
    filter wt is re-arranged like any weights."""
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(1200 + sum(shape))
    w = rng.integers(-4, 5, (K, C, R, S)).astype(np.float32)
    P, Q = oracle.out_dim(H, R, st, pd), oracle.out_dim(W, S, st, pd)
    dy = rng.integers(-4, 5, (N, K, P, Q)).astype(np.float32)
    plan = cd.Plan(N, K, P, Q, C, R, S, 1, R - 1 - pd, in_layout=cd.BLOCKED, out_layout=cd.BLOCKED)
    assert plan.output_dims() == (H, W) and plan.workspace_bytes() == 0
    wt = torch.empty((C, K, R, S), device="cuda")
    cd.dgrad_filter(_dev(w), wt)
    wtb = _nan((-(-C // KB), -(-K // CB), R, S, CB, KB))
    cd.pack_w(wt, wtb)
    dyb = _nan((N, -(-K // CB), P, Q, CB))
    cd.pack_act(_dev(dy), dyb)
    dxb = _nan((N, -(-C // CB), H, W, CB))
    plan.run(dyb, wtb, dxb)
    dx = _nan((N, C, H, W))
    cd.unpack_act(dxb, dx)
    torch.cuda.synchronize()
    plan.destroy()
    assert np.array_equal(dx.cpu().numpy().astype(np.float64), oracle.conv_dgrad(dy, w, H, W, st, pd))
