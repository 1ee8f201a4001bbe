"""Seeded random small shapes through every path the library offers for them: plain and
blocked forward (where a compiled variant serves the shape), fused tail, data gradient
(stride 1, square filters) and weight gradient (supported filter widths), each against
the oracle, bit for bit on integer inputs."""
import numpy as np
import pytest
import torch

from oracle import layout_ref as L
from paper_1809_10170_amd import conv_direct as cd

pytestmark = pytest.mark.gpu


def _shapes(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        R, S = (int(rng.integers(1, 6)),) * 2 if rng.random() < 0.7 else (int(rng.integers(1, 6)), int(rng.integers(1, 6)))
        st, pd = int(rng.integers(1, 4)), int(rng.integers(0, 4))
        H, W = int(rng.integers(1, 41)), int(rng.integers(1, 41))
        if H + 2 * pd < R or W + 2 * pd < S:
            continue
        out.append((int(rng.integers(1, 4)), int(rng.integers(1, 71)), H, W, int(rng.integers(1, 71)), R, S, st, pd))
    return out


SHAPES = _shapes(48, 20260) + _shapes(32, 20261)


def _ints(rng, shape, amp=3):
    return rng.integers(-amp, amp + 1, size=shape).astype(np.float32)


@pytest.mark.parametrize("shape", SHAPES)
def test_forward_plain_and_fused(oracle, shape):
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(sum(shape))
    x, w = _ints(rng, (N, C, H, W)), _ints(rng, (K, C, R, S))
    plan = cd.Plan(*shape)
    P, Q = plan.output_dims()
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    out = torch.full((N, K, P, Q), float("nan"), device="cuda")
    plan.run(xd, wd, out)
    torch.cuda.synchronize()
    want = oracle.conv_forward(x, w, st, pd)
    assert np.array_equal(out.cpu().numpy().astype(np.float64), want), plan.info()["variant"]
    if not plan.info()["variant"].startswith("generic"):
        b, r = _ints(rng, (K,), 20), _ints(rng, (N, K, P, Q), 20)
        out.fill_(float("nan"))
        plan.run(xd, wd, out, bias=torch.from_numpy(b).cuda(), residual=torch.from_numpy(r).cuda(), relu=True)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().astype(np.float64), oracle.apply_tail(want, b, r, True)), plan.info()["variant"]
    plan.destroy()


@pytest.mark.parametrize("shape", SHAPES)
def test_forward_blocked(oracle, shape):
    N, C, H, W, K, R, S, st, pd = shape
    plan = cd.Plan(*shape, in_layout=cd.BLOCKED, out_layout=cd.BLOCKED)
    rng = np.random.default_rng(1 + sum(shape))
    x, w = _ints(rng, (N, C, H, W)), _ints(rng, (K, C, R, S))
    P, Q = plan.output_dims()
    out = torch.full((N, -(-K // 4), P, Q, 4), float("nan"), device="cuda")
    plan.run(torch.from_numpy(L.pack_activations(x, 4)).cuda(), torch.from_numpy(L.pack_weights(w, 4, 32)).cuda(), out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert not np.isnan(got).any()
    assert np.array_equal(L.unpack_activations(got, K).astype(np.float64), oracle.conv_forward(x, w, st, pd)), plan.info()["variant"]
    plan.destroy()


@pytest.mark.parametrize("shape", SHAPES)
def test_data_gradient(oracle, shape):
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(2 + sum(shape))
    w = _ints(rng, (K, C, R, S))
    dy = _ints(rng, (N, K, oracle.out_dim(H, R, st, pd), oracle.out_dim(W, S, st, pd)))
    plan = cd.Plan.dgrad(*shape)
    wt = torch.empty((plan.dgrad_wt_elems(),), device="cuda")
    plan.dgrad_prepare(torch.from_numpy(w).cuda(), wt)
    dx = torch.full((N, C, H, W), float("nan"), device="cuda")
    dyd = torch.from_numpy(dy).cuda()
    assert cd.lib().conv_direct_run(plan._p, dyd.data_ptr(), wt.data_ptr(), dx.data_ptr(), None) == cd.OK
    torch.cuda.synchronize()
    assert np.array_equal(dx.cpu().numpy().astype(np.float64), oracle.conv_dgrad(dy, w, H, W, st, pd)), plan.info()["variant"]
    plan.destroy()


@pytest.mark.parametrize("shape", SHAPES)
def test_weight_gradient(oracle, shape):
    N, C, H, W, K, R, S, st, pd = shape
    try:
        plan = cd.Plan.wgrad(*shape)
    except cd.ConvDirectError as e:
        assert e.code == cd.EUNSUPPORTED
        pytest.skip("no weight-gradient variant for this filter width and stride")
    rng = np.random.default_rng(3 + sum(shape))
    x = _ints(rng, (N, C, H, W))
    dy = _ints(rng, (N, K, oracle.out_dim(H, R, st, pd), oracle.out_dim(W, S, st, pd)))
    dw = torch.full((K, C, R, S), float("nan"), device="cuda")
    plan.run_wgrad(torch.from_numpy(x).cuda(), torch.from_numpy(dy).cuda(), dw)
    torch.cuda.synchronize()
    assert np.array_equal(dw.cpu().numpy().astype(np.float64), oracle.conv_wgrad(x, dy, R, S, st, pd)), plan.info()["variant"]
    plan.destroy()
