"""The one entry point that allocates nothing, conv_direct_run_dgrad_static (for callers that cannot call
hipMalloc), through the C ABI against the existing entry points it is a variant of
(conv_direct_dgrad_prepare into a caller buffer + conv_direct_run): same kernels, so bit for bit; and both
against the oracle's adjoint definition.  Two calls in a row, the second on a smaller problem, so that
what the first call left in the library's static array lies behind and around what the second one uses."""
import numpy as np
import pytest
import torch

from paper_1809_10170_amd import conv_direct as cd

pytestmark = pytest.mark.gpu


def _both(oracle, shape, seed):
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(seed)
    w = rng.uniform(-1, 1, (K, C, R, S)).astype(np.float32)
    P, Q = oracle.out_dim(H, R, st, pd), oracle.out_dim(W, S, st, pd)
    dy = rng.uniform(-1, 1, (N, K, P, Q)).astype(np.float32)
    plan = cd.Plan.dgrad(*shape)
    assert plan.dgrad_wt_elems() <= cd.STATIC_WT_ELEMS
    dyd, wd = torch.from_numpy(dy).cuda(), torch.from_numpy(w).cuda()
    # the existing entry points, with a caller-owned transformed filter
    wt = torch.full((plan.dgrad_wt_elems(),), float("nan"), device="cuda")
    want = torch.full((N, C, H, W), float("nan"), device="cuda")
    plan.dgrad_prepare(wd, wt)
    plan.run(dyd, wt, want)
    torch.cuda.synchronize()
    # the entry point that allocates nothing: torch's allocator must not move, nor the device's free memory
    # (beyond what loading the code object on the very first launch takes, which has happened above)
    got = torch.full((N, C, H, W), float("nan"), device="cuda")
    torch.cuda.synchronize()
    alloc0, res0 = torch.cuda.memory_allocated(), torch.cuda.memory_reserved()
    free0, _ = torch.cuda.mem_get_info()
    plan.run_dgrad_static(dyd, wd, got)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert torch.cuda.memory_allocated() == alloc0 and torch.cuda.memory_reserved() == res0
    assert free1 >= free0, "device memory was taken during conv_direct_run_dgrad_static"
    plan.destroy()
    assert torch.isfinite(got).all()
    assert torch.equal(got, want), f"{shape}: static-array path differs from the caller-buffer path"
    ref = oracle.conv_dgrad(dy, w, H, W, st, pd)
    err = np.abs(got.cpu().numpy().astype(np.float64) - ref).max()
    assert err <= oracle.tolerance(K, R, S), (shape, err)


def test_two_calls_in_a_row_second_smaller(oracle):
    # stride 1 (one transformed filter of the weights' size), then a smaller strided layer (four phase filters)
    _both(oracle, (2, 40, 29, 31, 70, 3, 3, 1, 1), 1)
    _both(oracle, (2, 12, 21, 20, 33, 3, 3, 2, 1), 2)
    # and a still smaller stride-1 problem after the strided one
    _both(oracle, (1, 5, 9, 9, 6, 3, 3, 1, 1), 3)


def test_rejects_what_does_not_fit_before_any_launch():
    # 1024 x 1024 x 3 x 3 weights are 9.4 Mi floats, more than the static array's 4 Mi
    plan = cd.Plan.dgrad(1, 1024, 8, 8, 1024, 3, 3, 1, 1)
    assert plan.dgrad_wt_elems() > cd.STATIC_WT_ELEMS
    rc = cd.lib().conv_direct_run_dgrad_static(plan._p, 4096, 8192, 12288, None)
    assert rc == cd.ETOOBIG and "static array" in cd.strerror(rc)
    # a forward plan is no data gradient
    fwd = cd.Plan(1, 3, 8, 8, 4, 3, 3, 1, 1)
    assert cd.lib().conv_direct_run_dgrad_static(fwd._p, 4096, 8192, 12288, None) == cd.EINVAL
    assert cd.lib().conv_direct_run_dgrad_static(plan._p, 4097, 8192, 12288, None) == cd.EALIGN
    assert cd.lib().conv_direct_run_dgrad_static(plan._p, None, 8192, 12288, None) == cd.EINVAL
    plan.destroy()
    fwd.destroy()
