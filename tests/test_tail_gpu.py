"""GPU parity of the fused point-wise tail (bias, residual, ReLU) in every kernel family
and both output layouts."""
import numpy as np
import pytest
import torch

from oracle import layout_ref as L
from paper_1809_10170_amd import conv_direct as cd

pytestmark = pytest.mark.gpu

SHAPES = [
    # N, C, H, W, K, R, S, stride, pad
    (2, 7, 30, 61, 70, 3, 3, 1, 1),       # channel-pair family, ragged K (guarded stores) and whole blocks
    (3, 16, 13, 13, 130, 3, 3, 1, 1),     # flat tiling: tiles span images
    (2, 3, 99, 227, 96, 11, 11, 4, 0),    # row-pair family
    (2, 37, 19, 23, 65, 1, 1, 1, 0),      # pointwise family
    (2, 12, 57, 55, 130, 3, 3, 2, 1),     # stride 2
]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("parts", [(1, 0, 0), (0, 1, 0), (0, 0, 1), (1, 1, 1)])
@pytest.mark.parametrize("out_layout", [cd.PLAIN, cd.BLOCKED])
def test_fused_tail_integer_inputs_bit_exact(oracle, shape, parts, out_layout):
    N, C, H, W, K, R, S, st, pd = shape
    use_b, use_r, relu = parts
    rng = np.random.default_rng(700 + sum(shape) + 7 * sum(parts))
    x = rng.integers(-4, 5, (N, C, H, W)).astype(np.float32)
    w = rng.integers(-4, 5, (K, C, R, S)).astype(np.float32)
    plan = cd.Plan(N, C, H, W, K, R, S, st, pd, out_layout=out_layout)
    P, Q = plan.output_dims()
    b = rng.integers(-50, 51, (K,)).astype(np.float32) if use_b else None
    r = rng.integers(-50, 51, (N, K, P, Q)).astype(np.float32) if use_r else None
    assert C * R * S * 16 + 100 < 2 ** 24
    blocked = out_layout == cd.BLOCKED
    out = torch.full((N, -(-K // 4), P, Q, 4) if blocked else (N, K, P, Q), float("nan"), device="cuda")
    rd = None
    if r is not None:
        rd = torch.from_numpy(L.pack_activations(r, 4) if blocked else r).cuda()
    plan.run(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), out,
             bias=torch.from_numpy(b).cuda() if b is not None else None, residual=rd, relu=bool(relu))
    torch.cuda.synchronize()
    info = plan.info()
    plan.destroy()
    got = out.cpu().numpy()
    assert not np.isnan(got).any()
    if blocked:
        if K % 4:
            assert np.all(got[:, -1, :, :, K % 4:] == 0)
        got = L.unpack_activations(got, K)
    want = oracle.conv_forward_fused(x, w, st, pd, bias=b, residual=r, relu=bool(relu))
    assert np.array_equal(got.astype(np.float64), want), info["variant"]


def test_fused_tail_random_inputs_and_plain_run_unchanged(oracle):
    N, C, H, W, K, R, S, st, pd = 2, 16, 28, 28, 64, 3, 3, 1, 1
    rng = np.random.default_rng(9)
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    w = rng.uniform(-1, 1, (K, C, R, S)).astype(np.float32)
    b = rng.uniform(-1, 1, (K,)).astype(np.float32)
    r = rng.uniform(-1, 1, (N, K, H, W)).astype(np.float32)
    plan = cd.Plan(N, C, H, W, K, R, S, st, pd)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    o1, o2 = torch.empty((N, K, H, W), device="cuda"), torch.empty((N, K, H, W), device="cuda")
    plan.run(xd, wd, o1, bias=torch.from_numpy(b).cuda(), residual=torch.from_numpy(r).cuda(), relu=True)
    plan.run(xd, wd, o2)
    torch.cuda.synchronize()
    plan.destroy()
    tol = oracle.tolerance(C, R, S)
    assert np.abs(o1.cpu().numpy() - oracle.conv_forward_fused(x, w, st, pd, b, r, True)).max() <= tol
    assert np.abs(o2.cpu().numpy() - oracle.conv_forward(x, w, st, pd)).max() <= tol


def test_fallback_kernel_applies_the_tail_too(oracle):
    shape = (1, 2, 5, 300, 3, 1, 7, 1, 3)              # a shape only the runtime-shape kernel serves
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(21)
    x = rng.integers(-4, 5, (N, C, H, W)).astype(np.float32)
    w = rng.integers(-4, 5, (K, C, R, S)).astype(np.float32)
    for out_layout in (cd.PLAIN, cd.BLOCKED):
        plan = cd.Plan(*shape, out_layout=out_layout)
        assert plan.info()["variant"].startswith("generic")
        P, Q = plan.output_dims()
        b = rng.integers(-9, 10, (K,)).astype(np.float32)
        r = rng.integers(-9, 10, (N, K, P, Q)).astype(np.float32)
        blocked = out_layout == cd.BLOCKED
        out = torch.full((N, 1, P, Q, 4) if blocked else (N, K, P, Q), float("nan"), device="cuda")
        rd = torch.from_numpy(L.pack_activations(r, 4) if blocked else r).cuda()
        plan.run(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), out, bias=torch.from_numpy(b).cuda(),
                 residual=rd, relu=True)
        torch.cuda.synchronize()
        plan.destroy()
        got = out.cpu().numpy()
        if blocked:
            assert np.all(got[:, -1, :, :, K % 4:] == 0)
            got = L.unpack_activations(got, K)
        assert np.array_equal(got.astype(np.float64), oracle.conv_forward_fused(x, w, st, pd, b, r, True))
