"""The measured choice of a variant (conv_direct_create_tuned) on the GPU: it returns a
working plan of a variant that serves the shape, remembers it, and the result is right."""
import numpy as np
import pytest
import torch

from paper_1809_10170_amd import conv_direct as cd

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape,layouts", [
    ((4, 32, 28, 28, 96, 3, 3, 1, 1), (cd.PLAIN, cd.PLAIN)),
    ((4, 32, 28, 28, 96, 3, 3, 1, 1), (cd.BLOCKED, cd.BLOCKED)),
    ((2, 3, 64, 64, 32, 7, 7, 2, 3), (cd.PLAIN, cd.BLOCKED)),
    # pointwise layers: among the candidates are the tiles with a shared last block (no fused tail: the plan for them
    # comes with a second choice) and the walk over all output channels
    ((8, 256, 56, 56, 64, 1, 1, 1, 0), (cd.PLAIN, cd.PLAIN)),
    ((8, 64, 56, 56, 96, 1, 1, 1, 0), (cd.PLAIN, cd.PLAIN)),
])
def test_tuned_plan_is_correct_and_remembered(oracle, shape, layouts):
    from oracle import layout_ref as L
    N, C, H, W, K, R, S, st, pd = shape
    li, lo = layouts
    cd.tuning_clear()
    rng = np.random.default_rng(sum(shape))
    x = rng.integers(-4, 5, (N, C, H, W)).astype(np.float32)
    w = rng.integers(-4, 5, (K, C, R, S)).astype(np.float32)
    xd = torch.from_numpy(L.pack_activations(x, 4) if li == cd.BLOCKED else x).cuda()
    wd = torch.from_numpy(L.pack_weights(w, 4, 32) if li == cd.BLOCKED else w).cuda()
    P, Q = oracle.out_dim(H, R, st, pd), oracle.out_dim(W, S, st, pd)
    out = torch.full((N, -(-K // 4), P, Q, 4) if lo == cd.BLOCKED else (N, K, P, Q), float("nan"), device="cuda")
    plan = cd.Plan.tuned(xd, wd, out, *shape, in_layout=li, out_layout=lo, reps=3)
    name = plan.info()["variant"]
    assert name in cd.variant_names() and cd.tuning_size() == 1
    out.fill_(float("nan"))
    plan.run(xd, wd, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    if lo == cd.BLOCKED:
        got = L.unpack_activations(got, K)
    assert np.array_equal(got.astype(np.float64), oracle.conv_forward(x, w, st, pd)), name
    # later plans for the same problem take the measured choice; other problems are untouched
    again = cd.Plan(*shape, in_layout=li, out_layout=lo)
    assert again.info()["variant"] == name
    again.destroy()
    plan.destroy()
    cd.tuning_clear()
