"""GPU parity of the data gradient (stride 1) against the oracle's adjoint definition."""
import numpy as np
import pytest
import torch

from paper_1809_10170_amd import conv_direct as cd
from paper_1809_10170_amd import workloads

pytestmark = pytest.mark.gpu


def _dgrad(dy, w, H, W, pad):
    N, K, P, Q = dy.shape
    _, C, R, S = w.shape
    plan = cd.Plan.dgrad(N, C, H, W, K, R, S, 1, pad)
    assert plan.output_dims() == (H, W) and plan.workspace_bytes() == 0
    wd = torch.from_numpy(w).cuda()
    wt = torch.full((C, K, R, S), float("nan"), device="cuda")
    cd.dgrad_filter(wd, wt)
    dx = torch.full((N, C, H, W), float("nan"), device="cuda")
    plan.run(torch.from_numpy(dy).cuda(), wt, dx)
    torch.cuda.synchronize()
    info = plan.info()
    plan.destroy()
    return dx.cpu().numpy(), wt.cpu().numpy(), info


SMALL = [
    # N, C, H, W, K, R, S, pad
    (2, 7, 30, 61, 70, 3, 3, 1),
    (2, 3, 33, 47, 35, 3, 3, 0),
    (1, 9, 40, 40, 33, 5, 5, 2),
    (2, 37, 19, 23, 65, 1, 1, 0),
    (3, 16, 13, 13, 130, 3, 3, 1),
    (1, 5, 20, 22, 6, 4, 4, 3),
    (1, 4, 12, 12, 8, 3, 3, 2),
]


@pytest.mark.parametrize("shape", SMALL)
def test_small_shapes_integer_inputs_bit_exact(oracle, shape):
    N, C, H, W, K, R, S, pd = shape
    rng = np.random.default_rng(500 + sum(shape))
    w = rng.integers(-4, 5, (K, C, R, S)).astype(np.float32)
    P, Q = oracle.out_dim(H, R, 1, pd), oracle.out_dim(W, S, 1, pd)
    dy = rng.integers(-4, 5, (N, K, P, Q)).astype(np.float32)
    assert K * R * S * 16 < 2 ** 24
    got, wt, info = _dgrad(dy, w, H, W, pd)
    assert np.array_equal(wt, w[:, :, ::-1, ::-1].transpose(1, 0, 2, 3)), "dgrad_filter"
    assert np.array_equal(got.astype(np.float64), oracle.conv_dgrad(dy, w, H, W, 1, pd)), info["variant"]


@pytest.mark.parametrize("shape", SMALL)
def test_small_shapes_random_inputs(oracle, shape):
    N, C, H, W, K, R, S, pd = shape
    rng = np.random.default_rng(600 + sum(shape))
    w = rng.uniform(-1, 1, (K, C, R, S)).astype(np.float32)
    P, Q = oracle.out_dim(H, R, 1, pd), oracle.out_dim(W, S, 1, pd)
    dy = rng.uniform(-1, 1, (N, K, P, Q)).astype(np.float32)
    got, _, info = _dgrad(dy, w, H, W, pd)
    err = np.abs(got.astype(np.float64) - oracle.conv_dgrad(dy, w, H, W, 1, pd)).max()
    assert err <= oracle.tolerance(K, R, S), (info["variant"], err)   # the reduction runs over K*R*S


GENERAL = [
    # N, C, H, W, K, R, S, stride, pad: strided layers, unequal filter sides, pad > R-1
    (2, 8, 20, 20, 9, 3, 3, 2, 1),
    (2, 5, 23, 31, 7, 3, 5, 1, 1),
    (1, 6, 20, 22, 8, 3, 3, 1, 3),
    (2, 3, 75, 64, 10, 7, 7, 2, 3),
    (1, 3, 51, 47, 12, 11, 11, 4, 0),
    (2, 4, 17, 19, 5, 2, 4, 3, 2),
    (1, 7, 16, 16, 6, 1, 1, 2, 0),
    (2, 40, 29, 29, 70, 3, 3, 2, 1),       # phases: ragged channel chunks, several tiles per image
    (3, 16, 56, 56, 33, 3, 3, 2, 1),       # dy 28x28: the flat tiling, tiles across images
    (2, 9, 30, 33, 12, 4, 4, 2, 1),        # 4x4 stride 2: every phase has all four taps
    (2, 20, 31, 29, 33, 8, 8, 2, 3),       # 8x8 stride 2: 4x4 taps per phase
    (3, 24, 26, 30, 40, 4, 4, 1, 2),       # 4x4 stride 1 (one convolution; the 4x4 variant, or the fallback for so small a problem)
    (2, 6, 21, 20, 8, 3, 3, 2, 0),         # trailing input rows that no window of the forward pass reaches
    (1, 5, 25, 26, 7, 5, 5, 3, 2),         # stride 3: nine phases of 2x2 taps
    (2, 5, 40, 40, 9, 3, 3, 3, 1),         # R = stride: one tap per phase
    (16, 64, 28, 28, 70, 3, 3, 2, 1),      # dy 14x14: the split flat tiling for 15x15 phase results
    (16, 64, 14, 14, 70, 3, 3, 2, 1),      # dy 7x7
]


@pytest.mark.parametrize("shape", GENERAL)
def test_general_cases_strided_unequal_sides_large_pads(oracle, shape):
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(650 + sum(shape))
    w = rng.integers(-4, 5, (K, C, R, S)).astype(np.float32)
    P, Q = oracle.out_dim(H, R, st, pd), oracle.out_dim(W, S, st, pd)
    dy = rng.integers(-4, 5, (N, K, P, Q)).astype(np.float32)
    plan = cd.Plan.dgrad(*shape)
    info = plan.info()
    # strided layers with a square filter run as stride^2 small stride-1 convolutions (one per phase of the
    # input positions) on the compiled kernels; the rest on the runtime-shape kernel
    phases = st > 1 and R == S
    assert plan.output_dims() == (H, W)
    if phases:
        assert info["dgrad_phases"] == min(st, R) ** 2 and not info["variant"].startswith("generic")   # (phases a >= R have no tap)
    else:
        assert info["dgrad_phases"] == 0
    wt = torch.full((plan.dgrad_wt_elems(),), float("nan"), device="cuda")
    plan.dgrad_prepare(torch.from_numpy(w).cuda(), wt)
    dx = torch.full((N, C, H, W), float("nan"), device="cuda")
    assert cd.lib().conv_direct_run(plan._p, torch.from_numpy(dy).cuda().data_ptr(), wt.data_ptr(), dx.data_ptr(), None) == cd.OK
    torch.cuda.synchronize()
    plan.destroy()
    assert np.array_equal(dx.cpu().numpy().astype(np.float64), oracle.conv_dgrad(dy, w, H, W, st, pd))


@pytest.mark.parametrize("name", [l.name for l in workloads.ALL_LAYERS if l.N >= 32 and l.stride == 1 and l.C >= 16])
def test_benchmark_layers_full_size_sampled(oracle, name):
    """Full-size layers: 10^5 sampled dx elements and three whole images against the oracle.  The sample is
    computed through the flipped-filter identity (pinned on the CPU against the adjoint definition), which
    lets the oracle evaluate single elements; the whole images through the adjoint definition itself."""
    l = workloads.BY_NAME[name]
    _, w = workloads.make_inputs(l)
    rng = np.random.default_rng(11)
    dy = rng.uniform(-1, 1, (l.N, l.K, l.P, l.Q)).astype(np.float32)
    got, _, info = _dgrad(dy, w, l.H, l.W, l.pad)
    assert not np.isnan(got).any()
    pts = np.stack([rng.integers(0, d, 100000) for d in (l.N, l.C, l.H, l.W)], axis=1).astype(np.int32)
    wt = np.ascontiguousarray(w[:, :, ::-1, ::-1].transpose(1, 0, 2, 3))
    want = oracle.conv_forward_points(dy, wt, pts, 1, l.R - 1 - l.pad)
    err = np.abs(got[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]].astype(np.float64) - want).max()
    assert err <= oracle.tolerance(l.K, l.R, l.S), (info["variant"], err)
    for n in sorted({0, l.N // 2, l.N - 1}):   # three whole images against the adjoint definition itself
        want = oracle.conv_dgrad(np.ascontiguousarray(dy[n:n + 1]), w, l.H, l.W, 1, l.pad)
        err = np.abs(got[n:n + 1].astype(np.float64) - want).max()
        assert err <= oracle.tolerance(l.K, l.R, l.S), (info["variant"], n, err)


def test_strided_benchmark_layer_full_size_whole_images(oracle):
    """The 3x3 stride-2 layer of the suite at full size (four 2x2 phase convolutions, merged into the waves of one
    workgroup per tile, on the flat tiling):
    three whole images of dx against the oracle's adjoint (images are independent)."""
    l = workloads.BY_NAME["s2_c128_56_k256_3x3_n64"]
    _, w = workloads.make_inputs(l)
    rng = np.random.default_rng(12)
    dy = rng.uniform(-1, 1, (l.N, l.K, l.P, l.Q)).astype(np.float32)
    plan = cd.Plan.dgrad(*l.dims())
    info = plan.info()
    assert info["dgrad_phases"] == 4 and info["variant"].startswith("d2s1_flat28_k64m") and plan.workspace_bytes() == 0
    wt = torch.empty((plan.dgrad_wt_elems(),), device="cuda")
    plan.dgrad_prepare(torch.from_numpy(w).cuda(), wt)
    dx = torch.full((l.N, l.C, l.H, l.W), float("nan"), device="cuda")
    plan.run(torch.from_numpy(dy).cuda(), wt, dx)
    torch.cuda.synchronize()
    plan.destroy()
    assert torch.isfinite(dx).all()
    for n in (0, l.N // 2, l.N - 1):
        want = oracle.conv_dgrad(np.ascontiguousarray(dy[n:n + 1]), w, l.H, l.W, l.stride, l.pad)
        err = np.abs(dx[n:n + 1].cpu().numpy().astype(np.float64) - want).max()
        assert err <= oracle.tolerance(l.K, l.R, l.S), err


# ---- blocked layouts (dy [N][K/4][P][Q][4], dx [N][C/4][H][W][4]; the weights stay plain) ----
BLOCKED_CASES = [s[:7] + (1, s[7]) for s in SMALL] + GENERAL


@pytest.mark.parametrize("layouts", [(cd.BLOCKED, cd.BLOCKED), (cd.BLOCKED, cd.PLAIN), (cd.PLAIN, cd.BLOCKED)],
                         ids=["blocked-blocked", "blocked-plain", "plain-blocked"])
@pytest.mark.parametrize("shape", BLOCKED_CASES)
def test_blocked_layouts_integer_inputs_bit_exact(oracle, shape, layouts):
    """Every case of the plain-layout tests with dy and/or dx in the blocked activation layout, against the
    layout oracle (unpack, adjoint definition, pack); the spare channels of dx's last pencil must be zeros."""
    from oracle import layout_ref as L
    N, C, H, W, K, R, S, st, pd = shape
    dyl, dxl = layouts
    rng = np.random.default_rng(660 + sum(shape))
    w = rng.integers(-4, 5, (K, C, R, S)).astype(np.float32)
    P, Q = oracle.out_dim(H, R, st, pd), oracle.out_dim(W, S, st, pd)
    dy = rng.integers(-4, 5, (N, K, P, Q)).astype(np.float32)
    assert K * R * S * 16 < 2 ** 24
    plan = cd.Plan.dgrad(*shape, dy_layout=dyl, dx_layout=dxl)
    info = plan.info()
    assert plan.output_dims() == (H, W) and plan.workspace_bytes() == 0
    assert info["in_layout"] == ("blocked" if dyl == cd.BLOCKED else "plain")
    assert info["out_layout"] == ("blocked" if dxl == cd.BLOCKED else "plain")
    dy_in = L.pack_activations(dy, 4) if dyl == cd.BLOCKED else dy
    wt = torch.full((plan.dgrad_wt_elems(),), float("nan"), device="cuda")
    plan.dgrad_prepare(torch.from_numpy(w).cuda(), wt)
    dx = torch.full((N, -(-C // 4), H, W, 4) if dxl == cd.BLOCKED else (N, C, H, W), float("nan"), device="cuda")
    plan.run(torch.from_numpy(dy_in).cuda(), wt, dx)
    torch.cuda.synchronize()
    plan.destroy()
    want = oracle.conv_dgrad(dy, w, H, W, st, pd)
    if dxl == cd.BLOCKED:
        want = L.pack_activations(want, 4)
        assert np.array_equal(want, L.conv_dgrad_blocked(L.pack_activations(dy, 4), w, H, W, st, pd))
    assert np.array_equal(dx.cpu().numpy().astype(np.float64), want), info["variant"]


def test_blocked_layouts_strided_benchmark_layer_full_size(oracle):
    """The suite's 3x3 stride-2 layer in the blocked layouts at full size: the phases run on a compiled blocked
    variant; three whole images against the oracle."""
    from oracle import layout_ref as L
    l = workloads.BY_NAME["s2_c128_56_k256_3x3_n64"]
    _, w = workloads.make_inputs(l)
    rng = np.random.default_rng(13)
    dy = rng.uniform(-1, 1, (l.N, l.K, l.P, l.Q)).astype(np.float32)
    plan = cd.Plan.dgrad(*l.dims(), dy_layout=cd.BLOCKED, dx_layout=cd.BLOCKED)
    info = plan.info()
    assert info["dgrad_phases"] == 4 and info["variant"].startswith("b2s1_flat28_k64m") and plan.workspace_bytes() == 0
    wt = torch.empty((plan.dgrad_wt_elems(),), device="cuda")
    plan.dgrad_prepare(torch.from_numpy(w).cuda(), wt)
    dyb = torch.empty((l.N, l.K // 4, l.P, l.Q, 4), device="cuda")
    cd.pack_act(torch.from_numpy(dy).cuda(), dyb)
    dxb = torch.full((l.N, l.C // 4, l.H, l.W, 4), float("nan"), device="cuda")
    plan.run(dyb, wt, dxb)
    torch.cuda.synchronize()
    plan.destroy()
    assert torch.isfinite(dxb).all()
    for n in (0, l.N // 2, l.N - 1):
        want = L.conv_dgrad_blocked(L.pack_activations(np.ascontiguousarray(dy[n:n + 1]), 4), w, l.H, l.W, l.stride, l.pad)
        err = np.abs(dxb[n:n + 1].cpu().numpy().astype(np.float64) - want).max()
        assert err <= oracle.tolerance(l.K, l.R, l.S), err


MERGED_CASES = [
    # all four phases of a stride-2 layer in one workgroup (eight waves = phase x two blocks of 32 channels), forced
    ((2, 40, 29, 29, 70, 3, 3, 2, 1), "d2s1_8x28_k64m"),        # second channel block with 8 channels, ragged chunks
    ((2, 9, 30, 33, 12, 4, 4, 2, 1), "d2s1_8x28_k64m"),         # 4x4: every phase has all four taps; no second block
    ((3, 100, 20, 24, 33, 3, 3, 2, 1), "d2s1_8x28_k64m"),       # two channel tiles, the second with one block and a bit
    ((2, 6, 21, 20, 8, 3, 3, 2, 0), "d2s1_8x28_k64m"),          # trailing rows no window reaches: dx is cleared first
    ((3, 16, 56, 56, 33, 3, 3, 2, 1), "d2s1_flat28_k64m_b7"),
    ((2, 70, 56, 56, 40, 4, 4, 2, 1), "d2s1_flat28_k64m_b7"),
    ((16, 64, 28, 28, 70, 3, 3, 2, 1), "d2s1_flat14_k64m_b7"),
    ((5, 130, 28, 28, 24, 3, 3, 2, 1), "d2s1_flat14_k64m_b7"),
    ((16, 64, 14, 14, 70, 3, 3, 2, 1), "d2s1_flat7_k64m_b4"),
    ((2, 40, 29, 29, 70, 3, 3, 2, 1), "b2s1_8x28_k64m"),        # blocked dy and dx (the padded taps are multiplied too)
    ((3, 100, 20, 24, 33, 4, 4, 2, 1), "b2s1_8x28_k64m"),
    ((3, 16, 56, 56, 33, 3, 3, 2, 1), "b2s1_flat28_k64m_b7"),
]


def test_every_merged_phase_variant_has_a_case():
    names = {n for n in cd.variant_names() if n.endswith("m") or "k64m_" in n}
    assert names and names == {v for _, v in MERGED_CASES}


@pytest.mark.parametrize("shape,variant", MERGED_CASES)
def test_merged_phase_variants_integer_inputs_bit_exact(oracle, shape, variant):
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(670 + sum(shape))
    w = rng.integers(-4, 5, (K, C, R, S)).astype(np.float32)
    P, Q = oracle.out_dim(H, R, st, pd), oracle.out_dim(W, S, st, pd)
    dy = rng.integers(-4, 5, (N, K, P, Q)).astype(np.float32)
    blocked = variant.startswith("b")
    lay = cd.BLOCKED if blocked else cd.PLAIN
    plan = cd.Plan.dgrad(*shape, variant=variant, dy_layout=lay, dx_layout=lay)
    info = plan.info()
    assert info["variant"] == variant and info["dgrad_phases"] == 4 and plan.output_dims() == (H, W)
    wt = torch.full((plan.dgrad_wt_elems(),), float("nan"), device="cuda")
    plan.dgrad_prepare(torch.from_numpy(w).cuda(), wt)
    want = oracle.conv_dgrad(dy, w, H, W, st, pd)
    if blocked:
        from oracle import layout_ref as L
        dy, want = L.pack_activations(dy, 4), L.pack_activations(want, 4)
    dx = torch.full(want.shape, float("nan"), device="cuda")
    plan.run(torch.from_numpy(dy).cuda(), wt, dx)
    torch.cuda.synchronize()
    plan.destroy()
    assert np.array_equal(dx.cpu().numpy().astype(np.float64), want)


def test_a_merged_phase_variant_serves_only_stride_two():
    with pytest.raises(cd.ConvDirectError) as e:
        cd.Plan.dgrad(1, 5, 25, 26, 7, 5, 5, 3, 2, variant="d2s1_8x28_k64m")     # stride 3: nine phases
    assert e.value.code == cd.EUNSUPPORTED
    with pytest.raises(cd.ConvDirectError) as e:
        cd.Plan(2, 16, 20, 20, 32, 2, 2, 1, 0, variant="d2s1_8x28_k64m")          # a forward layer
    assert e.value.code == cd.EUNSUPPORTED
