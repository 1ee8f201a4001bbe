"""GPU parity of the weight gradient against the oracle's adjoint definition."""
import numpy as np
import pytest
import torch

from paper_1809_10170_amd import conv_direct as cd
from paper_1809_10170_amd import workloads

pytestmark = pytest.mark.gpu


def _wgrad(x, dy, R, S, st, pd, variant=None):
    N, C, H, W = x.shape
    K = dy.shape[1]
    plan = cd.Plan.wgrad(N, C, H, W, K, R, S, st, pd, variant=variant)
    assert plan.workspace_bytes() == 0
    dw = torch.full((K, C, R, S), float("nan"), device="cuda")
    plan.run_wgrad(torch.from_numpy(x).cuda(), torch.from_numpy(dy).cuda(), dw)
    torch.cuda.synchronize()
    info = plan.info()
    plan.destroy()
    return dw.cpu().numpy(), info


SMALL = [
    # N, C, H, W, K, R, S, stride, pad
    (2, 7, 30, 61, 70, 3, 3, 1, 1),        # ragged C and K, rows longer than a chunk
    (5, 40, 13, 13, 130, 3, 3, 1, 1),      # several images per workgroup, three channel groups
    (2, 3, 33, 47, 35, 3, 3, 1, 0),
    (1, 9, 40, 40, 33, 5, 5, 1, 2),
    (2, 37, 19, 23, 65, 1, 1, 1, 0),
    (2, 12, 57, 55, 130, 3, 3, 2, 1),
    (2, 3, 75, 230, 64, 7, 7, 2, 3),
    (2, 3, 99, 227, 96, 11, 11, 4, 0),
    (1, 4, 12, 12, 8, 3, 3, 1, 2),         # pad larger than usual: whole filter rows without an input row
    (3, 5, 20, 70, 6, 5, 3, 1, 1),         # R != S
    (3, 20, 14, 14, 40, 3, 3, 1, 1),       # small maps: chunks of whole rows (14, 28, 7, 27 wide; 13 above)
    (2, 9, 30, 28, 33, 3, 3, 1, 1),
    (5, 33, 7, 7, 70, 3, 3, 1, 1),
    (2, 10, 27, 27, 40, 5, 5, 1, 2),
    (2, 8, 22, 13, 16, 3, 3, 1, 1),        # 22 rows of 13: a ragged last group of rows
]


@pytest.mark.parametrize("shape", SMALL)
def test_small_shapes_integer_inputs_bit_exact(oracle, shape):
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(800 + sum(shape))
    x = rng.integers(-2, 3, (N, C, H, W)).astype(np.float32)
    P, Q = oracle.out_dim(H, R, st, pd), oracle.out_dim(W, S, st, pd)
    dy = rng.integers(-2, 3, (N, K, P, Q)).astype(np.float32)
    assert N * P * Q * 4 < 2 ** 24          # every partial sum exact in fp32, whatever the order
    got, info = _wgrad(x, dy, R, S, st, pd)
    assert not np.isnan(got).any()
    assert np.array_equal(got.astype(np.float64), oracle.conv_wgrad(x, dy, R, S, st, pd)), info["variant"]


@pytest.mark.parametrize("shape", SMALL[:6])
def test_small_shapes_random_inputs(oracle, shape):
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(900 + sum(shape))
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    P, Q = oracle.out_dim(H, R, st, pd), oracle.out_dim(W, S, st, pd)
    dy = rng.uniform(-1, 1, (N, K, P, Q)).astype(np.float32)
    got, info = _wgrad(x, dy, R, S, st, pd)
    # the reduction runs over N*P*Q products of magnitude <= 1: the forward bar with that length
    tol = 1e-4 * np.sqrt(N * P * Q)
    err = np.abs(got.astype(np.float64) - oracle.conv_wgrad(x, dy, R, S, st, pd)).max()
    assert err <= tol, (info["variant"], err)


ALL_ROWS_CASES = [
    ((2, 40, 20, 64, 48, 3, 3, 1, 1), "w3s1_ar_c64_k64_p32"),       # waves spread over two channel groups
    ((2, 20, 9, 56, 70, 3, 3, 1, 1), "w3s1_ar_c32_k128_p28"),       # rows of two 28-pixel chunks
    ((2, 70, 11, 64, 130, 3, 3, 1, 1), "w3s1_ar_c32_k128_p32"),     # three channel groups, two k tiles
    ((2, 64, 9, 56, 128, 3, 3, 1, 1), "w3s1_ar_c64_k128_p28"),       # eight waves: four k-blocks x two channel groups
    ((1, 128, 6, 64, 100, 3, 3, 1, 1), "w3s1_ar_c64_k128_p32"),
    ((1, 12, 21, 127, 40, 3, 3, 2, 1), "w3s2_ar_c32_k128_p32"),     # stride 2, rows of 64
    ((2, 12, 57, 55, 130, 3, 3, 2, 1), "w3s2_ar_c32_k128_p28"),     # stride 2, rows of 28
    ((3, 9, 4, 7, 33, 3, 3, 1, 1), "w3s1_ar_c32_k128_q7h"),         # 4 rows of 7 per chunk
    ((5, 33, 7, 7, 70, 3, 3, 1, 1), "w3s1_ar_c32_k128_q7"),         # whole 7x7 maps per chunk
    ((3, 20, 14, 14, 40, 3, 3, 1, 1), "w3s1_ar_c32_k128_q14h"),
    ((2, 8, 22, 13, 16, 3, 3, 1, 1), "w3s1_ar_c32_k128_q13h"),
    ((2, 2, 20, 40, 20, 3, 3, 1, 1), "w3s1_arpack1_k128_p32"),      # packed columns: 18 of 32
    ((2, 100, 9, 56, 40, 1, 1, 1, 0), "w1s1_ar_c128_k64_p28"),       # 1x1: two channel groups of 64
    ((2, 100, 9, 64, 40, 1, 1, 1, 0), "w1s1_ar_c128_k64_p32"),
    ((2, 37, 10, 64, 130, 1, 1, 1, 0), "w1s1_ar_c64_k128_p32"),
    ((2, 37, 19, 23, 65, 1, 1, 1, 0), "w1s1_ar_c64_k128_p28"),
    ((1, 40, 9, 64, 70, 5, 5, 1, 2), "w5s1_ar_c32_k64_p32"),        # 25 column blocks dealt out to four waves per k-block
    ((2, 10, 27, 27, 40, 5, 5, 1, 2), "w5s1_ar_c32_k64_p28"),
    ((2, 40, 30, 127, 70, 5, 5, 2, 2), "w5s2_ar_c32_k64_p32"),
    ((2, 40, 30, 55, 70, 5, 5, 2, 2), "w5s2_ar_c32_k64_p28"),
    ((2, 40, 30, 64, 70, 4, 4, 1, 1), "w4s1_ar_c32_k128_p32"),      # 4x4: 16 column blocks, two waves per k-block
    ((2, 40, 20, 53, 70, 4, 4, 1, 1), "w4s1_ar_c32_k128_p28"),
    ((2, 40, 41, 128, 70, 4, 4, 2, 1), "w4s2_ar_c32_k128_p32"),
    ((2, 40, 30, 56, 70, 4, 4, 2, 1), "w4s2_ar_c32_k128_p28"),
    ((2, 1, 30, 30, 10, 7, 7, 2, 3), "w7s2_arpack5_k64_p56"),       # one channel
    ((2, 3, 75, 230, 64, 7, 7, 2, 3), "w7s2_arpack5_k64_p64"),
    ((2, 3, 99, 227, 96, 11, 11, 4, 0), "w11s4_arpack12_k128_p28"),
    ((1, 3, 51, 135, 40, 11, 11, 4, 0), "w11s4_arpack12_k128_p32"),
    ((2, 3, 75, 230, 64, 7, 7, 2, 3), "w7s2_arpack5_k64_p56b2"),     # packed columns dealt out to two waves per k-block
    ((2, 2, 61, 120, 70, 7, 7, 2, 3), "w7s2_arpack5_k64_p28b2"),
    ((2, 3, 99, 227, 96, 11, 11, 4, 0), "w11s4_arpack12_k96_p28b2"),  # three k-blocks per workgroup
    ((2, 3, 67, 227, 100, 11, 11, 4, 0), "w11s4_arpack12_k96_p28b2"),
    ((1, 3, 99, 227, 130, 11, 11, 4, 0), "w11s4_arpack12_k128_p28b2"),
    ((2, 40, 20, 56, 48, 3, 3, 1, 1), "w3s1_ar_c64_k64_p28"),
]

def test_every_all_rows_variant_has_a_case():
    names = {n for n in cd.wgrad_variant_names() if "_ar" in n}
    assert names and names <= {v for _, v in ALL_ROWS_CASES}, names - {v for _, v in ALL_ROWS_CASES}


@pytest.mark.parametrize("shape,variant", ALL_ROWS_CASES)
def test_all_rows_variants_integer_inputs_bit_exact(oracle, shape, variant):
    """Every variant whose waves own all filter rows (columns = consecutive floats of dw), forced, on a
    shape with ragged edges in the dimensions the variant tiles."""
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(1000 + sum(shape))
    x = rng.integers(-2, 3, (N, C, H, W)).astype(np.float32)
    P, Q = oracle.out_dim(H, R, st, pd), oracle.out_dim(W, S, st, pd)
    dy = rng.integers(-2, 3, (N, K, P, Q)).astype(np.float32)
    got, info = _wgrad(x, dy, R, S, st, pd, variant=variant)
    assert info["variant"] == variant
    assert np.array_equal(got.astype(np.float64), oracle.conv_wgrad(x, dy, R, S, st, pd))


def test_non_finite_lds_leftovers_do_not_leak():
    """A chunk with an odd number of pixels reads one input position past its rows, times a zero of dy:
    run a kernel that leaves NaNs in LDS first, then a 7x7 map (49 pixels per chunk)."""
    N, C, H, W, K = 2, 32, 7, 7, 32
    bad = torch.full((N, C, H, W), float("nan"), device="cuda")
    dyb = torch.ones((N, K, H, W), device="cuda")
    dwb = torch.empty((K, C, 3, 3), device="cuda")
    plan = cd.Plan.wgrad(N, C, H, W, K, 3, 3, 1, 1)
    for _ in range(3):
        plan.run_wgrad(bad, dyb, dwb)      # fills the LDS of many CUs with NaNs
    x = torch.ones((N, C, H, W), device="cuda")
    dw = torch.empty((K, C, 3, 3), device="cuda")
    plan.run_wgrad(x, dyb, dw)
    torch.cuda.synchronize()
    plan.destroy()
    assert torch.isfinite(dw).all()
    assert float(dw[0, 0, 1, 1]) == N * H * W


def test_unsupported_stride_is_refused():
    with pytest.raises(cd.ConvDirectError) as e:
        cd.Plan.wgrad(2, 8, 40, 40, 8, 3, 3, 5, 1)
    assert e.value.code == cd.EUNSUPPORTED


@pytest.mark.parametrize("shape", [(2, 9, 21, 30, 40, 3, 4, 1, 1), (2, 70, 17, 19, 33, 2, 2, 2, 0), (1, 5, 30, 41, 8, 4, 6, 3, 2),
                                   (2, 6, 33, 37, 9, 3, 3, 4, 1)])
def test_fallback_for_other_filter_widths_and_strides(oracle, shape):
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(950 + sum(shape))
    x = rng.integers(-2, 3, (N, C, H, W)).astype(np.float32)
    dy = rng.integers(-2, 3, (N, K, oracle.out_dim(H, R, st, pd), oracle.out_dim(W, S, st, pd))).astype(np.float32)
    got, info = _wgrad(x, dy, R, S, st, pd)
    assert info["variant"].startswith("w_any")
    assert np.array_equal(got.astype(np.float64), oracle.conv_wgrad(x, dy, R, S, st, pd))


def test_wgrad_plan_is_not_a_forward_plan():
    plan = cd.Plan.wgrad(2, 8, 20, 20, 8, 3, 3, 1, 1)
    x = torch.zeros((2, 8, 20, 20), device="cuda")
    w = torch.zeros((8, 8, 3, 3), device="cuda")
    out = torch.zeros((2, 8, 20, 20), device="cuda")
    assert cd.lib().conv_direct_run(plan._p, x.data_ptr(), w.data_ptr(), out.data_ptr(), None) == cd.EINVAL
    plan.destroy()


@pytest.mark.parametrize("name", [l.name for l in workloads.ALL_LAYERS if l.N >= 32])
def test_benchmark_layers_full_size_sampled(oracle, name):
    """Full-size layers: a sample of dw's output channels in full against the oracle (its cost is that of
    the forward pass per output channel)."""
    l = workloads.BY_NAME[name]
    x, _ = workloads.make_inputs(l)
    rng = np.random.default_rng(13)
    dy = rng.uniform(-1, 1, (l.N, l.K, l.P, l.Q)).astype(np.float32)
    got, info = _wgrad(x, dy, l.R, l.S, l.stride, l.pad)
    assert not np.isnan(got).any()
    ks = sorted({0, l.K - 1, int(rng.integers(0, l.K))})
    want = oracle.conv_wgrad(x, np.ascontiguousarray(dy[:, ks]), l.R, l.S, l.stride, l.pad)
    tol = 1e-4 * np.sqrt(l.N * l.P * l.Q)
    err = np.abs(got[ks].astype(np.float64) - want).max()
    assert err <= tol, (info["variant"], err)


@pytest.mark.parametrize("shape", [(3, 40, 20, 56, 70, 3, 3, 1, 1), (4, 33, 13, 13, 40, 3, 3, 1, 1), (2, 3, 75, 230, 64, 7, 7, 2, 3),
                                   (3, 5, 20, 70, 6, 5, 3, 1, 1)])
def test_deterministic_plan_same_bits_every_run(oracle, shape):
    """One workgroup per tile of dw: plain stores into a buffer that was not cleared, and the same bits on every run
    (random inputs, whose sums do depend on the order of the additions)."""
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(1300 + sum(shape))
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    P, Q = oracle.out_dim(H, R, st, pd), oracle.out_dim(W, S, st, pd)
    dy = rng.uniform(-1, 1, (N, K, P, Q)).astype(np.float32)
    plan = cd.Plan.wgrad(*shape, deterministic=True)
    assert plan.info()["splits"] == 1
    xd, dyd = torch.from_numpy(x).cuda(), torch.from_numpy(dy).cuda()
    runs = []
    for fill in (float("nan"), 7.0, -1e30):
        dw = torch.full((K, C, R, S), fill, device="cuda")
        plan.run_wgrad(xd, dyd, dw)
        torch.cuda.synchronize()
        runs.append(dw.cpu().numpy())
    plan.destroy()
    assert np.array_equal(runs[0], runs[1]) and np.array_equal(runs[0], runs[2])
    err = np.abs(runs[0].astype(np.float64) - oracle.conv_wgrad(x, dy, R, S, st, pd)).max()
    assert err <= 1e-4 * np.sqrt(N * P * Q), err


# ---- blocked layouts (x [N][C/4][H][W][4], dy [N][K/4][P][Q][4], dw [K/32][C/4][R][S][4][32]) ----
FALLBACK_SHAPES = [(2, 9, 21, 30, 40, 3, 4, 1, 1), (2, 70, 17, 19, 33, 2, 2, 2, 0), (1, 5, 30, 41, 8, 4, 6, 3, 2), (2, 6, 33, 37, 9, 3, 3, 4, 1)]
BLOCKED_SHAPES = sorted(set(SMALL) | {s for s, _ in ALL_ROWS_CASES} | set(FALLBACK_SHAPES))
B, PL = cd.BLOCKED, cd.PLAIN


def _spare_nan(a, channels):
    """The spare channels that complete the last pencil of a blocked activation tensor, set to NaN."""
    a = a.copy()
    if channels % 4:
        a[:, -1, :, :, channels % 4:] = np.nan
    return a


@pytest.mark.parametrize("shape", BLOCKED_SHAPES)
def test_blocked_layouts_every_variant_that_serves_the_shape(oracle, shape):
    """Integer inputs, bit-exact against the layout oracle, for the planner's choice in several layout mixes (also the
    one-workgroup-per-tile plan) and for EVERY compiled variant that accepts the shape, all tensors blocked.  The spare
    channels of x's and dy's last pencils hold NaN: they may only meet results that are dropped; those of dw must
    come back as zeros."""
    from oracle import layout_ref as L
    N, C, H, W, K, R, S, st, pd = shape
    rng = np.random.default_rng(1400 + sum(shape))
    x = rng.integers(-2, 3, (N, C, H, W)).astype(np.float32)
    P, Q = oracle.out_dim(H, R, st, pd), oracle.out_dim(W, S, st, pd)
    dy = rng.integers(-2, 3, (N, K, P, Q)).astype(np.float32)
    want = oracle.conv_wgrad(x, dy, R, S, st, pd)
    xb, dyb = L.pack_activations(x, 4), L.pack_activations(dy, 4)
    wantb = L.conv_wgrad_blocked(xb, dyb, C, K, R, S, st, pd, cb=4, kb=32)
    assert np.array_equal(wantb, L.pack_weights(want, 4, 32))
    dev = {PL: (torch.from_numpy(x).cuda(), torch.from_numpy(dy).cuda()),
           B: (torch.from_numpy(_spare_nan(xb, C)).cuda(), torch.from_numpy(_spare_nan(dyb, K)).cuda())}
    cases = [(None, False, lay) for lay in ((B, B, B), (B, B, PL), (PL, B, B), (B, PL, PL), (PL, PL, B))]
    cases += [(None, True, (B, B, B))] + [(v, False, (B, B, B)) for v in cd.wgrad_variant_names()]
    ran = 0
    for variant, det, (xl, yl, wl) in cases:
        try:
            plan = cd.Plan.wgrad(*shape, variant=variant, deterministic=det, x_layout=xl, dy_layout=yl, dw_layout=wl)
        except cd.ConvDirectError as e:
            assert variant is not None and e.code == cd.EUNSUPPORTED, (variant, e.code)
            continue
        info = plan.info()
        assert (info["x_layout"], info["dy_layout"], info["dw_layout"]) == tuple("blocked" if v == B else "plain" for v in (xl, yl, wl))
        dw = torch.full(wantb.shape if wl == B else want.shape, float("nan"), device="cuda")
        plan.run_wgrad(dev[xl][0], dev[yl][1], dw)
        torch.cuda.synchronize()
        plan.destroy()
        assert np.array_equal(dw.cpu().numpy().astype(np.float64), wantb if wl == B else want), (info["variant"], det, xl, yl, wl)
        ran += 1
    assert ran >= 7


@pytest.mark.parametrize("name", [l.name for l in workloads.ALL_LAYERS if l.N >= 32])
def test_blocked_layouts_benchmark_layers_full_size_sampled(oracle, name):
    """Full-size layers with dy and dw blocked, x blocked unless it is a first layer's image (3 channels, kept
    plain as the forward pass keeps it): a sample of dw's output channels in full against the oracle."""
    from oracle import layout_ref as L
    l = workloads.BY_NAME[name]
    x, _ = workloads.make_inputs(l)
    rng = np.random.default_rng(14)
    dy = rng.uniform(-1, 1, (l.N, l.K, l.P, l.Q)).astype(np.float32)
    xl = PL if l.C < 4 else B
    plan = cd.Plan.wgrad(*l.dims(), x_layout=xl, dy_layout=B, dw_layout=B)
    xd = torch.from_numpy(x).cuda()
    if xl == B:
        xp = torch.empty((l.N, -(-l.C // 4), l.H, l.W, 4), device="cuda")
        cd.pack_act(xd, xp)
        xd = xp
    dyb = torch.empty((l.N, -(-l.K // 4), l.P, l.Q, 4), device="cuda")
    cd.pack_act(torch.from_numpy(dy).cuda(), dyb)
    dwb = torch.full((-(-l.K // 32), -(-l.C // 4), l.R, l.S, 4, 32), float("nan"), device="cuda")
    plan.run_wgrad(xd, dyb, dwb)
    torch.cuda.synchronize()
    info = plan.info()
    plan.destroy()
    got = L.unpack_weights(dwb.cpu().numpy(), l.K, l.C)
    assert not np.isnan(got).any()
    ks = sorted({0, l.K - 1, int(rng.integers(0, l.K))})
    want = oracle.conv_wgrad(x, np.ascontiguousarray(dy[:, ks]), l.R, l.S, l.stride, l.pad)
    err = np.abs(got[ks].astype(np.float64) - want).max()
    assert err <= 1e-4 * np.sqrt(l.N * l.P * l.Q), (info["variant"], err)
