"""GPU parity of the two special forms of the pointwise (1x1) family: the input-stationary walk over all
output channels (variants ..._kall) and the tiles with a shared last block (variants p1s1/b1s1 ..._sl)."""
import re

import numpy as np
import pytest
import torch

from oracle import layout_ref as L
from paper_1809_10170_amd import conv_direct as cd

pytestmark = pytest.mark.gpu

WALK = [n for n in cd.variant_names() if "_kall" in n]
SHARED = [n for n in cd.variant_names() if re.match(r"[pb]1s1_.*_sl\d", n)]


def test_the_forms_exist():
    assert WALK and SHARED


def _run(plan, x, w, K, blocked, bias=None, residual=None, relu=False, in_blocked=False):
    N, _, H, W = x.shape
    out = torch.full((N, -(-K // 4), H, W, 4) if blocked else (N, K, H, W), float("nan"), device="cuda")
    rd = None
    if residual is not None:
        rd = torch.from_numpy(L.pack_activations(residual, 4) if blocked else residual).cuda()
    if in_blocked:
        x, w = L.pack_activations(x, 4), L.pack_weights(w, 4, 32)
    plan.run(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), out,
             bias=torch.from_numpy(bias).cuda() if bias is not None else None, residual=rd, relu=relu)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert not np.isnan(got).any()
    return L.unpack_activations(got, K) if blocked else got


# N, H, W, K: the last tile partly filled and tiles that straddle images; one lane group in all; a map smaller
# than a wave's share; many channel blocks (each wave takes the shared block several times)
WALK_SHAPES = [(3, 20, 22, 96), (1, 2, 2, 32), (5, 6, 6, 256), (2, 40, 42, 416), (7, 14, 14, 64)]


@pytest.mark.parametrize("name", WALK)
@pytest.mark.parametrize("shape", WALK_SHAPES)
@pytest.mark.parametrize("out_layout", [cd.PLAIN, cd.BLOCKED])
@pytest.mark.parametrize("tail", [False, True])
def test_walk_over_all_output_channels_bit_exact_on_integers(oracle, name, shape, out_layout, tail):
    N, H, W, K = shape
    C = int(re.search(r"_c(\d+)_kall", name).group(1))
    rng = np.random.default_rng(4100 + sum(shape) + 3 * out_layout + tail)
    x = rng.integers(-4, 5, (N, C, H, W)).astype(np.float32)
    w = rng.integers(-4, 5, (K, C, 1, 1)).astype(np.float32)
    b = rng.integers(-50, 51, (K,)).astype(np.float32) if tail else None
    r = rng.integers(-50, 51, (N, K, H, W)).astype(np.float32) if tail else None
    assert C * 16 + 100 < 2 ** 24
    inb = name.startswith("b")          # the variant for blocked input and weights
    plan = cd.Plan(N, C, H, W, K, 1, 1, 1, 0, variant=name, in_layout=cd.BLOCKED if inb else cd.PLAIN, out_layout=out_layout)
    info = plan.info()
    assert info["variant"] == name and info["ktiles"] == 1 and info["tail_variant"] == "same"
    got = _run(plan, x, w, K, out_layout == cd.BLOCKED, b, r, tail, in_blocked=inb)
    plan.destroy()
    want = oracle.conv_forward_fused(x, w, 1, 0, bias=b, residual=r, relu=tail) if tail else oracle.conv_forward(x, w, 1, 0)
    assert np.array_equal(got.astype(np.float64), want)


@pytest.mark.parametrize("name", WALK)
def test_walk_random_inputs_within_tolerance(oracle, name):
    C = int(re.search(r"_c(\d+)_kall", name).group(1))
    N, H, W, K = 4, 28, 28, 160
    rng = np.random.default_rng(4200)
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    w = rng.uniform(-1, 1, (K, C, 1, 1)).astype(np.float32)
    inb = name.startswith("b")
    plan = cd.Plan(N, C, H, W, K, 1, 1, 1, 0, variant=name, in_layout=cd.BLOCKED if inb else cd.PLAIN)
    got = _run(plan, x, w, K, False, in_blocked=inb)
    plan.destroy()
    assert np.abs(got - oracle.conv_forward(x, w, 1, 0)).max() <= oracle.tolerance(C, 1, 1)


# N, C, H, W, K: ragged channels, tiles and last block; a map of exactly two tiles (the benchmark's case, scaled down in
# N); fewer pixels than one tile
SHARED_SHAPES = [(2, 37, 41, 43, 70), (2, 64, 56, 56, 64), (1, 8, 9, 9, 33), (3, 130, 30, 61, 96)]


@pytest.mark.parametrize("name", SHARED)
@pytest.mark.parametrize("shape", SHARED_SHAPES)
def test_shared_last_block_bit_exact_on_integers(oracle, name, shape):
    N, C, H, W, K = shape
    blocked = name.startswith("b")
    rng = np.random.default_rng(4300 + sum(shape))
    x = rng.integers(-4, 5, (N, C, H, W)).astype(np.float32)
    w = rng.integers(-4, 5, (K, C, 1, 1)).astype(np.float32)
    assert C * 16 < 2 ** 24
    lay = cd.BLOCKED if blocked else cd.PLAIN
    plan = cd.Plan(N, C, H, W, K, 1, 1, 1, 0, variant=name, in_layout=lay, out_layout=lay)
    assert plan.info()["variant"] == name
    out = torch.full((N, -(-K // 4), H, W, 4) if blocked else (N, K, H, W), float("nan"), device="cuda")
    xd = torch.from_numpy(L.pack_activations(x, 4) if blocked else x).cuda()
    wd = torch.from_numpy(L.pack_weights(w, 4, 32) if blocked else w).cuda()
    plan.run(xd, wd, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert not np.isnan(got).any()
    if blocked:
        got = L.unpack_activations(got, K)
    assert np.array_equal(got.astype(np.float64), oracle.conv_forward(x, w, 1, 0))

    # a call with a tail runs on the plan's second choice, same result as the definition
    tv = plan.info()["tail_variant"]
    assert tv != "same" and tv != name
    b = rng.integers(-50, 51, (K,)).astype(np.float32)
    r = rng.integers(-50, 51, (N, K, H, W)).astype(np.float32)
    out.fill_(float("nan"))
    rd = torch.from_numpy(L.pack_activations(r, 4) if blocked else r).cuda()
    plan.run(xd, wd, out, bias=torch.from_numpy(b).cuda(), residual=rd, relu=True)
    torch.cuda.synchronize()
    plan.destroy()
    got = out.cpu().numpy()
    assert not np.isnan(got).any()
    if blocked:
        got = L.unpack_activations(got, K)
    assert np.array_equal(got.astype(np.float64), oracle.conv_forward_fused(x, w, 1, 0, bias=b, residual=r, relu=True))


def test_benchmark_pointwise_layers_take_the_two_forms():
    p = cd.Plan(64, 64, 56, 56, 256, 1, 1, 1, 0)
    assert "_kall" in p.info()["variant"]
    p.destroy()
    p = cd.Plan(64, 256, 56, 56, 64, 1, 1, 1, 0)
    assert "_sl" in p.info()["variant"]
    p.destroy()
    p = cd.Plan(64, 64, 56, 56, 256, 1, 1, 1, 0, in_layout=cd.BLOCKED, out_layout=cd.BLOCKED)
    assert "_kall" in p.info()["variant"]
    p.destroy()
