"""Host-side checks of the C ABI and the planner.  No GPU: nothing here launches a kernel.

The library must load, export every symbol the header declares, reject bad arguments
with the documented codes, and plan a tiling that covers every output exactly once.
"""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_1809_10170_amd import conv_direct as cd
from paper_1809_10170_amd import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    with open(os.path.join(ROOT, "include", "conv_direct.h")) as f:
        text = re.sub(r"/\*.*?\*/", "", f.read(), flags=re.S)
    names = set(re.findall(r"\b(conv_direct_[a-z_]+)\s*\(", text))
    assert {"conv_direct_create", "conv_direct_run", "conv_direct_destroy"} <= names
    raw = ctypes.CDLL(cd.LIB_PATH)
    for nm in sorted(names):
        assert hasattr(raw, nm), f"{nm} declared in the header but not exported"


def test_error_codes():
    L = cd.lib()
    p = ctypes.c_void_p()
    good = [1, 3, 8, 8, 4, 3, 3, 1, 1]
    for pos, bad in [(0, 0), (1, -1), (2, 0), (3, 0), (4, 0), (5, 0), (6, 0), (7, 0), (8, -1)]:
        args = list(good)
        args[pos] = bad
        assert L.conv_direct_create(ctypes.byref(p), *args) == cd.EINVAL
        assert not p.value
    # filter larger than the padded input
    assert L.conv_direct_create(ctypes.byref(p), 1, 1, 2, 2, 1, 3, 3, 1, 0) == cd.EINVAL
    assert L.conv_direct_create(ctypes.byref(p), 1, 1, 2, 2, 1, 3, 3, 1, 1) == cd.OK
    assert L.conv_direct_destroy(p) == cd.OK
    # NULL plan pointer
    assert L.conv_direct_create(None, *good) == cd.EINVAL
    # a tensor with 2^31 or more elements
    assert L.conv_direct_create(ctypes.byref(p), 4096, 1024, 32, 32, 8, 1, 1, 1, 0) == cd.EUNSUPPORTED
    assert L.conv_direct_destroy(None) == cd.OK
    assert L.conv_direct_create_with_variant(ctypes.byref(p), b"no_such_variant", *good) == cd.EUNSUPPORTED
    assert L.conv_direct_create_with_variant(ctypes.byref(p), None, *good) == cd.EINVAL
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert cd.strerror(code)
    assert L.conv_direct_last_hip_error() == 0


def test_run_rejects_null_and_misaligned_pointers_before_any_launch():
    plan = cd.Plan(1, 3, 8, 8, 4, 3, 3, 1, 1)
    L = cd.lib()
    assert L.conv_direct_run(plan._p, None, 4096, 8192, None) == cd.EINVAL
    assert L.conv_direct_run(plan._p, 4096, None, 8192, None) == cd.EINVAL
    assert L.conv_direct_run(plan._p, 4096, 8192, None, None) == cd.EINVAL
    assert L.conv_direct_run(None, 4096, 8192, 12288, None) == cd.EINVAL
    assert L.conv_direct_run(plan._p, 4097, 8192, 12288, None) == cd.EALIGN
    assert L.conv_direct_run(plan._p, 4096, 8194, 12288, None) == cd.EALIGN
    assert L.conv_direct_run(plan._p, 4096, 8192, 12291, None) == cd.EALIGN
    assert L.conv_direct_output_dims(None, None, None) == cd.EINVAL
    plan.destroy()
    plan.destroy()   # idempotent


def _check_cover(info, exhaustive):
    N, K, P, Q = info["N"], info["K"], info["P"], info["Q"]
    TP, TQ, KT = info["TP"], info["TQ"], info["KT"]
    tP, tQ, tK = info["tilesP"], info["tilesQ"], info["ktiles"]
    assert (tK - 1) * KT < K <= tK * KT
    if info["flat"]:
        # flat tiling: tQ tiles of NPB*32 consecutive pixels numbered over all images
        npix = info["NPB"] * 32
        assert info["grid"] == tQ * tK and tP == 1
        assert (tQ - 1) * npix < N * P * Q <= tQ * npix
    elif info["pointwise"]:
        # every image is one row of P*Q pixels, cut into tQ tiles of TQ
        assert info["grid"] == tQ * tK * N and tP == 1 and TP == 1
        assert info["NPB"] * 32 == TQ
        assert (tQ - 1) * TQ < P * Q <= tQ * TQ
    else:
        assert info["grid"] == tP * tQ * tK * N
        assert info["NPB"] * 32 >= TP * TQ
        assert (tP - 1) * TP < P <= tP * TP
        assert (tQ - 1) * TQ < Q <= tQ * TQ
    assert info["lds_bytes"] <= 160 * 1024
    assert info["threads"] % 64 == 0 and 64 <= info["threads"] <= 1024
    assert info["workspace_bytes"] == 0
    assert 0.0 < info["mfma_efficiency"] <= 1.0
    if exhaustive and not info["flat"] and not info["pointwise"]:
        # replay the kernel's workgroup -> tile decode and count writers per output
        hits = np.zeros((N, K, P, Q), np.int32)
        for bid in range(info["grid"]):
            b = bid
            kt, b = b % tK, b // tK
            tq, b = b % tQ, b // tQ
            tp, n = b % tP, b // tP
            hits[n, kt * KT:(kt + 1) * KT, tp * TP:(tp + 1) * TP, tq * TQ:(tq + 1) * TQ] += 1
        assert hits.min() == 1 and hits.max() == 1


@pytest.mark.parametrize("layer", workloads.ALL_LAYERS + workloads.INCEPTION, ids=lambda l: l.name)
def test_plan_for_every_benchmark_layer(layer):
    plan = cd.Plan(*layer.dims())
    assert plan.output_dims() == (layer.P, layer.Q)
    assert plan.workspace_bytes() == 0
    info = plan.info()
    for k in ("N", "C", "H", "W", "K", "R", "S", "stride", "pad"):
        assert info[k] == getattr(layer, k)
    # a compiled (not runtime-shape) variant serves every batched benchmark layer
    if layer.N >= 32:
        assert not info["variant"].startswith("generic")
    _check_cover(info, exhaustive=layer.N * layer.K * layer.P * layer.Q <= 2_000_000)
    plan.destroy()


@pytest.mark.parametrize("shape", [
    (1, 1, 1, 1, 1, 1, 1, 1, 0), (2, 5, 9, 7, 33, 2, 4, 3, 2), (3, 4, 40, 70, 65, 4, 4, 1, 0),
    (1, 7, 33, 35, 130, 3, 3, 1, 1), (2, 3, 50, 50, 20, 9, 9, 5, 4), (1, 2, 5, 300, 3, 1, 7, 1, 3),
])
def test_plan_for_odd_shapes(shape):
    plan = cd.Plan(*shape)
    _check_cover(plan.info(), exhaustive=True)
    plan.destroy()


def _seeded_shapes(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        kind = rng.integers(0, 4)
        if kind == 0:      # pointwise, channel counts around the special forms' conditions
            R = S = 1
            st, pd = 1, 0
            C = int(rng.choice([64, 63, 65, 128, 256, 24]))
            K = int(rng.choice([32, 64, 96, 256, 70, 33]))
        else:
            R = int(rng.integers(1, 8))
            S = R if rng.random() < 0.7 else int(rng.integers(1, 8))
            st, pd = int(rng.integers(1, 4)), int(rng.integers(0, 4))
            C, K = int(rng.integers(1, 300)), int(rng.integers(1, 300))
        H, W = int(rng.integers(1, 120)), int(rng.integers(1, 120))
        if rng.random() < 0.3:
            H = W = int(rng.choice([7, 13, 14, 27, 28, 56]))
        if H + 2 * pd < R or W + 2 * pd < S:
            continue
        out.append((int(rng.integers(1, 70)), C, H, W, K, R, S, st, pd))
    return out


def test_planner_on_seeded_random_shapes():
    """Plans of every kind for a few hundred seeded shapes: each is created, describes a grid that covers its
    output, names a second choice exactly when its variant has no fused tail, and is destroyed."""
    for shape in _seeded_shapes(300, 77):
        N, C, H, W, K, R, S, st, pd = shape
        for li, lo in ((cd.PLAIN, cd.PLAIN), (cd.BLOCKED, cd.BLOCKED), (cd.PLAIN, cd.BLOCKED)):
            plan = cd.Plan(*shape, in_layout=li, out_layout=lo)
            info = plan.info()
            _check_cover(info, exhaustive=False)
            assert (info["tail_variant"] != "same") == ("_sl" in info["variant"] and info["variant"][1] == "1"), (shape, info["variant"])
            assert info["model_clocks"] > 0
            plan.destroy()
        if R == S or st == 1:
            plan = cd.Plan.dgrad(*shape)
            assert plan.info()["workspace_bytes"] == 0 and plan.dgrad_wt_elems() > 0
            plan.destroy()
        try:
            plan = cd.Plan.wgrad(*shape)
        except cd.ConvDirectError as e:
            assert e.code == cd.EUNSUPPORTED, shape      # (filter shapes the weight gradient has no variant for)
        else:
            assert plan.info()["kind"] == "wgrad"
            plan.destroy()


def test_every_variant_plans_a_matching_shape():
    names = cd.variant_names()
    assert len(names) == len(set(names)) and any(n.startswith("generic") for n in names)
    for nm in names:
        m = re.match(r"[fdrpb](\d+)s(\d+)_", nm)
        R, st = (int(m.group(1)), int(m.group(2))) if m else (4, 3)
        C = 3 if nm.startswith("r") else 6   # the row-pair family takes only a few channels
        fl = re.search(r"_flat(\d+)_", nm)     # flat tiling is compiled for one image size
        H, W = (int(fl.group(1)),) * 2 if fl else (37, 41)
        blocked = nm.startswith("b")               # variants for the blocked input / weight layouts
        if "k64m" in nm:
            # all phases of a stride-2 layer's data gradient in one workgroup: serves that, and no forward layer
            lay = cd.BLOCKED if blocked else cd.PLAIN
            with pytest.raises(cd.ConvDirectError) as e:
                cd.Plan(2, C, H, W, 70, R, R, st, R // 2, variant=nm, in_layout=lay, out_layout=lay)
            assert e.value.code == cd.EUNSUPPORTED
            plan = cd.Plan.dgrad(2, 70, 2 * H, 2 * W, C, 3, 3, 2, 1, variant=nm, dy_layout=lay, dx_layout=lay)   # (dy is H x W)
            info = plan.info()
            assert info["variant"] == nm and info["dgrad_phases"] == 4 and info["ktiles"] == 2
            _check_cover(info, exhaustive=True)
            plan.destroy()
            continue
        K = 70
        walk = re.search(r"_c(\d+)_kall", nm)
        if walk:
            # all output channels per workgroup, the input in registers: exactly that many input channels, whole blocks
            # of 32 output channels, pixels in fours; anything else is another variant's
            C, K, H, W = int(walk.group(1)), 96, 36, 41
            for bad in ((2, C, H, W, 70, 1, 1, 1, 0), (2, C, 37, 41, K, 1, 1, 1, 0), (2, C + 2, H, W, K, 1, 1, 1, 0)):
                with pytest.raises(cd.ConvDirectError) as e:
                    cd.Plan(*bad, variant=nm)
                assert e.value.code == cd.EUNSUPPORTED
        plan = cd.Plan(2, C, H, W, K, R, R, st, R // 2, variant=nm,
                       in_layout=cd.BLOCKED if blocked else cd.PLAIN, out_layout=cd.BLOCKED if blocked else cd.PLAIN)
        info = plan.info()
        assert info["variant"] == nm
        # a variant without the fused tail comes with a second choice that has one
        assert (info["tail_variant"] != "same") == ("_sl" in nm and nm[0] in "pb" and nm[1] == "1")
        assert info["in_layout"] == info["out_layout"] == ("blocked" if blocked else "plain")
        if not blocked and not nm.startswith("generic"):   # a compiled variant serves one input layout only
            with pytest.raises(cd.ConvDirectError) as e:
                cd.Plan(2, C, H, W, K, R, R, st, R // 2, variant=nm, in_layout=cd.BLOCKED)
            assert e.value.code == cd.EUNSUPPORTED
        _check_cover(info, exhaustive=True)
        plan.destroy()


def test_no_kernel_uses_private_scratch():
    """Zero workspace includes hidden memory: no kernel may spill registers to scratch
    or use a dynamic stack (read from the compiler's resource report of the last build)."""
    from paper_1809_10170_amd import build
    recs = [r for r in build.kernel_resources() if "conv_" in r["kernel"]]
    assert recs, "no resource report: build with `python -m paper_1809_10170_amd.build`"
    for r in recs:
        assert int(r["ScratchSize [bytes/lane]"]) == 0, r
        assert r["Dynamic Stack"] == "False", r
        assert int(r["VGPRs Spill"]) == 0, r


def test_huge_image_planes_fall_back_to_the_runtime_shape_kernel():
    """The compiled kernels reach the input with 31-bit byte offsets per channel chunk; an
    image whose chunk does not fit is planned onto the fallback (64-bit indexing)."""
    plan = cd.Plan(1, 4, 16384, 16384, 1, 3, 3, 1, 1)     # 4 x 1 GiB channel planes
    assert plan.info()["variant"].startswith("generic")
    plan.destroy()
    plan = cd.Plan(1, 4, 4096, 4096, 1, 3, 3, 1, 1)       # 64 MiB planes: compiled variant
    assert not plan.info()["variant"].startswith("generic")
    plan.destroy()


def test_tuning_table_round_trip_and_override(tmp_path):
    """The measured-choice table: loaded entries win over the model for exactly their problem,
    unknown or unusable entries fall back to it, malformed files change nothing."""
    cd.tuning_clear()
    shape = (2, 16, 30, 30, 64, 3, 3, 1, 1)
    default = cd.Plan(*shape).info()["variant"]
    other = next(n for n in ("d3s1_8x28_k128", "d3s1_14x14_k128", "d3s1_4x56_k128") if n != default)
    good = tmp_path / "tuned.txt"
    good.write_text("# measured choices\n"
                    + " ".join(map(str, shape)) + f" 0 0 {other}\n"
                    + "2 16 31 31 64 3 3 1 1 0 0 no_such_variant\n"
                    + "2 16 32 32 64 3 3 1 1 0 0 r11s4_4x55_k96\n")
    cd.tuning_load(str(good))
    assert cd.tuning_size() == 3
    assert cd.Plan(*shape).info()["variant"] == other
    assert cd.Plan(3, *shape[1:]).info()["variant"] == cd.Plan(3, *shape[1:], variant=None).info()["variant"]
    for hw in (31, 32):   # unknown variant / a variant that cannot run the shape: the model decides
        p = cd.Plan(2, 16, hw, hw, 64, 3, 3, 1, 1)
        assert p.info()["variant"] not in ("no_such_variant", "r11s4_4x55_k96")
    out = tmp_path / "saved.txt"
    cd.tuning_save(str(out))
    assert sorted(l.split() for l in out.read_text().splitlines()) == \
        sorted(l.split() for l in good.read_text().splitlines() if not l.startswith("#"))
    bad = tmp_path / "bad.txt"
    bad.write_text("1 2 3 4 5 6 7 8 9 0 0 d3s1_8x28_k128\n1 2 3 oops\n")
    with pytest.raises(cd.ConvDirectError) as e:
        cd.tuning_load(str(bad))
    assert e.value.code == cd.EINVAL and cd.tuning_size() == 3
    with pytest.raises(cd.ConvDirectError):
        cd.tuning_load(str(tmp_path / "missing.txt"))
    cd.tuning_clear()
    assert cd.tuning_size() == 0 and cd.Plan(*shape).info()["variant"] == default


def test_measured_choice_of_a_variant_without_tail_still_gets_a_second_plan(tmp_path):
    """A tuning-table entry that names a variant without the fused tail: the plan is that variant, its second
    choice (for calls with a tail) comes from the model among the variants that have one, and planning ends."""
    cd.tuning_clear()
    shape = (4, 256, 56, 56, 64, 1, 1, 1, 0)
    names = [n for n in cd.variant_names() if n.startswith("p1s1") and "_sl" in n]
    assert names
    f = tmp_path / "tuned.txt"
    f.write_text(" ".join(map(str, shape)) + f" 0 0 {names[0]}\n")
    cd.tuning_load(str(f))
    plan = cd.Plan(*shape)
    info = plan.info()
    assert info["variant"] == names[0] and info["tail_variant"] not in ("same", names[0])
    plan.destroy()
    cd.tuning_clear()


def test_layout_gradient_and_tail_entry_points_check_arguments_before_any_launch():
    L = cd.lib()
    import ctypes
    p = ctypes.c_void_p()
    dims = (2, 8, 20, 20, 8, 3, 3, 1, 1)
    # layouts
    assert L.conv_direct_create_layout(ctypes.byref(p), *dims, 2, 0) == cd.EINVAL and not p
    assert L.conv_direct_create_layout(ctypes.byref(p), *dims, 0, -1) == cd.EINVAL and not p
    assert L.conv_direct_create_ex(ctypes.byref(p), b"no_such_variant", *dims, 1, 1) == cd.EUNSUPPORTED and not p
    assert cd.blocked_act_elems(2, 5, 3, 4) == 2 * 8 * 3 * 4 and cd.blocked_act_elems(0, 5, 3, 4) == 0
    assert cd.blocked_w_elems(33, 5, 3, 3) == 64 * 8 * 9 and cd.blocked_w_elems(33, 5, 3, -1) == 0
    for fn in (L.conv_direct_pack_act, L.conv_direct_unpack_act, L.conv_direct_pack_w, L.conv_direct_dgrad_filter):
        assert fn(None, 4096, 2, 3, 4, 5, None) == cd.EINVAL
        assert fn(4096, 8192, 2, 0, 4, 5, None) == cd.EINVAL
        assert fn(4098, 8192, 2, 3, 4, 5, None) == cd.EALIGN
    assert L.conv_direct_pack_act(4096, 8196, 2, 3, 4, 5, None) == cd.EALIGN      # blocked destination: 16 bytes
    # gradients
    sd = cd.Plan.dgrad(2, 8, 20, 20, 8, 3, 3, 2, 1)                      # strided, square filter: one 2x2 convolution per phase
    assert sd.info()["variant"].startswith("d2s1") and sd.info()["dgrad_phases"] == 4 and sd.output_dims() == (20, 20)
    assert sd.dgrad_wt_elems() == 4 * 8 * 8 * 2 * 2 and sd.workspace_bytes() == 0
    assert L.conv_direct_dgrad_prepare(sd._p, None, 4096, None) == cd.EINVAL
    assert L.conv_direct_dgrad_prepare(sd._p, 4098, 4096, None) == cd.EALIGN
    sd.destroy()
    sd = cd.Plan.dgrad(2, 8, 20, 21, 8, 3, 5, 2, 1)                      # R != S: the runtime-shape kernel, stride-1 form of wt
    assert sd.info()["variant"].startswith("generic") and sd.output_dims() == (20, 21) and sd.dgrad_wt_elems() == 8 * 8 * 15
    sd.destroy()
    s1 = cd.Plan.dgrad(*dims)
    assert s1.dgrad_wt_elems() == 8 * 8 * 9 and s1.info()["dgrad_phases"] == 0
    s1.destroy()
    fw = cd.Plan(*dims)
    assert fw.dgrad_wt_elems() == 0 and L.conv_direct_dgrad_prepare(fw._p, 4096, 8192, None) == cd.EINVAL   # not a data gradient
    fw.destroy()
    assert L.conv_direct_create_dgrad(ctypes.byref(p), 2, 8, 20, 20, 8, 3, 3, 0, 1) == cd.EINVAL
    assert L.conv_direct_create_wgrad(ctypes.byref(p), 2, 8, 40, 40, 8, 3, 4, 5, 1) == cd.EUNSUPPORTED and not p
    assert L.conv_direct_create_wgrad(ctypes.byref(p), 2, 8, 20, 20, 0, 3, 3, 1, 1) == cd.EINVAL
    wg = cd.Plan.wgrad(*dims)
    info = wg.info()
    assert info["kind"] == "wgrad" and info["workspace_bytes"] == 0 and info["grid"] == info["ktiles"] * info["cgroups"] * (1 if "_ar" in info["variant"] else 3) * info["splits"]   # (all-rows variants: the filter row is no grid dimension)
    P, Q = ctypes.c_int(), ctypes.c_int()
    assert L.conv_direct_output_dims(wg._p, ctypes.byref(P), ctypes.byref(Q)) == cd.EINVAL      # not a forward plan
    assert L.conv_direct_run(wg._p, 4096, 8192, 12288, None) == cd.EINVAL
    assert L.conv_direct_run_wgrad(wg._p, 4096, 8192, 12290, None) == cd.EALIGN
    assert L.conv_direct_run_wgrad(wg._p, None, 8192, 12288, None) == cd.EINVAL
    fwd = cd.Plan(*dims)
    assert L.conv_direct_run_wgrad(fwd._p, 4096, 8192, 12288, None) == cd.EINVAL                 # not a wgrad plan
    assert L.conv_direct_run_fused(fwd._p, 4096, 8192, 4098, None, 0, 12288, None) == cd.EALIGN  # misaligned bias
    dg = cd.Plan.dgrad(*dims)
    assert dg.output_dims() == (20, 20) and dg.info()["C"] == 8 and dg.info()["pad"] == 1
    for pl in (wg, fwd, dg):
        pl.destroy()
    # measured choice: arguments
    assert L.conv_direct_create_tuned(ctypes.byref(p), *dims, 0, 0, None, 8192, 12288, None, 3) == cd.EINVAL
    assert L.conv_direct_create_tuned(ctypes.byref(p), *dims, 0, 0, 4096, 8192, 12288, None, 0) == cd.EINVAL
    assert L.conv_direct_create_tuned(ctypes.byref(p), *dims, 0, 3, 4096, 8192, 12288, None, 3) == cd.EINVAL


def test_data_gradient_create_rejects_a_null_plan_pointer():
    L = cd.lib()
    for dims in ([2, 8, 20, 20, 9, 3, 3, 1, 1], [2, 8, 20, 20, 9, 3, 3, 2, 1], [2, 5, 23, 31, 7, 3, 5, 1, 1]):
        assert L.conv_direct_create_dgrad(None, *dims) == cd.EINVAL


def test_images_of_four_gigabytes_are_not_given_to_32_bit_spans():
    """One image of C*H*W*4 >= 2^32 bytes (the whole tensor still below 2^31 elements): the rectangular
    channel-pair tiles bound their loads by a 32-bit byte count from the chunk's first channel to the
    image's end, so the planner must not choose them."""
    N, C, H, W = 1, 1024, 1024, 1024
    assert C * H * W * 4 >= 2 ** 32 and N * C * H * W < 2 ** 31
    L = cd.lib()
    p = ctypes.c_void_p()
    rc = L.conv_direct_create(ctypes.byref(p), N, C, H, W, 1, 3, 3, 1, 1)
    if rc == cd.OK:
        buf = ctypes.create_string_buffer(1024)
        L.conv_direct_plan_info(p, buf, len(buf))
        assert b"variant=generic" in buf.value, buf.value
        L.conv_direct_destroy(p)
    else:
        assert rc == cd.EUNSUPPORTED
    for nm in cd.variant_names():
        if nm.startswith("d3s1") and "flat" not in nm:
            assert L.conv_direct_create_with_variant(ctypes.byref(p), nm.encode(), N, C, H, W, 1, 3, 3, 1, 1) == cd.EUNSUPPORTED


def test_probe_rejects_bad_arguments_before_any_launch():
    L = cd.lib()
    assert L.conv_direct_mfma_probe(None, 10, None) == cd.EINVAL
    assert L.conv_direct_mfma_probe(4096, 0, None) == cd.EINVAL
    assert L.conv_direct_mfma_probe(4100, 10, None) == cd.EALIGN


def test_plan_info_states_the_data_gradient_s_extra_buffer():
    plan = cd.Plan.dgrad(2, 8, 20, 20, 9, 3, 3, 1, 1)
    assert plan.info()["extra_caller_bytes"] == 4 * 9 * 8 * 3 * 3 == 4 * plan.dgrad_wt_elems()
    assert plan.dims[:4] == (2, 9, 20, 20)
    plan.destroy()
    plan = cd.Plan.dgrad(2, 8, 20, 20, 9, 3, 3, 2, 1)     # four phase filters of 2 x 2 taps
    assert plan.info()["extra_caller_bytes"] == 4 * 4 * 9 * 8 * 2 * 2
    plan.destroy()
    fwd = cd.Plan(2, 8, 20, 20, 9, 3, 3, 1, 1)
    assert fwd.info()["extra_caller_bytes"] == 0 and fwd.info()["workspace_bytes"] == 0
    fwd.destroy()


def test_data_gradient_plans_take_layouts_and_size_the_filter_in_whole_blocks():
    """conv_direct_create_dgrad_layout: the blocked transformed filter holds whole blocks of 32 layer-input channels and
    pencils of 4 layer-output channels per phase; bad layouts are refused; a phase filter of more than 4x4 taps goes to
    the runtime-shape kernel (no compiled kernel re-maps its output)."""
    p = cd.Plan.dgrad(2, 40, 29, 29, 70, 3, 3, 2, 1, dy_layout=cd.BLOCKED, dx_layout=cd.BLOCKED)
    i = p.info()
    assert i["dgrad_phases"] == 4 and i["in_layout"] == "blocked" and i["out_layout"] == "blocked"
    assert p.dgrad_wt_elems() == 4 * 64 * 72 * 2 * 2 and i["extra_caller_bytes"] == 4 * p.dgrad_wt_elems()
    q = cd.Plan.dgrad(2, 40, 29, 29, 70, 3, 3, 2, 1)
    assert q.dgrad_wt_elems() == 4 * 40 * 70 * 2 * 2
    plan = ctypes.c_void_p(1)
    assert cd.lib().conv_direct_create_dgrad_layout(ctypes.byref(plan), 2, 40, 29, 29, 70, 3, 3, 2, 1, 2, 0) == cd.EINVAL
    assert plan.value is None
    big = cd.Plan.dgrad(1, 8, 20, 20, 8, 9, 9, 2, 4)
    assert big.info()["dgrad_phases"] == 0 and big.info()["variant"].startswith("generic")
