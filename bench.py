#!/usr/bin/env python3
"""Benchmark of the zero-workspace direct convolution on one MI355X.

A step is one forward pass of every layer of the chosen workload (one
conv_direct_run per layer) on seeded synthetic tensors already resident in HBM.
The default workload is the batched AlexNet-/VGG-shaped layer suite; `--workload
NAME` times a single layer (names: paper_1809_10170_amd/workloads.py).

Prints ONE JSON line: whole-workload TFLOP/s (2*N*K*C*R*S*P*Q per layer / time of the timed
passes, which carry HIP events around the launches of one layer only: the one that takes the
most time), per-layer figures (average, median and minimum launch time from HIP events on the
launch stream in as many further passes behind the timed ones, fraction of the nominal fp32 MFMA peak and of the peak at the clock a bare-MFMA
probe measures in the same run, error of sampled outputs against the CPU oracle), the
roofline record of the kernel that takes the most time, and the CPU oracle timed on a
bounded sample of the same workload on this host.  The default run (forward, plain
layouts, batched suite) also times, outside the headline step, the single-image layers
and the toy layer (`layers_single`) and the library's other paths over the same suite
(`other_paths`: blocked layouts, data gradient, weight gradient) and over the GoogLeNet-shaped
layers (`other_paths.inception_forward*`).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_CLOCK_MHZ = 2400.0
PEAK_FP32_MFMA_TFLOPS = 157.3     # MI355X: 256 CU x 256 flop/clk x 2.4 GHz
PEAK_HBM_GBPS = 8000.0
FLOP_PER_CLOCK = 256 * 256        # fp32 MFMA, whole chip
CHECK_POINTS = 2000               # sampled outputs per layer compared with the oracle in every run


def suite(name, workloads):
    if name == "suite_batched":
        return [l for l in workloads.ALL_LAYERS if l.N >= 32]
    if name == "suite_single":      # the single-image layers and the toy layer
        return [l for l in workloads.ALL_LAYERS if l.N == 1]
    if name == "suite_inception":   # GoogLeNet-shaped layers; a suite of its own, not the headline metric
        return list(workloads.INCEPTION)
    if name == "suite_all":
        return list(workloads.ALL_LAYERS)
    return [workloads.BY_NAME[name]]


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for ln in f:
                if ln.lower().startswith("model name"):
                    return ln.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(layers, budget_s=15.0):
    """The oracle, as it stands, on whole images of the workload: pass after pass over the
    layers, one image (full output) of each per pass, until about budget_s seconds of CPU
    work are spent."""
    import oracle
    from paper_1809_10170_amd import workloads
    oracle.build()
    flops, secs, done, inputs = 0, 0.0, {}, {}
    n_pass = 0
    while secs < budget_s:
        for l in layers:
            if secs >= budget_s:
                break
            if l.name not in inputs:
                inputs[l.name] = workloads.make_inputs(l, N=min(l.N, 4))
            x, w = inputs[l.name]
            n = n_pass % x.shape[0]
            t0 = time.perf_counter()
            oracle.conv_forward(x[n:n + 1], w, l.stride, l.pad)
            secs += time.perf_counter() - t0
            flops += l.flops // l.N
            done[l.name] = done.get(l.name, 0) + 1
        n_pass += 1
    sample = ", ".join(f"{v}x {k}" for k, v in done.items())
    return {"value": flops / secs / 1e12, "unit": "TFLOP/s", "cores": oracle.threads(), "cpu_model": cpu_model(),
            "kind": "oracle", "sample": f"single images, full output (the first 4 of each layer, in turn): {sample}",
            "seconds": round(secs, 2)}


TRAFFIC_SOURCE = "profiles/hbm_traffic.md"


def measured_traffic(layer_name, variant):
    """HBM bytes per launch of a layer's kernel from the committed rocprofv3 --pmc summary
    (FETCH_SIZE and WRITE_SIZE scaled by the copy-kernel calibration stated there), or
    None if the summary has no row for this layer and kernel variant."""
    path = os.path.join(ROOT, TRAFFIC_SOURCE)
    try:
        with open(path) as f:
            for ln in f:
                cells = [c.strip() for c in ln.split("|")]
                if len(cells) > 6 and cells[1] == layer_name and cells[2] == variant:
                    return int((2.0 * float(cells[4]) + 1.0 * float(cells[5])) * 1024)
    except OSError:
        pass
    return None


def copy_probe(nbytes=1 << 30, reps=5):
    """A plain device-to-device copy of known size: under `rocprofv3 --pmc FETCH_SIZE`
    (or WRITE_SIZE) its counter reading calibrates the same counter read for the
    convolution kernels."""
    import torch
    x = torch.empty(nbytes // 4, device="cuda", dtype=torch.float32).normal_()
    y = torch.empty_like(x)
    torch.cuda.synchronize()
    for _ in range(reps):
        y.copy_(x)
    torch.cuda.synchronize()
    print(json.dumps({"copy_probe_bytes_read": nbytes, "copy_probe_bytes_written": nbytes, "reps": reps}))


def measure_clock(cd, torch, stream, iters=20000, reps=2):
    """Bare-MFMA probe: the shader clock under a saturated fp32 matrix load, from the probe's own counters
    (shader-clock ticks per tick of the constant 100 MHz counter around its loop), and the flop rate it
    reaches.  The clock ramps up over the first tens of milliseconds of load, so each probe launch runs
    for about 60 ms and the last one counts."""
    buf = torch.empty(cd.PROBE_BYTES // 8, device="cuda", dtype=torch.int64)
    cd.mfma_probe(buf, iters, stream.cuda_stream)
    torch.cuda.synchronize()
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        cd.mfma_probe(buf, iters, stream.cuda_stream)
        e1.record(stream)
        e1.synchronize()
        ms = e0.elapsed_time(e1)
    tflops = cd.PROBE_FLOP_PER_ITER * iters / (ms * 1e-3) / 1e12
    ticks = buf[512 * 256 * 4 // 8:].cpu().numpy().reshape(512, 2)
    ratio = sorted((ticks[:, 0] / ticks[:, 1]).tolist())[256]
    return {"probe": "bare v_mfma_f32_32x32x2_f32 chains, 2 waves per SIMD, 60 ms", "clock_mhz": round(ratio * 100.0, 1),
            "probe_tflops": round(tflops, 2), "clock_mhz_from_rate": round(tflops * 1e12 / FLOP_PER_CLOCK / 1e6, 1),
            "nominal_clock_mhz": PEAK_CLOCK_MHZ}


class Runner:
    """Plans and device tensors of one path (direction x layout) over a list of layers."""

    def __init__(self, cd, torch, workloads, tensors, layers, direction, blocked, variant=None):
        self.cd, self.torch, self.workloads = cd, torch, workloads
        self.direction, self.blocked = direction, blocked
        dev = torch.device("cuda:0")
        self.items = []
        for l in layers:
            xd, wd = tensors(l)
            if direction == "wgrad":
                # blocked: dy and dw in their blocked layouts, x too unless it is a first layer's image (kept plain)
                lx = cd.BLOCKED if blocked and l.C >= 4 else cd.PLAIN
                lo = cd.BLOCKED if blocked else cd.PLAIN
                plan = cd.Plan.wgrad(*l.dims(), x_layout=lx, dy_layout=lo, dw_layout=lo)
                dyp = self._dy(l, dev)
                self.items.append(dict(layer=l, plan=plan, x=self._act(xd, lx), dy=self._act(dyp, lo), x_plain=xd, dy_plain=dyp,
                                       dw=torch.empty((-(-l.K // 32), -(-l.C // 4), l.R, l.S, 4, 32) if blocked else (l.K, l.C, l.R, l.S), device=dev)))
            elif direction == "dgrad":
                lo = cd.BLOCKED if blocked else cd.PLAIN
                plan = cd.Plan.dgrad(*l.dims(), dy_layout=lo, dx_layout=lo)
                dyp = self._dy(l, dev)
                self.items.append(dict(layer=l, plan=plan, dy=self._act(dyp, lo), dy_plain=dyp, w=wd, wt=torch.empty((plan.dgrad_wt_elems(),), device=dev),
                                       dx=torch.empty((l.N, -(-l.C // 4), l.H, l.W, 4) if blocked else (l.N, l.C, l.H, l.W), device=dev)))
            else:
                li = cd.BLOCKED if blocked and l.C >= 4 else cd.PLAIN
                lo = cd.BLOCKED if blocked else cd.PLAIN
                plan = cd.Plan(*l.dims(), variant=variant, in_layout=li, out_layout=lo)
                xin, win = xd, wd
                if li == cd.BLOCKED:   # re-arranged once, outside the timed region (the weights: a one-time cost; the
                    xin = torch.empty((l.N, -(-l.C // 4), l.H, l.W, 4), device=dev)       # input: a previous layer's output)
                    win = torch.empty((-(-l.K // 32), -(-l.C // 4), l.R, l.S, 4, 32), device=dev)
                    cd.pack_act(xd, xin)
                    cd.pack_w(wd, win)
                oshape = (l.N, -(-l.K // 4), l.P, l.Q, 4) if lo == cd.BLOCKED else (l.N, l.K, l.P, l.Q)
                self.items.append(dict(layer=l, plan=plan, x=xin, w=win, out=torch.empty(oshape, device=dev), x_plain=xd, w_plain=wd))
        torch.cuda.synchronize()

    def _act(self, plain, layout):
        # an activation tensor in the given layout (re-arranged once, outside the timed region)
        if layout == self.cd.PLAIN:
            return plain
        n, c, h, w = plain.shape
        return self.cd.pack_act(plain, self.torch.empty((n, -(-c // 4), h, w, 4), device=plain.device))

    def _plain(self, t, shape):
        # a (possibly blocked) activation tensor as a plain one
        return t if tuple(t.shape) == tuple(shape) else self.cd.unpack_act(t, self.torch.empty(shape, device=t.device))

    def _dy(self, l, dev):
        # dy stands in for the next layer's gradient: U[-1,1], seeded
        g = self.torch.Generator(device="cpu").manual_seed(4242 + l.K)
        return (self.torch.rand((l.N, l.K, l.P, l.Q), generator=g) * 2 - 1).to(dev)

    def launch(self, it, stream):
        if self.direction == "wgrad":   # (x, dy) -> dw: a fill and the reduction
            it["plan"].run_wgrad(it["x"], it["dy"], it["dw"], stream)
        elif self.direction == "dgrad":  # the filter transform belongs to the step (weights change every update)
            it["plan"].dgrad_prepare(it["w"], it["wt"], stream)
            it["plan"].run(it["dy"], it["wt"], it["dx"], stream)
        else:
            it["plan"].run(it["x"], it["w"], it["out"], stream)

    def _passes(self, count, stream, bracket):
        """`count` passes over the layers with a pair of events around the launches of the layers in `bracket`:
        (host seconds, {layer index: sorted launch times in ms})."""
        torch = self.torch
        ev = {i: [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(count)] for i in bracket}
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(count):
            for i, it in enumerate(self.items):
                if i in ev:
                    ev[i][s][0].record(stream)
                self.launch(it, stream.cuda_stream)
                if i in ev:
                    ev[i][s][1].record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return wall, {i: sorted(e0.elapsed_time(e1) for e0, e1 in pairs) for i, pairs in ev.items()}

    def time_step(self, steps, warmup, stream):
        """Whole passes over the layers.  A pair of events around every launch costs the pass about 2 % (28 markers between
        14 kernels), so the timed passes carry events around ONE layer only, the one that takes the most time (found in
        the warm-up passes, which carry them all); the per-layer times come from a further `steps` passes behind the
        timed region.  Returns (ms per pass from the host clock around the `steps` timed passes, per-layer sorted
        launch times of the further passes, index of the layer that takes the most time, its sorted launch times in the
        timed passes)."""
        torch = self.torch
        everything = range(len(self.items))
        _, warm = self._passes(warmup, stream, everything)
        if warmup:
            dom = max(everything, key=lambda i: sum(warm[i]))
        else:
            dom = max(everything, key=lambda i: self.items[i]["layer"].flops)
        alloc_before = torch.cuda.memory_allocated()
        wall, dom_times = self._passes(steps, stream, [dom])
        assert torch.cuda.memory_allocated() == alloc_before, "device memory was allocated during the timed region"
        wall_ev, times = self._passes(steps, stream, everything)
        self.ms_per_pass_with_events = wall_ev * 1e3 / steps
        return wall * 1e3 / steps, [times[i] for i in everything], dom, dom_times[dom]

    def time_each(self, steps, warmup, stream):
        """Every layer alone in a loop of its own (for layers that are no part of a step): per-layer sorted
        launch times.  Back-to-back launches of one small layer find its tensors in the caches."""
        torch = self.torch
        times = []
        for it in self.items:
            for _ in range(warmup):
                self.launch(it, stream.cuda_stream)
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
            torch.cuda.synchronize()
            for e0, e1 in ev:
                e0.record(stream)
                self.launch(it, stream.cuda_stream)
                e1.record(stream)
            torch.cuda.synchronize()
            times.append(sorted(e0.elapsed_time(e1) for e0, e1 in ev))
        return times

    def check(self, it, npts=CHECK_POINTS):
        """Sampled results of the last launch against the CPU oracle: (max |err|, tolerance, what was compared)."""
        import numpy as np
        import oracle
        cd, torch, l = self.cd, self.torch, it["layer"]
        if self.direction == "wgrad":
            # three output channels of dw in full (each costs the oracle a forward pass of one channel)
            ks = sorted({0, l.K - 1, l.K // 2})
            want = oracle.conv_wgrad(it["x_plain"].cpu().numpy(), np.ascontiguousarray(it["dy_plain"].cpu().numpy()[:, ks]), l.R, l.S, l.stride, l.pad)
            dw = it["dw"].cpu().numpy()
            if dw.ndim == 6:   # blocked [K/32][C/4][R][S][4][32] -> [K][C][R][S]
                dw = dw.transpose(0, 5, 1, 4, 2, 3).reshape(dw.shape[0] * 32, dw.shape[1] * 4, l.R, l.S)[:l.K, :l.C]
            err = float(np.abs(dw[ks].astype(np.float64) - want).max())
            return err, 1e-4 * (l.N * l.P * l.Q) ** 0.5, f"dw[{ks}] in full"
        if self.direction == "dgrad":
            if not (l.stride == 1 and l.R == l.S and l.pad <= l.R - 1):
                # no single-element form for these: the last image in full against the oracle's adjoint
                n = l.N - 1
                want = oracle.conv_dgrad(np.ascontiguousarray(it["dy_plain"][n:n + 1].cpu().numpy()), it["w"].cpu().numpy(), l.H, l.W, l.stride, l.pad)
                dx = self._plain(it["dx"], (l.N, l.C, l.H, l.W))
                err = float(np.abs(dx[n:n + 1].cpu().numpy().astype(np.float64) - want).max())
                return err, oracle.tolerance(l.K, l.R, l.S), f"image {n} of dx in full"
            # sampled dx elements through the flipped-filter identity (pinned on the CPU against the adjoint definition)
            rng = np.random.default_rng(5)
            pts = np.stack([rng.integers(0, d, npts) for d in (l.N, l.C, l.H, l.W)], axis=1).astype(np.int32)
            wt = np.ascontiguousarray(it["w"].cpu().numpy()[:, :, ::-1, ::-1].transpose(1, 0, 2, 3))
            want = oracle.conv_forward_points(it["dy_plain"].cpu().numpy(), wt, pts, 1, l.R - 1 - l.pad)
            got = self._gather(self._plain(it["dx"], (l.N, l.C, l.H, l.W)), pts)
            return float(np.abs(got - want).max()), oracle.tolerance(l.K, l.R, l.S), f"{npts} sampled elements of dx"
        pts = self.workloads.sample_points(l, npts)
        want = oracle.conv_forward_points(it["x_plain"].cpu().numpy(), it["w_plain"].cpu().numpy(), pts, l.stride, l.pad)
        out = it["out"]
        if it["plan"].out_layout == cd.BLOCKED:
            out = cd.unpack_act(out, torch.empty((l.N, l.K, l.P, l.Q), device=out.device))
        got = self._gather(out, pts)
        return float(np.abs(got - want).max()), oracle.tolerance(l.C, l.R, l.S), f"{npts} sampled outputs"

    def _gather(self, t, pts):
        import numpy as np
        idx = self.torch.from_numpy(pts.astype(np.int64)).to(t.device)
        return t[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]].cpu().numpy().astype(np.float64)

    def records(self, times, clock_mhz, check=True):
        """One record per layer from its sorted launch times."""
        peak_at_clock = PEAK_FP32_MFMA_TFLOPS * clock_mhz / PEAK_CLOCK_MHZ if clock_mhz else None
        out = []
        for it, ms in zip(self.items, times):
            l, info = it["layer"], it["plan"].info()
            avg, med = sum(ms) / len(ms), ms[len(ms) // 2]
            tf = l.flops / (avg * 1e-3) / 1e12
            rec = {"layer": l.name, "variant": info["variant"], "grid": info["grid"],
                   "gflop": round(l.flops / 1e9, 3), "ms_avg": round(avg, 5), "ms_median": round(med, 5), "ms_min": round(ms[0], 5),
                   "tflops": round(tf, 3), "frac_fp32_mfma_peak": round(tf / PEAK_FP32_MFMA_TFLOPS, 4),
                   "frac_at_measured_clock": round(tf / peak_at_clock, 4) if peak_at_clock else None,
                   "algorithmic_GBps": round(l.algorithmic_bytes / (avg * 1e-3) / 1e9, 1),
                   "workspace_bytes": it["plan"].workspace_bytes()}
            if info.get("extra_caller_bytes"):
                rec["extra_caller_bytes"] = info["extra_caller_bytes"]   # the transformed filter of a data gradient
            if check:
                err, tol, what = self.check(it)
                rec.update({"max_err": float(f"{err:.3e}"), "tol": float(f"{tol:.3e}"), "checked": what})
                assert err <= tol, (l.name, err, tol)
            out.append(rec)
        return out

    def destroy(self):
        for it in self.items:
            it["plan"].destroy()
        self.items = []


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="suite_batched")
    ap.add_argument("--variant", default=None, help="force a kernel variant (single-layer workloads)")
    ap.add_argument("--direction", default="forward", choices=["forward", "dgrad", "wgrad"],
                    help="dgrad: the data gradient of the suite's layers behind the first one (filter transform + convolution "
                         "of dy per step); wgrad: the weight gradient of every layer (clear + reduction per step); "
                         "plain layouts")
    ap.add_argument("--layout", default="plain", choices=["plain", "blocked"],
                    help="blocked: the paper's Section 4 layouts (activations [N][C/4][H][W][4], weights "
                         "[K/32][C/4][R][S][4][32]); first layers (C < 4) keep a plain input and write a blocked "
                         "output")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true", help="skip the comparison of sampled results with the oracle")
    ap.add_argument("--no-extras", action="store_true",
                    help="headline step only: no single-image layers, no other paths, no clock probe (for profiling runs)")
    ap.add_argument("--check", action="store_true", help="(kept for older command lines: the check is on by default)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="run only a 1 GiB device copy (calibration of the HBM traffic counters)")
    args = ap.parse_args()
    if args.copy_probe:
        return copy_probe()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only; --gpus must be 1 "
                 "(the forward pass shards over the batch with no exchange step; nothing here uses a second GPU)")

    import torch
    from paper_1809_10170_amd import conv_direct as cd
    from paper_1809_10170_amd import workloads

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    cd.lib()   # fail loudly if the HIP library is missing
    layers = suite(args.workload, workloads)
    blocked = args.layout == "blocked"

    def dgrad_layers(ls):
        # a suite: the layers whose data gradient runs on the compiled kernels (stride 1, or a strided layer as one
        # small convolution per phase), first layers left out (no network needs the gradient of its input image);
        # a layer named alone runs whatever its path
        return [l for l in ls if l.R == l.S and l.pad <= l.R - 1 and l.C >= 16] if len(ls) > 1 else ls

    if args.direction == "dgrad":
        layers = dgrad_layers(layers)
    if not layers:
        sys.exit("bench.py: no layer left to run")
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()
    check = not args.no_check

    cache = {}

    def tensors(l):   # the layer's seeded input and weights on the device, made once
        if l.name not in cache:
            x, w = workloads.make_inputs(l)
            cache[l.name] = (torch.from_numpy(x).to(dev), torch.from_numpy(w).to(dev))
        return cache[l.name]

    clock = None if args.no_extras else measure_clock(cd, torch, stream)
    clock_mhz = clock["clock_mhz"] if clock else None

    main_run = Runner(cd, torch, workloads, tensors, layers, args.direction, blocked, args.variant)
    ms_per_step, times, dom_index, dom_times = main_run.time_step(args.steps, args.warmup, stream)
    per_layer = main_run.records(times, clock_mhz, check)
    total_flops = sum(l.flops for l in layers)
    value = total_flops / (ms_per_step * 1e-3) / 1e12

    # the layer that takes the most time, from the events around its launches inside the timed passes
    dom = dict(per_layer[dom_index])
    dom["ms_avg"] = round(sum(dom_times) / len(dom_times), 5)
    dom["tflops"] = round(layers[dom_index].flops / (dom["ms_avg"] * 1e-3) / 1e12, 3)
    if clock_mhz:
        dom["frac_at_measured_clock"] = round(dom["tflops"] / (PEAK_FP32_MFMA_TFLOPS * clock_mhz / PEAK_CLOCK_MHZ), 4)
    kern = {"r": "conv_rows_kernel", "p": "conv_pw_kernel", "w": "conv_wgrad_kernel"}.get(dom["variant"][0], "conv_dma_kernel")
    traffic = measured_traffic(dom["layer"], dom["variant"])
    roofline = {"bound": "mfma", "kernel": f"{kern}<{dom['variant']}>", "layer": dom["layer"],
                "achieved": dom["tflops"], "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": round(dom["tflops"] / PEAK_FP32_MFMA_TFLOPS, 4),
                "frac_at_measured_clock": dom["frac_at_measured_clock"],
                "launch_ms": dom["ms_avg"], "launch_ms_source": f"HIP events around this layer's {len(dom_times)} launches in the timed passes, on the launch stream",
                "traffic": traffic,
                "traffic_source": (f"{TRAFFIC_SOURCE}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this layer with this "
                                   "variant, scaled by the copy calibration stated there; not measured in this run") if traffic else None,
                "algorithmic_bytes": workloads.BY_NAME[dom["layer"]].algorithmic_bytes}

    rec = {
        "metric": ("conv wgrad TFLOP/s (2*N*K*C*R*S*P*Q/t), fp32, zero workspace" if args.direction == "wgrad" else
                   "conv dgrad TFLOP/s (2*N*K*C*R*S*P*Q/t), fp32, zero workspace" if args.direction == "dgrad" else
                   "conv fwd TFLOP/s (2*N*K*C*R*S*P*Q/t), fp32, zero workspace"),
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "direction": args.direction, "layout": args.layout, "layers": [l.name for l in layers],
                   "frac_fp32_mfma_peak": round(value / PEAK_FP32_MFMA_TFLOPS, 4),
                   "frac_at_measured_clock": round(value / (PEAK_FP32_MFMA_TFLOPS * clock_mhz / PEAK_CLOCK_MHZ), 4) if clock_mhz else None,
                   "workspace_bytes": sum(r["workspace_bytes"] for r in per_layer),
                   "layer_times": f"per-layer figures: {args.steps} further passes behind the timed ones, with HIP events around every launch "
                                  "(kept out of the timed passes, which they slow by about 2 %)",
                   "ms_per_pass_with_layer_events": round(main_run.ms_per_pass_with_events, 4)},
        "roofline": roofline,
        "clock": clock,
        "layers": per_layer,
    }
    main_run.destroy()

    default_run = args.workload == "suite_batched" and args.direction == "forward" and not blocked and not args.variant
    if default_run and not args.no_extras:
        # the single-image layers and the toy layer: each alone in a loop (absolute TFLOP/s; these layers are bounded by
        # launch latency and by having less work than the chip has SIMDs, no fraction of the peak is aimed at)
        single = Runner(cd, torch, workloads, tensors, suite("suite_single", workloads), "forward", False)
        rec["layers_single"] = single.records(single.time_each(args.steps, args.warmup, stream), clock_mhz, check)
        single.destroy()
        # the other paths over the same suite, each timed as whole passes like the headline step
        other = {}
        for name, direction, blk, ls in (("forward_blocked", "forward", True, layers), ("dgrad", "dgrad", False, dgrad_layers(layers)),
                                         ("wgrad", "wgrad", False, layers), ("dgrad_blocked", "dgrad", True, dgrad_layers(layers)),
                                         ("wgrad_blocked", "wgrad", True, layers),
                                         ("inception_forward", "forward", False, suite("suite_inception", workloads)),
                                         ("inception_forward_blocked", "forward", True, suite("suite_inception", workloads))):
            run = Runner(cd, torch, workloads, tensors, ls, direction, blk)
            ms, tms, _, _ = run.time_step(args.steps, args.warmup, stream)
            fl = sum(l.flops for l in ls)
            recs = run.records(tms, clock_mhz, check)
            other[name] = {"value": round(fl / (ms * 1e-3) / 1e12, 3), "unit": "TFLOP/s", "ms_per_step": round(ms, 4),
                           "frac_fp32_mfma_peak": round(fl / (ms * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS, 4),
                           "n_layers": len(ls), "layers": recs}
            run.destroy()
        rec["other_paths"] = other
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(layers)
    print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
