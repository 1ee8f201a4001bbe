#!/usr/bin/env python3
"""Benchmark of the zero-workspace direct convolution on one MI355X.

A step is one forward pass of every layer of the chosen workload (one
conv_direct_run per layer) on seeded synthetic tensors already resident in HBM.
The default workload is the batched AlexNet-/VGG-shaped layer suite; `--workload
NAME` times a single layer (names: paper_1809_10170_amd/workloads.py).

Prints ONE JSON line: whole-workload TFLOP/s (2*N*K*C*R*S*P*Q per layer / time),
per-layer figures, the roofline record of the kernel that takes the most time, and
the CPU oracle timed on a bounded sample of the same workload on this host.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3     # MI355X: 256 CU x 256 flop/clk x 2.4 GHz
PEAK_HBM_GBPS = 8000.0


def suite(name, workloads):
    if name == "suite_batched":
        return [l for l in workloads.ALL_LAYERS if l.N >= 32]
    if name == "suite_inception":   # GoogLeNet-shaped layers; a suite of its own, not the headline metric
        return list(workloads.INCEPTION)
    if name == "suite_all":
        return list(workloads.ALL_LAYERS)
    return [workloads.BY_NAME[name]]


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
    return {"value": flops / secs / 1e12, "unit": "TFLOP/s", "cores": oracle.threads(),
            "kind": "oracle", "sample": f"single images, full output (the first 4 of each layer, in turn): {sample}",
            "seconds": round(secs, 2)}


def measured_traffic(layer_name, variant):
    """HBM bytes per launch of a layer's kernel from the committed rocprofv3 --pmc summary
    (FETCH_SIZE and WRITE_SIZE scaled by the copy-kernel calibration stated there), or
    None if the summary has no row for this layer and kernel variant."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.md")
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
    ap.add_argument("--check", action="store_true", help="also verify sampled outputs against the oracle")
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
    dgrad = args.direction == "dgrad"
    wgrad = args.direction == "wgrad"
    if (dgrad or wgrad) and blocked:
        sys.exit("bench.py: the gradients run in plain layouts")
    if dgrad and len(layers) > 1:
        # a suite: the layers whose data gradient runs on the compiled kernels (stride 1, or a strided layer as one
        # small convolution per phase), first layers left out (no network needs the gradient of its input image);
        # a layer named alone runs whatever its path
        layers = [l for l in layers if l.R == l.S and l.pad <= l.R - 1 and l.C >= 16]
    if not layers:
        sys.exit("bench.py: no layer left to run")
    dev = torch.device("cuda:0")

    items = []
    for l in layers:
        x, w = workloads.make_inputs(l)
        xd, wd = torch.from_numpy(x).to(dev), torch.from_numpy(w).to(dev)
        if wgrad:
            g = torch.Generator(device="cpu").manual_seed(4242 + l.K)
            dy = (torch.rand((l.N, l.K, l.P, l.Q), generator=g) * 2 - 1).to(dev)
            plan = cd.Plan.wgrad(*l.dims())
            dw = torch.empty((l.K, l.C, l.R, l.S), device=dev)
            items.append((l, plan, xd, dy, dw, "wgrad"))
            del x, w
            continue
        if dgrad:
            # dy stands in for the next layer's gradient: U[-1,1], seeded
            g = torch.Generator(device="cpu").manual_seed(4242 + l.K)
            dy = (torch.rand((l.N, l.K, l.P, l.Q), generator=g) * 2 - 1).to(dev)
            plan = cd.Plan.dgrad(*l.dims())
            wt = torch.empty((plan.dgrad_wt_elems(),), device=dev)
            dx = torch.empty((l.N, l.C, l.H, l.W), device=dev)
            items.append((l, plan, dy, wt, dx, wd))
            del x, w
            continue
        li = cd.BLOCKED if blocked and l.C >= 4 else cd.PLAIN
        lo = cd.BLOCKED if blocked else cd.PLAIN
        plan = cd.Plan(*l.dims(), variant=args.variant, in_layout=li, out_layout=lo)
        if li == cd.BLOCKED:   # re-arranged once, outside the timed region (the weights: a one-time cost; the
            xb = torch.empty((l.N, -(-l.C // 4), l.H, l.W, 4), device=dev)       # input: a previous layer's output)
            wb = torch.empty((-(-l.K // 32), -(-l.C // 4), l.R, l.S, 4, 32), device=dev)
            cd.pack_act(xd, xb)
            cd.pack_w(wd, wb)
            torch.cuda.synchronize()
            xd, wd = xb, wb
        oshape = (l.N, -(-l.K // 4), l.P, l.Q, 4) if lo == cd.BLOCKED else (l.N, l.K, l.P, l.Q)
        out = torch.empty(oshape, device=dev, dtype=torch.float32)
        items.append((l, plan, xd, wd, out, None))
        del x, w
    torch.cuda.synchronize()
    alloc_before = torch.cuda.memory_allocated()

    stream = torch.cuda.current_stream()

    def launch(item):
        l, plan, xd, wd, out, w_plain = item
        if isinstance(w_plain, str):   # wgrad: (x, dy) -> dw
            return plan.run_wgrad(xd, wd, out, stream.cuda_stream)
        if w_plain is not None:   # dgrad: the filter transform belongs to the step (weights change every update)
            plan.dgrad_prepare(w_plain, wd, stream.cuda_stream)
        plan.run(xd, wd, out, stream.cuda_stream)

    for _ in range(args.warmup):
        for item in items:
            launch(item)
    torch.cuda.synchronize()

    # per-layer events inside the timed region, on the stream the kernels run on
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in items] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        for i, item in enumerate(items):
            ev[s][i][0].record(stream)
            launch(item)
            ev[s][i][1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    assert torch.cuda.memory_allocated() == alloc_before, "device memory was allocated during the timed region"

    per_layer = []
    for i, (l, plan, xd, wd, out, _) in enumerate(items):
        ms = sorted(ev[s][i][0].elapsed_time(ev[s][i][1]) for s in range(args.steps))
        avg = sum(ms) / len(ms)
        info = plan.info()
        per_layer.append({
            "layer": l.name, "variant": info["variant"], "grid": info["grid"],
            "gflop": round(l.flops / 1e9, 3), "ms_avg": round(avg, 5), "ms_min": round(ms[0], 5),
            "tflops": round(l.flops / (avg * 1e-3) / 1e12, 3),
            "frac_fp32_mfma_peak": round(l.flops / (avg * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS, 4),
            "algorithmic_GBps": round(l.algorithmic_bytes / (avg * 1e-3) / 1e9, 1),
            "workspace_bytes": plan.workspace_bytes(),
        })
    total_flops = sum(l.flops for l in layers)
    ms_per_step = wall * 1e3 / args.steps
    value = total_flops / (ms_per_step * 1e-3) / 1e12

    dom = max(per_layer, key=lambda r: r["ms_avg"])
    kern = {"r": "conv_rows_kernel", "p": "conv_pw_kernel", "w": "conv_wgrad_kernel"}.get(dom["variant"][0], "conv_dma_kernel")
    roofline = {"bound": "mfma", "kernel": f"{kern}<{dom['variant']}>", "layer": dom["layer"],
                "achieved": dom["tflops"], "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": round(dom["tflops"] / PEAK_FP32_MFMA_TFLOPS, 4),
                "launch_ms": dom["ms_avg"], "traffic": measured_traffic(dom["layer"], dom["variant"]),
                "algorithmic_bytes": workloads.BY_NAME[dom["layer"]].algorithmic_bytes}

    if args.check:
        import oracle
        for l, plan, xd, wd, out, w_plain in items:
            if isinstance(w_plain, str):
                # three output channels of dw in full (each costs the oracle a forward pass of one channel)
                import numpy as np
                ks = sorted({0, l.K - 1, l.K // 2})
                want = oracle.conv_wgrad(xd.cpu().numpy(), np.ascontiguousarray(wd.cpu().numpy()[:, ks]), l.R, l.S, l.stride, l.pad)
                err = float(abs(out.cpu().numpy()[ks] - want).max())
                assert err <= 1e-4 * (l.N * l.P * l.Q) ** 0.5, (l.name, err)
                continue
            if w_plain is not None and not (l.stride == 1 and l.R == l.S and l.pad <= l.R - 1):
                # no single-element form for these: two whole images against the oracle's adjoint (images are independent)
                import numpy as np
                dyh, wh = xd.cpu().numpy(), w_plain.cpu().numpy()
                for n in sorted({0, l.N - 1}):
                    want = oracle.conv_dgrad(np.ascontiguousarray(dyh[n:n + 1]), wh, l.H, l.W, l.stride, l.pad)
                    err = float(abs(out[n:n + 1].cpu().numpy() - want).max())
                    assert err <= oracle.tolerance(l.K, l.R, l.S), (l.name, err)
                continue
            if w_plain is not None:
                # sampled dx elements through the flipped-filter identity (pinned on the CPU against the adjoint definition)
                import numpy as np
                rng = np.random.default_rng(5)
                pts = np.stack([rng.integers(0, d, 4000) for d in (l.N, l.C, l.H, l.W)], axis=1).astype(np.int32)
                wt = np.ascontiguousarray(w_plain.cpu().numpy()[:, :, ::-1, ::-1].transpose(1, 0, 2, 3))
                want = oracle.conv_forward_points(xd.cpu().numpy(), wt, pts, 1, l.R - 1 - l.pad)
                got = out.cpu().numpy()[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]]
                err = float(abs(got - want).max())
                assert err <= oracle.tolerance(l.K, l.R, l.S), (l.name, err)
                continue
            pts = workloads.sample_points(l, 4000)
            x, w = workloads.make_inputs(l)
            want = oracle.conv_forward_points(x, w, pts, l.stride, l.pad)
            if plan.out_layout == cd.BLOCKED:
                out = cd.unpack_act(out, torch.empty((l.N, l.K, l.P, l.Q), device=dev))
                torch.cuda.synchronize()
            got = out.cpu().numpy()[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]]
            err = float(abs(got - want).max())
            assert err <= oracle.tolerance(l.C, l.R, l.S), (l.name, err)

    rec = {
        "metric": ("conv wgrad TFLOP/s (2*N*K*C*R*S*P*Q/t), fp32, zero workspace" if wgrad else
                   "conv dgrad TFLOP/s (2*N*K*C*R*S*P*Q/t), fp32, zero workspace" if dgrad else
                   "conv fwd TFLOP/s (2*N*K*C*R*S*P*Q/t), fp32, zero workspace"),
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "direction": args.direction, "layout": args.layout, "layers": [l.name for l in layers],
                   "frac_fp32_mfma_peak": round(value / PEAK_FP32_MFMA_TFLOPS, 4),
                   "workspace_bytes": 0},
        "roofline": roofline,
        "layers": per_layer,
    }
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(layers)
    for _, plan, *_ in items:
        plan.destroy()
    print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
