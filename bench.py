#!/usr/bin/env python3
"""Benchmark of the 2D selective scan on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 2] [--all]

A step is one pass of the scan over one batch of synthetic input (forward; forward + backward
for the training workload).  Inputs are resident in HBM before the timed region; the steps
cycle through several independent buffer sets so that consecutive launches do not hit the
256 MB Infinity Cache.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2412_00678_amd import workloads as wl  # noqa: E402

HBM_PEAK_GBS = 8000.0            # MI355X published HBM3E bandwidth
# fp32 vector peak without packed-FP32 instructions (they are disabled in this build):
# 256 CUs x 4 SIMDs x 16 lanes x 2 flop (FMA) x 2.4 GHz = 78.6 TFLOP/s; the published
# 157.3 TFLOP/s counts two FMAs per lane per clock through the packed forms.
ALU_PEAK_TFLOPS = 78.6
FLOPS_PER_UNIT_FWD = 9.0         # exp + 2 mul + 3 FMA per (position, channel, state)
FLOPS_PER_UNIT_BWD = 32.0        # rebuilt states (7) + two reverse scans and local gradients (25)

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (see profiles/);
# None where no counter run has been recorded for the workload.
MEASURED_TRAFFIC_BYTES = {
    # forward: FETCH_SIZE 49,475 KiB x 2.00 (copy-kernel scale) + WRITE_SIZE 32,768 KiB x 1.00 per launch
    "wsi_256x256_bf16_mask50": int((49475 * 2.0 + 32768) * 1024),
}


def device_sets(s2d, inp, dtype, nsets, backward):
    import torch
    base = s2d.to_device(inp, dtype)
    sets = [base]
    for _ in range(nsets - 1):
        sets.append({k: (None if v is None else v.clone()) for k, v in base.items()})
    for s in sets:
        s["y"] = torch.empty_like(s["x"])
    return sets


def time_launches(fn, sets, steps, warmup):
    """Average duration of one launch in ms, from events on the launch stream."""
    import torch
    for i in range(warmup):
        fn(sets[i % len(sets)])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        fn(sets[i % len(sets)])
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return e0.elapsed_time(e1) / steps, wall_ms / steps


def bench_workload(s2d, w, steps, warmup, with_bwd, force_sets=None):
    import torch
    inp = wl.make_inputs(w, seed=0)
    set_bytes = w.fwd_bytes() + (w.bwd_bytes() if with_bwd else 0)
    nsets = int(min(16, max(2, np.ceil(1.2e9 / set_bytes))))
    free, _ = torch.cuda.mem_get_info()
    nsets = int(max(1, min(nsets, free // (4 * set_bytes))))
    if force_sets:
        nsets = int(force_sets)
    sets = device_sets(s2d, inp, w.dtype, nsets, with_bwd)
    desc = s2d.make_desc(sets[0]["x"], sets[0]["A"])
    wf = s2d.workspace_bytes(desc, s2d.PASS_FWD)
    ws_f = torch.empty(max(wf, 16), dtype=torch.uint8, device="cuda:0")

    def fwd(s):
        s2d.scan2d_fwd(s["x"], s["delta"], s["A"], s["Bm"], s["Cm"], s["Dskip"], s["mask"], y=s["y"], workspace=ws_f)

    ms_f, wall_f = time_launches(fwd, sets, steps, warmup)
    out = {"workload": w.name, "shape": [w.Bt, w.Dc, w.N, w.H, w.W], "dtype": "bf16" if w.dtype == wl.BF16 else "fp32",
           "buffer_sets": nsets, "fwd_ms": ms_f, "fwd_gunits_s": w.units / ms_f / 1e6,
           "fwd_algorithmic_GBs": w.fwd_bytes() / ms_f / 1e6, "fwd_bytes": w.fwd_bytes()}
    if with_bwd:
        wb = s2d.workspace_bytes(desc, s2d.PASS_BWD)
        ws_b = torch.empty(max(wb, 16), dtype=torch.uint8, device="cuda:0")

        def bwd(s):
            s2d.scan2d_bwd(s["x"], s["delta"], s["A"], s["Bm"], s["Cm"], s["Dskip"], s["mask"], s["dy"], workspace=ws_b)

        ms_b, _ = time_launches(bwd, sets, max(3, steps // 8), max(1, warmup // 8))
        out.update({"bwd_ms": ms_b, "bwd_gunits_s": w.units / ms_b / 1e6, "bwd_algorithmic_GBs": w.bwd_bytes() / ms_b / 1e6,
                    "fwd_bwd_gunits_s": w.units / (ms_f + ms_b) / 1e6, "bwd_workspace_bytes": wb})
    del sets
    torch.cuda.empty_cache()
    return out, inp


def bench_softplus(s2d, w, steps, warmup):
    """scan2d_fwd_softplus (and scan2d_bwd_softplus for the training workload) on the workload's tensors."""
    import torch
    inp = wl.make_inputs(w, seed=0)
    set_bytes = w.fwd_bytes() + (w.bwd_bytes() if w.backward else 0)
    nsets = int(min(16, max(2, np.ceil(1.2e9 / set_bytes))))
    sets = device_sets(s2d, inp, w.dtype, nsets, w.backward)
    bias = torch.zeros(w.Dc, dtype=torch.float32, device="cuda:0")
    desc = s2d.make_desc(sets[0]["x"], sets[0]["A"])
    ws_f = torch.empty(max(s2d.workspace_bytes(desc, s2d.PASS_FWD), 16), dtype=torch.uint8, device="cuda:0")

    def fwd(s):
        s2d.scan2d_fwd_softplus(s["x"], s["delta"], bias, s["A"], s["Bm"], s["Cm"], s["Dskip"], s["mask"], y=s["y"], workspace=ws_f)

    ms_f, _ = time_launches(fwd, sets, steps, warmup)
    out = {"fwd_ms": ms_f, "fwd_gunits_s": w.units / ms_f / 1e6}
    if w.backward:
        ws_b = torch.empty(max(s2d.workspace_bytes(desc, s2d.PASS_BWD_SOFTPLUS), 16), dtype=torch.uint8, device="cuda:0")

        def bwd(s):
            s2d.scan2d_bwd_softplus(s["x"], s["delta"], bias, s["A"], s["Bm"], s["Cm"], s["Dskip"], s["mask"], s["dy"], workspace=ws_b)

        ms_b, _ = time_launches(bwd, sets, max(3, steps // 8), max(1, warmup // 8))
        out.update({"bwd_ms": ms_b, "bwd_gunits_s": w.units / ms_b / 1e6})
    return out


def bench_gated(s2d, w, steps, warmup):
    """scan2d_fwd_softplus_gated (training form: both outputs written; and scan2d_bwd_softplus_gated for the
    training workload) on the workload's tensors plus a gate branch z."""
    import torch
    inp = wl.make_inputs(w, seed=0)
    set_bytes = w.fwd_bytes() + (w.bwd_bytes() if w.backward else 0)
    nsets = int(min(16, max(2, np.ceil(1.2e9 / set_bytes))))
    sets = device_sets(s2d, inp, w.dtype, nsets, w.backward)
    g = torch.Generator(device="cuda:0").manual_seed(7)
    for s in sets:
        s["z"] = (2.0 * torch.randn(s["x"].shape, device="cuda:0", generator=g)).to(s["x"].dtype)
        s["y_scan"] = torch.empty_like(s["x"])
    bias = torch.zeros(w.Dc, dtype=torch.float32, device="cuda:0")
    desc = s2d.make_desc(sets[0]["x"], sets[0]["A"])
    ws_f = torch.empty(max(s2d.workspace_bytes(desc, s2d.PASS_FWD), 16), dtype=torch.uint8, device="cuda:0")

    def fwd(s):
        s2d.scan2d_fwd_softplus_gated(s["x"], s["delta"], bias, s["A"], s["Bm"], s["Cm"], s["Dskip"], s["mask"], s["z"],
                                      workspace=ws_f, y=s["y"], y_scan=s["y_scan"])

    def fwd_infer(s):
        s2d.scan2d_fwd_softplus_gated(s["x"], s["delta"], bias, s["A"], s["Bm"], s["Cm"], s["Dskip"], s["mask"], s["z"],
                                      want_y_scan=False, workspace=ws_f, y=s["y"])

    ms_f, _ = time_launches(fwd, sets, steps, warmup)
    ms_i, _ = time_launches(fwd_infer, sets, steps, warmup)
    out = {"fwd_ms": ms_f, "fwd_gunits_s": w.units / ms_f / 1e6, "fwd_without_y_scan_ms": ms_i}
    if w.backward:
        ws_b = torch.empty(max(s2d.workspace_bytes(desc, s2d.PASS_BWD_GATED), 16), dtype=torch.uint8, device="cuda:0")

        def bwd(s):
            s2d.scan2d_bwd_softplus_gated(s["x"], s["delta"], bias, s["A"], s["Bm"], s["Cm"], s["Dskip"], s["mask"], s["z"],
                                          s["y_scan"], s["dy"], workspace=ws_b)

        ms_b, _ = time_launches(bwd, sets, max(3, steps // 8), max(1, warmup // 8))
        out.update({"bwd_ms": ms_b, "bwd_gunits_s": w.units / ms_b / 1e6})
    return out


def cpu_baseline(w, inp):
    """The oracle as it stands, all host cores, forward of the same workload repeated for ~10 s."""
    import oracle
    cores = oracle.num_procs()

    def once():
        t0 = time.perf_counter()
        oracle.scan2d_fwd(inp["x"], inp["delta"], inp["A"], inp["Bm"], inp["Cm"], inp["Dskip"], inp["mask"],
                          dtype=w.dtype, threads=cores)
        return time.perf_counter() - t0

    first = once()
    reps = int(min(200, max(1, round(10.0 / max(first, 1e-3)))))
    total = sum(once() for _ in range(reps))
    return {"value": w.units * reps / total / 1e9, "unit": "G(pos*ch*state)/s", "cores": cores, "kind": "oracle",
            "sample": f"{reps} forward passes of {w.name} ({w.units} units each) in {total:.2f} s, all host cores"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", type=int, default=2, help="index into the five configurations (default: the 256x256 WSI grid)")
    ap.add_argument("--all", action="store_true", help="also time the other configurations (reported under 'others')")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--gated", action="store_true",
                    help="also time the block form: softplus step and output gate y * SiLU(z) in the kernels, reported under 'gated'")
    ap.add_argument("--softplus", action="store_true",
                    help="also time the entry points that compute the step themselves, delta = softplus(raw + bias) "
                         "(same tensors, delta read as the raw projection), reported under 'softplus'")
    ap.add_argument("--paper-shapes", action="store_true",
                    help="also time the grids the paper times (14x14, 56x56, 200x200; N = 16): 128-channel maps and "
                         "batches of single-channel maps, reported under 'paper_shapes' as feature maps per second")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: the scan shards over channels with no exchange in forward; "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    from paper_2412_00678_amd import scan2d as s2d   # raises if the library is missing

    torch.cuda.set_device(0)
    w = wl.CONFIGS[args.workload]
    res, inp = bench_workload(s2d, w, args.steps, args.warmup, with_bwd=w.backward)
    ms = res["fwd_ms"] + res.get("bwd_ms", 0.0)
    flops = w.units * (FLOPS_PER_UNIT_FWD + (FLOPS_PER_UNIT_BWD if w.backward else 0.0))
    alu = flops / (ms * 1e-3) / 1e12
    hbm_bytes = w.fwd_bytes() + (w.bwd_bytes() if w.backward else 0)
    hbm = hbm_bytes / (ms * 1e-3) / 1e9
    traffic = MEASURED_TRAFFIC_BYTES.get(w.name)
    line = {
        "metric": "2D-scan G(pos*ch*state)/s (forward; forward+backward for the training workload)",
        "value": w.units / ms / 1e6, "unit": "G(pos*ch*state)/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "shape_Bt_Dc_N_H_W": [w.Bt, w.Dc, w.N, w.H, w.W],
                   "storage": res["dtype"], "pass": "fwd+bwd" if w.backward else "fwd", "buffer_sets": res["buffer_sets"]},
        # the kernel issues ~15 fp32 VALU instructions per unit against 0.39 algorithmic bytes:
        # the vector ALU, not HBM, is the roof that binds; both are reported
        "roofline": {"bound": "alu", "achieved": alu, "peak": ALU_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": alu / ALU_PEAK_TFLOPS, "traffic": traffic},
        "roofline_hbm": {"bound": "hbm", "achieved": hbm, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": hbm / HBM_PEAK_GBS, "algorithmic_bytes": hbm_bytes, "traffic": traffic},
        "detail": res,
    }
    if args.all:
        others = []
        for k, ow in enumerate(wl.CONFIGS):
            if k == args.workload:
                continue
            r, _ = bench_workload(s2d, ow, max(20, args.steps // 3), max(5, args.warmup // 3), with_bwd=ow.backward)
            others.append(r)
        line["others"] = others
    if args.gated:
        line["gated"] = bench_gated(s2d, w, max(20, args.steps // 3), max(5, args.warmup // 3))
    if args.softplus:
        line["softplus"] = bench_softplus(s2d, w, max(20, args.steps // 3), max(5, args.warmup // 3))
    if args.paper_shapes:
        rows = []
        for side in (14, 56, 200):
            for label, Bt, Dc in (("128-channel map, batch 8", 8, 128), ("single-channel maps, batch 4096", 4096, 1)):
                pw = wl.Workload(f"paper_{side}x{side}_{Dc}ch", Bt, Dc, 16, side, side, wl.F32)
                r, _ = bench_workload(s2d, pw, max(20, args.steps // 3), max(5, args.warmup // 3), with_bwd=False)
                rows.append({"grid": side, "what": label, "fwd_ms": r["fwd_ms"], "maps_per_s": Bt / (r["fwd_ms"] * 1e-3),
                             "gunits_s": r["fwd_gunits_s"], "algorithmic_GBs": r["fwd_algorithmic_GBs"],
                             "hbm_frac": r["fwd_algorithmic_GBs"] / HBM_PEAK_GBS})
        line["paper_shapes"] = rows
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(w, inp)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
