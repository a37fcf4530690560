"""Text summaries of rocprofv3 runs of bench.py, and the traffic record that bench.py reports.

    python -m paper_2412_00678_amd.profile_summary commands RUNS   # prints the rocprofv3 command lines, one per run
    python -m paper_2412_00678_amd.profile_summary write RUNS      # reads RUNS/*, writes profiles/*.md and profiles/traffic.json

`commands` prints one shell line per run (kernel trace, FETCH_SIZE, WRITE_SIZE and issue counters, each a run
of its own, plus the copy-kernel runs that calibrate the two size counters); run them on the GPU from /tmp with
TMPDIR=/tmp.  `write` turns the result databases into short tables.  Everything in the written files is a measured
or derived figure, the plan strings come from the library (scan2d_describe_plan via bench.py's JSON line), and
profiles/traffic.json carries the sha256 of the kernel sources it was measured on: bench.py reports `traffic`
only while that hash still matches.
"""
from __future__ import annotations

import json
import os
import re
import sqlite3
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROFILES = os.path.join(ROOT, "profiles")
SQ = ("SQ_INSTS_VALU SQ_INSTS_SALU SQ_INSTS_LDS SQ_INSTS_VMEM_RD SQ_WAVE_CYCLES SQ_BUSY_CYCLES SQ_WAIT_INST_ANY "
      "SQ_ACTIVE_INST_VALU")
SIMDS = 1024                     # 256 compute units x 4 SIMDs
COPY_KIB = 1048576.0             # roofprobe --copy moves 2^30 bytes each way per launch

# run name -> (rocprofv3 options, program and its arguments, file that takes the program's stdout or None)
TRACE_STEPS = {1: "--steps 300 --warmup 200", 2: "--steps 300 --warmup 200", 3: "--steps 200 --warmup 100", 4: "--steps 40 --warmup 20"}
PMC_STEPS = {1: "--steps 20 --warmup 4", 2: "--steps 20 --warmup 4", 3: "--steps 12 --warmup 4", 4: "--steps 8 --warmup 4"}


def runs():
    out = []
    for w in (1, 2, 3, 4):
        b = f"python3 bench.py --no-cpu --workload {w}"
        out.append((f"trace_{w}", "--kernel-trace --stats", f"{b} {TRACE_STEPS[w]}", f"trace_{w}.json"))
        out.append((f"fetch_{w}", "--pmc FETCH_SIZE", f"{b} {PMC_STEPS[w]}", None))
        out.append((f"write_{w}", "--pmc WRITE_SIZE", f"{b} {PMC_STEPS[w]}", None))
        out.append((f"sq_{w}", f"--pmc {SQ}", f"{b} {PMC_STEPS[w]}", None))
    out.append(("grbm_2", "--pmc GRBM_GUI_ACTIVE", "python3 bench.py --no-cpu --workload 2 --steps 20 --warmup 4", None))
    out.append(("trace_all", "--kernel-trace --stats", "python3 bench.py --no-cpu --all --paper-shapes --steps 300 --warmup 200", "trace_all.json"))
    out.append(("trace_block", "--kernel-trace --stats", "python3 bench.py --no-cpu --workload 4 --softplus --gated --steps 40 --warmup 8",
                "trace_block.json"))
    # the same two commands without the profiler: kernel tracing adds several microseconds to every launch
    out.append(("plain_all", None, "python3 bench.py --no-cpu --all --paper-shapes --steps 300 --warmup 200", "plain_all.json"))
    out.append(("plain_block", None, "python3 bench.py --no-cpu --workload 4 --softplus --gated --steps 40 --warmup 8", "plain_block.json"))
    # the producers in front of the scan (convolution + SiLU, projections) and the chain into the gated scan
    for w in (2, 3):
        b = f"python3 bench.py --no-cpu --block --workload {w} --steps 150 --warmup 100"
        out.append((f"trace_producers_{w}", "--kernel-trace --stats", b, f"trace_producers_{w}.json"))
        out.append((f"plain_producers_{w}", None, b, f"plain_producers_{w}.json"))
    out.append(("fetch_copy", "--pmc FETCH_SIZE", "./paper_2412_00678_amd/roofprobe --copy 5", None))
    out.append(("write_copy", "--pmc WRITE_SIZE", "./paper_2412_00678_amd/roofprobe --copy 5", None))
    return out


def command(run, runs_dir):
    name, opts, prog, stdout = run
    prog = prog.replace("bench.py", os.path.join(ROOT, "bench.py")).replace("./paper_2412_00678_amd", os.path.join(ROOT, "paper_2412_00678_amd"))
    line = prog if opts is None else f"rocprofv3 {opts} -d {runs_dir}/{name} -o r -- {prog}"
    return line + (f" > {runs_dir}/{stdout}" if stdout else " > /dev/null")


def shown(run):
    """The command as the summaries quote it: relative paths, output folder elided."""
    name, opts, prog, _ = run
    if opts is None:
        return prog
    return f"cd /tmp && export TMPDIR=/tmp && rocprofv3 {opts} -d <out>/{name} -o r -- {prog}"


def db_path(runs_dir, name):
    for base, _, files in os.walk(os.path.join(runs_dir, name)):
        for f in files:
            if f.endswith("_results.db"):
                return os.path.join(base, f)
    raise FileNotFoundError(f"no rocprofv3 database under {runs_dir}/{name}")


def query(path, sql, args=()):
    con = sqlite3.connect(path)
    try:
        return con.execute(sql, args).fetchall()
    finally:
        con.close()


def short(name: str) -> str:
    """Kernel name without return type, namespaces and parameter list; template arguments stay."""
    n = name.replace("void ", "").replace("scan2d::(anonymous namespace)::", "").replace("scan2d::", "")
    depth = 0
    for k, ch in enumerate(n):
        depth += ch == "<"
        depth -= ch == ">"
        if ch == "(" and depth == 0:
            return n[:k]
    return n


def kernel_table(runs_dir, name):
    rows = query(db_path(runs_dir, name), "select name,total_calls,total_duration,average,percentage from top_kernels")
    out = ["| kernel | calls | total (us) | average (us) | % |", "|---|---|---|---|---|"]
    for n, calls, total, avg, pct in rows:
        out.append(f"| `{short(n)[:110]}` | {calls} | {total:.1f} | {avg:.2f} | {pct:.2f} |")
    return "\n".join(out)


def counters(runs_dir, name, like="%scan2d%"):
    """{kernel: {counter: (mean per dispatch, dispatches, mean duration in us)}}"""
    rows = query(db_path(runs_dir, name),
                 "select kernel_name,counter_name,avg(value),count(*),avg(duration) from counters_collection "
                 "where kernel_name like ? group by kernel_name,counter_name", (like,))
    out = {}
    for n, cn, v, k, d in rows:
        out.setdefault(short(n), {})[cn] = (v, k, d / 1e3)
    return out


def pair_weights(table):
    """Launches per reported step for a run of the training workload, which times scan2d_fwd + scan2d_bwd and then the
    training pair scan2d_fwd_saving + scan2d_bwd_saved (the reported step): the plain forward and the checkpoint sweep
    are not part of the pair, the kernels both backward calls share run once per step.  None for other runs."""
    def keepy(k):                                         # <T, LG, K, NW, NG, WAVES, RPB, SP, UA, CK, CF, KEEPY, GATE>
        args = k[k.index("<") + 1:k.rindex(">")].split(", ")
        return len(args) >= 12 and args[11] == "true"
    saving = [k for k in table if k.startswith("scan2d_fwd_shared_kernel") and keepy(k)]
    if not saving:
        return None
    w = {}
    for k in table:
        if k.startswith("scan2d_fwd_shared_kernel"):
            w[k] = 1.0 if k in saving else 0.0
        else:
            w[k] = 0.5                                    # dispatched by scan2d_bwd and by scan2d_bwd_saved
    return w


def per_step(table, counter):
    """Sum over kernels of (mean per dispatch x dispatches per step).  A step is one bench.py step; the kernel
    with the fewest dispatches runs once per step and every other count must be a multiple of it."""
    counts = {k: v[counter][1] for k, v in table.items() if counter in v}
    steps = min(counts.values())
    weights = pair_weights(table)
    total, rows = 0.0, []
    for k, c in sorted(counts.items()):
        if c % steps:
            raise ValueError(f"{k}: {c} dispatches is not a multiple of {steps} steps")
        mean, _, dur = table[k][counter]
        n = (c // steps) * (weights[k] if weights else 1.0)
        total += mean * n
        rows.append((k, n, mean, dur))
    return total, rows, steps


def copy_scales(runs_dir):
    f = counters(runs_dir, "fetch_copy", "%k_copy%")
    w = counters(runs_dir, "write_copy", "%k_copy%")
    fetch = next(iter(f.values()))["FETCH_SIZE"][0]
    write = next(iter(w.values()))["WRITE_SIZE"][0]
    return COPY_KIB / fetch, COPY_KIB / write, fetch, write


def clock_ghz(runs_dir):
    t = counters(runs_dir, "grbm_2")
    k = max(t, key=lambda n: t[n]["GRBM_GUI_ACTIVE"][2])
    cycles, _, us = t[k]["GRBM_GUI_ACTIVE"]
    return cycles / 8.0 / us / 1e3, k                      # the counter sums the 8 XCDs


def workload_summary(runs_dir, w, bench, fs, ws, ghz):
    """Per-kernel rows and per-step totals of one bench.py workload."""
    units = bench["detail"]["shape"]
    units = units[0] * units[1] * units[2] * units[3] * units[4]
    fe, wr, sq = counters(runs_dir, f"fetch_{w}"), counters(runs_dir, f"write_{w}"), counters(runs_dir, f"sq_{w}")
    fetch_kib, frows, _ = per_step(fe, "FETCH_SIZE")
    write_kib, wrows, _ = per_step(wr, "WRITE_SIZE")
    valu, vrows, _ = per_step(sq, "SQ_INSTS_VALU")
    wmap = {k: (n, m) for k, n, m, _ in wrows}
    vmap = {k: (m, d) for k, _, m, d in vrows}
    lines = ["| kernel | launches per step | duration (us) | VALU lane-instructions per unit | VALU utilisation | HBM read (MB) | HBM written (MB) |",
             "|---|---|---|---|---|---|---|"]
    for k, n, mean, dur in frows:
        v, vd = vmap.get(k, (0.0, dur))
        util = v * 4.0 / SIMDS / (ghz * 1e3) / vd if vd else 0.0
        lines.append(f"| `{k[:100]}` | {n:g} | {vd:.1f} | {v * 64 * max(n, 1) / units:.2f} | {100 * util:.0f} % | {mean * fs * 1024 / 1e6:.1f} | "
                     f"{wmap[k][1] * ws * 1024 / 1e6:.1f} |")
    rec = {"hbm_bytes_per_launch": int(round((fetch_kib * fs + write_kib * ws) * 1024)),
           "hbm_read_bytes": int(round(fetch_kib * fs * 1024)), "hbm_written_bytes": int(round(write_kib * ws * 1024)),
           "fetch_size_kib_raw": fetch_kib, "write_size_kib_raw": write_kib, "fetch_scale": fs, "write_scale": ws,
           "valu_lane_instructions_per_unit": valu * 64 / units, "units_per_launch": units,
           "commands": [shown(r) for r in runs() if r[0] in (f"fetch_{w}", f"write_{w}", f"sq_{w}", "fetch_copy", "write_copy")]}
    return "\n".join(lines), rec


def raw_counter_table(runs_dir, name):
    t = counters(runs_dir, name)
    out = ["| kernel | counter | mean per dispatch | dispatches | mean duration (us) |", "|---|---|---|---|---|"]
    for k in sorted(t):
        for cn in sorted(t[k]):
            v, n, d = t[k][cn]
            out.append(f"| `{k[:90]}` | {cn} | {v:.6g} | {n} | {d:.2f} |")
    return "\n".join(out)


# sources that the recorded workloads (scan2d_fwd / scan2d_bwd on the benchmark configurations) do not run: the probe
# and the layers around the scan
NOT_IN_DIGEST = ("roofprobe", "scan2d_block", "scan2d_pool", "scan2d_linear", "scan2d_norm")


def kernel_source_digest() -> str:
    """sha256 over the sources of the scan kernels and their dispatcher: traffic.json is valid while it matches."""
    import hashlib
    h = hashlib.sha256()
    src = os.path.join(ROOT, "paper_2412_00678_amd", "csrc")
    for name in sorted(os.listdir(src)):
        if name.endswith((".hip", ".hpp")) and not name.startswith(NOT_IN_DIGEST):
            h.update(name.encode())
            with open(os.path.join(src, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()


def plans(detail):
    out = [f"- forward: `{detail['fwd_plan']}`"]
    if "bwd_plan" in detail:
        out.append(f"- backward: `{detail['bwd_plan']}`")
    return "\n".join(out)


def write(runs_dir):
    by_name = {r[0]: r for r in runs()}
    fs, ws, fetch_copy, write_copy = copy_scales(runs_dir)
    ghz, clock_kernel = clock_ghz(runs_dir)
    traffic = {"kernel_source_sha256": kernel_source_digest(), "clock_ghz": ghz, "workloads": {}}
    titles = {1: ("scan2d_fwd_wsi64_fp32.md", "scan2d_fwd on the 64x64 fp32 WSI grid with 40 % of the positions masked (configuration 1)"),
              2: ("scan2d_fwd_wsi256_bf16.md", "scan2d_fwd on the 256x256 bf16 WSI grid (configuration 2)"),
              3: ("scan2d_fwd_vmamba56_bf16.md", "scan2d_fwd on the 56x56 bf16 backbone stage, batch 32 (configuration 3)"),
              4: ("scan2d_train128x192_fp32.md", "scan2d_fwd + scan2d_bwd on the 128x192 fp32 training configuration (configuration 4)")}
    for w, (fname, title) in titles.items():
        with open(os.path.join(runs_dir, f"trace_{w}.json")) as f:
            bench = json.loads(f.read().strip().splitlines()[-1])
        table, rec = workload_summary(runs_dir, w, bench, fs, ws, ghz)
        d = bench["detail"]
        rec["algorithmic_bytes"] = bench["roofline"]["algorithmic_bytes"]
        traffic["workloads"][d["workload"]] = rec
        timing = f"forward {d['fwd_ms'] * 1e3:.1f} us (median {d['fwd_ms_median'] * 1e3:.1f}, minimum {d['fwd_ms_min'] * 1e3:.1f})"
        if "bwd_ms" in d:
            timing += f", backward {d['bwd_ms'] * 1e3:.1f} us (median {d['bwd_ms_median'] * 1e3:.1f}, minimum {d['bwd_ms_min'] * 1e3:.1f})"
        if "pair_fwd_ms" in d:
            timing += (f"; training pair (the reported step; launches per step below are those of the pair): scan2d_fwd_saving "
                       f"{d['pair_fwd_ms'] * 1e3:.1f} us, scan2d_bwd_saved {d['pair_bwd_ms'] * 1e3:.1f} us, "
                       f"{d['pair_saved_bytes'] / 1e6:.0f} MB of checkpoints handed over")
        with open(os.path.join(PROFILES, fname), "w") as f:
            f.write(f"""# {title}

Plans (scan2d_describe_plan):

{plans(d)}

## Kernel trace

`{shown(by_name[f'trace_{w}'])}`

{kernel_table(runs_dir, f'trace_{w}')}

bench.py's own event timing in the same run: {timing} per step.  The kernel averages above include the run's second
pass over a single buffer set (inputs resident in the Infinity Cache), so they sit between the two figures bench.py
prints.

## Issue counters and HBM traffic per kernel

`{shown(by_name[f'sq_{w}'])}`, and the same command with `--pmc FETCH_SIZE` and with `--pmc WRITE_SIZE` (KiB per
dispatch, scaled x{fs:.3f} / x{ws:.3f}: what a copy kernel of known size reads on the same counters, see
roofprobe_mi355x.md).  A unit is one (position, channel, state): {rec['units_per_launch']:,} per launch.  VALU
utilisation = wavefront instructions x 4 cycles / {SIMDS} SIMDs / {ghz:.2f} GHz / duration.

{table}

Per step: {rec['hbm_read_bytes'] / 1e6:.1f} MB read + {rec['hbm_written_bytes'] / 1e6:.1f} MB written =
{rec['hbm_bytes_per_launch'] / 1e6:.1f} MB of HBM traffic against {rec['algorithmic_bytes'] / 1e6:.1f} MB algorithmic
({rec['hbm_bytes_per_launch'] / rec['algorithmic_bytes']:.2f}x); {rec['valu_lane_instructions_per_unit']:.2f} VALU
lane-instructions per unit over all kernels of the step.

## Raw counters

{raw_counter_table(runs_dir, f'sq_{w}')}
""")
    with open(os.path.join(PROFILES, "traffic.json"), "w") as f:
        json.dump(traffic, f, indent=1, sort_keys=True)
        f.write("\n")

    probe_path = os.path.join(runs_dir, "roofprobe.txt")
    probe = open(probe_path).read().strip() if os.path.exists(probe_path) else "(not run)"
    with open(os.path.join(PROFILES, "roofprobe_mi355x.md"), "w") as f:
        f.write(f"""# Roofline probe and counter calibration on the MI355X box

`./paper_2412_00678_amd/roofprobe` (built by `python -m paper_2412_00678_amd.build`):

```
{probe}
```

256 CUs x 64 lanes x 2.4 GHz = 39.3 T lane-op/s is the nominal fp32 vector issue ceiling (78.6 TFLOP/s counting an
FMA as two); the clock measured under the forward kernel (`{shown(by_name['grbm_2'])}`, counter summed over
the 8 XCDs, kernel `{clock_kernel[:60]}`) was {ghz:.2f} GHz.

## Counter calibration (copy kernel, 2^30 bytes read and 2^30 bytes written per launch)

`{shown(by_name['fetch_copy'])}` and `{shown(by_name['write_copy'])}`

| counter | mean per dispatch (KiB) | true KiB | scale factor |
|---|---|---|---|
| FETCH_SIZE | {fetch_copy:,.0f} | 1,048,576 | {fs:.3f} |
| WRITE_SIZE | {write_copy:,.0f} | 1,048,576 | {ws:.3f} |
""")

    with open(os.path.join(runs_dir, "plain_all.json")) as f:
        ball = json.loads(f.read().strip().splitlines()[-1])
    rows = ["| workload | pass | plan | time by bench.py events (us) | G units/s | algorithmic GB/s |", "|---|---|---|---|---|---|"]
    for r in [ball["detail"]] + ball["others"]:
        rows.append(f"| {r['workload']} | fwd | `{r['fwd_plan']}` | {r['fwd_ms'] * 1e3:.1f} | {r['fwd_gunits_s']:.0f} | {r['fwd_algorithmic_GBs']:.0f} |")
        if "bwd_ms" in r:
            rows.append(f"| {r['workload']} | bwd | `{r['bwd_plan']}` | {r['bwd_ms'] * 1e3:.1f} | {r['bwd_gunits_s']:.0f} | {r['bwd_algorithmic_GBs']:.0f} |")
    prow = ["| grid | maps | time (us) | feature maps/s | G units/s | algorithmic GB/s |", "|---|---|---|---|---|---|"]
    for r in ball["paper_shapes"]:
        prow.append(f"| {r['grid']}x{r['grid']} | {r['what']} | {r['fwd_ms'] * 1e3:.1f} | {r['maps_per_s']:.0f} | {r['gunits_s']:.0f} | {r['algorithmic_GBs']:.0f} |")
    with open(os.path.join(PROFILES, "scan2d_all_workloads.md"), "w") as f:
        f.write(f"""# Every configuration and the paper's timed grids in one process

`{shown(by_name['trace_all'])}`

One process times all workloads, so a kernel instantiation that serves several workloads shows their average.

{kernel_table(runs_dir, 'trace_all')}

Timings by bench.py's own events on the launch stream, from the same command without the profiler
(`{shown(by_name['plain_all'])}`; kernel tracing adds several microseconds to every launch, which would double the
figures of the workloads that take a dozen microseconds):

""" + "\n".join(rows) + """

Grids of the paper's speed table (N = 16, fp32):

""" + "\n".join(prow) + "\n")

    with open(os.path.join(runs_dir, "plain_block.json")) as f:
        bb = json.loads(f.read().strip().splitlines()[-1])
    us = lambda d, k: f"{d[k] * 1e3:.0f}"
    with open(os.path.join(PROFILES, "scan2d_block_form_train128x192_fp32.md"), "w") as f:
        f.write(f"""# The block form on the 128x192 fp32 training configuration: softplus step and output gate

`{shown(by_name['trace_block'])}`

One process times the plain, the softplus and the gated entry points one after the other.

{kernel_table(runs_dir, 'trace_block')}

bench.py's own event timings, from the same command without the profiler (us per call):

| entry points | forward | backward |
|---|---|---|
| scan2d_fwd / scan2d_bwd | {us(bb['detail'], 'fwd_ms')} | {us(bb['detail'], 'bwd_ms')} |
| scan2d_fwd_softplus / scan2d_bwd_softplus | {us(bb['softplus'], 'fwd_ms')} | {us(bb['softplus'], 'bwd_ms')} |
| scan2d_fwd_softplus_gated (y_scan and y / y only) / scan2d_bwd_softplus_gated | {us(bb['gated'], 'fwd_ms')} / {us(bb['gated'], 'fwd_without_y_scan_ms')} | {us(bb['gated'], 'bwd_ms')} |
""")


def write_producers(runs_dir, by_name):
    names = {2: "scan2d_block_producers_wsi256_bf16.md", 3: "scan2d_block_producers_vmamba56_bf16.md"}
    for w, fname in names.items():
        with open(os.path.join(runs_dir, f"plain_producers_{w}.json")) as f:
            bench = json.loads(f.read().strip().splitlines()[-1])
        blk = bench["block"]
        rows = ["| step | time by bench.py events (us) | algorithmic MB | GB/s | % of 8 TB/s |", "|---|---|---|---|---|"]
        for key, label in (("conv_silu", "scan2d_block_conv_silu (3x3 depth-wise + SiLU)"), ("xproj", "scan2d_block_xproj (step, B, C projections)")):
            r = blk[key + "_roofline"]
            rows.append(f"| {label} | {blk[key + '_ms'] * 1e3:.1f} | {r['algorithmic_bytes'] / 1e6:.1f} | {r['achieved']:.0f} | {100 * r['frac']:.1f} |")
        rows.append(f"| scan2d_fwd_softplus_gated on their outputs | {blk['gated_scan_ms'] * 1e3:.1f} | | | |")
        rows.append(f"| the three calls back to back | {blk['chain_ms'] * 1e3:.1f} | | | |")
        r = blk["norm_roofline"]
        rows.append(f"| scan2d_block_norm (layer norm over the {blk['model_width']} channels of the model width) | {blk['norm_ms'] * 1e3:.1f} | {r['algorithmic_bytes'] / 1e6:.1f} | {r['achieved']:.0f} | {100 * r['frac']:.1f} |")
        for key, label in (("in_proj", f"scan2d_block_linear, model width {blk['model_width']} -> inner width (one of the two input projections)"),
                           ("out_proj", "scan2d_block_linear, inner width -> model width, plus the skip connection")):
            r = blk[key + "_roofline"]
            rows.append(f"| {label} ({blk[key + '_tflops']:.0f} TFLOP/s) | {blk[key + '_ms'] * 1e3:.1f} | {r['algorithmic_bytes'] / 1e6:.1f} | {r['achieved']:.0f} | {100 * r['frac']:.1f} |")
        rows.append(f"| the whole block forward: layer norm, two input projections, convolution, projections, gated scan, output projection | {blk['whole_block_ms'] * 1e3:.1f} | | | |")
        r = blk["attn_pool_roofline"]
        rows.append(f"| scan2d_block_attn_pool (M = {blk['attn_pool_shape']['M']} channels, D = {blk['attn_pool_shape']['D']} hidden units; three launches) | "
                    f"{blk['attn_pool_ms'] * 1e3:.1f} | {r['algorithmic_bytes'] / 1e6:.1f} | {r['achieved']:.0f} | {100 * r['frac']:.1f} |")
        with open(os.path.join(PROFILES, fname), "w") as f:
            f.write(f"""# The layers around the scan on {bench['detail']['workload']}: convolution + SiLU, projections (MFMA), gated scan, linear layers, aggregator

`{shown(by_name[f'trace_producers_{w}'])}`

{kernel_table(runs_dir, f'trace_producers_{w}')}

The kernel averages above cover both of the run's passes (buffer sets cycling, then one set resident in the Infinity
Cache).  bench.py's own event timings from the same command without the profiler (`{shown(by_name[f'plain_producers_{w}'])}`,
buffer sets cycling; low-rank step R = {blk['R']}; the projection runs at {blk['xproj_tflops']:.0f} TFLOP/s, far below
the matrix cores' rate: it is bound by the bytes of x and delta_raw):

""" + "\n".join(rows) + "\n")


def main(argv):
    if len(argv) != 3 or argv[1] not in ("commands", "write"):
        print(__doc__, file=sys.stderr)
        return 2
    runs_dir = os.path.abspath(argv[2])
    if argv[1] == "commands":
        for r in runs():
            print(command(r, runs_dir))
        print(f"{os.path.join(ROOT, 'paper_2412_00678_amd', 'roofprobe')} > {runs_dir}/roofprobe.txt")
        return 0
    write(runs_dir)
    write_producers(runs_dir, {r[0]: r for r in runs()})
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
