"""Builds the gfx950 shared library `libscan2d.so` (and the roofline probe) with hipcc.

Every translation unit is compiled for gfx950 only, with packed-FP32 instruction selection
switched off, then linked in-tree next to this file.  Run as `python -m paper_2412_00678_amd.build`.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libscan2d.so")
PROBE = os.path.join(HERE, "roofprobe")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall", "-Wno-unused-value",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
UNITS = ["scan2d_api.hip", "scan2d_elementwise.hip", "scan2d_fwd_f32.hip", "scan2d_fwd_bf16.hip", "scan2d_fwd_f32_sp.hip", "scan2d_fwd_bf16_sp.hip", "scan2d_fwd_f32_um.hip", "scan2d_fwd_bf16_um.hip", "scan2d_fwd_bf16_ua.hip", "scan2d_fwd_f32_sp_um.hip", "scan2d_fwd_bf16_sp_um.hip", "scan2d_fwd_bf16_sp_ua.hip",
         "scan2d_bwd.hip", "scan2d_bwd_f32.hip", "scan2d_bwd_bf16.hip", "scan2d_bwd_f32_sp.hip", "scan2d_bwd_bf16_sp.hip"]


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError("command failed: " + " ".join(cmd) + "\n" + out)
    return out


def _newest_header() -> float:
    t = 0.0
    for root in (CSRC, os.path.join(HERE, "..", "include")):
        for f in os.listdir(root):
            if f.endswith((".hpp", ".h")):
                t = max(t, os.path.getmtime(os.path.join(root, f)))
    return t


def build(force: bool = True, jobs: int = 4, verbose: bool = True) -> str:
    """Compile all units (always, unless force=False and objects are newer than sources) and link."""
    os.makedirs(OBJ, exist_ok=True)
    hdr = _newest_header()
    todo = []
    for u in UNITS:
        src = os.path.join(CSRC, u)
        obj = os.path.join(OBJ, u.replace(".hip", ".o"))
        stale = force or not os.path.exists(obj) or os.path.getmtime(obj) < max(os.path.getmtime(src), hdr)
        if stale:
            todo.append([HIPCC, *FLAGS, "-c", src, "-o", obj])
    with ThreadPoolExecutor(max_workers=max(1, jobs)) as ex:
        for out in ex.map(_run, todo):
            if verbose and out.strip():
                print(out)
    objs = [os.path.join(OBJ, u.replace(".hip", ".o")) for u in UNITS]
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    probe_src = os.path.join(CSRC, "roofprobe.hip")
    if os.path.exists(probe_src):
        _run([HIPCC, *FLAGS, "-o", PROBE, probe_src])
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(force="--incremental" not in sys.argv)
