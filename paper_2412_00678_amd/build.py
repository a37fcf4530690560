"""Builds the gfx950 shared library `libscan2d.so` (and the roofline probe) with hipcc.

Every translation unit is compiled for gfx950 only, with packed-FP32 instruction selection
switched off, then linked in-tree next to this file.  Run as `python -m paper_2412_00678_amd.build`.
"""
from __future__ import annotations

import os
import re
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
# scan2d_api.hip is compiled last: it includes the register table generated from the remarks of the forward units
UNITS = ["scan2d_elementwise.hip", "scan2d_block.hip", "scan2d_pool.hip", "scan2d_linear.hip", "scan2d_norm.hip", "scan2d_fwd_f32.hip", "scan2d_fwd_bf16.hip", "scan2d_fwd_f32_sp.hip", "scan2d_fwd_bf16_sp.hip", "scan2d_fwd_f32_um.hip", "scan2d_fwd_bf16_um.hip", "scan2d_fwd_bf16_ua.hip", "scan2d_fwd_f32_sp_um.hip", "scan2d_fwd_bf16_sp_um.hip", "scan2d_fwd_bf16_sp_ua.hip",
         "scan2d_fwd_shared_f32.hip", "scan2d_fwd_shared_bf16.hip", "scan2d_fwd_shared_gate.hip", "scan2d_fwd_skew.hip", "scan2d_fwd_shared_f32_cf.hip", "scan2d_fwd_shared_bf16_cf.hip", "scan2d_fwd_av.hip", "scan2d_fwd_tile16.hip",
         "scan2d_bwd.hip", "scan2d_bwd_f32.hip", "scan2d_bwd_bf16.hip", "scan2d_bwd_f32_sp.hip", "scan2d_bwd_bf16_sp.hip",
         "scan2d_bwd_shared_f32.hip", "scan2d_bwd_shared_bf16.hip", "scan2d_bwd_shared_f32_cf.hip", "scan2d_bwd_shared_bf16_cf.hip", "scan2d_bwd_av.hip"]
API_UNIT = "scan2d_api.hip"
REGS_UNITS = ("scan2d_fwd_f32.hip", "scan2d_fwd_bf16.hip", "scan2d_fwd_shared_f32.hip", "scan2d_fwd_shared_bf16.hip")
REGS_INC = "scan2d_fwd_regs.inc"


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError("command failed: " + " ".join(cmd) + "\n" + out)
    return out


_REMARK = re.compile(r"remark: .*\[-Rpass-analysis=kernel-resource-usage\]")
_KERNEL = re.compile(r"scan2d_fwd(_shared)?_kernelI(f|NS_6bf16_tE)((?:L[ib]\d+E)+)E")


def _split_remarks(out: str):
    """Separates the compiler's resource-usage remarks from its other output; returns (other, {mangled: VGPRs + AGPRs})."""
    regs, cur, rest = {}, None, []
    lines = out.splitlines()
    k = 0
    while k < len(lines):
        line = lines[k]
        if _REMARK.search(line):
            m = re.search(r"Function Name: (\S+)", line)
            if m:
                cur = m.group(1)
                regs[cur] = 0
            m = re.search(r" (VGPRs|AGPRs): (\d+)", line)
            if m and cur:
                regs[cur] += int(m.group(2))
            k += 1
            while k < len(lines) and not re.match(r"\S+:\d+:\d+: ", lines[k]) and not lines[k].startswith(("clang", "hipcc", "In file")):
                k += 1          # the source line and caret that follow a remark
            continue
        rest.append(line)
        k += 1
    other = "\n".join(rest)
    if "warning:" not in other and "error:" not in other:
        other = ""              # only the include trails of the remarks are left
    return other, regs


def _write_regs_inc(regs: dict, path: str) -> None:
    """The register table the forward dispatcher ranks its variants with, from this build's own kernels.

    Plain kernels <T, LG, K, NW, WAVES, EXACT, FAST, MULTI, SP, MA, UA, AV>: per (K, NW) the largest count over the
    unguarded instantiations (EXACT, FAST, !MULTI, !SP, MA, !UA, !AV), bf16 and fp32 storage.
    Shared-producer kernels <T, LG, K, NW, NG, WAVES, RPB, SP, UA, CK, CF, KEEPY, GATE, SKEW>: the count of each (!SP, !UA, CK = 0, !CF, !KEEPY, !GATE, !SKEW) instantiation."""
    plain, shared = {}, {}
    for name, n in regs.items():
        m = _KERNEL.search(name)
        if not m:
            continue
        bf16 = m.group(2) != "f"
        a = [int(t) for t in re.findall(r"L[ib](\d+)E", m.group(3))]
        if m.group(1):
            if len(a) == 13 and a[6:] == [0, 0, 0, 0, 0, 0, 0]:  # !SP, !UA, forward (not the checkpoint mode), rows first, !KEEPY, !GATE
                shared[(int(bf16), *a[:6])] = n
        elif len(a) == 11 and a[4:] == [1, 1, 0, 0, 1, 0, 0]:
            key = (a[1], a[2])
            cur = plain.setdefault(key, [0, 0])
            cur[0 if bf16 else 1] = max(cur[0 if bf16 else 1], n)
    if not plain or not shared:
        raise RuntimeError("no resource-usage remarks found for the forward kernels (plain: %d, shared: %d): "
                           "the kernel names or template lists no longer match _KERNEL" % (len(plain), len(shared)))
    with open(path, "w") as f:
        f.write("// Generated by paper_2412_00678_amd/build.py from the compiler's resource-usage remarks of this build.\n")
        f.write("// {K, NW, VGPRs+AGPRs bf16, fp32}: largest count over the unguarded plain forward instantiations\n")
        f.write("static const PlainRegs kPlainRegs[] = {\n")
        for (K, NW), (b, f32) in sorted(plain.items()):
            f.write("    {%d, %d, %d, %d},\n" % (K, NW, b or 300, f32 or 300))
        f.write("};\n// {bf16, LG, K, NW, NG, WAVES, RPB, VGPRs+AGPRs} of the shared-producer forward instantiations\n")
        f.write("static const SharedRegs kSharedRegs[] = {\n")
        for key, n in sorted(shared.items()):
            f.write("    {%s, %d},\n" % (", ".join(str(t) for t in key), n))
        f.write("};\n")


def _newest_header() -> float:
    t = 0.0
    for root in (CSRC, os.path.join(HERE, "..", "include")):
        for f in os.listdir(root):
            if f.endswith((".hpp", ".h")):
                t = max(t, os.path.getmtime(os.path.join(root, f)))
    return t


def build(force: bool = True, jobs: int = 6, verbose: bool = True) -> str:
    """Compile all units (always, unless force=False and objects are newer than sources) and link."""
    os.makedirs(OBJ, exist_ok=True)
    hdr = _newest_header()
    todo = []
    for u in UNITS:
        src = os.path.join(CSRC, u)
        obj = os.path.join(OBJ, u.replace(".hip", ".o"))
        stale = force or not os.path.exists(obj) or os.path.getmtime(obj) < max(os.path.getmtime(src), hdr)
        remarks = os.path.join(OBJ, u.replace(".hip", ".regs"))
        if u in REGS_UNITS and not os.path.exists(remarks):
            stale = True
        if stale:
            extra = ["-Rpass-analysis=kernel-resource-usage"] if u in REGS_UNITS else []
            todo.append((u, [HIPCC, *FLAGS, *extra, "-c", src, "-o", obj]))
    with ThreadPoolExecutor(max_workers=max(1, jobs)) as ex:
        for (u, _), out in zip(todo, ex.map(_run, [c for _, c in todo])):
            if u in REGS_UNITS:
                out, regs = _split_remarks(out)
                with open(os.path.join(OBJ, u.replace(".hip", ".regs")), "w") as f:
                    f.write("".join("%s %d\n" % kv for kv in sorted(regs.items())))
            if verbose and out.strip():
                print(out)
    # the dispatcher's register table, from the kernels just compiled (or compiled earlier and unchanged)
    regs = {}
    for u in REGS_UNITS:
        with open(os.path.join(OBJ, u.replace(".hip", ".regs"))) as f:
            for line in f:
                name, n = line.split()
                regs[name] = int(n)
    _write_regs_inc(regs, os.path.join(OBJ, REGS_INC))
    out = _run([HIPCC, *FLAGS, "-I", OBJ, "-c", os.path.join(CSRC, API_UNIT), "-o", os.path.join(OBJ, API_UNIT.replace(".hip", ".o"))])
    if verbose and out.strip():
        print(out)
    objs = [os.path.join(OBJ, u.replace(".hip", ".o")) for u in UNITS + [API_UNIT]]
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    probe_src = os.path.join(CSRC, "roofprobe.hip")
    if os.path.exists(probe_src):
        _run([HIPCC, *FLAGS, "-o", PROBE, probe_src])
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(force="--incremental" not in sys.argv)
