"""Prints the register table that the forward dispatcher ranks its variants with.

    python -m paper_2412_00678_amd.fwd_regs_table

Compiles the two forward translation units with the compiler's resource-usage remarks and prints,
for every (K, NW), the largest VGPR + AGPR count over the unguarded variants (bf16 and fp32 storage)
in the form of the table `fwd_regs()` of csrc/scan2d_api.hip.  Run it after changing the forward
kernel and paste the rows: the dispatcher derives the waves per SIMD of a variant from them.
"""
from __future__ import annotations

import os
import re
import subprocess
import sys

from . import build as hip_build

HERE = os.path.dirname(os.path.abspath(__file__))


def usage(unit: str) -> dict:
    cmd = [hip_build.HIPCC, *hip_build.FLAGS, "-Rpass-analysis=kernel-resource-usage", "-c",
           os.path.join(hip_build.CSRC, unit), "-o", os.devnull]
    err = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True).stderr
    out, cur = {}, None
    for line in err.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            cur = subprocess.run(["c++filt", m.group(1)], stdout=subprocess.PIPE, text=True).stdout.strip()
            out[cur] = 0
            continue
        m = re.search(r" (VGPRs|AGPRs): (\d+)", line)
        if m and cur:
            out[cur] += int(m.group(2))
    return out


def table(unit: str) -> dict:
    best = {}
    for name, regs in usage(unit).items():
        # EXACT, FAST, !MULTI, !SP, MA, !UA: the plain unguarded variants
        m = re.search(r"scan2d_fwd_kernel<[^,]+, \d+, (\d+), (\d+), \d+, true, true, false, false, true, false>", name)
        if m:
            key = (int(m.group(1)), int(m.group(2)))
            best[key] = max(best.get(key, 0), regs)
    return best


def main() -> int:
    b, f = table("scan2d_fwd_bf16.hip"), table("scan2d_fwd_f32.hip")
    for key in sorted(set(b) | set(f)):
        print("{%d, %d, %d, %d}," % (key[0], key[1], b.get(key, 300), f.get(key, 300)))
    return 0


if __name__ == "__main__":
    sys.exit(main())
