"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares,
and rejects bad arguments before touching a device (no compute call is made here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "scan2d.h")
LIB = os.path.join(ROOT, "paper_2412_00678_amd", "libscan2d.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail(f"{LIB} not built: run `python -m paper_2412_00678_amd.build` first")
    from paper_2412_00678_amd import scan2d
    return scan2d


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(scan2d_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    assert declared_functions() == sorted(
        ["scan2d_fwd", "scan2d_fwd_softplus", "scan2d_fwd_softplus_gated", "scan2d_bwd", "scan2d_bwd_softplus",
         "scan2d_bwd_softplus_gated", "scan2d_workspace_bytes", "scan2d_describe_plan", "scan2d_strerror",
         "scan2d_version", "scan2d_debug_force_variant", "scan2d_bwd_static_scratch", "scan2d_fwd_variants", "scan2d_bwd_variants",
         "scan2d_block_conv_silu", "scan2d_block_xproj", "scan2d_saved_bytes", "scan2d_fwd_saving", "scan2d_bwd_saved",
         "scan2d_block_attn_pool", "scan2d_block_linear", "scan2d_block_norm"])


def test_library_exports_every_declared_symbol(lib):
    raw = ctypes.CDLL(LIB)
    for name in declared_functions():
        assert hasattr(raw, name), name
    assert sorted(lib.EXPORTS) == declared_functions()
    assert lib.version() >= 100


def test_error_strings_are_distinct_and_static(lib):
    seen = {lib.strerror(c) for c in range(0, -10, -1)}
    assert len(seen) == 10
    assert "unknown" in lib.strerror(-99)


def test_descriptor_validation_needs_no_device(lib):
    D = lib.Desc
    call = lambda d: lib.lib.scan2d_fwd(ctypes.byref(d), *([None] * 8), None, 0, None)
    assert call(D(0, 1, 1, 1, 1, 0, 0)) == -2
    assert call(D(1, 1, 1, 1, 65, 0, 0)) == -2
    assert call(D(1, 1, 1, -3, 4, 0, 0)) == -2
    assert call(D(1, 1, 4096, 4096, 16, 0, 0)) == -2          # N*H*W >= 2^27
    assert call(D(1, 1, 8, 8, 4, 7, 0)) == -3
    assert call(D(1, 1, 8, 8, 4, 0, 4)) == -4                    # an unknown flag bit
    assert call(D(1, 1, 8, 8, 4, 0, 3)) != -4                    # SCAN2D_FLAG_IDENTITY_CELLS | SCAN2D_FLAG_COLUMNS_FIRST
    assert call(D(1, 1, 8, 8, 4, 0, 0)) == -1                  # NULL tensors
    assert lib.lib.scan2d_fwd(None, *([None] * 8), None, 0, None) == -1
    bwd = lambda d: lib.lib.scan2d_bwd(ctypes.byref(d), *([None] * 14), None, 0, None)
    assert bwd(D(1, 0, 1, 1, 1, 0, 0)) == -2
    assert bwd(D(1, 1, 8, 8, 4, 1, 0)) == -1


def test_misaligned_pointers_are_rejected_before_any_launch(lib):
    d = lib.Desc(1, 1, 8, 8, 4, 0, 0)
    ok, bad = 4096, 4100                                       # fake addresses: never dereferenced
    args = [ok] * 5 + [None, None, ok]
    for k in (0, 1, 2, 3, 4, 7):                               # exactly one misaligned pointer each time
        a = list(args)
        a[k] = bad
        assert lib.lib.scan2d_fwd(ctypes.byref(d), *a, None, 0, None) == -6


def test_workspace_query(lib):
    small = lib.Desc(1, 16, 16, 16, 4, 0, 0)
    assert lib.workspace_bytes(small, lib.PASS_FWD) == 0       # one panel: no carry buffer
    wide = lib.Desc(1, 2, 8, 3000, 4, 0, 0)
    assert lib.workspace_bytes(wide, lib.PASS_FWD) == 1 * 2 * 4 * 8 * 4
    assert lib.workspace_bytes(lib.Desc(0, 1, 1, 1, 1, 0, 0), lib.PASS_FWD) == 0
    assert lib.workspace_bytes(small, 9) == 0                 # an unknown pass
    # the gated backward adds one map-sized buffer (dy * SiLU(z), storage type), rounded up to 256 bytes
    for dt, eb in ((0, 4), (1, 2)):
        d = lib.Desc(2, 8, 20, 40, 16, dt, 0)
        assert lib.workspace_bytes(d, lib.PASS_BWD_GATED) == lib.workspace_bytes(d, lib.PASS_BWD_SOFTPLUS) + ((2 * 8 * 20 * 40 * eb + 255) // 256) * 256
        # the shared-producer sweeps (16 states here) apply the softplus themselves: no step buffer
        assert lib.workspace_bytes(d, lib.PASS_BWD_SOFTPLUS) == lib.workspace_bytes(d, lib.PASS_BWD)
        # the plain sweeps keep the step in the workspace (one fp32 map-sized buffer)
        d5 = lib.Desc(2, 8, 20, 40, 5, dt, 0)
        extra = ((2 * 8 * 20 * 40 * 4 + 255) // 256) * 256 + 256      # and room behind it for reads past the last row
        assert lib.workspace_bytes(d5, lib.PASS_BWD_SOFTPLUS) == lib.workspace_bytes(d5, lib.PASS_BWD) + extra
    assert lib.workspace_bytes(lib.Desc(1, 2, 8, 3000, 4, 0, 0), lib.PASS_BWD_GATED) > 0       # wide maps: column panels
    # columns first inside the kernels (a shared-producer tiling takes the shape): the workspace of the plain call;
    # through transposes otherwise (here: 5 states): the transposed copies (x, delta, y; Bm, Cm; mask) behind the
    # workspace of the swapped shape; identity cells: one more copy of the step
    r256 = lambda v: (v + 255) // 256 * 256
    d = lib.Desc(2, 8, 20, 40, 16, 0, lib.FLAG_COLUMNS_FIRST)
    assert lib.workspace_bytes(d, lib.PASS_FWD) == 0
    assert lib.describe_plan(d, lib.PASS_FWD).startswith("columns-first(in-kernel) fwd form=shared")
    assert lib.describe_plan(d, lib.PASS_BWD).startswith("columns-first(in-kernel) bwd form=banded-shared")
    assert lib.workspace_bytes(d, lib.PASS_BWD) == lib.workspace_bytes(lib.Desc(2, 8, 20, 40, 16, 0, 0), lib.PASS_BWD)
    d = lib.Desc(2, 8, 20, 40, 5, 0, lib.FLAG_COLUMNS_FIRST)
    assert lib.describe_plan(d, lib.PASS_FWD).startswith("columns-first(transposed) fwd")
    assert lib.workspace_bytes(d, lib.PASS_FWD) == 3 * r256(2 * 8 * 800 * 4) + 2 * r256(2 * 5 * 800 * 4) + r256(2 * 800)
    # the two timed configurations run columns first inside the kernels, forward and backward
    for shape in ((1, 256, 256, 256, 16, 1), (8, 256, 128, 192, 16, 0)):
        d = lib.Desc(*shape, lib.FLAG_COLUMNS_FIRST)
        assert lib.describe_plan(d, lib.PASS_FWD).startswith("columns-first(in-kernel)")
    assert lib.describe_plan(lib.Desc(8, 256, 128, 192, 16, 0, lib.FLAG_COLUMNS_FIRST), lib.PASS_BWD).startswith("columns-first(in-kernel)")
    assert lib.workspace_bytes(lib.Desc(2, 8, 20, 40, 16, 1, lib.FLAG_IDENTITY_CELLS), lib.PASS_FWD) == r256(2 * 8 * 800 * 2)
    assert lib.workspace_bytes(lib.Desc(1, 2, 3000, 8, 4, 0, lib.FLAG_COLUMNS_FIRST), lib.PASS_BWD) > 0    # 3000 columns after the swap


# ------------------------------------------------------------------ host logic: variant choice and launch plans

def plan(lib, d, which):
    fields = {}
    for tok in lib.describe_plan(d, which).split()[1:]:
        k, v = tok.split("=")
        fields[k] = v if k == "form" else int(v)
    return fields


SWEEP_W = [1, 2, 3, 7, 13, 14, 15, 16, 17, 20, 28, 30, 31, 32, 33, 56, 60, 63, 64, 65, 100, 127, 128, 129, 132, 190, 192,
           193, 200, 250, 255, 256, 257, 300, 500, 512, 513, 777, 1000, 1024, 1025, 3000]
SWEEP_N = [1, 3, 4, 5, 8, 15, 16, 17, 24, 40, 63, 64]


def test_every_shape_has_a_forward_plan_within_the_hardware_limits(lib):
    for dtype in (0, 1):
        for W in SWEEP_W:
            for N in SWEEP_N:
                for (Bt, Dc, H) in ((1, 1, 1), (2, 7, 9), (4, 256, 64)):
                    d = lib.Desc(Bt, Dc, H, W, N, dtype, 0)
                    f = plan(lib, d, lib.PASS_FWD)
                    where = f"dtype {dtype} W {W} N {N} Bt {Bt} Dc {Dc} H {H}: {f}"
                    assert f["lds"] <= 160 * 1024, where
                    assert f["waves"] in (4, 8, 16), where
                    if f["form"] == "tile16":                 # few tiny maps: one workgroup per map
                        assert W <= 16 and H <= 16 and N <= 16 and Bt * Dc <= 1024, where
                        assert f["wgs"] == Bt * Dc and f["workspace"] == 0, where
                    elif f["form"] == "small":
                        assert W <= 16 * f["K"] and 4 * f["NW"] >= N, where
                        assert f["wgs"] == -(-Bt * Dc // 4), where
                    else:
                        assert f["NG"] * f["NW"] >= N and f["NG"] <= f["waves"] * 64 // f["LG"], where
                        assert f["panels"] * f["LG"] * f["K"] >= W, where
                        assert f["wgs"] * f["MPW"] >= Bt * Dc, where
                        assert (f["workspace"] > 0) == (f["panels"] > 1), where
                        assert f["fast"] == (f["panels"] == 1), where      # unguarded loads whenever one panel covers the row
                        if f["exact"]:
                            assert N % f["NW"] == 0, where
                    assert f["workspace"] == lib.workspace_bytes(d, lib.PASS_FWD), where


def test_backward_plans_cover_every_shape_the_forward_accepts(lib):
    for dtype in (0, 1):
        for W in SWEEP_W:
            for N in SWEEP_N:
                for (Bt, Dc, H) in ((1, 1, 1), (2, 7, 9), (4, 512, 128)):
                    d = lib.Desc(Bt, Dc, H, W, N, dtype, 0)
                    f = plan(lib, d, lib.PASS_BWD)            # every width and state count the forward accepts
                    where = f"dtype {dtype} W {W} N {N} Bt {Bt} Dc {Dc} H {H}: {f}"
                    assert f["lds"] <= 160 * 1024, where
                    assert f["workspace"] == lib.workspace_bytes(d, lib.PASS_BWD), where
                    assert 1 <= f["GS"] <= 8 and f["CG"] == -(-Dc // f["GS"]), where
                    if f["form"] == "small":
                        assert W <= 16 and H <= 16 and N <= 16 and 4 * f["NW"] >= N, where
                    else:
                        assert f["LG"] * f["K"] * f["panels"] >= W, where
                        assert f["panels"] == 1 or (f["LG"] * f["K"] == 256 and f["panels"] == -(-W // 256)), where
                        assert f["bands"] == -(-H // f["RB"]), where
                        # checkpoints + partial sums over channel groups + partial sums over batch items
                        ck = Bt * Dc * f["bands"] * N * W * 4
                        part = 2 * Bt * f["CG"] * N * H * W * 4 if f["CG"] > 1 else 0
                        assert f["workspace"] >= ck + part, where
                        # ... + the padded copies of the tensors' last rows
                        tail = (W + 16) * (5 * (4 if dtype == 0 else 2) + 1)
                        # ... + the carries between column panels (row-end states per border, a*q twice)
                        carries = (f["panels"] + 1) * (Bt * Dc * N * H * 4 + 256) if f["panels"] > 1 else 0
                        # (checkpoint rows of the shared-producer sweeps are padded to the lane grid LG * K)
                        wide = max(W, f["LG"] * f["K"]) if f["form"] == "banded-shared" else W
                        ck_max = Bt * Dc * f["bands"] * N * wide * 4
                        part_max = 2 * Bt * f["CG"] * N * H * wide * 4 if f["CG"] > 1 else 0
                        assert f["workspace"] <= ck_max + part_max + Bt * Dc * (N + 2) * 4 + tail + carries + 7 * 256, where


def test_benchmark_configurations_take_the_intended_forms(lib):
    f = plan(lib, lib.Desc(1, 256, 256, 256, 16, 1, 0), lib.PASS_FWD)
    # one map per compute unit: one state per lane on 16 wavefronts (four per SIMD); with more maps than compute units
    # two states per lane on 8 wavefronts, two workgroups per compute unit
    assert (f["form"], f["LG"], f["K"], f["NW"], f["waves"]) == ("shared", 64, 4, 1, 16) and f["fast"] and f["wgs"] == 256
    f = plan(lib, lib.Desc(2, 256, 256, 256, 16, 1, 0), lib.PASS_FWD)
    assert (f["form"], f["LG"], f["K"], f["NW"], f["waves"]) == ("shared", 64, 4, 2, 8) and f["wgs"] == 512
    f = plan(lib, lib.Desc(32, 192, 56, 56, 16, 1, 0), lib.PASS_FWD)
    assert f["form"] == "shared" and f["LG"] == 16 and f["K"] == 4 and f["fast"]
    f = plan(lib, lib.Desc(1, 256, 64, 64, 16, 0, 0), lib.PASS_FWD)
    assert (f["form"], f["LG"], f["K"], f["NW"]) == ("shared", 16, 4, 1)
    f = plan(lib, lib.Desc(1, 16, 16, 16, 4, 0, 0), lib.PASS_FWD)
    assert f["form"] == "tile16" and f["wgs"] == 16          # few tiny maps: rows and columns as parallel scans
    f = plan(lib, lib.Desc(8, 128, 14, 14, 16, 0, 0), lib.PASS_FWD)
    assert f["form"] == "tile16" and f["wgs"] == 1024
    f = plan(lib, lib.Desc(64, 128, 14, 14, 16, 0, 0), lib.PASS_FWD)
    assert f["form"] == "small"                              # many of them: four maps per workgroup, row by row
    b = plan(lib, lib.Desc(4, 512, 128, 192, 16, 0, 0), lib.PASS_BWD)
    assert (b["form"], b["LG"], b["K"], b["NW"]) == ("banded-shared", 16, 12, 1) and b["wgs"] * b["GS"] >= 4 * 512 // 1


def test_wide_grids_take_the_shared_producer_forms(lib):
    # 257 to 1024 columns, 16 states, one map per compute unit: wave-wide groups with 8, 12 or 16 columns per lane
    for W, K in ((300, 8), (400, 8), (512, 8), (513, 12), (600, 12), (768, 12), (769, 16), (1000, 16), (1024, 16)):
        for dtype in (0, 1):
            f = plan(lib, lib.Desc(1, 256, 200, W, 16, dtype, 0), lib.PASS_FWD)
            assert (f["form"], f["LG"], f["K"], f["panels"]) == ("shared", 64, K, 1) and f["workspace"] == 0, (W, dtype, f)
    f = plan(lib, lib.Desc(1, 256, 200, 1025, 16, 1, 0), lib.PASS_FWD)
    assert f["form"] == "general" and f["panels"] > 1
    # their backward: panels of 256 columns; with 16 states the shared-producer main sweep, two states per lane
    b = plan(lib, lib.Desc(1, 256, 400, 400, 16, 1, 0), lib.PASS_BWD)
    assert (b["form"], b["LG"], b["K"], b["NW"], b["waves"], b["panels"]) == ("banded-shared", 64, 4, 2, 8, 2)
    b = plan(lib, lib.Desc(1, 256, 400, 400, 8, 1, 0), lib.PASS_BWD)
    assert (b["form"], b["LG"], b["K"], b["panels"]) == ("banded", 64, 4, 2)
