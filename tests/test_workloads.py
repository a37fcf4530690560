"""Host-side checks of the seeded input recipe (shapes, distributions, mask structure)."""
import numpy as np
import pytest

from paper_2412_00678_amd import workloads as wl


def test_config_table_matches_the_five_benchmark_shapes():
    shapes = [(c.Bt, c.Dc, c.N, c.H, c.W, c.dtype) for c in wl.CONFIGS]
    assert shapes == [(1, 16, 4, 16, 16, wl.F32), (1, 256, 16, 64, 64, wl.F32),
                      (1, 256, 16, 256, 256, wl.BF16), (32, 192, 16, 56, 56, wl.BF16),
                      (4, 512, 16, 128, 192, wl.F32)]
    assert [c.units for c in wl.CONFIGS] == [16384, 16777216, 268435456, 308281344, 805306368]
    assert wl.CONFIGS[2].fwd_bytes() == pytest.approx(104.9e6, rel=2e-3)
    assert wl.CONFIGS[4].fwd_bytes() == pytest.approx(616.7e6, rel=2e-3)
    assert wl.CONFIGS[4].bwd_bytes() == pytest.approx(1031.8e6, rel=2e-3)


def test_inputs_are_seeded_and_distributed_as_stated():
    c = wl.CONFIGS[1]
    a, b = wl.make_inputs(c, seed=0), wl.make_inputs(c, seed=0)
    for k in a:
        assert (a[k] is None and b[k] is None) or np.array_equal(a[k], b[k])
    assert not np.array_equal(a["x"], wl.make_inputs(c, seed=1)["x"])
    assert a["x"].shape == (1, 256, 64, 64) and a["Bm"].shape == (1, 16, 64, 64)
    assert a["A"].shape == (256, 16) and (a["A"] < 0).all()
    assert (a["delta"] > 0).all()
    # softplus(N(-2, 0.5)): median = softplus(-2)
    assert np.median(a["delta"]) == pytest.approx(np.log1p(np.exp(-2.0)), rel=0.02)
    assert np.median(np.log(-a["A"])) == pytest.approx(0.0, abs=0.05)
    m = a["mask"]
    assert m.dtype == np.uint8 and m.sum() == round(0.40 * 64 * 64)
    assert not a["x"][0, :, m[0] != 0].any()                  # x = 0 under the mask
    keep = a["x"][0, :, m[0] == 0]
    assert keep.std() == pytest.approx(1.0, rel=0.02)
    # blobs, not salt-and-pepper: most background cells have a background right-neighbour
    same = (m[0, :, 1:] == m[0, :, :-1]).mean()
    assert same > 0.9
    assert a["dy"] is None


def test_bf16_round_trip_and_ties():
    f = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38, 1e-40, np.inf], np.float32)
    bits = wl.f32_to_bf16_bits(f)
    back = wl.bf16_bits_to_f32(bits)
    assert back[0] == 1.0 and back[1] == 1.0            # 1 + 2^-8 is a tie -> even
    assert back[2] == np.float32(1.015625)              # 1 + 3*2^-8 is a tie -> even (1 + 2^-6)
    assert back[3] == -2.5 and np.isinf(back[6])
    assert np.array_equal(wl.f32_to_bf16_bits(back), bits)   # idempotent
    assert np.isnan(wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(np.array([np.nan], np.float32)))[0])


def test_poison_under_mask_keeps_everything_else():
    c = wl.Workload("t", 2, 3, 2, 12, 10, wl.F32, mask_frac=0.25)
    a = wl.make_inputs(c, seed=4)
    p = wl.make_inputs(c, seed=4, poison_under_mask=np.nan)
    m = np.broadcast_to(a["mask"][:, None] != 0, a["x"].shape)
    assert np.isnan(p["x"][m]).all() and np.array_equal(p["x"][~m], a["x"][~m])
    assert a["mask"].reshape(2, -1).sum(1).tolist() == [30, 30]


def test_small_and_degenerate_grids_generate():
    for H, W in [(1, 1), (1, 7), (5, 1), (3, 2)]:
        c = wl.Workload("t", 1, 2, 3, H, W, wl.BF16, mask_frac=0.5, backward=True)
        a = wl.make_inputs(c)
        assert a["x"].dtype == np.uint16 and a["dy"].shape == (1, 2, H, W)
        assert a["mask"].sum() == round(0.5 * H * W)
