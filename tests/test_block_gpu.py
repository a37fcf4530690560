"""GPU parity of the producers in front of the scan (scan2d_block_conv_silu, scan2d_block_xproj) against
oracle/block.py, through the C ABI, and of the chain conv -> projections -> gated scan against the oracle's chain."""
import numpy as np
import pytest

import oracle
from oracle import block
from paper_2412_00678_amd import workloads as wl

pytestmark = pytest.mark.gpu

# max|gpu - ref| / max|ref| per tensor: fp32 arithmetic on both products and one rounding to the storage type
TOL_BLOCK = {wl.F32: 1e-5, wl.BF16: 2.0 ** -7}
TOL_SCAN = {wl.F32: 1e-4, wl.BF16: 2e-2}


@pytest.fixture(scope="module")
def s2d():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2412_00678_amd import scan2d
    return scan2d


def rel_err(got, ref):
    return float(np.max(np.abs(got - ref)) / max(float(np.max(np.abs(ref))), 1e-30))


CONV_CASES = [
    # Bt, Dc, H, W, dtype, KH, KW, PH, PW
    (2, 5, 13, 17, wl.F32, 3, 3, 1, 1), (1, 3, 14, 14, wl.BF16, 3, 3, 1, 1), (2, 4, 9, 30, wl.BF16, 1, 4, 0, 3),
    (1, 2, 7, 5, wl.F32, 7, 7, 3, 3), (1, 2, 5, 9, wl.F32, 2, 5, 1, 0), (1, 3, 1, 1, wl.BF16, 3, 3, 1, 1),
    (1, 2, 6, 64, wl.BF16, 5, 3, 4, 2), (3, 2, 33, 3, wl.F32, 3, 1, 0, 0), (1, 64, 56, 56, wl.BF16, 3, 3, 1, 1),
]


@pytest.mark.parametrize("case", CONV_CASES, ids=lambda c: "x".join(map(str, c[:4])) + ("bf16" if c[4] else "f32") + f"-k{c[5]}x{c[6]}")
def test_conv_silu_matches_oracle(s2d, case):
    import torch
    Bt, Dc, H, W, dtype, KH, KW, PH, PW = case
    w_ = wl.Workload("conv", Bt, Dc, 1, H, W, dtype)
    inp = wl.make_block_inputs(w_, R=1, KH=KH, KW=KW, seed=41)
    print(f"conv case {case}", flush=True)
    d = s2d.to_device({k: inp[k] for k in ("u", "w", "bias")}, dtype)
    for bias in (d["bias"], None):
        x = s2d.block_conv_silu(d["u"], d["w"], bias, PH, PW)
        torch.cuda.synchronize()
        ref = block.conv_silu(inp["u"], inp["w"], None if bias is None else inp["bias"], PH, PW, dtype=dtype)
        got = wl.to_float(s2d.to_host(x), dtype)
        assert np.isfinite(got).all()
        assert rel_err(got, wl.to_float(ref, dtype)) <= TOL_BLOCK[dtype]
        if dtype == wl.BF16:                              # one rounding: almost every output has the oracle's bits
            assert np.mean(s2d.to_host(x) == ref) > 0.99


XPROJ_CASES = [
    # Bt, Dc, N, H, W, dtype, R
    (1, 256, 16, 37, 41, wl.BF16, 8), (2, 64, 16, 8, 24, wl.BF16, 4), (1, 100, 5, 9, 20, wl.F32, 7), (1, 37, 3, 5, 7, wl.BF16, 2),
    (1, 96, 64, 6, 22, wl.F32, 64), (1, 1024, 16, 4, 16, wl.BF16, 64), (2, 30, 4, 1, 1, wl.F32, 1), (1, 256, 16, 64, 64, wl.F32, 8),
    (1, 130, 8, 3, 70, wl.BF16, 5), (1, 600, 16, 5, 30, wl.BF16, 10), (2, 300, 16, 7, 19, wl.F32, 9), (1, 512, 64, 2, 40, wl.F32, 33),
    # the kernel for the common case (H*W a multiple of 64, Dc a multiple of 16 within one chunk, at most 48 rows of Wx):
    # both storage types, every size class of the low-rank step, several tiles per workgroup
    (2, 128, 16, 8, 16, wl.F32, 8), (1, 256, 16, 16, 16, wl.BF16, 12), (1, 64, 8, 8, 8, wl.BF16, 20), (1, 16, 4, 8, 8, wl.F32, 3),
    (3, 192, 16, 56, 56, wl.BF16, 6), (1, 48, 16, 32, 1200, wl.BF16, 16), (1, 112, 12, 16, 20, wl.F32, 24),
    # the kernel for more channels than one chunk (up to 512, low-rank step of at most 16 rows): whole chunks and a
    # ragged last chunk, both storage types and both size classes of the low-rank step, several tiles per workgroup
    (1, 512, 16, 16, 64, wl.F32, 16), (2, 144, 16, 8, 8, wl.F32, 5), (1, 384, 16, 24, 32, wl.BF16, 12), (1, 272, 8, 8, 16, wl.BF16, 3),
    (1, 512, 16, 64, 300, wl.BF16, 16), (3, 320, 12, 8, 40, wl.F32, 9),
]


@pytest.mark.parametrize("case", XPROJ_CASES, ids=lambda c: "x".join(map(str, c[:5])) + ("bf16" if c[5] else "f32") + f"-R{c[6]}")
def test_xproj_matches_oracle(s2d, case):
    import torch
    Bt, Dc, N, H, W, dtype, R = case
    w_ = wl.Workload("xproj", Bt, Dc, N, H, W, dtype)
    inp = wl.make_block_inputs(w_, R=R, seed=42)
    print(f"xproj case {case}", flush=True)
    d = s2d.to_device({"x": inp["u"], "Wx": inp["Wx"], "Wdt": inp["Wdt"]}, dtype)
    delta_raw, Bm, Cm = s2d.block_xproj(d["x"], d["Wx"], d["Wdt"], N)
    torch.cuda.synchronize()
    refs = block.xproj(inp["u"], inp["Wx"], inp["Wdt"], N, dtype=dtype)
    for name, g, r in zip(("delta_raw", "Bm", "Cm"), (delta_raw, Bm, Cm), refs):
        got = wl.to_float(s2d.to_host(g), dtype)
        assert np.isfinite(got).all(), name
        e = rel_err(got, wl.to_float(r, dtype))
        assert e <= TOL_BLOCK[dtype], f"{name}: rel err {e:.3e}"


def test_block_entry_points_reject_bad_arguments(s2d):
    import torch
    u = torch.zeros((1, 4, 8, 8), device="cuda")
    w = torch.zeros((4, 3, 3), device="cuda")
    with pytest.raises(s2d.Scan2dError) as e:
        s2d.block_conv_silu(u, w, None, 3, 1)            # the first tap's offset must lie inside the filter
    assert e.value.code == -2
    with pytest.raises(s2d.Scan2dError) as e:
        s2d.block_conv_silu(u, w, None, 1, 1, x=u)       # in place
    assert e.value.code == -2
    with pytest.raises(s2d.Scan2dError) as e:
        s2d.block_conv_silu(u, torch.zeros((4, 9, 3), device="cuda"), None, 1, 1)
    assert e.value.code == -2
    x = torch.zeros((1, 64, 4, 4), device="cuda", dtype=torch.bfloat16)
    with pytest.raises(s2d.Scan2dError) as e:            # more than 64 low-rank rows
        s2d.block_xproj(x, torch.zeros((65 + 32, 64), device="cuda", dtype=torch.bfloat16), torch.zeros((64, 65), device="cuda"), 16)
    assert e.value.code == -2


@pytest.mark.parametrize("shape", [(2, 24, 16, 21, 40, wl.F32, 4), (1, 64, 16, 56, 56, wl.BF16, 4), (1, 32, 16, 30, 255, wl.BF16, 2)],
                         ids=["21x40-f32", "56x56-bf16", "30x255-bf16"])
def test_conv_projections_and_gated_scan_chain_matches_the_oracle_chain(s2d, shape):
    """u -> conv + SiLU -> x -> (delta_raw, Bm, Cm) -> softplus step, 2D scan, gate -> y, every tensor between the stages
    in the storage type on both sides."""
    import torch
    Bt, Dc, N, H, W, dtype, R = shape
    w_ = wl.Workload("chain", Bt, Dc, N, H, W, dtype, mask_frac=0.3)
    inp = wl.make_block_inputs(w_, R=R, seed=43)
    d = s2d.to_device(inp, dtype)
    x = s2d.block_conv_silu(d["u"], d["w"], d["bias"])
    delta_raw, Bm, Cm = s2d.block_xproj(x, d["Wx"], d["Wdt"], N)
    _, y = s2d.scan2d_fwd_softplus_gated(x, delta_raw, d["delta_bias"], d["A"], Bm, Cm, d["Dskip"], d["mask"], d["z"], want_y_scan=False)
    torch.cuda.synchronize()
    xr = block.conv_silu(inp["u"], inp["w"], inp["bias"], 1, 1, dtype=dtype)
    dr, Br, Cr = block.xproj(xr, inp["Wx"], inp["Wdt"], N, dtype=dtype)
    _, yr = oracle.scan2d_fwd_softplus_gated(xr, dr, inp["delta_bias"], inp["A"], Br, Cr, inp["Dskip"], inp["mask"], inp["z"], dtype=dtype)
    got = wl.to_float(s2d.to_host(y), dtype)
    assert np.isfinite(got).all()
    assert rel_err(wl.to_float(s2d.to_host(x), dtype), wl.to_float(xr, dtype)) <= TOL_BLOCK[dtype]
    assert rel_err(wl.to_float(s2d.to_host(delta_raw), dtype), wl.to_float(dr, dtype)) <= 2 * TOL_BLOCK[dtype]
    assert rel_err(got, wl.to_float(yr, dtype)) <= TOL_SCAN[dtype]


@pytest.mark.parametrize("k", [2, 3, 4], ids=["wsi-256x256-bf16", "vmamba-56x56-bf16", "train-128x192-fp32"])
def test_producers_at_full_size_on_sampled_outputs(s2d, k):
    """The launch configuration bench.py --block times.  The convolution is checked on whole sampled maps, the
    projections (independent per position) on sampled positions of every batch item, against the oracle."""
    import torch
    w = wl.CONFIGS[k]
    R = max(1, (w.Dc // 2 + 15) // 16)
    inp = wl.make_block_inputs(w, R=R, seed=0)
    d = s2d.to_device({key: inp[key] for key in ("u", "w", "bias", "Wx", "Wdt")}, w.dtype)
    x = s2d.block_conv_silu(d["u"], d["w"], d["bias"])
    delta_raw, Bm, Cm = s2d.block_xproj(x, d["Wx"], d["Wdt"], w.N)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    xh = s2d.to_host(x)
    for _ in range(6):                                   # whole maps of the convolution
        b, c = int(rng.integers(w.Bt)), int(rng.integers(w.Dc))
        ref = block.conv_silu(inp["u"][b:b + 1, c:c + 1], inp["w"][c:c + 1], inp["bias"][c:c + 1], 1, 1, dtype=w.dtype)
        assert rel_err(wl.to_float(xh[b, c], w.dtype), wl.to_float(ref[0, 0], w.dtype)) <= TOL_BLOCK[w.dtype]
    # sampled positions: a 1 x P' problem made of the sampled columns of x as the GPU produced it
    P = w.H * w.W
    pos = np.unique(np.concatenate([rng.integers(0, P, 400), [0, 63, 64, P - 65, P - 64, P - 1]]))
    dh, Bh, Ch = (s2d.to_host(t).reshape(w.Bt, -1, P) for t in (delta_raw, Bm, Cm))
    xs = xh.reshape(w.Bt, w.Dc, P)
    for b in sorted({0, w.Bt - 1, int(rng.integers(w.Bt))}):
        sub = np.ascontiguousarray(xs[b][:, pos]).reshape(1, w.Dc, 1, len(pos))
        refs = block.xproj(sub, inp["Wx"], inp["Wdt"], w.N, dtype=w.dtype)
        for name, got, ref in zip(("delta_raw", "Bm", "Cm"), (dh, Bh, Ch), refs):
            e = rel_err(wl.to_float(got[b][:, pos], w.dtype), wl.to_float(ref[0, :, 0, :], w.dtype))
            assert e <= TOL_BLOCK[w.dtype], f"{name} of batch item {b}: rel err {e:.3e}"


# ------------------------------------------------------------------------------------------------ aggregator
# fp32 sums and a tanh / exp of about 1e-6 relative accuracy against double precision: the attention weights carry
# the absolute error of the scores (a few 1e-6 for scores of a few units) as a relative one
TOL_POOL = 2e-5

POOL_CASES = [
    # Bt, M, H, W, dtype, D, mask_frac
    (1, 128, 16, 16, wl.BF16, 128, 0.0), (2, 64, 9, 21, wl.F32, 128, 0.3), (1, 37, 5, 7, wl.BF16, 50, 0.4), (3, 5, 1, 1, wl.F32, 1, 0.0),
    (1, 300, 8, 24, wl.BF16, 128, 0.5), (2, 200, 7, 19, wl.F32, 96, 0.2), (1, 128, 3, 70, wl.F32, 128, 0.0), (1, 16, 64, 65, wl.BF16, 17, 0.3),
    (2, 256, 40, 40, wl.BF16, 128, 0.5),
]


@pytest.mark.parametrize("case", POOL_CASES, ids=lambda c: "x".join(map(str, c[:4])) + ("bf16" if c[4] else "f32") + f"-D{c[5]}-m{c[6]}")
def test_attn_pool_matches_oracle(s2d, case):
    import torch
    Bt, M, H, W, dtype, D, mf = case
    w_ = wl.Workload("pool", Bt, M, 1, H, W, dtype, mask_frac=mf)
    inp = wl.make_pool_inputs(w_, D=D, seed=44)
    print(f"attn_pool case {case}", flush=True)
    d = s2d.to_device(inp, dtype)
    z, attn = s2d.block_attn_pool(d["h"], d["V"], d["w"], d["mask"])
    torch.cuda.synchronize()
    zr, ar = block.attn_pool(inp["h"], inp["V"], inp["w"], inp["mask"], dtype=dtype)
    zg, ag = s2d.to_host(z).astype(np.float64), s2d.to_host(attn).astype(np.float64)
    assert np.isfinite(zg).all() and np.isfinite(ag).all()
    assert rel_err(ag, ar) <= TOL_POOL and rel_err(zg, zr) <= TOL_POOL
    if inp["mask"] is not None:
        assert not ag[inp["mask"] != 0].any()                               # exactly zero outside the bag
    np.testing.assert_allclose(ag.reshape(Bt, -1).sum(axis=1), 1.0, rtol=1e-5)


def test_attn_pool_edge_cases(s2d):
    import torch
    rng = np.random.default_rng(45)
    Bt, M, H, W, D = 2, 24, 6, 10, 128
    w_ = wl.Workload("pool", Bt, M, 1, H, W, wl.F32, mask_frac=0.3)
    inp = wl.make_pool_inputs(w_, D=D, seed=46)
    # what lies under the mask is never read into the result: NaN there changes nothing
    hp = inp["h"].copy()
    hp[np.broadcast_to(inp["mask"][:, None] != 0, hp.shape)] = np.nan
    d = s2d.to_device(inp, wl.F32)
    z0, a0 = s2d.block_attn_pool(d["h"], d["V"], d["w"], d["mask"])
    z1, a1 = s2d.block_attn_pool(torch.from_numpy(hp).cuda(), d["V"], d["w"], d["mask"])
    torch.cuda.synchronize()
    assert torch.equal(z0, z1) and torch.equal(a0, a1)
    # an empty bag (batch item 1) gives zeros, the other item is unchanged; a bag of one returns that embedding
    m2 = inp["mask"].copy()
    m2[1] = 1
    z2, a2 = s2d.block_attn_pool(d["h"], d["V"], d["w"], torch.from_numpy(m2).cuda())
    torch.cuda.synchronize()
    assert torch.equal(z2[0], z0[0]) and not z2[1].any() and not a2[1].any()
    m3 = np.ones_like(m2)
    m3[0, 2, 3] = 0
    m3[1, 5, 9] = 0
    z3, a3 = s2d.block_attn_pool(d["h"], d["V"], d["w"], torch.from_numpy(m3).cuda())
    torch.cuda.synchronize()
    assert a3[0, 2, 3] == 1.0 and a3[1, 5, 9] == 1.0 and float(a3.sum()) == 2.0
    assert np.array_equal(s2d.to_host(z3)[0], inp["h"][0, :, 2, 3]) and np.array_equal(s2d.to_host(z3)[1], inp["h"][1, :, 5, 9])
    # w = 0: uniform attention over the bag, z = mean embedding
    z4, a4 = s2d.block_attn_pool(d["h"], d["V"], torch.zeros(D, device="cuda"), d["mask"])
    torch.cuda.synchronize()
    for b in range(Bt):
        mem = inp["mask"][b] == 0
        np.testing.assert_allclose(s2d.to_host(a4)[b][mem], 1.0 / mem.sum(), rtol=1e-6)
        np.testing.assert_allclose(s2d.to_host(z4)[b], inp["h"][b][:, mem].astype(np.float64).mean(axis=1), rtol=1e-4, atol=1e-6)
    # scores of +-1000 (saturated tanh times large w) neither overflow nor lose the normalisation
    z5, a5 = s2d.block_attn_pool(d["h"], d["V"], d["w"] * 100.0, d["mask"])
    torch.cuda.synchronize()
    assert torch.isfinite(z5).all() and abs(float(a5[0].sum()) - 1.0) < 1e-5
    # two calls give the same bits; more than 128 hidden units are refused
    z6, a6 = s2d.block_attn_pool(d["h"], d["V"], d["w"], d["mask"])
    torch.cuda.synchronize()
    assert torch.equal(z6, z0) and torch.equal(a6, a0)
    with pytest.raises(s2d.Scan2dError) as e:
        s2d.block_attn_pool(d["h"], torch.zeros((129, M), device="cuda"), torch.zeros(129, device="cuda"))
    assert e.value.code == -2


@pytest.mark.parametrize("k", [2, 3], ids=["wsi-256x256-bf16", "vmamba-56x56-bf16"])
def test_attn_pool_at_full_size(s2d, k):
    """The launch configuration bench.py --block times: embeddings of half the scan's channel count (the block's model
    width for an expansion of 2), 128 hidden units, the workload's mask."""
    import torch
    w = wl.CONFIGS[k]
    w_ = wl.Workload("pool", w.Bt, w.Dc // 2, 1, w.H, w.W, w.dtype, mask_frac=w.mask_frac)
    inp = wl.make_pool_inputs(w_, D=128, seed=0)
    d = s2d.to_device(inp, w.dtype)
    z, attn = s2d.block_attn_pool(d["h"], d["V"], d["w"], d["mask"])
    torch.cuda.synchronize()
    zr, ar = block.attn_pool(inp["h"], inp["V"], inp["w"], inp["mask"], dtype=w.dtype)
    assert rel_err(s2d.to_host(attn).astype(np.float64), ar) <= TOL_POOL
    assert rel_err(s2d.to_host(z).astype(np.float64), zr) <= TOL_POOL


# ------------------------------------------------------------------------------------------------ linear layers
LINEAR_CASES = [
    # Bt, Cin, Cout, H, W, dtype, bias, residual
    (1, 128, 256, 16, 32, wl.BF16, True, False), (2, 64, 128, 8, 16, wl.F32, False, False), (1, 256, 128, 16, 24, wl.BF16, True, True),
    (1, 36, 50, 5, 12, wl.F32, True, True), (3, 100, 130, 7, 20, wl.BF16, False, True), (1, 4, 1, 2, 2, wl.F32, True, False),
    (1, 512, 300, 3, 44, wl.BF16, True, False), (2, 96, 192, 56, 56, wl.BF16, False, False), (1, 160, 96, 20, 52, wl.F32, True, True),
    # neither H*W nor the channel count a multiple of 4: the kernel with one thread per output
    (2, 37, 19, 5, 7, wl.BF16, True, True), (1, 30, 64, 3, 9, wl.F32, True, False), (1, 64, 10, 1, 1, wl.F32, False, True),
]


@pytest.mark.parametrize("case", LINEAR_CASES, ids=lambda c: "x".join(map(str, c[:5])) + ("bf16" if c[5] else "f32") + ("-b" if c[6] else "") + ("-r" if c[7] else ""))
def test_linear_matches_oracle(s2d, case):
    import torch
    Bt, Cin, Cout, H, W, dtype, has_bias, has_res = case
    print(f"linear case {case}", flush=True)
    rng = np.random.default_rng(47)
    cast = (lambda a: wl.f32_to_bf16_bits(a.astype(np.float32))) if dtype == wl.BF16 else (lambda a: a.astype(np.float32))
    inp = {"x": cast(rng.standard_normal((Bt, Cin, H, W))), "Wt": cast(rng.standard_normal((Cout, Cin)) / np.sqrt(Cin)),
           "bias": rng.standard_normal(Cout).astype(np.float32) if has_bias else None,
           "res": cast(rng.standard_normal((Bt, Cout, H, W))) if has_res else None}
    d = s2d.to_device(inp, dtype)
    out = s2d.block_linear(d["x"], d["Wt"], d["bias"], d["res"])
    torch.cuda.synchronize()
    ref = block.linear(inp["x"], inp["Wt"], inp["bias"], inp["res"], dtype=dtype)
    got = wl.to_float(s2d.to_host(out), dtype)
    assert np.isfinite(got).all()
    assert rel_err(got, wl.to_float(ref, dtype)) <= TOL_BLOCK[dtype]
    if dtype == wl.BF16:
        assert np.mean(s2d.to_host(out) == ref) > 0.99
    if has_res:                                           # the skip connection accumulated in place
        acc = d["res"].clone()
        s2d.block_linear(d["x"], d["Wt"], d["bias"], acc, out=acc)
        torch.cuda.synchronize()
        assert torch.equal(acc, out)


def test_linear_rejects_bad_arguments(s2d):
    import torch
    x = torch.zeros((1, 8, 4, 4), device="cuda")
    with pytest.raises(s2d.Scan2dError) as e:
        s2d.block_linear(x, torch.zeros((8, 8), device="cuda"), out=x)                   # in place on the input
    assert e.value.code == -2
    with pytest.raises(ValueError):
        s2d.block_linear(x, torch.zeros((8, 7), device="cuda"))


@pytest.mark.parametrize("k", [2, 3], ids=["wsi-256x256-bf16", "vmamba-56x56-bf16"])
def test_linear_at_full_size_on_sampled_positions(s2d, k):
    """The block's input projection (model width Dc / 2 -> inner width Dc) and output projection with the skip
    connection (Dc -> Dc / 2), in the launch configuration bench.py --block times, on sampled positions."""
    import torch
    w = wl.CONFIGS[k]
    Dm, P = w.Dc // 2, w.H * w.W
    rng = np.random.default_rng(48)
    cast = lambda a: wl.f32_to_bf16_bits(a.astype(np.float32))
    inp = {"t": cast(rng.standard_normal((w.Bt, Dm, w.H, w.W))), "Win": cast(rng.standard_normal((w.Dc, Dm)) / np.sqrt(Dm)),
           "Wout": cast(rng.standard_normal((Dm, w.Dc)) / np.sqrt(w.Dc)), "bias": rng.standard_normal(w.Dc).astype(np.float32)}
    d = s2d.to_device(inp, w.dtype)
    u = s2d.block_linear(d["t"], d["Win"], d["bias"])
    back = s2d.block_linear(u, d["Wout"], None, d["t"])
    torch.cuda.synchronize()
    pos = np.unique(np.concatenate([rng.integers(0, P, 300), [0, 127, 128, P - 129, P - 128, P - 1]]))
    uh, bh, th = (s2d.to_host(t).reshape(w.Bt, -1, P) for t in (u, back, d["t"]))
    for b in sorted({0, w.Bt - 1}):
        sub = np.ascontiguousarray(th[b][:, pos]).reshape(1, Dm, 1, len(pos))
        ur = block.linear(sub, inp["Win"], inp["bias"], None, dtype=w.dtype)
        assert rel_err(wl.to_float(uh[b][:, pos], w.dtype), wl.to_float(ur[0, :, 0, :], w.dtype)) <= TOL_BLOCK[w.dtype]
        usub = np.ascontiguousarray(uh[b][:, pos]).reshape(1, w.Dc, 1, len(pos))
        br = block.linear(usub, inp["Wout"], None, sub, dtype=w.dtype)
        assert rel_err(wl.to_float(bh[b][:, pos], w.dtype), wl.to_float(br[0, :, 0, :], w.dtype)) <= TOL_BLOCK[w.dtype]


# ------------------------------------------------------------------------------------------------ normalisation
NORM_CASES = [
    # Bt, C, H, W, dtype, kind, beta
    (1, 128, 16, 32, wl.BF16, 0, True), (2, 64, 8, 16, wl.F32, 1, False), (1, 100, 5, 12, wl.F32, 0, True), (3, 37, 7, 9, wl.BF16, 0, False),
    (1, 1, 4, 4, wl.F32, 1, True), (2, 5, 1, 1, wl.F32, 0, True), (1, 192, 56, 56, wl.BF16, 1, True), (1, 512, 3, 70, wl.F32, 0, True),
    (1, 19, 64, 65, wl.BF16, 1, False),
]


@pytest.mark.parametrize("case", NORM_CASES, ids=lambda c: "x".join(map(str, c[:4])) + ("bf16" if c[4] else "f32") + ("-rms" if c[5] else "-ln") + ("-b" if c[6] else ""))
def test_norm_matches_oracle(s2d, case):
    import torch
    Bt, C, H, W, dtype, kind, has_beta = case
    print(f"norm case {case}", flush=True)
    rng = np.random.default_rng(49)
    cast = (lambda a: wl.f32_to_bf16_bits(a.astype(np.float32))) if dtype == wl.BF16 else (lambda a: a.astype(np.float32))
    # a mean of several standard deviations: the variance must not come from a difference of large sums
    inp = {"x": cast(rng.standard_normal((Bt, C, H, W)) * 0.5 + 4.0), "gamma": rng.standard_normal(C).astype(np.float32),
           "beta": rng.standard_normal(C).astype(np.float32) if has_beta else None}
    d = s2d.to_device(inp, dtype)
    out = s2d.block_norm(d["x"], d["gamma"], d["beta"], 1e-5, kind)
    torch.cuda.synchronize()
    ref = block.norm(inp["x"], inp["gamma"], inp["beta"], 1e-5, kind, dtype=dtype)
    got = wl.to_float(s2d.to_host(out), dtype)
    assert np.isfinite(got).all()
    assert rel_err(got, wl.to_float(ref, dtype)) <= TOL_BLOCK[dtype]
    if dtype == wl.BF16:
        assert np.mean(s2d.to_host(out) == ref) > 0.99
    inplace = d["x"].clone()
    s2d.block_norm(inplace, d["gamma"], d["beta"], 1e-5, kind, out=inplace)
    torch.cuda.synchronize()
    assert torch.equal(inplace, out)


def test_norm_rejects_bad_arguments(s2d):
    import torch
    x = torch.zeros((1, 8, 4, 4), device="cuda")
    g = torch.ones(8, device="cuda")
    for kind, eps in ((2, 1e-5), (0, -1.0), (0, float("nan"))):
        with pytest.raises(s2d.Scan2dError) as e:
            s2d.block_norm(x, g, None, eps, kind)
        assert e.value.code == -2


@pytest.mark.parametrize("shape", [(1, 32, 16, 16, 24, wl.BF16, 4), (2, 16, 8, 9, 20, wl.F32, 2)], ids=["16x24-bf16", "9x20-f32"])
def test_whole_block_forward_matches_the_oracle_chain(s2d, shape):
    """Layer norm -> the two input projections -> convolution + SiLU -> step / B / C projections -> softplus step, 2D
    scan, gate -> output projection with the skip connection, every tensor between the stages in the storage type on
    both sides (Fig. 2)."""
    import torch
    Bt, Dm, N, H, W, dtype, R = shape
    Dc = 2 * Dm
    w_ = wl.Workload("block", Bt, Dc, N, H, W, dtype, mask_frac=0.3)
    inp = wl.make_block_inputs(w_, R=R, seed=50)
    rng = np.random.default_rng(51)
    cast = (lambda a: wl.f32_to_bf16_bits(a.astype(np.float32))) if dtype == wl.BF16 else (lambda a: a.astype(np.float32))
    ext = {"t": cast(rng.standard_normal((Bt, Dm, H, W))), "Win_x": cast(rng.standard_normal((Dc, Dm)) / np.sqrt(Dm)),
           "Win_z": cast(rng.standard_normal((Dc, Dm)) / np.sqrt(Dm)), "Wout": cast(rng.standard_normal((Dm, Dc)) / np.sqrt(Dc)),
           "gamma": rng.normal(1.0, 0.1, Dm).astype(np.float32), "beta": rng.normal(0.0, 0.1, Dm).astype(np.float32)}
    d = s2d.to_device({**inp, **ext}, dtype)
    tn = s2d.block_norm(d["t"], d["gamma"], d["beta"], 1e-5, s2d.LAYER_NORM)
    u = s2d.block_linear(tn, d["Win_x"])
    z = s2d.block_linear(tn, d["Win_z"])
    x = s2d.block_conv_silu(u, d["w"], d["bias"])
    delta_raw, Bm, Cm = s2d.block_xproj(x, d["Wx"], d["Wdt"], N)
    _, y = s2d.scan2d_fwd_softplus_gated(x, delta_raw, d["delta_bias"], d["A"], Bm, Cm, d["Dskip"], d["mask"], z, want_y_scan=False)
    t_out = s2d.block_linear(y, d["Wout"], None, d["t"])
    torch.cuda.synchronize()
    tnr = block.norm(ext["t"], ext["gamma"], ext["beta"], 1e-5, block.LAYER_NORM, dtype=dtype)
    ur = block.linear(tnr, ext["Win_x"], dtype=dtype)
    zr = block.linear(tnr, ext["Win_z"], dtype=dtype)
    xr = block.conv_silu(ur, inp["w"], inp["bias"], 1, 1, dtype=dtype)
    dr, Br, Cr = block.xproj(xr, inp["Wx"], inp["Wdt"], N, dtype=dtype)
    _, yr = oracle.scan2d_fwd_softplus_gated(xr, dr, inp["delta_bias"], inp["A"], Br, Cr, inp["Dskip"], inp["mask"], zr, dtype=dtype)
    tr = block.linear(yr, ext["Wout"], None, ext["t"], dtype=dtype)
    got = wl.to_float(s2d.to_host(t_out), dtype)
    assert np.isfinite(got).all()
    # roundings of the storage type between seven stages: a few units in the last place of bf16 at the end
    tol = {wl.F32: 2e-5, wl.BF16: 3e-2}[dtype]
    assert rel_err(wl.to_float(s2d.to_host(u), dtype), wl.to_float(ur, dtype)) <= 2 * TOL_BLOCK[dtype]
    assert rel_err(got, wl.to_float(tr, dtype)) <= tol


@pytest.mark.parametrize("dtype", [wl.BF16, wl.F32], ids=["bf16", "f32"])
def test_whole_block_and_aggregator_replay_from_a_hip_graph(s2d, dtype):
    """The layers around the scan only enqueue kernels on the caller's stream (no allocation, no memset, no
    synchronisation), so a whole block forward plus the aggregator can be captured; every replay equals the eager
    result bit for bit, also after the inputs changed and eager work ran in between.  fp32 takes the linear kernel
    that needs more than 64 KB of dynamic LDS (the attribute is raised once, outside the capture)."""
    import torch
    Bt, Dm, N, H, W, R = 2, 32, 16, 16, 32, 4
    Dc = 2 * Dm
    w_ = wl.Workload("graph_block", Bt, Dc, N, H, W, dtype, mask_frac=0.3)
    cast = (lambda a: wl.f32_to_bf16_bits(a.astype(np.float32))) if dtype == wl.BF16 else (lambda a: a.astype(np.float32))

    def draw(seed):
        inp = wl.make_block_inputs(w_, R=R, seed=seed)
        rng = np.random.default_rng(seed + 100)
        inp.update({"t": cast(rng.standard_normal((Bt, Dm, H, W))), "Win_x": cast(rng.standard_normal((Dc, Dm)) / np.sqrt(Dm)),
                    "Win_z": cast(rng.standard_normal((Dc, Dm)) / np.sqrt(Dm)), "Wout": cast(rng.standard_normal((Dm, Dc)) / np.sqrt(Dc)),
                    "gamma": rng.normal(1.0, 0.1, Dm).astype(np.float32), "beta": rng.normal(0.0, 0.1, Dm).astype(np.float32),
                    "V": cast(rng.standard_normal((128, Dm)) / np.sqrt(Dm)), "wp": rng.standard_normal(128).astype(np.float32)})
        return inp

    sets = [draw(61), draw(62)]
    st = s2d.to_device(sets[0], dtype)
    like = lambda C: torch.empty((Bt, C, H, W), dtype=st["t"].dtype, device="cuda:0")
    buf = {"tn": like(Dm), "u": like(Dc), "zb": like(Dc), "x": like(Dc), "y": like(Dc), "t_out": like(Dm),
           "proj": (like(Dc), like(N), like(N)), "pool": (torch.empty((Bt, Dm), device="cuda:0"), torch.empty((Bt, H, W), device="cuda:0"))}
    desc = s2d.make_desc(buf["x"], st["A"])
    ws = torch.empty(max(16, s2d.workspace_bytes(desc, s2d.PASS_FWD)), dtype=torch.uint8, device="cuda:0")

    def run():
        s2d.block_norm(st["t"], st["gamma"], st["beta"], 1e-5, s2d.LAYER_NORM, out=buf["tn"])
        s2d.block_linear(buf["tn"], st["Win_x"], out=buf["u"])
        s2d.block_linear(buf["tn"], st["Win_z"], out=buf["zb"])
        s2d.block_conv_silu(buf["u"], st["w"], st["bias"], x=buf["x"])
        s2d.block_xproj(buf["x"], st["Wx"], st["Wdt"], N, out=buf["proj"])
        s2d.scan2d_fwd_softplus_gated(buf["x"], buf["proj"][0], st["delta_bias"], st["A"], buf["proj"][1], buf["proj"][2], st["Dskip"],
                                      st["mask"], buf["zb"], want_y_scan=False, workspace=ws, y=buf["y"])
        s2d.block_linear(buf["y"], st["Wout"], None, st["t"], out=buf["t_out"])
        s2d.block_attn_pool(buf["t_out"], st["V"], st["wp"], st["mask"], out=buf["pool"])

    def snapshot():
        torch.cuda.synchronize()
        return [s2d.to_host(buf["t_out"]).copy(), s2d.to_host(buf["pool"][0]).copy(), s2d.to_host(buf["pool"][1]).copy()]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                       # warm-up outside the capture
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for k in (0, 1, 0):
        new = s2d.to_device(sets[k], dtype)
        for name, t in st.items():
            if t is not None:
                t.copy_(new[name])
        for t in (buf["t_out"], buf["pool"][0], buf["pool"][1]):
            t.fill_(float("nan"))
        graph.replay()
        got = snapshot()
        run()                                           # eager work between the replays
        ref = snapshot()
        for a, b in zip(got, ref):
            assert np.array_equal(a, b)
    # and the replayed result is the oracle's chain (first draw)
    i0 = sets[0]
    tnr = block.norm(i0["t"], i0["gamma"], i0["beta"], 1e-5, block.LAYER_NORM, dtype=dtype)
    xr = block.conv_silu(block.linear(tnr, i0["Win_x"], dtype=dtype), i0["w"], i0["bias"], 1, 1, dtype=dtype)
    dr, Br, Cr = block.xproj(xr, i0["Wx"], i0["Wdt"], N, dtype=dtype)
    _, yr = oracle.scan2d_fwd_softplus_gated(xr, dr, i0["delta_bias"], i0["A"], Br, Cr, i0["Dskip"], i0["mask"], block.linear(tnr, i0["Win_z"], dtype=dtype), dtype=dtype)
    tr = block.linear(yr, i0["Wout"], None, i0["t"], dtype=dtype)
    assert rel_err(wl.to_float(got[0], dtype), wl.to_float(tr, dtype)) <= {wl.F32: 2e-5, wl.BF16: 3e-2}[dtype]
