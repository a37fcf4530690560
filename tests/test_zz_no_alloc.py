"""scan2d_bwd_static_scratch (the backward for callers that cannot allocate) against scan2d_bwd, through the C ABI."""
import numpy as np
import pytest

from paper_2412_00678_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def s2d():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2412_00678_amd import scan2d          # raises if the library is not built
    return scan2d


def _outputs(torch, d):
    x, A, Bm = d["x"], d["A"], d["Bm"]
    return (torch.empty_like(x), torch.empty_like(x), torch.empty_like(A),
            torch.empty(Bm.shape, dtype=torch.float32, device=x.device),
            torch.empty(Bm.shape, dtype=torch.float32, device=x.device),
            None if d["Dskip"] is None else torch.empty_like(d["Dskip"]))


def _both(s2d, w, seed):
    import torch
    inp = wl.make_inputs(w, seed=seed)
    d = s2d.to_device(inp, w.dtype)
    need = s2d.workspace_bytes(s2d.make_desc(d["x"], d["A"]), s2d.PASS_BWD)
    assert 0 < need <= s2d.STATIC_SCRATCH_BYTES, need
    print(f"static scratch case Bt={w.Bt} Dc={w.Dc} N={w.N} H={w.H} W={w.W} dtype={w.dtype} workspace={need}", flush=True)
    ref = s2d.scan2d_bwd(d["x"], d["delta"], d["A"], d["Bm"], d["Cm"], d["Dskip"], d["mask"], d["dy"])
    torch.cuda.synchronize()
    out = _outputs(torch, d)
    for t in out:
        if t is not None:
            t.fill_(float("nan"))                       # every element must be written by the call
    torch.cuda.synchronize()
    got = s2d.scan2d_bwd_static_scratch(d["x"], d["delta"], d["A"], d["Bm"], d["Cm"], d["Dskip"], d["mask"], d["dy"], out)
    torch.cuda.synchronize()
    for name, g, r in zip(("dx", "ddelta", "dA", "dBm", "dCm", "dDskip"), got, ref):
        if r is None:
            assert g is None
            continue
        # the same kernels on the same inputs, reductions in a fixed order: bit-identical
        assert np.array_equal(s2d.to_host(g).view(np.uint8), s2d.to_host(r).view(np.uint8)), name


def test_static_scratch_backward_matches_scan2d_bwd_twice_in_a_row(s2d):
    # the second call is smaller and reuses the array that still holds the first call's checkpoints and sums
    _both(s2d, wl.Workload("noalloc_a", 2, 12, 16, 40, 72, wl.F32, mask_frac=0.3, backward=True), seed=21)
    _both(s2d, wl.Workload("noalloc_b", 1, 5, 16, 23, 50, wl.BF16, mask_frac=0.2, backward=True), seed=22)
    _both(s2d, wl.Workload("noalloc_c", 3, 7, 8, 12, 14, wl.F32, mask_frac=0.0, backward=True), seed=23)   # small-map form


def test_static_scratch_refuses_what_does_not_fit(s2d):
    import torch
    w = wl.Workload("noalloc_big", 1, 64, 16, 128, 192, wl.F32, mask_frac=0.0, backward=True)
    inp = wl.make_inputs(w, seed=1)
    d = s2d.to_device(inp, w.dtype)
    assert s2d.workspace_bytes(s2d.make_desc(d["x"], d["A"]), s2d.PASS_BWD) > s2d.STATIC_SCRATCH_BYTES
    out = _outputs(torch, d)
    for t in out:
        t.fill_(7.0)
    with pytest.raises(s2d.Scan2dError) as e:
        s2d.scan2d_bwd_static_scratch(d["x"], d["delta"], d["A"], d["Bm"], d["Cm"], d["Dskip"], d["mask"], d["dy"], out)
    assert e.value.code == s2d.ERR_SCRATCH_LIMIT
    assert "scratch" in s2d.strerror(e.value.code)
    torch.cuda.synchronize()
    assert all(bool((t == 7.0).all()) for t in out)     # nothing was enqueued
