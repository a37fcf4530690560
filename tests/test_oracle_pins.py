"""Pins for the CPU oracle: everything here checks `oracle.scan2d_fwd/bwd` against facts the
paper or plain mathematics fix, never against the oracle itself or the GPU path.

Sources: 2DMamba Eq. 1-2 (1D recurrence), Eq. 3 (discretisation), Eq. 5-6 (the two scans),
Eq. 7 and its derivation in Supp. C (closed form), Eq. 8 (printed 3x3 exponents), the remark
that y[i,j] only sees its upper-left quadrant (below Eq. 7), Supp. B (identity padding).
"""
import os

import numpy as np
import pytest

import oracle
from paper_2412_00678_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
F64 = oracle.F64


def rand_problem(rng, Bt, Dc, N, H, W, with_mask=True, with_skip=True):
    x = rng.standard_normal((Bt, Dc, H, W))
    delta = np.logaddexp(0.0, rng.normal(-1.0, 0.7, (Bt, Dc, H, W)))
    A = (-np.exp(rng.normal(0.0, 0.5, (Dc, N)))).astype(np.float32)
    Bm = rng.standard_normal((Bt, N, H, W))
    Cm = rng.standard_normal((Bt, N, H, W))
    Dskip = rng.standard_normal(Dc).astype(np.float32) if with_skip else None
    mask = (rng.random((Bt, H, W)) < 0.3).astype(np.uint8) if with_mask else None
    return x, delta, A, Bm, Cm, Dskip, mask


def brute_force_y(x, delta, A, Bm, Cm, Dskip, mask):
    """Closed form (Eq. 7 with the position subscripts kept): every source (i',j') reaches
    (i,j) by moving right along row i' and then down column j; the weight is the product of
    the a's of the cells entered on the way.  Pure loops, no recurrence."""
    Bt, Dc, H, W = x.shape
    N = A.shape[1]
    y = np.zeros((Bt, Dc, H, W))
    for b in range(Bt):
        for c in range(Dc):
            for i in range(H):
                for j in range(W):
                    acc = 0.0
                    for n in range(N):
                        a = np.exp(delta[b, c] * float(A[c, n]))
                        hsum = 0.0
                        for i2 in range(i + 1):
                            for j2 in range(j + 1):
                                xe = 0.0 if (mask is not None and mask[b, i2, j2]) else x[b, c, i2, j2]
                                w = 1.0
                                for s in range(j2 + 1, j + 1):
                                    w *= a[i2, s]
                                for r in range(i2 + 1, i + 1):
                                    w *= a[r, j]
                                hsum += w * delta[b, c, i2, j2] * Bm[b, n, i2, j2] * xe
                        acc += Cm[b, n, i, j] * hsum
                    xe = 0.0 if (mask is not None and mask[b, i, j]) else x[b, c, i, j]
                    y[b, c, i, j] = acc + (float(Dskip[c]) * xe if Dskip is not None else 0.0)
    return y


def read_eq8():
    blocks, cur = {}, None
    for line in open(os.path.join(GOLDEN, "eq8_exponents.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line in ("2D", "1D"):
            cur = line
            blocks[cur] = []
        else:
            blocks[cur].append([int(t) for t in line.split()])
    return np.array(blocks["2D"]), np.array(blocks["1D"])


# ----------------------------------------------------------------------------- forward pins

def test_eq8_printed_exponents_2d_and_1d():
    """Constant A-bar = alpha, unit impulse at (i',j'): h[3,3] must be alpha^k with k as printed."""
    e2d, e1d = read_eq8()
    A = np.array([[np.log(0.5)]], np.float32)
    alpha = np.exp(float(A[0, 0]))          # delta = 1 -> a = exp(A)
    ones = np.ones((1, 1, 3, 3))
    for i2 in range(3):
        for j2 in range(3):
            Bm = np.zeros((1, 1, 3, 3))
            Bm[0, 0, i2, j2] = 1.0
            y = oracle.scan2d_fwd(ones, ones, A, Bm, ones, None, None, dtype=F64)
            assert y[0, 0, 2, 2] == pytest.approx(alpha ** e2d[i2, j2], rel=1e-14)
            # the same map flattened row-major and scanned as one row (H = 1): the 1D scan
            y1 = oracle.scan2d_fwd(ones.reshape(1, 1, 1, 9), ones.reshape(1, 1, 1, 9), A,
                                   Bm.reshape(1, 1, 1, 9), ones.reshape(1, 1, 1, 9), None, None, dtype=F64)
            assert y1[0, 0, 0, 8] == pytest.approx(alpha ** e1d[i2, j2], rel=1e-14)
    # the contrast the paper draws: Manhattan distance 4 instead of flattened distance 8
    assert e2d[0, 0] == 4 and e1d[0, 0] == 8


@pytest.mark.parametrize("shape", [(1, 2, 3, 4, 5), (2, 1, 2, 6, 3), (1, 1, 1, 5, 6)])
def test_brute_force_closed_form(shape):
    Bt, Dc, N, H, W = shape
    rng = np.random.default_rng(11 + H * W)
    p = rand_problem(rng, Bt, Dc, N, H, W)
    y = oracle.scan2d_fwd(*p, dtype=F64)
    np.testing.assert_allclose(y, brute_force_y(*p), rtol=1e-11, atol=1e-12)


def scan1d(a, u):
    """Eq. 1: h_t = a_t h_{t-1} + u_t, h_0 = 0."""
    h, out = 0.0, []
    for at, ut in zip(a, u):
        h = at * h + ut
        out.append(h)
    return np.array(out)


@pytest.mark.parametrize("axis", ["row", "col"])
def test_single_row_or_column_is_the_1d_selective_scan(axis):
    rng = np.random.default_rng(5)
    L, N, Dc = 13, 3, 2
    shape = (1, Dc, 1, L) if axis == "row" else (1, Dc, L, 1)
    sshape = (1, N, 1, L) if axis == "row" else (1, N, L, 1)
    x = rng.standard_normal(shape)
    delta = np.logaddexp(0, rng.normal(-1, 0.5, shape))
    A = (-np.exp(rng.normal(0, 0.5, (Dc, N)))).astype(np.float32)
    Bm, Cm = rng.standard_normal(sshape), rng.standard_normal(sshape)
    Dskip = rng.standard_normal(Dc).astype(np.float32)
    y = oracle.scan2d_fwd(x, delta, A, Bm, Cm, Dskip, None, dtype=F64).reshape(Dc, L)
    for c in range(Dc):
        xs, ds = x[0, c].reshape(L), delta[0, c].reshape(L)
        ref = float(Dskip[c]) * xs
        for n in range(N):
            h = scan1d(np.exp(ds * float(A[c, n])), ds * Bm[0, n].reshape(L) * xs)
            ref = ref + Cm[0, n].reshape(L) * h           # Eq. 2
        np.testing.assert_allclose(y[c], ref, rtol=1e-12, atol=1e-13)


def test_unit_decay_gives_summed_area_table():
    """A = 0 -> a = exp(0) = 1 exactly -> h is the inclusive 2D prefix sum of u."""
    rng = np.random.default_rng(7)
    H, W = 9, 7
    x = rng.standard_normal((1, 1, H, W))
    delta = np.logaddexp(0, rng.normal(-1, 0.5, (1, 1, H, W)))
    Bm = rng.standard_normal((1, 1, H, W))
    ones = np.ones((1, 1, H, W))
    y = oracle.scan2d_fwd(x, delta, np.zeros((1, 1), np.float32), Bm, ones, None, None, dtype=F64)
    sat = np.cumsum(np.cumsum(delta * Bm * x, axis=-1), axis=-2)
    np.testing.assert_allclose(y, sat, rtol=1e-12, atol=1e-13)


def test_constant_decay_is_separable_matmul():
    """Constant alpha: h = G_H u G_W^T with G[k,l] = alpha^(k-l) for k >= l (Eq. 7 verbatim)."""
    rng = np.random.default_rng(8)
    H, W = 6, 8
    A = np.array([[-0.75]], np.float32)
    dl = 0.5
    alpha = np.exp(dl * float(A[0, 0]))
    x = rng.standard_normal((1, 1, H, W))
    Bm = rng.standard_normal((1, 1, H, W))
    delta = np.full((1, 1, H, W), dl)
    ones = np.ones((1, 1, H, W))
    y = oracle.scan2d_fwd(x, delta, A, Bm, ones, None, None, dtype=F64)[0, 0]

    def G(n):
        k = np.arange(n)
        d = k[:, None] - k[None, :]
        return np.where(d >= 0, alpha ** np.maximum(d, 0), 0.0)

    u = (delta * Bm * x)[0, 0]
    np.testing.assert_allclose(y, G(H) @ u @ G(W).T, rtol=1e-12, atol=1e-13)


def test_linear_in_x_and_skip_term():
    rng = np.random.default_rng(9)
    x, delta, A, Bm, Cm, Dskip, mask = rand_problem(rng, 1, 2, 3, 5, 6)
    x2 = rng.standard_normal(x.shape)
    f = lambda xx, D=Dskip: oracle.scan2d_fwd(xx, delta, A, Bm, Cm, D, mask, dtype=F64)
    np.testing.assert_allclose(f(2.0 * x - 3.0 * x2), 2.0 * f(x) - 3.0 * f(x2), rtol=1e-11, atol=1e-12)
    # the skip term is exactly Dskip[c] * x_eff added on top
    xe = np.where(mask[:, None] != 0, 0.0, x)
    np.testing.assert_allclose(f(x) - f(x, None), Dskip[None, :, None, None] * xe, rtol=1e-11, atol=1e-12)


def test_causality_upper_left_quadrant_only():
    rng = np.random.default_rng(10)
    p = list(rand_problem(rng, 1, 2, 2, 6, 7, with_mask=False))
    y0 = oracle.scan2d_fwd(*p, dtype=F64)
    i0, j0 = 3, 4
    q = [None if t is None else t.copy() for t in p]
    for k in (0, 1):                       # x, delta [b,c,i,j]
        q[k][..., i0 + 1:, :] += 5.0
        q[k][..., :, j0 + 1:] += 5.0
    for k in (3, 4):                       # Bm, Cm
        q[k][..., i0 + 1:, :] -= 2.0
        q[k][..., :, j0 + 1:] -= 2.0
    y1 = oracle.scan2d_fwd(*q, dtype=F64)
    assert np.array_equal(y0[..., :i0 + 1, :j0 + 1], y1[..., :i0 + 1, :j0 + 1])
    assert not np.array_equal(y0, y1)


def test_mask_is_a_select_on_x():
    rng = np.random.default_rng(12)
    x, delta, A, Bm, Cm, Dskip, mask = rand_problem(rng, 2, 3, 2, 5, 5)
    m4 = mask[:, None] != 0
    y_mask = oracle.scan2d_fwd(x, delta, A, Bm, Cm, Dskip, mask, dtype=F64)
    y_zero = oracle.scan2d_fwd(np.where(m4, 0.0, x), delta, A, Bm, Cm, Dskip, None, dtype=F64)
    assert np.array_equal(y_mask, y_zero)
    for poison in (np.nan, np.inf, 1e300):
        y_p = oracle.scan2d_fwd(np.where(m4, poison, x), delta, A, Bm, Cm, Dskip, mask, dtype=F64)
        assert np.array_equal(y_mask, y_p)
    full = np.ones_like(mask)
    assert not oracle.scan2d_fwd(x, delta, A, Bm, Cm, Dskip, full, dtype=F64).any()
    # decay still acts at background cells: y there is generally non-zero (state flows through)
    assert np.abs(y_mask[np.broadcast_to(m4, y_mask.shape)]).max() > 0


# ------------------------------------------------------------------------ storage precisions

def test_bf16_rounding_is_single_and_ties_to_even():
    """The oracle rounds its double result to bf16 once, to nearest-even (no fp32 detour)."""
    ulp = 2.0 ** -7                                   # bf16 spacing in [1, 2)
    cases = {
        1.0 + 0.5 * ulp: 1.0,                         # tie -> even mantissa
        1.0 + 1.5 * ulp: 1.0 + 2 * ulp,               # tie -> even mantissa
        1.0 + 0.5 * ulp + 2.0 ** -30: 1.0 + ulp,      # just above a tie; an fp32 detour drops 2^-30
        1.0 + 0.5 * ulp - 2.0 ** -40: 1.0,
        -3.0 - 2.0 ** -8: -3.0,                       # spacing 2^-6 in [2, 4): below half stays
        2.0 ** -130: 2.0 ** -130,                     # bf16 sub-normal, representable
    }
    for v, want in cases.items():
        assert _round_via_oracle(v) == np.float32(want), v
    rng = np.random.default_rng(3)
    vals = rng.standard_normal(200).astype(np.float32)
    got = np.array([_round_via_oracle(float(v)) for v in vals])
    np.testing.assert_array_equal(got, wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(vals)))


def _round_via_oracle(v):
    """Make the oracle produce the double v and round it: with A = 0 (a = 1) and
    delta = Bm = Cm = 1 the last state of a 1 x K row is the exact sum of the K inputs, which
    are bf16-representable terms adding up to v."""
    terms = _split_bf16_exact(v)
    K = len(terms)
    x = wl.f32_to_bf16_bits(np.array(terms, np.float32)).reshape(1, 1, 1, K)
    assert np.array_equal(wl.bf16_bits_to_f32(x).reshape(-1), np.array(terms, np.float32))
    one = wl.f32_to_bf16_bits(np.ones((1, 1, 1, K), np.float32))
    A = np.zeros((1, 1), np.float32)
    y = oracle.scan2d_fwd(x, one, A, one, one, None, None, dtype=oracle.BF16)
    return wl.bf16_bits_to_f32(y)[0, 0, 0, K - 1]


def _split_bf16_exact(v):
    """Greedy split of a double into bf16-representable terms that sum to it exactly."""
    terms, r = [], float(v)
    while r != 0.0 and len(terms) < 12:
        t = float(wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(np.array([r], np.float32)))[0])
        if t == 0.0:
            break
        terms.append(t)
        r -= t
    assert r == 0.0, "value not exactly representable as a short sum of bf16 terms"
    return terms or [0.0]


@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_low_precision_storage_matches_double_path(dtype):
    rng = np.random.default_rng(21)
    x, delta, A, Bm, Cm, Dskip, mask = rand_problem(rng, 2, 3, 4, 7, 9)

    def store(a):
        a32 = a.astype(np.float32)
        return wl.f32_to_bf16_bits(a32) if dtype == oracle.BF16 else a32

    xs, ds, Bs, Cs = store(x), store(delta), store(Bm), store(Cm)
    y = oracle.scan2d_fwd(xs, ds, A, Bs, Cs, Dskip, mask, dtype=dtype)
    wide = [wl.to_float(t, dtype) for t in (xs, ds, Bs, Cs)]
    y64 = oracle.scan2d_fwd(wide[0], wide[1], A, wide[2], wide[3], Dskip, mask, dtype=F64)
    if dtype == oracle.BF16:
        # one rounding of the double result, to nearest: within half a bf16 ulp, and idempotent
        yf = wl.bf16_bits_to_f32(y).astype(np.float64)
        assert np.all(np.abs(yf - y64) <= 2.0 ** -8 * np.abs(y64) + 1e-40)
    else:
        np.testing.assert_array_equal(y, y64.astype(np.float32))


# ---------------------------------------------------------------------------- backward pins

def loss(p, dy):
    return float(np.sum(dy * oracle.scan2d_fwd(*p, dtype=F64)))


def test_backward_matches_central_differences_for_every_input():
    rng = np.random.default_rng(31)
    Bt, Dc, N, H, W = 2, 2, 3, 4, 5
    x, delta, A, Bm, Cm, Dskip, mask = rand_problem(rng, Bt, Dc, N, H, W)
    # fp32 parameters on a dyadic grid so that +-eps is exact in fp32
    A = (np.round(A * 64) / 64).astype(np.float32)
    Dskip = (np.round(Dskip * 64) / 64).astype(np.float32)
    dy = rng.standard_normal(x.shape)
    p = [x, delta, A, Bm, Cm, Dskip, mask]
    dx, ddelta, dA, dBm, dCm, dD = oracle.scan2d_bwd(x, delta, A, Bm, Cm, Dskip, mask, dy, dtype=F64)
    grads = {0: dx, 1: ddelta, 2: dA, 3: dBm, 4: dCm, 5: dD}
    for k, g in grads.items():
        eps = 2.0 ** -12 if k in (2, 5) else 1e-6
        fd = np.zeros(p[k].shape)
        it = np.nditer(p[k], flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            hi = [t if t is None else t.copy() for t in p]
            lo = [t if t is None else t.copy() for t in p]
            hi[k][idx] += eps
            lo[k][idx] -= eps
            fd[idx] = (loss(hi, dy) - loss(lo, dy)) / (2 * eps)
        tol = 2e-6 if k in (2, 5) else 1e-7       # dA, dDskip come back rounded to fp32
        np.testing.assert_allclose(g, fd, rtol=tol, atol=tol * np.abs(fd).max(), err_msg=f"input {k}")
    # background cells get exactly zero dx
    assert not dx[np.broadcast_to(mask[:, None] != 0, dx.shape)].any()


def test_backward_adjoint_identity_in_x():
    """x -> y is linear (mask and skip included): <dy, y(x)> == <dx(dy), x>."""
    rng = np.random.default_rng(32)
    x, delta, A, Bm, Cm, Dskip, mask = rand_problem(rng, 1, 3, 4, 6, 5)
    dy = rng.standard_normal(x.shape)
    y = oracle.scan2d_fwd(x, delta, A, Bm, Cm, Dskip, mask, dtype=F64)
    dx = oracle.scan2d_bwd(x, delta, A, Bm, Cm, Dskip, mask, dy, dtype=F64)[0]
    assert np.sum(dy * y) == pytest.approx(np.sum(dx * x), rel=1e-12)


def test_backward_single_row_is_the_1d_reverse_recurrence():
    rng = np.random.default_rng(33)
    L, N = 11, 2
    x = rng.standard_normal((1, 1, 1, L))
    delta = np.logaddexp(0, rng.normal(-1, 0.5, (1, 1, 1, L)))
    A = np.array([[-0.5, -1.25]], np.float32)
    Bm, Cm = rng.standard_normal((1, N, 1, L)), rng.standard_normal((1, N, 1, L))
    dy = rng.standard_normal((1, 1, 1, L))
    dx, ddelta, dA, dBm, dCm, _ = oracle.scan2d_bwd(x, delta, A, Bm, Cm, None, None, dy, dtype=F64)
    xs, ds, dys = x.reshape(L), delta.reshape(L), dy.reshape(L)
    dx_ref, dd_ref = np.zeros(L), np.zeros(L)
    for n in range(N):
        a = np.exp(ds * float(A[0, n]))
        u = ds * Bm[0, n, 0] * xs
        h = scan1d(a, u)
        dh = np.zeros(L)                    # reverse recurrence of Eq. 1
        carry = 0.0
        for t in range(L - 1, -1, -1):
            dh[t] = dys[t] * Cm[0, n, 0, t] + carry
            carry = a[t] * dh[t]
        hprev = np.concatenate([[0.0], h[:-1]])
        da = dh * hprev
        dx_ref += dh * ds * Bm[0, n, 0]
        dd_ref += da * a * float(A[0, n]) + dh * Bm[0, n, 0] * xs
        np.testing.assert_allclose(dBm[0, n, 0], dh * ds * xs, rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(dCm[0, n, 0], dys * h, rtol=1e-6, atol=1e-7)
        assert dA[0, n] == pytest.approx(np.sum(da * a * ds), rel=1e-6)
    np.testing.assert_allclose(dx.reshape(L), dx_ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(ddelta.reshape(L), dd_ref, rtol=1e-12, atol=1e-13)


def test_backward_unit_decay_is_reverse_summed_area_table():
    rng = np.random.default_rng(34)
    H, W = 5, 6
    x = rng.standard_normal((1, 1, H, W))
    delta = np.logaddexp(0, rng.normal(-1, 0.5, (1, 1, H, W)))
    Bm, Cm = rng.standard_normal((1, 1, H, W)), rng.standard_normal((1, 1, H, W))
    dy = rng.standard_normal((1, 1, H, W))
    Dskip = np.array([0.5], np.float32)
    dx, *_ , dD = oracle.scan2d_bwd(x, delta, np.zeros((1, 1), np.float32), Bm, Cm, Dskip, None, dy, dtype=F64)
    q = np.flip(np.cumsum(np.cumsum(np.flip(dy * Cm, (-1, -2)), axis=-1), axis=-2), (-1, -2))
    np.testing.assert_allclose(dx, q * delta * Bm + 0.5 * dy, rtol=1e-12, atol=1e-13)
    assert dD[0] == pytest.approx(np.sum(dy * x), rel=1e-6)


@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_backward_low_precision_storage_matches_double_path(dtype):
    rng = np.random.default_rng(35)
    x, delta, A, Bm, Cm, Dskip, mask = rand_problem(rng, 2, 3, 2, 5, 6)
    dy = rng.standard_normal(x.shape)

    def store(a):
        a32 = a.astype(np.float32)
        return wl.f32_to_bf16_bits(a32) if dtype == oracle.BF16 else a32

    s = [store(t) for t in (x, delta, Bm, Cm, dy)]
    w = [wl.to_float(t, dtype) for t in s]
    lo = oracle.scan2d_bwd(s[0], s[1], A, s[2], s[3], Dskip, mask, s[4], dtype=dtype)
    hi = oracle.scan2d_bwd(w[0], w[1], A, w[2], w[3], Dskip, mask, w[4], dtype=F64)
    for k in range(6):
        a = wl.to_float(lo[k], dtype) if k < 2 else lo[k].astype(np.float64)
        rel = 2.0 ** -8 if (dtype == oracle.BF16 and k < 2) else 2.0 ** -23
        assert np.all(np.abs(a - hi[k]) <= rel * np.abs(hi[k]) + 1e-30), k


def test_thread_count_does_not_change_results():
    rng = np.random.default_rng(36)
    x, delta, A, Bm, Cm, Dskip, mask = rand_problem(rng, 2, 5, 3, 6, 7)
    dy = rng.standard_normal(x.shape)
    y1 = oracle.scan2d_fwd(x, delta, A, Bm, Cm, Dskip, mask, dtype=F64, threads=1)
    y4 = oracle.scan2d_fwd(x, delta, A, Bm, Cm, Dskip, mask, dtype=F64, threads=4)
    assert np.array_equal(y1, y4)
    g1 = oracle.scan2d_bwd(x, delta, A, Bm, Cm, Dskip, mask, dy, dtype=F64, threads=1)
    g4 = oracle.scan2d_bwd(x, delta, A, Bm, Cm, Dskip, mask, dy, dtype=F64, threads=4)
    for a, b in zip(g1, g4):
        np.testing.assert_allclose(a, b, rtol=1e-6, atol=1e-9)   # channel sums re-associate


# ---------------------------------------------------------------------------- softplus step (Eq. 3)

def test_softplus_step_is_log1p_exp_with_its_asymptotes():
    """delta = softplus(raw + bias[c]) (Eq. 3; bias as in the supplementary algorithm): against
    math.log1p(math.exp(t)) element by element, and against its two asymptotes (t for large t,
    exp(t) for very negative t)."""
    import math
    rng = np.random.default_rng(41)
    Bt, Dc, N, H, W = 1, 2, 2, 3, 4
    x, _, A, Bm, Cm, Dskip, mask = rand_problem(rng, Bt, Dc, N, H, W)
    raw = rng.normal(0.0, 3.0, x.shape)
    bias = np.array([0.25, -1.5], np.float32)
    delta = np.empty_like(raw)
    for idx in np.ndindex(raw.shape):
        delta[idx] = math.log1p(math.exp(raw[idx] + float(bias[idx[1]])))
    want = oracle.scan2d_fwd(x, delta, A, Bm, Cm, Dskip, mask, dtype=F64)
    got = oracle.scan2d_fwd_softplus(x, raw, bias, A, Bm, Cm, Dskip, mask, dtype=F64)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-13)
    # no bias = zero bias
    np.testing.assert_array_equal(oracle.scan2d_fwd_softplus(x, raw, None, A, Bm, Cm, Dskip, mask, dtype=F64),
                                  oracle.scan2d_fwd_softplus(x, raw, np.zeros(Dc, np.float32), A, Bm, Cm, Dskip, mask, dtype=F64))
    # asymptotes: softplus(t) -> t (t = 40: the difference is e^-40), -> exp(t) (t = -40)
    big = np.full(x.shape, 40.0)
    np.testing.assert_allclose(oracle.scan2d_fwd_softplus(x, big, None, A, Bm, Cm, Dskip, mask, dtype=F64),
                               oracle.scan2d_fwd(x, big, A, Bm, Cm, Dskip, mask, dtype=F64), rtol=1e-12, atol=1e-12)
    small = np.full(x.shape, -40.0)
    np.testing.assert_allclose(oracle.scan2d_fwd_softplus(x, small, None, A, Bm, Cm, Dskip, mask, dtype=F64),
                               oracle.scan2d_fwd(x, np.exp(small), A, Bm, Cm, Dskip, mask, dtype=F64), rtol=1e-12, atol=1e-30)


def test_softplus_backward_matches_central_differences_and_the_logistic_chain_rule():
    from scipy.special import expit
    rng = np.random.default_rng(43)
    Bt, Dc, N, H, W = 2, 2, 3, 3, 4
    x, _, A, Bm, Cm, Dskip, mask = rand_problem(rng, Bt, Dc, N, H, W)
    raw = rng.normal(-0.5, 1.5, x.shape)
    bias = (np.round(rng.normal(0, 1, Dc) * 64) / 64).astype(np.float32)
    dy = rng.standard_normal(x.shape)

    def f(r, b):
        return float(np.sum(dy * oracle.scan2d_fwd_softplus(x, r, b, A, Bm, Cm, Dskip, mask, dtype=F64)))

    dx, draw, dbias, dA, dBm, dCm, dD = oracle.scan2d_bwd_softplus(x, raw, bias, A, Bm, Cm, Dskip, mask, dy, dtype=F64)
    fd = np.zeros(raw.shape)
    for idx in np.ndindex(raw.shape):
        hi, lo = raw.copy(), raw.copy()
        hi[idx] += 1e-6
        lo[idx] -= 1e-6
        fd[idx] = (f(hi, bias) - f(lo, bias)) / 2e-6
    np.testing.assert_allclose(draw, fd, rtol=1e-7, atol=1e-7 * np.abs(fd).max())
    eps = 2.0 ** -12
    for c in range(Dc):
        hi, lo = bias.copy(), bias.copy()
        hi[c] += eps
        lo[c] -= eps
        assert abs((f(raw, hi) - f(raw, lo)) / (2 * eps) - dbias[c]) <= 2e-6 * max(1.0, abs(dbias[c]))
    # chain rule with a library logistic function on top of the plain backward
    t = raw + bias[None, :, None, None].astype(np.float64)
    plain = oracle.scan2d_bwd(x, np.logaddexp(0.0, t), A, Bm, Cm, Dskip, mask, dy, dtype=F64)
    np.testing.assert_allclose(draw, plain[1] * expit(t), rtol=1e-12, atol=1e-14)
    for a, b in zip((dx, dA, dBm, dCm, dD), (plain[0], plain[2], plain[3], plain[4], plain[5])):
        np.testing.assert_array_equal(a, b)
    assert oracle.scan2d_bwd_softplus(x, raw, None, A, Bm, Cm, Dskip, mask, dy, dtype=F64)[2] is None


@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_softplus_low_precision_storage_rounds_once(dtype):
    rng = np.random.default_rng(47)
    Bt, Dc, N, H, W = 1, 3, 4, 5, 6
    x, _, A, Bm, Cm, Dskip, mask = rand_problem(rng, Bt, Dc, N, H, W)
    raw = rng.normal(-1.0, 1.0, x.shape)
    bias = rng.normal(0, 1, Dc).astype(np.float32)
    st = lambda a: wl.f32_to_bf16_bits(a.astype(np.float32)) if dtype == oracle.BF16 else a.astype(np.float32)
    xs, rs, Bs, Cs = st(x), st(raw), st(Bm), st(Cm)
    wide = lambda a: wl.to_float(a, dtype).astype(np.float64)
    y = oracle.scan2d_fwd_softplus(xs, rs, bias, A, Bs, Cs, Dskip, mask, dtype=dtype)
    y64 = oracle.scan2d_fwd_softplus(wide(xs), wide(rs), bias, A, wide(Bs), wide(Cs), Dskip, mask, dtype=F64)
    want = wl.f32_to_bf16_bits(y64.astype(np.float32)) if dtype == oracle.BF16 else y64.astype(np.float32)
    if dtype == oracle.F32:
        np.testing.assert_array_equal(y, want)
    else:   # double -> fp32 -> bf16 may differ from the single rounding by one unit in rare ties
        assert np.abs(y.astype(np.int32) - want.astype(np.int32)).max() <= 1


# ---------------------------------------------------------------------------- output gate (Fig. 2)

def test_output_gate_is_silu_of_z_times_the_scan_output():
    """y = y_scan * z / (1 + exp(-z)): against math.exp element by element, the values SiLU(1),
    SiLU(-1) and SiLU(0) = 0, and the asymptote SiLU(z) -> z."""
    import math
    rng = np.random.default_rng(51)
    Bt, Dc, N, H, W = 2, 2, 3, 3, 5
    x, _, A, Bm, Cm, Dskip, mask = rand_problem(rng, Bt, Dc, N, H, W)
    raw = rng.normal(-0.5, 1.0, x.shape)
    z = rng.normal(0.0, 2.0, x.shape)
    ys, y = oracle.scan2d_fwd_softplus_gated(x, raw, None, A, Bm, Cm, Dskip, mask, z, dtype=F64)
    np.testing.assert_array_equal(ys, oracle.scan2d_fwd_softplus(x, raw, None, A, Bm, Cm, Dskip, mask, dtype=F64))
    for idx in np.ndindex(z.shape):
        assert abs(y[idx] - ys[idx] * z[idx] / (1.0 + math.exp(-z[idx]))) <= 1e-14 * max(1.0, abs(y[idx]))
    one = np.ones(x.shape)
    np.testing.assert_allclose(oracle.scan2d_fwd_softplus_gated(x, raw, None, A, Bm, Cm, Dskip, mask, one, dtype=F64)[1],
                               ys * 0.7310585786300049, rtol=1e-14)
    np.testing.assert_allclose(oracle.scan2d_fwd_softplus_gated(x, raw, None, A, Bm, Cm, Dskip, mask, -one, dtype=F64)[1],
                               ys * -0.2689414213699951, rtol=1e-14)
    assert not oracle.scan2d_fwd_softplus_gated(x, raw, None, A, Bm, Cm, Dskip, mask, 0 * one, dtype=F64)[1].any()
    np.testing.assert_allclose(oracle.scan2d_fwd_softplus_gated(x, raw, None, A, Bm, Cm, Dskip, mask, 40 * one, dtype=F64)[1],
                               ys * 40.0, rtol=1e-14)


def test_gated_backward_matches_central_differences_in_every_input():
    rng = np.random.default_rng(53)
    Bt, Dc, N, H, W = 2, 2, 2, 3, 3
    x, _, A, Bm, Cm, Dskip, mask = rand_problem(rng, Bt, Dc, N, H, W)
    raw = rng.normal(-0.5, 1.0, x.shape)
    bias = (np.round(rng.normal(0, 1, Dc) * 64) / 64).astype(np.float32)
    z = rng.normal(0.0, 1.5, x.shape)
    dy = rng.standard_normal(x.shape)
    A64 = A.astype(np.float64)

    def f(x_=x, raw_=raw, z_=z, Bm_=Bm, Cm_=Cm):
        return float(np.sum(dy * oracle.scan2d_fwd_softplus_gated(x_, raw_, bias, A, Bm_, Cm_, Dskip, mask, z_, dtype=F64)[1]))

    grads = oracle.scan2d_bwd_softplus_gated(x, raw, bias, A, Bm, Cm, Dskip, mask, z, dy, dtype=F64)
    dx, draw, dbias, dA, dBm, dCm, dD, dz = grads
    for name, arr, got in (("x_", x, dx), ("raw_", raw, draw), ("z_", z, dz), ("Bm_", Bm, dBm), ("Cm_", Cm, dCm)):
        fd = np.zeros(arr.shape)
        for idx in np.ndindex(arr.shape):
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += 1e-6
            lo[idx] -= 1e-6
            fd[idx] = (f(**{name: hi}) - f(**{name: lo})) / 2e-6
        if name == "x_":
            fd[np.broadcast_to(mask[:, None] != 0, fd.shape)] = 0.0     # x under the mask does not exist
        np.testing.assert_allclose(got, fd, rtol=2e-7, atol=2e-7 * max(1e-30, np.abs(fd).max()), err_msg=name)
    # the gate changes nothing but dy: every other gradient is the ungated backward fed dy * SiLU(z)
    s = 1.0 / (1.0 + np.exp(-z))
    plain = oracle.scan2d_bwd_softplus(x, raw, bias, A, Bm, Cm, Dskip, mask, dy * z * s, dtype=F64)
    for a, b in zip(grads[:7], plain):
        np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-15)
    assert A64.shape == dA.shape


@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_gated_output_is_rounded_once_from_the_unrounded_scan(dtype):
    rng = np.random.default_rng(57)
    Bt, Dc, N, H, W = 1, 3, 4, 5, 6
    x, _, A, Bm, Cm, Dskip, mask = rand_problem(rng, Bt, Dc, N, H, W)
    raw = rng.normal(-1.0, 1.0, x.shape)
    z = rng.normal(0.0, 1.5, x.shape)
    st = lambda a: wl.f32_to_bf16_bits(a.astype(np.float32)) if dtype == oracle.BF16 else a.astype(np.float32)
    xs, rs, Bs, Cs, zs = st(x), st(raw), st(Bm), st(Cm), st(z)
    wide = lambda a: wl.to_float(a, dtype).astype(np.float64)
    ys, y = oracle.scan2d_fwd_softplus_gated(xs, rs, None, A, Bs, Cs, Dskip, mask, zs, dtype=dtype)
    ys64, y64 = oracle.scan2d_fwd_softplus_gated(wide(xs), wide(rs), None, A, wide(Bs), wide(Cs), Dskip, mask, wide(zs), dtype=F64)
    for got, ref in ((ys, ys64), (y, y64)):
        want = wl.f32_to_bf16_bits(ref.astype(np.float32)) if dtype == oracle.BF16 else ref.astype(np.float32)
        if dtype == oracle.F32:
            np.testing.assert_array_equal(got, want)
        else:
            assert np.abs(got.astype(np.int32) - want.astype(np.int32)).max() <= 1


# ---------------------------------------------------------------------------- identity cells (skip mask mode)

def test_skipped_row_or_column_behaves_as_if_it_were_not_there():
    """A fully masked row (column) of identity cells passes the state through: every other output equals
    that of the map with the row (column) deleted (Supp. "Tiling and edge cases": A-bar = 1, x = 0)."""
    rng = np.random.default_rng(61)
    Bt, Dc, N, H, W = 2, 3, 3, 5, 6
    x, delta, A, Bm, Cm, Dskip, _ = rand_problem(rng, Bt, Dc, N, H, W)
    for axis, idx in ((2, 2), (3, 4), (2, 0), (3, 0), (2, H - 1)):
        mask = np.zeros((Bt, H, W), np.uint8)
        if axis == 2:
            mask[:, idx, :] = 1
        else:
            mask[:, :, idx] = 1
        y = oracle.scan2d_fwd_skip(x, delta, A, Bm, Cm, Dskip, mask, dtype=F64)
        cut = lambda a: np.ascontiguousarray(np.delete(a, idx, axis=axis))
        y_cut = oracle.scan2d_fwd(cut(x), cut(delta), A, cut(Bm), cut(Cm), Dskip, None, dtype=F64)
        np.testing.assert_allclose(cut(y), y_cut, rtol=1e-13, atol=1e-13)
    # without masked cells the mode changes nothing; the zero-token mode does not have the property
    none = np.zeros((Bt, H, W), np.uint8)
    np.testing.assert_array_equal(oracle.scan2d_fwd_skip(x, delta, A, Bm, Cm, Dskip, none, dtype=F64),
                                  oracle.scan2d_fwd(x, delta, A, Bm, Cm, Dskip, none, dtype=F64))
    mask = np.zeros((Bt, H, W), np.uint8)
    mask[:, 2, :] = 1
    y0 = oracle.scan2d_fwd(x, delta, A, Bm, Cm, Dskip, mask, dtype=F64)
    cut = lambda a: np.ascontiguousarray(np.delete(a, 2, axis=2))
    assert np.abs(cut(y0) - oracle.scan2d_fwd(cut(x), cut(delta), A, cut(Bm), cut(Cm), Dskip, None, dtype=F64)).max() > 1e-3


def test_skip_mode_backward_matches_central_differences():
    rng = np.random.default_rng(63)
    Bt, Dc, N, H, W = 1, 2, 2, 4, 4
    x, delta, A, Bm, Cm, Dskip, mask = rand_problem(rng, Bt, Dc, N, H, W)
    mask[0, 1, 2] = 1
    mask[0, 3, 0] = 1
    dy = rng.standard_normal(x.shape)
    m4 = np.broadcast_to(mask[:, None] != 0, x.shape)

    def f(x_=x, d_=delta, Bm_=Bm, Cm_=Cm):
        return float(np.sum(dy * oracle.scan2d_fwd_skip(x_, d_, A, Bm_, Cm_, Dskip, mask, dtype=F64)))

    dx, dd, dA, dBm, dCm, dD = oracle.scan2d_bwd_skip(x, delta, A, Bm, Cm, Dskip, mask, dy, dtype=F64)
    for name, arr, got in (("x_", x, dx), ("d_", delta, dd), ("Bm_", Bm, dBm), ("Cm_", Cm, dCm)):
        fd = np.zeros(arr.shape)
        for idx in np.ndindex(arr.shape):
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += 1e-6
            lo[idx] -= 1e-6
            fd[idx] = (f(**{name: hi}) - f(**{name: lo})) / 2e-6
        if name in ("x_", "d_"):
            assert not np.abs(fd[m4]).max() > 0          # the function does not depend on x or the step under the mask
            assert not got[m4].any()
        np.testing.assert_allclose(got, fd, rtol=2e-7, atol=2e-7 * max(1e-30, np.abs(fd).max()), err_msg=name)


# ---------------------------------------------------------------------------- columns first (scan order ablation)

def test_columns_first_is_the_two_recurrences_in_the_other_order():
    """v[i,j] = a v[i-1,j] + u, then h[i,j] = a h[i,j-1] + v, written as loops; equal to the row-first scan
    when the decay does not depend on the position (the two scans then commute), different otherwise."""
    rng = np.random.default_rng(71)
    Bt, Dc, N, H, W = 2, 2, 3, 4, 5
    x, delta, A, Bm, Cm, Dskip, mask = rand_problem(rng, Bt, Dc, N, H, W)
    y = oracle.scan2d_fwd_columns_first(x, delta, A, Bm, Cm, Dskip, mask, dtype=F64)
    want = np.zeros_like(y)
    for b in range(Bt):
        for c in range(Dc):
            for n in range(N):
                v = np.zeros((H, W))
                h = np.zeros((H, W))
                for i in range(H):
                    for j in range(W):
                        xe = 0.0 if mask[b, i, j] else x[b, c, i, j]
                        a = np.exp(delta[b, c, i, j] * float(A[c, n]))
                        u = delta[b, c, i, j] * Bm[b, n, i, j] * xe
                        v[i, j] = a * (v[i - 1, j] if i > 0 else 0.0) + u
                        h[i, j] = a * (h[i, j - 1] if j > 0 else 0.0) + v[i, j]
                want[b, c] += Cm[b, n] * h
            xe = np.where(mask[b] != 0, 0.0, x[b, c])
            want[b, c] += float(Dskip[c]) * xe
    np.testing.assert_allclose(y, want, rtol=1e-12, atol=1e-13)
    assert np.abs(y - oracle.scan2d_fwd(x, delta, A, Bm, Cm, Dskip, mask, dtype=F64)).max() > 1e-3
    const = np.full_like(delta, 0.37)                  # position-independent decay: the scans commute
    np.testing.assert_allclose(oracle.scan2d_fwd_columns_first(x, const, A, Bm, Cm, Dskip, mask, dtype=F64),
                               oracle.scan2d_fwd(x, const, A, Bm, Cm, Dskip, mask, dtype=F64), rtol=1e-12, atol=1e-13)


def test_columns_first_backward_matches_central_differences():
    rng = np.random.default_rng(73)
    Bt, Dc, N, H, W = 1, 2, 2, 3, 4
    x, delta, A, Bm, Cm, Dskip, mask = rand_problem(rng, Bt, Dc, N, H, W)
    dy = rng.standard_normal(x.shape)

    def f(x_=x, d_=delta, Bm_=Bm, Cm_=Cm):
        return float(np.sum(dy * oracle.scan2d_fwd_columns_first(x_, d_, A, Bm_, Cm_, Dskip, mask, dtype=F64)))

    dx, dd, dA, dBm, dCm, dD = oracle.scan2d_bwd_columns_first(x, delta, A, Bm, Cm, Dskip, mask, dy, dtype=F64)
    for name, arr, got in (("x_", x, dx), ("d_", delta, dd), ("Bm_", Bm, dBm), ("Cm_", Cm, dCm)):
        fd = np.zeros(arr.shape)
        for idx in np.ndindex(arr.shape):
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += 1e-6
            lo[idx] -= 1e-6
            fd[idx] = (f(**{name: hi}) - f(**{name: lo})) / 2e-6
        if name == "x_":
            fd[np.broadcast_to(mask[:, None] != 0, fd.shape)] = 0.0
        np.testing.assert_allclose(got, fd, rtol=2e-7, atol=2e-7 * max(1e-30, np.abs(fd).max()), err_msg=name)


# ----------------------------------------------------------------------------- padding token, independent vertical decay
# oracle.scan2d_fwd_variants / scan2d_bwd_variants (Eq. 4 and the padding-token ablation; the supplement's ablation
# of re-using A-bar for the vertical scan).

def brute_force_variants(x, delta, A, A_v, Bm, Cm, Dskip, mask, pad):
    """Path-product closed form with its own decay on the vertical leg: right along row i' with a = exp(delta A),
    then down column j with a_v = exp(delta A_v); x under the mask is pad[c].  Pure loops, no recurrence."""
    Bt, Dc, H, W = x.shape
    N = A.shape[1]
    y = np.zeros((Bt, Dc, H, W))
    for b in range(Bt):
        for c in range(Dc):
            xe = np.where(mask[b] != 0, float(pad[c]) if pad is not None else 0.0, x[b, c]) if mask is not None else x[b, c]
            for i in range(H):
                for j in range(W):
                    acc = 0.0
                    for n in range(N):
                        a = np.exp(delta[b, c] * float(A[c, n]))
                        av = np.exp(delta[b, c] * float((A_v if A_v is not None else A)[c, n]))
                        hsum = 0.0
                        for i2 in range(i + 1):
                            for j2 in range(j + 1):
                                w = 1.0
                                for s in range(j2 + 1, j + 1):
                                    w *= a[i2, s]
                                for r in range(i2 + 1, i + 1):
                                    w *= av[r, j]
                                hsum += w * delta[b, c, i2, j2] * Bm[b, n, i2, j2] * xe[i2, j2]
                        acc += Cm[b, n, i, j] * hsum
                    y[b, c, i, j] = acc + (float(Dskip[c]) * xe[i, j] if Dskip is not None else 0.0)
    return y


def _variant_problem(seed, Bt=2, Dc=2, N=3, H=4, W=5):
    rng = np.random.default_rng(seed)
    x, delta, A, Bm, Cm, Dskip, mask = rand_problem(rng, Bt, Dc, N, H, W)
    A = (np.round(A * 64) / 64).astype(np.float32)
    A_v = (np.round(-np.exp(rng.normal(0.3, 0.5, A.shape)) * 64) / 64).astype(np.float32)
    Dskip = (np.round(Dskip * 64) / 64).astype(np.float32)
    pad = (np.round(rng.standard_normal(Dc) * 64) / 64).astype(np.float32)
    return rng, x, delta, A, A_v, Bm, Cm, Dskip, mask, pad


@pytest.mark.parametrize("use_av,use_pad", [(True, True), (True, False), (False, True)])
def test_variants_match_the_brute_force_path_products(use_av, use_pad):
    _, x, delta, A, A_v, Bm, Cm, Dskip, mask, pad = _variant_problem(71, 1, 2, 2, 4, 4)
    A_v, pad = (A_v if use_av else None), (pad if use_pad else None)
    y = oracle.scan2d_fwd_variants(x, delta, A, Bm, Cm, Dskip, mask, A_v=A_v, pad=pad, dtype=F64)
    np.testing.assert_allclose(y, brute_force_variants(x, delta, A, A_v, Bm, Cm, Dskip, mask, pad), rtol=1e-12, atol=1e-12)


def test_variants_reduce_to_the_plain_operator():
    """A_v = A is the paper's default (A-bar re-used); pad = 0 is the fixed zero token: bit for bit."""
    rng, x, delta, A, A_v, Bm, Cm, Dskip, mask, pad = _variant_problem(72, 2, 3, 4, 6, 5)
    dy = rng.standard_normal(x.shape)
    base_y = oracle.scan2d_fwd(x, delta, A, Bm, Cm, Dskip, mask, dtype=F64)
    base_g = oracle.scan2d_bwd(x, delta, A, Bm, Cm, Dskip, mask, dy, dtype=F64)
    zero = np.zeros_like(pad)
    for av, pd in ((None, None), (A, None), (None, zero), (A, zero)):
        assert np.array_equal(oracle.scan2d_fwd_variants(x, delta, A, Bm, Cm, Dskip, mask, A_v=av, pad=pd, dtype=F64), base_y)
        dx, dd, dA, dAv, dB, dC, dD, dP = oracle.scan2d_bwd_variants(x, delta, A, Bm, Cm, Dskip, mask, dy, A_v=av, pad=pd, dtype=F64)
        assert np.array_equal(dx, base_g[0]) and np.array_equal(dB, base_g[3]) and np.array_equal(dC, base_g[4])
        assert np.array_equal(dD, base_g[5])
        np.testing.assert_allclose(dd, base_g[1], rtol=1e-13, atol=1e-13)
        # one parameter driving both decays: its gradient is the sum of the two
        np.testing.assert_allclose(dA if av is None else dA.astype(np.float64) + dAv, base_g[2], rtol=2e-6)


def test_vertical_decay_only_acts_down_the_columns():
    """With a single row the vertical decay never acts; with a single column only it acts on the way down."""
    _, x, delta, A, A_v, Bm, Cm, Dskip, mask, pad = _variant_problem(73, 1, 2, 3, 1, 7)
    y = oracle.scan2d_fwd_variants(x, delta, A, Bm, Cm, Dskip, mask, A_v=A_v, dtype=F64)
    assert np.array_equal(y, oracle.scan2d_fwd(x, delta, A, Bm, Cm, Dskip, mask, dtype=F64))
    _, x, delta, A, A_v, Bm, Cm, Dskip, mask, pad = _variant_problem(74, 1, 2, 3, 7, 1)
    y = oracle.scan2d_fwd_variants(x, delta, A, Bm, Cm, Dskip, mask, A_v=A_v, dtype=F64)
    # a single column: h[i] = a_v[i] h[i-1] + u[i], the 1D recurrence (Eq. 1-2) with A_v as its parameter
    assert np.allclose(y, oracle.scan2d_fwd(x, delta, A_v, Bm, Cm, Dskip, mask, dtype=F64), rtol=1e-13, atol=1e-13)


def test_padding_token_is_x_replaced_under_the_mask():
    """The operator only sees x_eff: storing pad[c] into x under the mask and dropping the mask gives the same y."""
    _, x, delta, A, A_v, Bm, Cm, Dskip, mask, pad = _variant_problem(75, 2, 3, 4, 5, 6)
    y = oracle.scan2d_fwd_variants(x, delta, A, Bm, Cm, Dskip, mask, pad=pad, dtype=F64)
    xr = np.where(mask[:, None] != 0, pad.astype(np.float64)[None, :, None, None], x)
    assert np.array_equal(y, oracle.scan2d_fwd(xr, delta, A, Bm, Cm, Dskip, None, dtype=F64))
    poisoned = np.where(mask[:, None] != 0, np.nan, x)           # a select: what is stored under the mask never leaks
    assert np.array_equal(y, oracle.scan2d_fwd_variants(poisoned, delta, A, Bm, Cm, Dskip, mask, pad=pad, dtype=F64))


def test_variants_backward_matches_central_differences_for_every_input():
    rng, x, delta, A, A_v, Bm, Cm, Dskip, mask, pad = _variant_problem(76)
    dy = rng.standard_normal(x.shape)
    dx, dd, dA, dAv, dB, dC, dD, dP = oracle.scan2d_bwd_variants(x, delta, A, Bm, Cm, Dskip, mask, dy, A_v=A_v, pad=pad, dtype=F64)
    p = {"x": x, "delta": delta, "A": A, "A_v": A_v, "Bm": Bm, "Cm": Cm, "Dskip": Dskip, "pad": pad}
    grads = {"x": dx, "delta": dd, "A": dA, "A_v": dAv, "Bm": dB, "Cm": dC, "Dskip": dD, "pad": dP}

    def f(q):
        y = oracle.scan2d_fwd_variants(q["x"], q["delta"], q["A"], q["Bm"], q["Cm"], q["Dskip"], mask, A_v=q["A_v"], pad=q["pad"], dtype=F64)
        return float(np.sum(dy * y))

    for k, g in grads.items():
        fp32 = p[k].dtype == np.float32
        eps = 2.0 ** -12 if fp32 else 1e-6
        fd = np.zeros(p[k].shape)
        it = np.nditer(p[k], flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            hi = {n: t.copy() for n, t in p.items()}
            lo = {n: t.copy() for n, t in p.items()}
            hi[k][idx] += eps
            lo[k][idx] -= eps
            fd[idx] = (f(hi) - f(lo)) / (2 * eps)
        tol = 2e-6 if fp32 else 1e-7                     # fp32 outputs come back rounded
        np.testing.assert_allclose(g, fd, rtol=tol, atol=tol * max(np.abs(fd).max(), 1e-30), err_msg=k)
    assert not dx[np.broadcast_to(mask[:, None] != 0, dx.shape)].any()      # x under the mask has no influence


def test_variants_low_precision_storage_rounds_once():
    rng, x, delta, A, A_v, Bm, Cm, Dskip, mask, pad = _variant_problem(77, 1, 3, 4, 6, 7)
    for dtype in (oracle.F32, oracle.BF16):
        cast = (lambda t: wl.f32_to_bf16_bits(t.astype(np.float32))) if dtype == oracle.BF16 else (lambda t: t.astype(np.float32))
        xs, ds, Bs, Cs = cast(x), cast(delta), cast(Bm), cast(Cm)
        y = oracle.scan2d_fwd_variants(xs, ds, A, Bs, Cs, Dskip, mask, A_v=A_v, pad=pad, dtype=dtype)
        wide = [wl.to_float(t, dtype) for t in (xs, ds, Bs, Cs)]
        y64 = oracle.scan2d_fwd_variants(wide[0], wide[1], A, wide[2], wide[3], Dskip, mask, A_v=A_v, pad=pad, dtype=F64)
        expect = wl.f32_to_bf16_bits(y64.astype(np.float32)) if dtype == oracle.BF16 else y64.astype(np.float32)
        if dtype == oracle.F32:
            assert np.array_equal(y, expect)
        else:                                             # double -> bf16 directly; via fp32 may differ in rare double-rounding ties
            assert np.mean(y == expect) > 0.999
