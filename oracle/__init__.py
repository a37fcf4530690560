"""CPU oracle for the 2D selective scan (2DMamba Eq. 3, 5, 6; output rule below Eq. 7).

TEST INFRASTRUCTURE ONLY.  The arithmetic lives in ``scan2d_oracle.c`` (plain C loops in
double precision).  This module compiles it with gcc and wraps it with ctypes on numpy
arrays.  Nothing here is shared with, or imported by, the GPU library; only tests, the
smoke check and the benchmark's ``cpu_baseline`` leg may import it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "scan2d_oracle.c")
_SRC_VARIANTS = os.path.join(_HERE, "scan2d_oracle_variants.c")     # padding token, independent vertical decay
_LIB = os.path.join(_HERE, "liboracle_scan2d.so")

F32, BF16, F64 = 0, 1, 2
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle (gcc -O2, no fast-math, OpenMP over independent maps)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_VARIANTS))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        cmd = ["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-fopenmp", "-shared", "-fPIC",
               "-o", _LIB, _SRC, _SRC_VARIANTS, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, ip = ctypes.c_void_p, ctypes.c_int
        lib.oracle_scan2d_fwd.argtypes = [ip] * 6 + [vp] * 8 + [ip]
        lib.oracle_scan2d_fwd.restype = ip
        lib.oracle_scan2d_bwd.argtypes = [ip] * 6 + [vp] * 14 + [ip]
        lib.oracle_scan2d_bwd.restype = ip
        lib.oracle_scan2d_fwd_variants.argtypes = [ip] * 6 + [vp] * 10
        lib.oracle_scan2d_fwd_variants.restype = ip
        lib.oracle_scan2d_bwd_variants.argtypes = [ip] * 6 + [vp] * 18
        lib.oracle_scan2d_bwd_variants.restype = ip
        lib.oracle_num_procs.restype = ip
        lib.oracle_round_to_bf16.argtypes = [vp, vp, ctypes.c_size_t]
        lib.oracle_round_to_bf16.restype = None
        _lib = lib
    return _lib


def num_procs() -> int:
    return int(_load().oracle_num_procs())


def _storage(dtype: int):
    if dtype == F32:
        return np.float32
    if dtype == BF16:
        return np.uint16
    if dtype == F64:
        return np.float64
    raise ValueError("dtype must be 0 (fp32), 1 (bf16 bits in uint16) or 2 (double, tests only)")


def _chk(a, np_dtype, shape, name, optional=False):
    if a is None:
        if optional:
            return None
        raise ValueError(f"{name} is required")
    a = np.ascontiguousarray(a)
    if a.dtype != np_dtype or tuple(a.shape) != tuple(shape):
        raise ValueError(f"{name}: expected {np_dtype} {tuple(shape)}, got {a.dtype} {a.shape}")
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def scan2d_fwd(x, delta, A, Bm, Cm, Dskip=None, mask=None, dtype=F32, threads=0):
    """y = 2D selective scan of x.  bf16 tensors are uint16 arrays holding the bf16 bits.

    x, delta: [Bt, Dc, H, W]; A: [Dc, N] fp32; Bm, Cm: [Bt, N, H, W]; Dskip: [Dc] fp32 or None;
    mask: [Bt, H, W] uint8 (nonzero = background) or None.  Returns y like x.
    """
    st = _storage(dtype)
    x = np.ascontiguousarray(x)
    Bt, Dc, H, W = x.shape
    N = np.asarray(A).shape[1]
    x = _chk(x, st, (Bt, Dc, H, W), "x")
    delta = _chk(delta, st, (Bt, Dc, H, W), "delta")
    A = _chk(A, np.float32, (Dc, N), "A")
    Bm = _chk(Bm, st, (Bt, N, H, W), "Bm")
    Cm = _chk(Cm, st, (Bt, N, H, W), "Cm")
    Dskip = _chk(Dskip, np.float32, (Dc,), "Dskip", optional=True)
    mask = _chk(mask, np.uint8, (Bt, H, W), "mask", optional=True)
    y = np.empty_like(x)
    rc = _load().oracle_scan2d_fwd(Bt, Dc, H, W, N, dtype, _ptr(x), _ptr(delta), _ptr(A),
                                   _ptr(Bm), _ptr(Cm), _ptr(Dskip), _ptr(mask), _ptr(y),
                                   int(threads))
    if rc != 0:
        raise RuntimeError(f"oracle_scan2d_fwd failed ({rc})")
    return y


def scan2d_bwd(x, delta, A, Bm, Cm, Dskip, mask, dy, dtype=F32, threads=0):
    """Gradients (dx, ddelta, dA, dBm, dCm, dDskip) of sum(dy * y); dDskip is None iff Dskip is."""
    st = _storage(dtype)
    x = np.ascontiguousarray(x)
    Bt, Dc, H, W = x.shape
    N = np.asarray(A).shape[1]
    x = _chk(x, st, (Bt, Dc, H, W), "x")
    delta = _chk(delta, st, (Bt, Dc, H, W), "delta")
    dy = _chk(dy, st, (Bt, Dc, H, W), "dy")
    A = _chk(A, np.float32, (Dc, N), "A")
    Bm = _chk(Bm, st, (Bt, N, H, W), "Bm")
    Cm = _chk(Cm, st, (Bt, N, H, W), "Cm")
    Dskip = _chk(Dskip, np.float32, (Dc,), "Dskip", optional=True)
    mask = _chk(mask, np.uint8, (Bt, H, W), "mask", optional=True)
    dx = np.empty_like(x)
    ddelta = np.empty_like(x)
    dA = np.empty((Dc, N), np.float32)
    dBm = np.empty((Bt, N, H, W), np.float32)
    dCm = np.empty((Bt, N, H, W), np.float32)
    dDskip = None if Dskip is None else np.empty((Dc,), np.float32)
    rc = _load().oracle_scan2d_bwd(Bt, Dc, H, W, N, dtype, _ptr(x), _ptr(delta), _ptr(A),
                                   _ptr(Bm), _ptr(Cm), _ptr(Dskip), _ptr(mask), _ptr(dy),
                                   _ptr(dx), _ptr(ddelta), _ptr(dA), _ptr(dBm), _ptr(dCm),
                                   _ptr(dDskip), int(threads))
    if rc != 0:
        raise RuntimeError(f"oracle_scan2d_bwd failed ({rc})")
    return dx, ddelta, dA, dBm, dCm, dDskip


# ----------------------------------------------------------------------------------------------
# Step fused in front of the scan (2DMamba Eq. 3: the step is softplus of a projection; the
# supplementary algorithm adds a bias inside the softplus): delta = softplus(raw + bias[c]).
# Written as a composition: the library routine numpy.logaddexp(0, t) = log(1 + exp(t)) in double,
# then the plain scan above on double storage, then one rounding to the storage type.  The
# backward is the chain rule: d softplus(t) / dt = 1 / (1 + exp(-t)).

def _widen(a, dtype):
    a = np.ascontiguousarray(a)
    if dtype == BF16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def _narrow(a, dtype):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if dtype == F32:
        return a.astype(np.float32)
    if dtype == F64:
        return a
    out = np.empty(a.shape, np.uint16)
    _load().oracle_round_to_bf16(_ptr(a), _ptr(out), a.size)
    return out


def _step(delta_raw, delta_bias, dtype):
    t = _widen(delta_raw, dtype)
    if delta_bias is not None:
        t = t + np.asarray(delta_bias, np.float64)[None, :, None, None]
    return t, np.logaddexp(0.0, t)


def scan2d_fwd_softplus(x, delta_raw, delta_bias, A, Bm, Cm, Dskip=None, mask=None, dtype=F32, threads=0):
    """y of the scan with delta = softplus(delta_raw + delta_bias[c]) (delta_bias: [Dc] fp32 or None)."""
    _, delta = _step(delta_raw, delta_bias, dtype)
    y = scan2d_fwd(_widen(x, dtype), delta, A, _widen(Bm, dtype), _widen(Cm, dtype), Dskip, mask,
                   dtype=F64, threads=threads)
    return _narrow(y, dtype)


def scan2d_bwd_softplus(x, delta_raw, delta_bias, A, Bm, Cm, Dskip, mask, dy, dtype=F32, threads=0):
    """Gradients (dx, ddelta_raw, ddelta_bias, dA, dBm, dCm, dDskip); ddelta_bias is None iff delta_bias is."""
    t, delta = _step(delta_raw, delta_bias, dtype)
    dx, dd, dA, dBm, dCm, dD = scan2d_bwd(_widen(x, dtype), delta, A, _widen(Bm, dtype), _widen(Cm, dtype),
                                          Dskip, mask, _widen(dy, dtype), dtype=F64, threads=threads)
    draw = dd / (1.0 + np.exp(-t))
    dbias = None if delta_bias is None else draw.sum(axis=(0, 2, 3)).astype(np.float32)
    return _narrow(dx, dtype), _narrow(draw, dtype), dbias, dA, dBm, dCm, dD


# ------------------------------------------------------------------ output gate of the block
# The 2DMamba block is the Mamba block with the scan swapped for the 2D one (Sec. 3.2, Fig. 2):
# the scan's output is multiplied element-wise by SiLU(z) = z / (1 + exp(-z)) of the block's
# gate branch z [Bt][Dc][H][W].  The gate acts on the unrounded scan output; the gated output
# is rounded once to the storage type (the ungated output, which a backward pass needs for
# dz, is rounded on its own).  d SiLU(z) / dz = s (1 + z (1 - s)) with s = 1 / (1 + exp(-z)).

def _silu(z):
    s = 1.0 / (1.0 + np.exp(-z))
    return z * s, s * (1.0 + z * (1.0 - s))


def scan2d_fwd_softplus_gated(x, delta_raw, delta_bias, A, Bm, Cm, Dskip, mask, z, dtype=F32, threads=0):
    """(y_scan, y): the scan output with the softplus step, and y = y_scan * SiLU(z)."""
    _, delta = _step(delta_raw, delta_bias, dtype)
    y = scan2d_fwd(_widen(x, dtype), delta, A, _widen(Bm, dtype), _widen(Cm, dtype), Dskip, mask,
                   dtype=F64, threads=threads)
    gate, _ = _silu(_widen(z, dtype))
    return _narrow(y, dtype), _narrow(y * gate, dtype)


def scan2d_bwd_softplus_gated(x, delta_raw, delta_bias, A, Bm, Cm, Dskip, mask, z, dy, dtype=F32, threads=0):
    """Gradients of sum(dy * y) for the gated output y:
    (dx, ddelta_raw, ddelta_bias, dA, dBm, dCm, dDskip, dz)."""
    t, delta = _step(delta_raw, delta_bias, dtype)
    xw, Bw, Cw, zw, dyw = (_widen(a, dtype) for a in (x, Bm, Cm, z, dy))
    y = scan2d_fwd(xw, delta, A, Bw, Cw, Dskip, mask, dtype=F64, threads=threads)
    gate, dgate = _silu(zw)
    dz = dyw * y * dgate
    dx, dd, dA, dBm, dCm, dD = scan2d_bwd(xw, delta, A, Bw, Cw, Dskip, mask, dyw * gate, dtype=F64, threads=threads)
    draw = dd / (1.0 + np.exp(-t))
    dbias = None if delta_bias is None else draw.sum(axis=(0, 2, 3)).astype(np.float32)
    return _narrow(dx, dtype), _narrow(draw, dtype), dbias, dA, dBm, dCm, dD, _narrow(dz, dtype)


# ------------------------------------------------------------------ identity cells ("skip" mask mode)
# Supp. "Tiling and edge cases": cells that are not part of the map are padded with A-bar = 1 and x = 0,
# so that the state passes through them unchanged.  As a mask mode: a masked cell has step 0 (a = exp(0) = 1,
# u = 0) besides x = 0.  That is the plain scan on a step that is zero under the mask; the gradient of the
# step under the mask is zero because the step there is the constant 0.

def _skip_step(delta, mask):
    d = np.array(delta, copy=True)
    if mask is not None:
        d[np.broadcast_to(np.asarray(mask)[:, None] != 0, d.shape)] = 0      # +0 in every storage type
    return d


def scan2d_fwd_skip(x, delta, A, Bm, Cm, Dskip=None, mask=None, dtype=F32, threads=0):
    return scan2d_fwd(x, _skip_step(delta, mask), A, Bm, Cm, Dskip, mask, dtype=dtype, threads=threads)


def scan2d_bwd_skip(x, delta, A, Bm, Cm, Dskip, mask, dy, dtype=F32, threads=0):
    dx, dd, dA, dBm, dCm, dD = scan2d_bwd(x, _skip_step(delta, mask), A, Bm, Cm, Dskip, mask, dy, dtype=dtype, threads=threads)
    return dx, _skip_step(dd, mask), dA, dBm, dCm, dD


# ------------------------------------------------------------------ columns first (scan order ablation)
# The supplement ablates the order of the two scans.  Columns first: v[i,j] = a[i,j] v[i-1,j] + u[i,j] down each
# column, then h[i,j] = a[i,j] h[i,j-1] + v[i,j] along each row, y = C h + D x.  Exchanging the roles of i and
# j turns these two lines into Eq. 5 and Eq. 6, so this is the row-first scan of the transposed maps,
# transposed back (tests/test_oracle_pins.py checks it against the two recurrences written as loops).

def _tr(a):
    return None if a is None else np.ascontiguousarray(np.swapaxes(a, -1, -2))


def scan2d_fwd_columns_first(x, delta, A, Bm, Cm, Dskip=None, mask=None, dtype=F32, threads=0):
    return _tr(scan2d_fwd(_tr(x), _tr(delta), A, _tr(Bm), _tr(Cm), Dskip, _tr(mask), dtype=dtype, threads=threads))


def scan2d_bwd_columns_first(x, delta, A, Bm, Cm, Dskip, mask, dy, dtype=F32, threads=0):
    dx, dd, dA, dBm, dCm, dD = scan2d_bwd(_tr(x), _tr(delta), A, _tr(Bm), _tr(Cm), Dskip, _tr(mask), _tr(dy),
                                          dtype=dtype, threads=threads)
    return _tr(dx), _tr(dd), dA, _tr(dBm), _tr(dCm), dD


# ----------------------------------------------------------------------------------------------
# The two variants the paper ablates besides the scan order (scan2d_oracle_variants.c): a learnable padding
# token under the mask (Eq. 4: x_eff = pad[c] there) and an independent decay parameter A_v for the vertical
# scan (the supplement's ablation of re-using A-bar).  None = the default of the operator.

def scan2d_fwd_variants(x, delta, A, Bm, Cm, Dskip=None, mask=None, A_v=None, pad=None, dtype=F32):
    st = _storage(dtype)
    x = np.ascontiguousarray(x)
    Bt, Dc, H, W = x.shape
    N = np.asarray(A).shape[1]
    x = _chk(x, st, (Bt, Dc, H, W), "x")
    delta = _chk(delta, st, (Bt, Dc, H, W), "delta")
    A = _chk(A, np.float32, (Dc, N), "A")
    A_v = _chk(A_v, np.float32, (Dc, N), "A_v", optional=True)
    Bm = _chk(Bm, st, (Bt, N, H, W), "Bm")
    Cm = _chk(Cm, st, (Bt, N, H, W), "Cm")
    Dskip = _chk(Dskip, np.float32, (Dc,), "Dskip", optional=True)
    mask = _chk(mask, np.uint8, (Bt, H, W), "mask", optional=True)
    pad = _chk(pad, np.float32, (Dc,), "pad", optional=True)
    y = np.empty_like(x)
    rc = _load().oracle_scan2d_fwd_variants(Bt, Dc, H, W, N, dtype, _ptr(x), _ptr(delta), _ptr(A), _ptr(A_v),
                                            _ptr(Bm), _ptr(Cm), _ptr(Dskip), _ptr(mask), _ptr(pad), _ptr(y))
    if rc != 0:
        raise RuntimeError(f"oracle_scan2d_fwd_variants failed ({rc})")
    return y


def scan2d_bwd_variants(x, delta, A, Bm, Cm, Dskip, mask, dy, A_v=None, pad=None, dtype=F32):
    """Gradients (dx, ddelta, dA, dA_v, dBm, dCm, dDskip, dpad); dA_v / dDskip / dpad are None iff their input is."""
    st = _storage(dtype)
    x = np.ascontiguousarray(x)
    Bt, Dc, H, W = x.shape
    N = np.asarray(A).shape[1]
    x = _chk(x, st, (Bt, Dc, H, W), "x")
    delta = _chk(delta, st, (Bt, Dc, H, W), "delta")
    dy = _chk(dy, st, (Bt, Dc, H, W), "dy")
    A = _chk(A, np.float32, (Dc, N), "A")
    A_v = _chk(A_v, np.float32, (Dc, N), "A_v", optional=True)
    Bm = _chk(Bm, st, (Bt, N, H, W), "Bm")
    Cm = _chk(Cm, st, (Bt, N, H, W), "Cm")
    Dskip = _chk(Dskip, np.float32, (Dc,), "Dskip", optional=True)
    mask = _chk(mask, np.uint8, (Bt, H, W), "mask", optional=True)
    pad = _chk(pad, np.float32, (Dc,), "pad", optional=True)
    dx, ddelta = np.empty_like(x), np.empty_like(x)
    dA = np.empty((Dc, N), np.float32)
    dA_v = None if A_v is None else np.empty((Dc, N), np.float32)
    dBm = np.empty((Bt, N, H, W), np.float32)
    dCm = np.empty((Bt, N, H, W), np.float32)
    dDskip = None if Dskip is None else np.empty((Dc,), np.float32)
    dpad = None if pad is None else np.empty((Dc,), np.float32)
    rc = _load().oracle_scan2d_bwd_variants(Bt, Dc, H, W, N, dtype, _ptr(x), _ptr(delta), _ptr(A), _ptr(A_v),
                                            _ptr(Bm), _ptr(Cm), _ptr(Dskip), _ptr(mask), _ptr(pad), _ptr(dy),
                                            _ptr(dx), _ptr(ddelta), _ptr(dA), _ptr(dA_v), _ptr(dBm), _ptr(dCm),
                                            _ptr(dDskip), _ptr(dpad))
    if rc != 0:
        raise RuntimeError(f"oracle_scan2d_bwd_variants failed ({rc})")
    return dx, ddelta, dA, dA_v, dBm, dCm, dDskip, dpad
