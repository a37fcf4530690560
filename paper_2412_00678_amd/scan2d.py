"""Thin ctypes binding of the C-ABI library `libscan2d.so` (see include/scan2d.h).

Argument marshalling only: every step of the scan runs in the HIP kernels.  PyTorch is used
for device memory and the current stream, nothing else.  Importing this module loads the
shared library and raises if it has not been built (there is no fallback path).
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libscan2d.so")

F32, BF16 = 0, 1
PASS_FWD, PASS_BWD, PASS_BWD_GATED, PASS_BWD_SOFTPLUS, PASS_FWD_VARIANTS, PASS_BWD_VARIANTS = 0, 1, 2, 3, 4, 5

EXPORTS = ("scan2d_fwd", "scan2d_fwd_softplus", "scan2d_fwd_softplus_gated", "scan2d_bwd", "scan2d_bwd_softplus",
           "scan2d_bwd_softplus_gated", "scan2d_workspace_bytes", "scan2d_describe_plan", "scan2d_strerror",
           "scan2d_version", "scan2d_debug_force_variant", "scan2d_bwd_static_scratch", "scan2d_fwd_variants", "scan2d_bwd_variants",
           "scan2d_block_conv_silu", "scan2d_block_xproj", "scan2d_saved_bytes", "scan2d_fwd_saving", "scan2d_bwd_saved",
           "scan2d_block_attn_pool", "scan2d_block_linear", "scan2d_block_norm")
STATIC_SCRATCH_BYTES = 32 * 1024 * 1024
ERR_SCRATCH_LIMIT = -9
TUNE_FWD, TUNE_FWD_SHARED, TUNE_BWD = 0, 1, 2


class Desc(ctypes.Structure):
    _fields_ = [("Bt", ctypes.c_int32), ("Dc", ctypes.c_int32), ("H", ctypes.c_int32),
                ("W", ctypes.c_int32), ("N", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("flags", ctypes.c_uint32)]


class Variants(ctypes.Structure):
    _fields_ = [("A_v", ctypes.c_void_p), ("pad", ctypes.c_void_p), ("dA_v", ctypes.c_void_p), ("dpad", ctypes.c_void_p)]


class ConvShape(ctypes.Structure):
    _fields_ = [("KH", ctypes.c_int32), ("KW", ctypes.c_int32), ("PH", ctypes.c_int32), ("PW", ctypes.c_int32)]


class Scan2dError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where} failed with code {code}: {strerror(code)}")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2412_00678_amd.build` "
            "(there is no CPU or PyTorch fallback for the scan)")
    lib = ctypes.CDLL(LIB_PATH)
    vp = ctypes.c_void_p
    lib.scan2d_fwd.argtypes = [ctypes.POINTER(Desc)] + [vp] * 8 + [vp, ctypes.c_size_t, vp]
    lib.scan2d_fwd.restype = ctypes.c_int
    lib.scan2d_fwd_softplus.argtypes = [ctypes.POINTER(Desc)] + [vp] * 9 + [vp, ctypes.c_size_t, vp]
    lib.scan2d_fwd_softplus.restype = ctypes.c_int
    lib.scan2d_bwd.argtypes = [ctypes.POINTER(Desc)] + [vp] * 14 + [vp, ctypes.c_size_t, vp]
    lib.scan2d_bwd.restype = ctypes.c_int
    lib.scan2d_fwd_variants.argtypes = [ctypes.POINTER(Desc)] + [vp] * 7 + [ctypes.POINTER(Variants), vp, vp, ctypes.c_size_t, vp]
    lib.scan2d_fwd_variants.restype = ctypes.c_int
    lib.scan2d_bwd_variants.argtypes = [ctypes.POINTER(Desc)] + [vp] * 7 + [ctypes.POINTER(Variants)] + [vp] * 7 + [vp, ctypes.c_size_t, vp]
    lib.scan2d_bwd_variants.restype = ctypes.c_int
    lib.scan2d_bwd_static_scratch.argtypes = [ctypes.POINTER(Desc)] + [vp] * 14 + [vp]
    lib.scan2d_bwd_static_scratch.restype = ctypes.c_int
    lib.scan2d_bwd_softplus.argtypes = [ctypes.POINTER(Desc)] + [vp] * 16 + [vp, ctypes.c_size_t, vp]
    lib.scan2d_bwd_softplus.restype = ctypes.c_int
    lib.scan2d_fwd_softplus_gated.argtypes = [ctypes.POINTER(Desc)] + [vp] * 11 + [vp, ctypes.c_size_t, vp]
    lib.scan2d_fwd_softplus_gated.restype = ctypes.c_int
    lib.scan2d_bwd_softplus_gated.argtypes = [ctypes.POINTER(Desc)] + [vp] * 19 + [vp, ctypes.c_size_t, vp]
    lib.scan2d_bwd_softplus_gated.restype = ctypes.c_int
    lib.scan2d_block_conv_silu.argtypes = [ctypes.POINTER(Desc), ctypes.POINTER(ConvShape)] + [vp] * 5
    lib.scan2d_block_conv_silu.restype = ctypes.c_int
    lib.scan2d_block_xproj.argtypes = [ctypes.POINTER(Desc), ctypes.c_int] + [vp] * 7
    lib.scan2d_block_xproj.restype = ctypes.c_int
    lib.scan2d_block_attn_pool.argtypes = [ctypes.POINTER(Desc), ctypes.c_int] + [vp] * 7
    lib.scan2d_block_attn_pool.restype = ctypes.c_int
    lib.scan2d_block_linear.argtypes = [ctypes.POINTER(Desc), ctypes.c_int] + [vp] * 6
    lib.scan2d_block_linear.restype = ctypes.c_int
    lib.scan2d_block_norm.argtypes = [ctypes.POINTER(Desc), ctypes.c_int, ctypes.c_float] + [vp] * 5
    lib.scan2d_block_norm.restype = ctypes.c_int
    lib.scan2d_saved_bytes.argtypes = [ctypes.POINTER(Desc)]
    lib.scan2d_saved_bytes.restype = ctypes.c_size_t
    lib.scan2d_fwd_saving.argtypes = [ctypes.POINTER(Desc)] + [vp] * 8 + [vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp]
    lib.scan2d_fwd_saving.restype = ctypes.c_int
    lib.scan2d_bwd_saved.argtypes = [ctypes.POINTER(Desc)] + [vp] * 8 + [vp, ctypes.c_size_t] + [vp] * 6 + [vp, ctypes.c_size_t, vp]
    lib.scan2d_bwd_saved.restype = ctypes.c_int
    lib.scan2d_workspace_bytes.argtypes = [ctypes.POINTER(Desc), ctypes.c_int]
    lib.scan2d_workspace_bytes.restype = ctypes.c_size_t
    lib.scan2d_strerror.argtypes = [ctypes.c_int]
    lib.scan2d_strerror.restype = ctypes.c_char_p
    lib.scan2d_version.restype = ctypes.c_int
    lib.scan2d_describe_plan.argtypes = [ctypes.POINTER(Desc), ctypes.c_int, ctypes.c_char_p, ctypes.c_size_t]
    lib.scan2d_describe_plan.restype = ctypes.c_int
    lib.scan2d_debug_force_variant.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_int), ctypes.c_int]
    lib.scan2d_debug_force_variant.restype = ctypes.c_int
    return lib


lib = _load()


def strerror(code: int) -> str:
    return lib.scan2d_strerror(int(code)).decode()


def version() -> int:
    return int(lib.scan2d_version())


def force_variant(kind: int, values=None) -> None:
    """Test hook: force a kernel variant for the whole process (None or "" clears the override).

    `values` is a sequence of ints or a comma-separated string, in the order the header gives for `kind`."""
    if isinstance(values, str):
        values = [int(t) for t in values.split(",") if t.strip()]
    values = list(values or [])
    arr = (ctypes.c_int * max(1, len(values)))(*values)
    rc = lib.scan2d_debug_force_variant(int(kind), arr, len(values))
    if rc != 0:
        raise Scan2dError(rc, "scan2d_debug_force_variant")


class forced_variant:
    """Context manager around force_variant: the override is cleared on exit."""

    def __init__(self, kind: int, values=None):
        self.kind, self.values = kind, values

    def __enter__(self):
        if self.values is not None:
            force_variant(self.kind, self.values)
        return self

    def __exit__(self, *exc):
        if self.values is not None:
            force_variant(self.kind, None)
        return False


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"x must be float32 or bfloat16, got {t.dtype}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _check(t: Optional[torch.Tensor], name: str, dtype, shape, optional=False):
    if t is None:
        if optional:
            return
        raise ValueError(f"{name} is required")
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    if t.dtype != dtype or tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected {dtype} {tuple(shape)}, got {t.dtype} {tuple(t.shape)}")


FLAG_IDENTITY_CELLS = 1      # masked cells pass the state through unchanged (step 0) instead of only holding x = 0
FLAG_COLUMNS_FIRST = 2       # columns are scanned first, then rows


def make_desc(x: torch.Tensor, A: torch.Tensor, flags: int = 0) -> Desc:
    Bt, Dc, H, W = x.shape
    return Desc(Bt, Dc, H, W, A.shape[1], _dtype_code(x), flags)


def describe_plan(desc: Desc, which: int) -> str:
    """One line naming the kernel form and launch shape the library would use (diagnostic)."""
    buf = ctypes.create_string_buffer(512)
    rc = lib.scan2d_describe_plan(ctypes.byref(desc), which, buf, len(buf))
    if rc != 0:
        raise Scan2dError(rc, "scan2d_describe_plan")
    return buf.value.decode()


def workspace_bytes(desc: Desc, which: int) -> int:
    return int(lib.scan2d_workspace_bytes(ctypes.byref(desc), which))


def _workspace(desc: Desc, which: int, device) -> Tuple[Optional[torch.Tensor], int]:
    n = workspace_bytes(desc, which)
    if n == 0:
        return None, 0
    return torch.empty(n, dtype=torch.uint8, device=device), n


def _stream_ptr() -> int:
    return torch.cuda.current_stream().cuda_stream


def scan2d_fwd(x, delta, A, Bm, Cm, Dskip=None, mask=None, y=None, workspace=None, flags=0):
    """y = 2D selective scan; enqueued on torch's current stream.  Returns y (allocated if None)."""
    desc = make_desc(x, A, flags)
    Bt, Dc, H, W, N = desc.Bt, desc.Dc, desc.H, desc.W, desc.N
    _check(x, "x", x.dtype, (Bt, Dc, H, W))
    _check(delta, "delta", x.dtype, (Bt, Dc, H, W))
    _check(A, "A", torch.float32, (Dc, N))
    _check(Bm, "Bm", x.dtype, (Bt, N, H, W))
    _check(Cm, "Cm", x.dtype, (Bt, N, H, W))
    _check(Dskip, "Dskip", torch.float32, (Dc,), optional=True)
    _check(mask, "mask", torch.uint8, (Bt, H, W), optional=True)
    if y is None:
        y = torch.empty_like(x)
    _check(y, "y", x.dtype, (Bt, Dc, H, W))
    if workspace is None:
        workspace, wbytes = _workspace(desc, PASS_FWD, x.device)
    else:
        wbytes = workspace.numel() * workspace.element_size()
    rc = lib.scan2d_fwd(ctypes.byref(desc), _ptr(x), _ptr(delta), _ptr(A), _ptr(Bm), _ptr(Cm),
                        _ptr(Dskip), _ptr(mask), _ptr(y), _ptr(workspace), wbytes, _stream_ptr())
    if rc != 0:
        raise Scan2dError(rc, "scan2d_fwd")
    return y


class Prepared:
    """An entry point with its arguments marshalled once.  Calling the object enqueues the same call again on torch's
    current stream: same tensors (their contents may change between calls), same workspace.  For loops that issue
    one short call after another, where checking and converting a dozen arguments costs more than the kernel."""

    def __init__(self, fn, name, args, keep):
        self._fn, self._name, self._args, self._keep = fn, name, args, keep      # keep: the tensors stay alive

    def __call__(self):
        rc = self._fn(*self._args, torch.cuda.current_stream().cuda_stream)
        if rc != 0:
            raise Scan2dError(rc, self._name)


def prepare_fwd(x, delta, A, Bm, Cm, Dskip, mask, y, workspace=None, flags=0) -> Prepared:
    """scan2d_fwd with the argument checks and conversions done now; see Prepared."""
    desc = make_desc(x, A, flags)
    Bt, Dc, H, W, N = desc.Bt, desc.Dc, desc.H, desc.W, desc.N
    _check(x, "x", x.dtype, (Bt, Dc, H, W))
    _check(delta, "delta", x.dtype, (Bt, Dc, H, W))
    _check(A, "A", torch.float32, (Dc, N))
    _check(Bm, "Bm", x.dtype, (Bt, N, H, W))
    _check(Cm, "Cm", x.dtype, (Bt, N, H, W))
    _check(Dskip, "Dskip", torch.float32, (Dc,), optional=True)
    _check(mask, "mask", torch.uint8, (Bt, H, W), optional=True)
    _check(y, "y", x.dtype, (Bt, Dc, H, W))
    if workspace is None:
        workspace, wbytes = _workspace(desc, PASS_FWD, x.device)
    else:
        wbytes = workspace.numel() * workspace.element_size()
    args = (ctypes.byref(desc), _ptr(x), _ptr(delta), _ptr(A), _ptr(Bm), _ptr(Cm), _ptr(Dskip), _ptr(mask), _ptr(y), _ptr(workspace), wbytes)
    return Prepared(lib.scan2d_fwd, "scan2d_fwd", args, (desc, x, delta, A, Bm, Cm, Dskip, mask, y, workspace))


def prepare_bwd(x, delta, A, Bm, Cm, Dskip, mask, dy, out, workspace=None, flags=0) -> Prepared:
    """scan2d_bwd with the argument checks and conversions done now; out = (dx, ddelta, dA, dBm, dCm, dDskip)."""
    desc = make_desc(x, A, flags)
    Bt, Dc, H, W, N = desc.Bt, desc.Dc, desc.H, desc.W, desc.N
    for t, name, dt, shape in ((x, "x", x.dtype, (Bt, Dc, H, W)), (delta, "delta", x.dtype, (Bt, Dc, H, W)), (A, "A", torch.float32, (Dc, N)),
                               (Bm, "Bm", x.dtype, (Bt, N, H, W)), (Cm, "Cm", x.dtype, (Bt, N, H, W)), (dy, "dy", x.dtype, (Bt, Dc, H, W)),
                               (out[0], "dx", x.dtype, (Bt, Dc, H, W)), (out[1], "ddelta", x.dtype, (Bt, Dc, H, W)),
                               (out[2], "dA", torch.float32, (Dc, N)), (out[3], "dBm", torch.float32, (Bt, N, H, W)),
                               (out[4], "dCm", torch.float32, (Bt, N, H, W))):
        _check(t, name, dt, shape)
    _check(Dskip, "Dskip", torch.float32, (Dc,), optional=True)
    _check(out[5], "dDskip", torch.float32, (Dc,), optional=True)
    _check(mask, "mask", torch.uint8, (Bt, H, W), optional=True)
    if workspace is None:
        workspace, wbytes = _workspace(desc, PASS_BWD, x.device)
    else:
        wbytes = workspace.numel() * workspace.element_size()
    args = (ctypes.byref(desc), _ptr(x), _ptr(delta), _ptr(A), _ptr(Bm), _ptr(Cm), _ptr(Dskip), _ptr(mask), _ptr(dy),
            _ptr(out[0]), _ptr(out[1]), _ptr(out[2]), _ptr(out[3]), _ptr(out[4]), _ptr(out[5]), _ptr(workspace), wbytes)
    return Prepared(lib.scan2d_bwd, "scan2d_bwd", args, (desc, x, delta, A, Bm, Cm, Dskip, mask, dy, out, workspace))


def saved_bytes(desc: Desc) -> int:
    """Bytes of the buffer that scan2d_fwd_saving leaves for scan2d_bwd_saved (0: this shape has no saving forward)."""
    return int(lib.scan2d_saved_bytes(ctypes.byref(desc)))


def prepare_training_pair(x, delta, A, Bm, Cm, Dskip, mask, y, dy, out, workspace_fwd=None, workspace_bwd=None):
    """(forward, backward, saved): scan2d_fwd_saving and scan2d_bwd_saved on these tensors as Prepared calls that share
    the buffer `saved` (None when the shape has no saving forward: the calls are then scan2d_fwd and scan2d_bwd)."""
    desc = make_desc(x, A, 0)
    Bt, Dc, H, W, N = desc.Bt, desc.Dc, desc.H, desc.W, desc.N
    for t, name, dt, shape in ((x, "x", x.dtype, (Bt, Dc, H, W)), (delta, "delta", x.dtype, (Bt, Dc, H, W)), (A, "A", torch.float32, (Dc, N)),
                               (Bm, "Bm", x.dtype, (Bt, N, H, W)), (Cm, "Cm", x.dtype, (Bt, N, H, W)), (y, "y", x.dtype, (Bt, Dc, H, W)),
                               (dy, "dy", x.dtype, (Bt, Dc, H, W)), (out[0], "dx", x.dtype, (Bt, Dc, H, W)),
                               (out[1], "ddelta", x.dtype, (Bt, Dc, H, W)), (out[2], "dA", torch.float32, (Dc, N)),
                               (out[3], "dBm", torch.float32, (Bt, N, H, W)), (out[4], "dCm", torch.float32, (Bt, N, H, W))):
        _check(t, name, dt, shape)
    _check(Dskip, "Dskip", torch.float32, (Dc,), optional=True)
    _check(out[5], "dDskip", torch.float32, (Dc,), optional=True)
    _check(mask, "mask", torch.uint8, (Bt, H, W), optional=True)
    nsaved = saved_bytes(desc)
    saved = torch.empty(nsaved, dtype=torch.uint8, device=x.device) if nsaved > 0 else None
    if workspace_fwd is None:
        workspace_fwd, _ = _workspace(desc, PASS_FWD, x.device)
    if workspace_bwd is None:
        workspace_bwd, _ = _workspace(desc, PASS_BWD, x.device)
    nbytes = lambda t: 0 if t is None else t.numel() * t.element_size()
    fargs = (ctypes.byref(desc), _ptr(x), _ptr(delta), _ptr(A), _ptr(Bm), _ptr(Cm), _ptr(Dskip), _ptr(mask), _ptr(y), _ptr(saved), nsaved,
             _ptr(workspace_fwd), nbytes(workspace_fwd))
    bargs = (ctypes.byref(desc), _ptr(x), _ptr(delta), _ptr(A), _ptr(Bm), _ptr(Cm), _ptr(Dskip), _ptr(mask), _ptr(dy), _ptr(saved), nsaved,
             _ptr(out[0]), _ptr(out[1]), _ptr(out[2]), _ptr(out[3]), _ptr(out[4]), _ptr(out[5]), _ptr(workspace_bwd), nbytes(workspace_bwd))
    keep = (desc, x, delta, A, Bm, Cm, Dskip, mask, y, dy, out, saved, workspace_fwd, workspace_bwd)
    return (Prepared(lib.scan2d_fwd_saving, "scan2d_fwd_saving", fargs, keep), Prepared(lib.scan2d_bwd_saved, "scan2d_bwd_saved", bargs, keep),
            saved)


def scan2d_fwd_softplus(x, delta_raw, delta_bias, A, Bm, Cm, Dskip=None, mask=None, y=None, workspace=None, flags=0):
    """y of the scan with delta = softplus(delta_raw + delta_bias[c]) computed in the kernels."""
    desc = make_desc(x, A, flags)
    Bt, Dc, H, W, N = desc.Bt, desc.Dc, desc.H, desc.W, desc.N
    _check(x, "x", x.dtype, (Bt, Dc, H, W))
    _check(delta_raw, "delta_raw", x.dtype, (Bt, Dc, H, W))
    _check(delta_bias, "delta_bias", torch.float32, (Dc,), optional=True)
    _check(A, "A", torch.float32, (Dc, N))
    _check(Bm, "Bm", x.dtype, (Bt, N, H, W))
    _check(Cm, "Cm", x.dtype, (Bt, N, H, W))
    _check(Dskip, "Dskip", torch.float32, (Dc,), optional=True)
    _check(mask, "mask", torch.uint8, (Bt, H, W), optional=True)
    if y is None:
        y = torch.empty_like(x)
    _check(y, "y", x.dtype, (Bt, Dc, H, W))
    if workspace is None:
        workspace, wbytes = _workspace(desc, PASS_FWD, x.device)
    else:
        wbytes = workspace.numel() * workspace.element_size()
    rc = lib.scan2d_fwd_softplus(ctypes.byref(desc), _ptr(x), _ptr(delta_raw), _ptr(delta_bias), _ptr(A), _ptr(Bm),
                                 _ptr(Cm), _ptr(Dskip), _ptr(mask), _ptr(y), _ptr(workspace), wbytes, _stream_ptr())
    if rc != 0:
        raise Scan2dError(rc, "scan2d_fwd_softplus")
    return y


def scan2d_bwd(x, delta, A, Bm, Cm, Dskip, mask, dy, workspace=None, flags=0, out=None):
    """Gradients (dx, ddelta, dA, dBm, dCm, dDskip) of sum(dy * y); dDskip is None iff Dskip is.
    `out`: the six tensors to write into (nothing is allocated then when a workspace is given too)."""
    desc = make_desc(x, A, flags)
    Bt, Dc, H, W, N = desc.Bt, desc.Dc, desc.H, desc.W, desc.N
    _check(x, "x", x.dtype, (Bt, Dc, H, W))
    _check(delta, "delta", x.dtype, (Bt, Dc, H, W))
    _check(dy, "dy", x.dtype, (Bt, Dc, H, W))
    _check(A, "A", torch.float32, (Dc, N))
    _check(Bm, "Bm", x.dtype, (Bt, N, H, W))
    _check(Cm, "Cm", x.dtype, (Bt, N, H, W))
    _check(Dskip, "Dskip", torch.float32, (Dc,), optional=True)
    _check(mask, "mask", torch.uint8, (Bt, H, W), optional=True)
    if out is not None:
        dx, ddelta, dA, dBm, dCm, dDskip = out
        _check(dx, "dx", x.dtype, (Bt, Dc, H, W))
        _check(ddelta, "ddelta", x.dtype, (Bt, Dc, H, W))
        _check(dA, "dA", torch.float32, (Dc, N))
        _check(dBm, "dBm", torch.float32, (Bt, N, H, W))
        _check(dCm, "dCm", torch.float32, (Bt, N, H, W))
        _check(dDskip, "dDskip", torch.float32, (Dc,), optional=True)
    else:
        dx = torch.empty_like(x)
        ddelta = torch.empty_like(x)
        dA = torch.empty((Dc, N), dtype=torch.float32, device=x.device)
        dBm = torch.empty((Bt, N, H, W), dtype=torch.float32, device=x.device)
        dCm = torch.empty((Bt, N, H, W), dtype=torch.float32, device=x.device)
        dDskip = None if Dskip is None else torch.empty((Dc,), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace, wbytes = _workspace(desc, PASS_BWD, x.device)
    else:
        wbytes = workspace.numel() * workspace.element_size()
    rc = lib.scan2d_bwd(ctypes.byref(desc), _ptr(x), _ptr(delta), _ptr(A), _ptr(Bm), _ptr(Cm),
                        _ptr(Dskip), _ptr(mask), _ptr(dy), _ptr(dx), _ptr(ddelta), _ptr(dA),
                        _ptr(dBm), _ptr(dCm), _ptr(dDskip), _ptr(workspace), wbytes, _stream_ptr())
    if rc != 0:
        raise Scan2dError(rc, "scan2d_bwd")
    return dx, ddelta, dA, dBm, dCm, dDskip


def scan2d_fwd_variants(x, delta, A, Bm, Cm, Dskip, mask, A_v=None, pad=None):
    """The forward scan with an independent vertical decay parameter A_v [Dc][N] and / or a padding token pad [Dc]."""
    desc = make_desc(x, A, 0)
    Bt, Dc, H, W, N = desc.Bt, desc.Dc, desc.H, desc.W, desc.N
    _check(A_v, "A_v", torch.float32, (Dc, N), optional=True)
    _check(pad, "pad", torch.float32, (Dc,), optional=True)
    y = torch.empty_like(x)
    workspace, wbytes = _workspace(desc, PASS_FWD_VARIANTS, x.device)
    v = Variants(_ptr(A_v), _ptr(pad), None, None)
    rc = lib.scan2d_fwd_variants(ctypes.byref(desc), _ptr(x), _ptr(delta), _ptr(A), _ptr(Bm), _ptr(Cm), _ptr(Dskip), _ptr(mask),
                                 ctypes.byref(v), _ptr(y), _ptr(workspace), wbytes, _stream_ptr())
    if rc != 0:
        raise Scan2dError(rc, "scan2d_fwd_variants")
    return y


def scan2d_bwd_variants(x, delta, A, Bm, Cm, Dskip, mask, dy, A_v=None, pad=None):
    """Gradients (dx, ddelta, dA, dA_v, dBm, dCm, dDskip, dpad); dA_v / dDskip / dpad are None iff their input is."""
    desc = make_desc(x, A, 0)
    Bt, Dc, H, W, N = desc.Bt, desc.Dc, desc.H, desc.W, desc.N
    _check(A_v, "A_v", torch.float32, (Dc, N), optional=True)
    _check(pad, "pad", torch.float32, (Dc,), optional=True)
    dx, ddelta = torch.empty_like(x), torch.empty_like(x)
    dA = torch.empty((Dc, N), dtype=torch.float32, device=x.device)
    dA_v = None if A_v is None else torch.empty((Dc, N), dtype=torch.float32, device=x.device)
    dBm = torch.empty((Bt, N, H, W), dtype=torch.float32, device=x.device)
    dCm = torch.empty((Bt, N, H, W), dtype=torch.float32, device=x.device)
    dDskip = None if Dskip is None else torch.empty((Dc,), dtype=torch.float32, device=x.device)
    dpad = None if pad is None else torch.empty((Dc,), dtype=torch.float32, device=x.device)
    workspace, wbytes = _workspace(desc, PASS_BWD_VARIANTS, x.device)
    v = Variants(_ptr(A_v), _ptr(pad), _ptr(dA_v), _ptr(dpad))
    rc = lib.scan2d_bwd_variants(ctypes.byref(desc), _ptr(x), _ptr(delta), _ptr(A), _ptr(Bm), _ptr(Cm), _ptr(Dskip), _ptr(mask),
                                 ctypes.byref(v), _ptr(dy), _ptr(dx), _ptr(ddelta), _ptr(dA), _ptr(dBm), _ptr(dCm), _ptr(dDskip),
                                 _ptr(workspace), wbytes, _stream_ptr())
    if rc != 0:
        raise Scan2dError(rc, "scan2d_bwd_variants")
    return dx, ddelta, dA, dA_v, dBm, dCm, dDskip, dpad


def scan2d_bwd_static_scratch(x, delta, A, Bm, Cm, Dskip, mask, dy, out, flags=0):
    """scan2d_bwd with the library's built-in scratch array as workspace.  Nothing is allocated, here or in the
    library: `out` = (dx, ddelta, dA, dBm, dCm, dDskip) are the caller's tensors (dDskip None iff Dskip is)."""
    desc = make_desc(x, A, flags)
    dx, ddelta, dA, dBm, dCm, dDskip = out
    rc = lib.scan2d_bwd_static_scratch(ctypes.byref(desc), _ptr(x), _ptr(delta), _ptr(A), _ptr(Bm), _ptr(Cm),
                                       _ptr(Dskip), _ptr(mask), _ptr(dy), _ptr(dx), _ptr(ddelta), _ptr(dA),
                                       _ptr(dBm), _ptr(dCm), _ptr(dDskip), _stream_ptr())
    if rc != 0:
        raise Scan2dError(rc, "scan2d_bwd_static_scratch")
    return out


def scan2d_bwd_softplus(x, delta_raw, delta_bias, A, Bm, Cm, Dskip, mask, dy, workspace=None, flags=0):
    """Gradients (dx, ddelta_raw, ddelta_bias, dA, dBm, dCm, dDskip) with the step computed in the kernels."""
    desc = make_desc(x, A, flags)
    Bt, Dc, H, W, N = desc.Bt, desc.Dc, desc.H, desc.W, desc.N
    _check(x, "x", x.dtype, (Bt, Dc, H, W))
    _check(delta_raw, "delta_raw", x.dtype, (Bt, Dc, H, W))
    _check(delta_bias, "delta_bias", torch.float32, (Dc,), optional=True)
    _check(dy, "dy", x.dtype, (Bt, Dc, H, W))
    _check(A, "A", torch.float32, (Dc, N))
    _check(Bm, "Bm", x.dtype, (Bt, N, H, W))
    _check(Cm, "Cm", x.dtype, (Bt, N, H, W))
    _check(Dskip, "Dskip", torch.float32, (Dc,), optional=True)
    _check(mask, "mask", torch.uint8, (Bt, H, W), optional=True)
    dx = torch.empty_like(x)
    draw = torch.empty_like(x)
    dbias = None if delta_bias is None else torch.empty((Dc,), dtype=torch.float32, device=x.device)
    dA = torch.empty((Dc, N), dtype=torch.float32, device=x.device)
    dBm = torch.empty((Bt, N, H, W), dtype=torch.float32, device=x.device)
    dCm = torch.empty((Bt, N, H, W), dtype=torch.float32, device=x.device)
    dDskip = None if Dskip is None else torch.empty((Dc,), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace, wbytes = _workspace(desc, PASS_BWD_SOFTPLUS, x.device)
    else:
        wbytes = workspace.numel() * workspace.element_size()
    rc = lib.scan2d_bwd_softplus(ctypes.byref(desc), _ptr(x), _ptr(delta_raw), _ptr(delta_bias), _ptr(A), _ptr(Bm),
                                 _ptr(Cm), _ptr(Dskip), _ptr(mask), _ptr(dy), _ptr(dx), _ptr(draw), _ptr(dbias),
                                 _ptr(dA), _ptr(dBm), _ptr(dCm), _ptr(dDskip), _ptr(workspace), wbytes, _stream_ptr())
    if rc != 0:
        raise Scan2dError(rc, "scan2d_bwd_softplus")
    return dx, draw, dbias, dA, dBm, dCm, dDskip


def scan2d_fwd_softplus_gated(x, delta_raw, delta_bias, A, Bm, Cm, Dskip, mask, z, want_y_scan=True, workspace=None,
                              y=None, y_scan=None, flags=0):
    """(y_scan or None, y) with y = y_scan * SiLU(z), step and gate computed in the kernel."""
    desc = make_desc(x, A, flags)
    Bt, Dc, H, W, N = desc.Bt, desc.Dc, desc.H, desc.W, desc.N
    _check(x, "x", x.dtype, (Bt, Dc, H, W))
    _check(delta_raw, "delta_raw", x.dtype, (Bt, Dc, H, W))
    _check(delta_bias, "delta_bias", torch.float32, (Dc,), optional=True)
    _check(z, "z", x.dtype, (Bt, Dc, H, W))
    _check(A, "A", torch.float32, (Dc, N))
    _check(Bm, "Bm", x.dtype, (Bt, N, H, W))
    _check(Cm, "Cm", x.dtype, (Bt, N, H, W))
    _check(Dskip, "Dskip", torch.float32, (Dc,), optional=True)
    _check(mask, "mask", torch.uint8, (Bt, H, W), optional=True)
    if y is None:
        y = torch.empty_like(x)
    else:
        _check(y, "y", x.dtype, (Bt, Dc, H, W))
    if not want_y_scan:
        y_scan = None
    elif y_scan is None:
        y_scan = torch.empty_like(x)
    else:
        _check(y_scan, "y_scan", x.dtype, (Bt, Dc, H, W))
    if workspace is None:
        workspace, wbytes = _workspace(desc, PASS_FWD, x.device)
    else:
        wbytes = workspace.numel() * workspace.element_size()
    rc = lib.scan2d_fwd_softplus_gated(ctypes.byref(desc), _ptr(x), _ptr(delta_raw), _ptr(delta_bias), _ptr(A), _ptr(Bm),
                                       _ptr(Cm), _ptr(Dskip), _ptr(mask), _ptr(z), _ptr(y_scan), _ptr(y),
                                       _ptr(workspace), wbytes, _stream_ptr())
    if rc != 0:
        raise Scan2dError(rc, "scan2d_fwd_softplus_gated")
    return y_scan, y


def scan2d_bwd_softplus_gated(x, delta_raw, delta_bias, A, Bm, Cm, Dskip, mask, z, y_scan, dy, workspace=None, flags=0):
    """Gradients (dx, ddelta_raw, ddelta_bias, dA, dBm, dCm, dDskip, dz) of the gated operator."""
    desc = make_desc(x, A, flags)
    Bt, Dc, H, W, N = desc.Bt, desc.Dc, desc.H, desc.W, desc.N
    _check(x, "x", x.dtype, (Bt, Dc, H, W))
    _check(delta_raw, "delta_raw", x.dtype, (Bt, Dc, H, W))
    _check(delta_bias, "delta_bias", torch.float32, (Dc,), optional=True)
    _check(z, "z", x.dtype, (Bt, Dc, H, W))
    _check(y_scan, "y_scan", x.dtype, (Bt, Dc, H, W))
    _check(dy, "dy", x.dtype, (Bt, Dc, H, W))
    _check(A, "A", torch.float32, (Dc, N))
    _check(Bm, "Bm", x.dtype, (Bt, N, H, W))
    _check(Cm, "Cm", x.dtype, (Bt, N, H, W))
    _check(Dskip, "Dskip", torch.float32, (Dc,), optional=True)
    _check(mask, "mask", torch.uint8, (Bt, H, W), optional=True)
    dx = torch.empty_like(x)
    draw = torch.empty_like(x)
    dz = torch.empty_like(x)
    dbias = None if delta_bias is None else torch.empty((Dc,), dtype=torch.float32, device=x.device)
    dA = torch.empty((Dc, N), dtype=torch.float32, device=x.device)
    dBm = torch.empty((Bt, N, H, W), dtype=torch.float32, device=x.device)
    dCm = torch.empty((Bt, N, H, W), dtype=torch.float32, device=x.device)
    dDskip = None if Dskip is None else torch.empty((Dc,), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace, wbytes = _workspace(desc, PASS_BWD_GATED, x.device)
    else:
        wbytes = workspace.numel() * workspace.element_size()
    rc = lib.scan2d_bwd_softplus_gated(ctypes.byref(desc), _ptr(x), _ptr(delta_raw), _ptr(delta_bias), _ptr(A), _ptr(Bm),
                                       _ptr(Cm), _ptr(Dskip), _ptr(mask), _ptr(z), _ptr(y_scan), _ptr(dy), _ptr(dx),
                                       _ptr(draw), _ptr(dbias), _ptr(dA), _ptr(dBm), _ptr(dCm), _ptr(dDskip), _ptr(dz),
                                       _ptr(workspace), wbytes, _stream_ptr())
    if rc != 0:
        raise Scan2dError(rc, "scan2d_bwd_softplus_gated")
    return dx, draw, dbias, dA, dBm, dCm, dDskip, dz


def block_conv_silu(u, w, bias=None, PH=None, PW=None, x=None):
    """x = SiLU(depth-wise correlation of u [Bt][Dc][H][W] with w [Dc][KH][KW] + bias [Dc]); PH, PW: offset of the
    filter's first tap (default: centred)."""
    Bt, Dc, H, W = u.shape
    KH, KW = int(w.shape[1]), int(w.shape[2])
    desc = Desc(Bt, Dc, H, W, 1, _dtype_code(u), 0)
    _check(u, "u", u.dtype, (Bt, Dc, H, W))
    _check(w, "w", torch.float32, (Dc, KH, KW))
    _check(bias, "bias", torch.float32, (Dc,), optional=True)
    if x is None:
        x = torch.empty_like(u)
    else:
        _check(x, "x", u.dtype, (Bt, Dc, H, W))
    shape = ConvShape(KH, KW, KH // 2 if PH is None else PH, KW // 2 if PW is None else PW)
    rc = lib.scan2d_block_conv_silu(ctypes.byref(desc), ctypes.byref(shape), _ptr(u), _ptr(w), _ptr(bias), _ptr(x), _stream_ptr())
    if rc != 0:
        raise Scan2dError(rc, "scan2d_block_conv_silu")
    return x


def block_xproj(x, Wx, Wdt, N, out=None):
    """(delta_raw, Bm, Cm) from x [Bt][Dc][H][W], Wx [(R + 2N)][Dc] (type of x) and Wdt [Dc][R] fp32."""
    Bt, Dc, H, W = x.shape
    R = int(Wdt.shape[1])
    desc = Desc(Bt, Dc, H, W, N, _dtype_code(x), 0)
    _check(x, "x", x.dtype, (Bt, Dc, H, W))
    _check(Wx, "Wx", x.dtype, (R + 2 * N, Dc))
    _check(Wdt, "Wdt", torch.float32, (Dc, R))
    if out is None:
        out = (torch.empty_like(x), torch.empty((Bt, N, H, W), dtype=x.dtype, device=x.device),
               torch.empty((Bt, N, H, W), dtype=x.dtype, device=x.device))
    else:
        _check(out[0], "delta_raw", x.dtype, (Bt, Dc, H, W))
        _check(out[1], "Bm", x.dtype, (Bt, N, H, W))
        _check(out[2], "Cm", x.dtype, (Bt, N, H, W))
    rc = lib.scan2d_block_xproj(ctypes.byref(desc), R, _ptr(x), _ptr(Wx), _ptr(Wdt), _ptr(out[0]), _ptr(out[1]), _ptr(out[2]), _stream_ptr())
    if rc != 0:
        raise Scan2dError(rc, "scan2d_block_xproj")
    return out


def block_linear(x, Wt, bias=None, residual=None, out=None):
    """out [Bt][Cout][H][W] = Wt [Cout][Cin] (type of x) applied at every position of x [Bt][Cin][H][W], plus
    bias [Cout] fp32 and residual [Bt][Cout][H][W] (type of x), both optional."""
    Bt, Cin, H, W = x.shape
    Cout = int(Wt.shape[0])
    desc = Desc(Bt, Cin, H, W, 1, _dtype_code(x), 0)
    _check(x, "x", x.dtype, (Bt, Cin, H, W))
    _check(Wt, "Wt", x.dtype, (Cout, Cin))
    if bias is not None:
        _check(bias, "bias", torch.float32, (Cout,))
    if residual is not None:
        _check(residual, "residual", x.dtype, (Bt, Cout, H, W))
    if out is None:
        out = torch.empty((Bt, Cout, H, W), dtype=x.dtype, device=x.device)
    else:
        _check(out, "out", x.dtype, (Bt, Cout, H, W))
    rc = lib.scan2d_block_linear(ctypes.byref(desc), Cout, _ptr(x), _ptr(Wt), _ptr(bias), _ptr(residual), _ptr(out), _stream_ptr())
    if rc != 0:
        raise Scan2dError(rc, "scan2d_block_linear")
    return out


LAYER_NORM, RMS_NORM = 0, 1


def block_norm(x, gamma, beta=None, eps=1e-5, kind=LAYER_NORM, out=None):
    """Layer norm or RMS norm over the channels of every position of x [Bt][C][H][W]; gamma, beta: [C] fp32."""
    Bt, C, H, W = x.shape
    desc = Desc(Bt, C, H, W, 1, _dtype_code(x), 0)
    _check(x, "x", x.dtype, (Bt, C, H, W))
    _check(gamma, "gamma", torch.float32, (C,))
    if beta is not None:
        _check(beta, "beta", torch.float32, (C,))
    if out is None:
        out = torch.empty_like(x)
    else:
        _check(out, "out", x.dtype, (Bt, C, H, W))
    rc = lib.scan2d_block_norm(ctypes.byref(desc), int(kind), float(eps), _ptr(x), _ptr(gamma), _ptr(beta), _ptr(out), _stream_ptr())
    if rc != 0:
        raise Scan2dError(rc, "scan2d_block_norm")
    return out


def block_attn_pool(h, V, w, mask=None, out=None):
    """(z [Bt][M] fp32, attn [Bt][H][W] fp32) from h [Bt][M][H][W], V [D][M] (type of h), w [D] fp32 and an optional
    mask [Bt][H][W] uint8 (non-zero = not in the bag)."""
    Bt, M, H, W = h.shape
    D = int(w.shape[0])
    desc = Desc(Bt, M, H, W, 1, _dtype_code(h), 0)
    _check(h, "h", h.dtype, (Bt, M, H, W))
    _check(V, "V", h.dtype, (D, M))
    _check(w, "w", torch.float32, (D,))
    if mask is not None:
        _check(mask, "mask", torch.uint8, (Bt, H, W))
    if out is None:
        out = (torch.empty((Bt, M), dtype=torch.float32, device=h.device), torch.empty((Bt, H, W), dtype=torch.float32, device=h.device))
    else:
        _check(out[0], "z", torch.float32, (Bt, M))
        _check(out[1], "attn", torch.float32, (Bt, H, W))
    rc = lib.scan2d_block_attn_pool(ctypes.byref(desc), D, _ptr(h), _ptr(V), _ptr(w), _ptr(mask) if mask is not None else None,
                                    _ptr(out[1]), _ptr(out[0]), _stream_ptr())
    if rc != 0:
        raise Scan2dError(rc, "scan2d_block_attn_pool")
    return out


def to_device(arrs: dict, dtype_code: int, device="cuda:0") -> dict:
    """numpy tensors of a workload (bf16 as uint16 bit patterns) -> device tensors."""
    import numpy as np

    out = {}
    for k, v in arrs.items():
        if v is None:
            out[k] = None
        elif v.dtype == np.uint16 and dtype_code == BF16:
            out[k] = torch.from_numpy(v.view(np.int16)).to(device).view(torch.bfloat16)
        else:
            out[k] = torch.from_numpy(v).to(device)
    return out


def to_host(t: torch.Tensor):
    """Device tensor -> numpy (bf16 comes back as its uint16 bit patterns)."""
    import numpy as np

    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()
