"""Seeded synthetic inputs for the 2D selective scan.

This module only draws random tensors with the shapes, value distributions and mask
structure of the workloads; it contains none of the scan's arithmetic and is the one
module that both the GPU path's callers and the CPU oracle's callers may share.

The tensors stand in for whole-slide-image patch-feature grids and VMamba stage feature
maps (2DMamba Sec. 4 measures on such grids; the datasets themselves are not used here).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np

F32, BF16 = 0, 1


@dataclass(frozen=True)
class Workload:
    name: str
    Bt: int
    Dc: int
    N: int
    H: int
    W: int
    dtype: int                 # F32 or BF16 (storage of x, delta, Bm, Cm, y, dy)
    mask_frac: float = 0.0     # fraction of background cells (0 = no mask tensor)
    delta_mu: float = -2.0     # delta = softplus(N(delta_mu, 0.5))
    backward: bool = False     # also draw dy

    @property
    def units(self) -> int:
        """(position x channel x state) triples: the throughput metric's denominator."""
        return self.Bt * self.Dc * self.H * self.W * self.N

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == BF16 else 4

    def fwd_bytes(self) -> int:
        """Algorithmic HBM bytes of one forward: x, delta read, y written, Bm, Cm, A, Dskip, mask read."""
        e = self.elem_bytes
        M = self.Bt * self.Dc * self.H * self.W
        S = self.Bt * self.N * self.H * self.W
        m = self.Bt * self.H * self.W if self.mask_frac > 0 else 0
        return 3 * M * e + 2 * S * e + self.Dc * self.N * 4 + self.Dc * 4 + m

    def bwd_bytes(self) -> int:
        """Algorithmic HBM bytes of one backward: x, delta, dy, Bm, Cm read; dx, ddelta, dBm, dCm written."""
        e = self.elem_bytes
        M = self.Bt * self.Dc * self.H * self.W
        S = self.Bt * self.N * self.H * self.W
        m = self.Bt * self.H * self.W if self.mask_frac > 0 else 0
        return 5 * M * e + 2 * S * e + 2 * S * 4 + 2 * (self.Dc * self.N * 4 + self.Dc * 4) + m


# The five benchmark configurations (index = configuration number).
CONFIGS = (
    Workload("tiny_16x16_fp32", 1, 16, 4, 16, 16, F32),
    Workload("wsi_64x64_fp32_mask40", 1, 256, 16, 64, 64, F32, mask_frac=0.40),
    Workload("wsi_256x256_bf16_mask50", 1, 256, 16, 256, 256, BF16, mask_frac=0.50),
    Workload("vmamba_56x56_bf16_b32", 32, 192, 16, 56, 56, BF16, delta_mu=-3.0),
    Workload("train_128x192_fp32_mask30", 4, 512, 16, 128, 192, F32, mask_frac=0.30, backward=True),
)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (nearest, ties to even); returns the 16 bits as uint16."""
    w = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    nan = (w & 0x7FFFFFFF) > 0x7F800000
    r = (w + (0x7FFF + ((w >> 16) & 1))) >> 16
    r = np.where(nan, (w >> 16) | 0x0040, r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp32, exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def to_float(a: np.ndarray, dtype: int) -> np.ndarray:
    """Stored tensor -> float64 values (bf16 bits widened exactly)."""
    if dtype == BF16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return np.asarray(a, dtype=np.float64)


def _smooth_axis(a: np.ndarray, sigma: float, axis: int) -> np.ndarray:
    """Gaussian smoothing along one axis with reflect padding (kernel radius 3 sigma)."""
    n = a.shape[axis]
    r = min(int(np.ceil(3.0 * sigma)), n - 1)
    if r <= 0:
        return a
    t = np.arange(-r, r + 1, dtype=np.float64)
    k = np.exp(-0.5 * (t / sigma) ** 2)
    k /= k.sum()
    pad = [(0, 0)] * a.ndim
    pad[axis] = (r, r)
    p = np.pad(a, pad, mode="reflect")
    out = np.zeros_like(a)
    for s in range(2 * r + 1):
        sl = [slice(None)] * a.ndim
        sl[axis] = slice(s, s + n)
        out += k[s] * p[tuple(sl)]
    return out


def blob_mask(noise: np.ndarray, frac: float) -> np.ndarray:
    """Background mask made of contiguous blobs: smooth the noise, mark the lowest `frac` cells.

    noise: [Bt, H, W] float64.  Exactly round(frac*H*W) cells per batch item are marked
    (ties broken by flat index).  Returns uint8 [Bt, H, W], 1 = background.
    """
    Bt, H, W = noise.shape
    sigma = max(1.0, min(H, W) / 16.0)
    sm = _smooth_axis(_smooth_axis(noise, sigma, 2), sigma, 1)
    k = int(round(frac * H * W))
    mask = np.zeros((Bt, H * W), np.uint8)
    for b in range(Bt):
        order = np.argsort(sm[b].reshape(-1), kind="stable")
        mask[b, order[:k]] = 1
    return mask.reshape(Bt, H, W)


def _softplus(t: np.ndarray) -> np.ndarray:
    return np.logaddexp(0.0, t)


def make_inputs(wl: Workload, seed: int = 0, poison_under_mask: Optional[float] = None
                ) -> Dict[str, Optional[np.ndarray]]:
    """Draw every tensor of a workload.  Draw order is fixed: x, delta, A, Bm, Cm, Dskip,
    mask noise (only if the workload has a mask), dy (only if it has a backward).

    x is zero under the mask in the stored tensor unless `poison_under_mask` is given, in
    which case that value (e.g. NaN) is stored there instead (for the mask-is-a-select test).
    bf16 workloads are rounded once here; both sides consume the same bits (uint16 arrays).
    """
    rng = np.random.default_rng(seed)
    Bt, Dc, N, H, W = wl.Bt, wl.Dc, wl.N, wl.H, wl.W

    def cast(a64: np.ndarray) -> np.ndarray:
        a32 = a64.astype(np.float32)
        return f32_to_bf16_bits(a32) if wl.dtype == BF16 else a32

    x64 = rng.standard_normal((Bt, Dc, H, W))
    delta = cast(_softplus(rng.normal(wl.delta_mu, 0.5, (Bt, Dc, H, W))))
    A = (-np.exp(rng.normal(0.0, 0.5, (Dc, N)))).astype(np.float32)
    Bm = cast(rng.standard_normal((Bt, N, H, W)))
    Cm = cast(rng.standard_normal((Bt, N, H, W)))
    Dskip = rng.standard_normal((Dc,)).astype(np.float32)
    mask = None
    if wl.mask_frac > 0:
        mask = blob_mask(rng.standard_normal((Bt, H, W)), wl.mask_frac)
        fill = 0.0 if poison_under_mask is None else poison_under_mask
        x64 = np.where(mask[:, None, :, :] != 0, fill, x64)
    x = cast(x64)
    del x64
    out = {"x": x, "delta": delta, "A": A, "Bm": Bm, "Cm": Cm, "Dskip": Dskip, "mask": mask, "dy": None}
    if wl.backward:
        out["dy"] = cast(rng.standard_normal((Bt, Dc, H, W)))
    return out


def make_block_inputs(wl: Workload, R: int, KH: int = 3, KW: int = 3, seed: int = 0) -> Dict[str, Optional[np.ndarray]]:
    """Tensors of the producers in front of the scan for a workload's shape (the paper trains these weights; here they
    are drawn): the block's pre-convolution activations u ~ N(0,1), a depth-wise filter w ~ N(0,1)/sqrt(KH*KW) with bias
    ~ N(0, 0.1), the projection Wx ~ N(0,1)/sqrt(Dc) [(R + 2N)][Dc] in the storage type, the step expansion
    Wdt ~ N(0,1)/sqrt(R) [Dc][R] with the step bias delta_bias ~ N(delta_mu, 0.5) (so that the softplus step has the
    workloads' distribution), the gate branch z ~ N(0,1), and A, Dskip, mask as make_inputs draws them.
    Draw order: u, w, bias, Wx, Wdt, delta_bias, z, A, Dskip, mask noise."""
    rng = np.random.default_rng(seed)
    Bt, Dc, N, H, W = wl.Bt, wl.Dc, wl.N, wl.H, wl.W

    def cast(a64: np.ndarray) -> np.ndarray:
        a32 = a64.astype(np.float32)
        return f32_to_bf16_bits(a32) if wl.dtype == BF16 else a32

    u = cast(rng.standard_normal((Bt, Dc, H, W)))
    w = (rng.standard_normal((Dc, KH, KW)) / np.sqrt(KH * KW)).astype(np.float32)
    bias = rng.normal(0.0, 0.1, (Dc,)).astype(np.float32)
    Wx = cast(rng.standard_normal((R + 2 * N, Dc)) / np.sqrt(Dc))
    Wdt = (rng.standard_normal((Dc, R)) / np.sqrt(R)).astype(np.float32)
    delta_bias = rng.normal(wl.delta_mu, 0.5, (Dc,)).astype(np.float32)
    z = cast(rng.standard_normal((Bt, Dc, H, W)))
    A = (-np.exp(rng.normal(0.0, 0.5, (Dc, N)))).astype(np.float32)
    Dskip = rng.standard_normal((Dc,)).astype(np.float32)
    mask = blob_mask(rng.standard_normal((Bt, H, W)), wl.mask_frac) if wl.mask_frac > 0 else None
    return {"u": u, "w": w, "bias": bias, "Wx": Wx, "Wdt": Wdt, "delta_bias": delta_bias, "z": z, "A": A, "Dskip": Dskip, "mask": mask}


def make_pool_inputs(wl: Workload, D: int = 128, seed: int = 0) -> Dict[str, Optional[np.ndarray]]:
    """Tensors of the aggregator for a workload's shape (the paper trains V and w; here they are drawn): embeddings
    h ~ N(0,1) [Bt][Dc][H][W] in the storage type, V ~ N(0,1)/sqrt(Dc) [D][Dc] in the storage type (hidden units of
    unit variance before the tanh), w ~ N(0,1) [D] fp32 (scores with a spread of a few units, so the attention is
    neither uniform nor one-hot), and the workload's mask.  Draw order: h, V, w, mask noise."""
    rng = np.random.default_rng(seed)
    Bt, Dc, H, W = wl.Bt, wl.Dc, wl.H, wl.W

    def cast(a64: np.ndarray) -> np.ndarray:
        a32 = a64.astype(np.float32)
        return f32_to_bf16_bits(a32) if wl.dtype == BF16 else a32

    h = cast(rng.standard_normal((Bt, Dc, H, W)))
    V = cast(rng.standard_normal((D, Dc)) / np.sqrt(Dc))
    w = rng.standard_normal((D,)).astype(np.float32)
    mask = blob_mask(rng.standard_normal((Bt, H, W)), wl.mask_frac) if wl.mask_frac > 0 else None
    return {"h": h, "V": V, "w": w, "mask": mask}
