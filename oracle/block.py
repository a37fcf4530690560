"""CPU oracle for the two producers in front of the scan inside a 2DMamba block (Sec. 3.2, Fig. 2).

TEST INFRASTRUCTURE ONLY: plain numpy in double precision, nothing shared with the GPU library.

The paper takes the design of the original Mamba block and swaps the scan (Sec. 3.2); it names the layers in front
of the scan only as "normalization, projection, and convolution" (Sec. 3.3) and Eq. 3 only says that Delta, B and C
are learnable linear functions of x.  Readings taken here (both stated in the design notes):

* convolution: depth-wise (one filter per channel) cross-correlation over the 2D map, zero outside the map, with the
  offset of the filter's first tap given explicitly, followed by SiLU:
      t[b,c,i,j] = bias[c] + sum_{p<KH, q<KW} w[c,p,q] * u[b,c,i+p-PH,j+q-PW],    x = t / (1 + exp(-t)).
  KH = KW = 3, PH = PW = 1 is the "same" 3x3 filter; KH = 1, KW = 4, PW = 3 is the causal filter of the 1D block
  applied along the rows.
* projections: one matrix Wx [(R + 2N)][Dc] applied at every position gives a low-rank step (R rows), B (N rows)
  and C (N rows); a second matrix Wdt [Dc][R] expands the low-rank step to one raw step per channel.  Its bias is
  the `delta_bias` of the softplus step (Eq. 3: Delta = softplus(Delta(x))) and is not added here.
      low[b,m,i,j]  = sum_c Wx[m,c] * x[b,c,i,j]
      delta_raw[b,c,i,j] = sum_r Wdt[c,r] * low[b,r,i,j],   Bm = low[:, R:R+N],   Cm = low[:, R+N:R+2N]
  The low-rank step is not rounded between the two products; every output is rounded once to the storage type.
"""
from __future__ import annotations

import numpy as np

from . import BF16, F32, F64, _narrow, _widen  # storage conversions only (exact widening, one nearest-even rounding)


def conv_silu(u, w, bias, PH, PW, dtype=F32):
    """x [Bt][Dc][H][W] (storage type) = SiLU(depth-wise correlation of u with w [Dc][KH][KW] + bias [Dc] or None)."""
    uw = _widen(u, dtype)
    w = np.asarray(w, np.float64)
    Bt, Dc, H, W = uw.shape
    KH, KW = w.shape[1:]
    t = np.zeros_like(uw)
    for p in range(KH):
        for q in range(KW):
            di, dj = p - PH, q - PW                      # the tap reads u[i + di, j + dj]
            i0, i1 = max(0, -di), min(H, H - di)
            j0, j1 = max(0, -dj), min(W, W - dj)
            if i0 < i1 and j0 < j1:
                t[:, :, i0:i1, j0:j1] += w[None, :, p, q, None, None] * uw[:, :, i0 + di:i1 + di, j0 + dj:j1 + dj]
    if bias is not None:
        t += np.asarray(bias, np.float64)[None, :, None, None]
    return _narrow(t / (1.0 + np.exp(-t)), dtype)


def xproj(x, Wx, Wdt, N, dtype=F32):
    """(delta_raw [Bt][Dc][H][W], Bm [Bt][N][H][W], Cm [Bt][N][H][W]) in the storage type.
    Wx: [(R + 2N)][Dc] in the storage type of x (the projection runs on the stored values); Wdt: [Dc][R] fp32."""
    xw = _widen(x, dtype)
    Wxw = _widen(Wx, dtype)
    Wdt = np.asarray(Wdt, np.float64)
    R = Wdt.shape[1]
    if Wxw.shape != (R + 2 * N, xw.shape[1]) or Wdt.shape[0] != xw.shape[1]:
        raise ValueError("Wx must be [(R + 2N)][Dc] and Wdt [Dc][R]")
    low = np.einsum("mc,bchw->bmhw", Wxw, xw)
    delta_raw = np.einsum("cr,brhw->bchw", Wdt, low[:, :R])
    return _narrow(delta_raw, dtype), _narrow(low[:, R:R + N], dtype), _narrow(low[:, R + N:], dtype)
