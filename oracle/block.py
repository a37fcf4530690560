"""CPU oracle for the layers around the scan: the two producers in front of it inside a 2DMamba block (Sec. 3.2,
Fig. 2) and the aggregator behind the last block (Supp. A "Aggregator", the two equations of the attention pooling).

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
* aggregator: the bag is the set of positions of a map that are not background (the paper pools "a bag of K
  embeddings"; with no mask every position is a member).  With V [D][M] and w [D] (D = 128 in the paper):
      s_k = sum_d w[d] * tanh(sum_m V[d,m] * h[m,k]),    a_k = exp(s_k) / sum_{j in bag} exp(s_j),    z = sum_k a_k h_k.
  Positions outside the bag get a = 0; an empty bag gives a = 0 and z = 0.  The outputs stay in double precision
  (the library returns fp32).
* linear layers of the block (Fig. 2: the projections into and out of the block's inner width; Sec. 3.2 keeps the
  original block's design): applied at every position of a channel-major map,
      out[b,o,i,j] = bias[o] + sum_c Wt[o,c] * in[b,c,i,j] (+ residual[b,o,i,j]),
  weights in the storage type, bias fp32, one rounding at the end.  The residual is the block's skip connection
  around the whole block (Fig. 2) and is added before that rounding.
* normalisation in front of the block (Sec. 3.3 lists "normalization, projection, and convolution" and does not say
  which): over the channels of each position, either of the two the Mamba blocks in use take,
      layer norm: out = (x - mean_c x) / sqrt(var_c x + eps) * gamma[c] + beta[c]     (biased variance)
      RMS norm:   out = x / sqrt(mean_c x^2 + eps) * gamma[c]                         (+ beta[c] if given)
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


def attn_pool(h, V, w, mask=None, dtype=F32):
    """Attention pooling over the positions of each batch item (Supp. A, the weighted sum and its attention weights).
    h: [Bt][M][H][W] and V: [D][M] in the storage type; w: [D] fp32; mask: [Bt][H][W] uint8 (non-zero = not in the
    bag) or None.  Returns (z [Bt][M], a [Bt][H][W]) as float64."""
    hw = _widen(h, dtype)
    Vw = _widen(V, dtype)
    w = np.asarray(w, np.float64)
    Bt, M, H, W = hw.shape
    if Vw.shape != (w.shape[0], M):
        raise ValueError("V must be [D][M] and w [D]")
    z = np.zeros((Bt, M))
    a = np.zeros((Bt, H, W))
    for b in range(Bt):
        bag = hw[b].reshape(M, H * W)                        # column k = embedding h_k
        member = np.ones(H * W, bool) if mask is None else (np.asarray(mask[b]).reshape(-1) == 0)
        if not member.any():
            continue
        members = bag[:, member]                             # what lies outside the bag is never read
        s = w @ np.tanh(Vw @ members)
        e = np.exp(s - s.max())
        am = e / e.sum()
        a[b].reshape(-1)[member] = am
        z[b] = members @ am
    return z, a


def linear(x, Wt, bias=None, residual=None, dtype=F32):
    """out [Bt][Cout][H][W] (storage type) = Wt [Cout][Cin] applied to x [Bt][Cin][H][W] at every position, plus
    bias [Cout] (fp32 or None), plus residual [Bt][Cout][H][W] (storage type or None)."""
    xw = _widen(x, dtype)
    Ww = _widen(Wt, dtype)
    if Ww.ndim != 2 or Ww.shape[1] != xw.shape[1]:
        raise ValueError("Wt must be [Cout][Cin]")
    out = np.einsum("oc,bchw->bohw", Ww, xw)
    if bias is not None:
        out = out + np.asarray(bias, np.float64)[None, :, None, None]
    if residual is not None:
        out = out + _widen(residual, dtype)
    return _narrow(out, dtype)


LAYER_NORM, RMS_NORM = 0, 1


def norm(x, gamma, beta=None, eps=1e-5, kind=LAYER_NORM, dtype=F32):
    """Normalisation over the channel axis of x [Bt][C][H][W] at every position; gamma, beta: [C] fp32 (beta or None)."""
    xw = _widen(x, dtype)
    g = np.asarray(gamma, np.float64)[None, :, None, None]
    if kind == LAYER_NORM:
        mean = xw.mean(axis=1, keepdims=True)
        var = ((xw - mean) ** 2).mean(axis=1, keepdims=True)
        out = (xw - mean) / np.sqrt(var + eps) * g
    elif kind == RMS_NORM:
        out = xw / np.sqrt((xw ** 2).mean(axis=1, keepdims=True) + eps) * g
    else:
        raise ValueError("kind must be LAYER_NORM or RMS_NORM")
    if beta is not None:
        out = out + np.asarray(beta, np.float64)[None, :, None, None]
    return _narrow(out, dtype)
