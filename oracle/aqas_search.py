"""CPU oracle of the AQAS scale search (Sec. 3.2, Eq. 1; App. A.4) -- TEST INFRASTRUCTURE ONLY.

The paper fixes the objective (Eq. 1: squared error of the quantized layer's output against the
unquantized product on calibration activations), the representatives (maximum magnitude per input
channel, for activations and for weights), the method (a grid search, as in the scaling work it
builds on) and a final adjustment (clipping the weights).  It prints neither the grid nor the
clipping rule; the readings taken here are

  * search space  s_k(alpha) = ax_k^alpha / aw_k^(1 - alpha),  ax_k = max_t |X[t,k]|,
    aw_k = max_n |W[n,k]|, alpha = j / 16 for j = 0..16.  A sixteenth power is a chain of correctly
    rounded binary32 square roots, so x^(j/16) is a fixed sequence of IEEE operations (the product
    of x^(1/2), x^(1/4), x^(1/8), x^(1/16) selected by the bits of j, multiplied in that order;
    x itself for j = 16, 1 for j = 0) and two implementations agree bit for bit;
    channels with ax_k = 0 or aw_k = 0 get s_k = 1; s is clamped to [1e-4, 1e4];
  * loss(alpha) = sum_{t,n} (Yq[t,n] - Y[t,n])^2 with Yq the fp16 output of the quantized layer
    and Y = X W^T in float64; the first minimal alpha wins;
  * weight clipping: with the chosen s, each output channel n tries range factors
    rho_i = 1 - 0.05 i, i = 0..10, applied to the (zero-containing) min / max of every group of
    that channel (one binary32 multiply each), step and zero-point from the shrunk range by the
    usual rule, and keeps the factor with the smallest output error of that channel
    (first minimum: the largest rho).

Every arithmetic step that decides codes is one IEEE binary32 operation (numpy float32 ops);
the losses are float64.  Built on the pinned functions of w4a8_oracle.
"""
from __future__ import annotations

import numpy as np

from . import w4a8_oracle as orc

__all__ = ["GRID", "CLIP_STEPS", "channel_absmax", "pow_sixteenths", "aqas_scale", "layer_output",
           "aqas_losses", "aqas_search", "clip_factor", "clipped_params", "clip_search"]

GRID = 16          # alpha = j / GRID, j = 0..GRID
CLIP_STEPS = 11    # rho_i = 1 - 0.05 i
F32 = np.float32


def channel_absmax(A):
    """max over rows of |A[r, k]| as float32 [K] (exact)."""
    A = np.asarray(A)
    return np.abs(A.astype(F32)).max(axis=0) if A.shape[0] else np.zeros(A.shape[1], F32)


def pow_sixteenths(x, j: int):
    """x^(j/16) for float32 x >= 0, as the fixed chain of square roots and products."""
    x = np.asarray(x, F32)
    if j == GRID:
        return x.copy()
    out = np.ones_like(x)
    r = x
    for bit in (3, 2, 1, 0):           # x^(1/2), x^(1/4), x^(1/8), x^(1/16)
        r = np.sqrt(r)                 # correctly rounded binary32
        if (j >> bit) & 1:
            out = out * r              # one binary32 multiply
    return out


def aqas_scale(ax, aw, j: int):
    """s_k = ax_k^(j/16) / aw_k^(1 - j/16), clamped to [1e-4, 1e4]; 1 where ax_k or aw_k is 0."""
    ax = np.asarray(ax, F32)
    aw = np.asarray(aw, F32)
    num = pow_sixteenths(ax, j)
    den = pow_sixteenths(aw, GRID - j)
    with np.errstate(divide="ignore", invalid="ignore"):
        s = (num / den).astype(F32)
    s = np.minimum(np.maximum(s, F32(1e-4)), F32(1e4))
    return np.where((ax == 0) | (aw == 0), F32(1.0), s).astype(F32)


def layer_output(X, W, s, group_size=0, step=None, zero=None):
    """fp16 output of the quantized layer, widened to float64 (and the intermediates)."""
    if step is None:
        r = orc.linear_w4a8(X, W, s, group_size)
    else:
        Xq, sx = orc.quantize_act_int8(X, s)
        codes, st, z = orc.quantize_weight_dint4(W, s, group_size, step=step, zero=zero)
        packed = orc.pack_dint4(codes)
        acc = orc.int_gemm(Xq, packed, z, group_size)
        y32, y64 = orc.dequant_epilogue(acc, sx, st)
        r = dict(Xq=Xq, sx=sx, codes=codes, step=st, zero=z, acc=acc, Y32=y32, Y64=y64)
    r["Y16"] = orc.cast_output(r["Y32"], "f16").astype(np.float64)
    return r


def _reference(X, W):
    return np.asarray(X, np.float64) @ np.asarray(W, np.float64).T


def aqas_losses(X, W, group_size=0):
    """loss[j] (float64) and s[j] for every grid point."""
    ax, aw = channel_absmax(X), channel_absmax(W)
    Y = _reference(X, W)
    losses = np.empty(GRID + 1, np.float64)
    scales = []
    for j in range(GRID + 1):
        s = aqas_scale(ax, aw, j)
        d = layer_output(X, W, s, group_size)["Y16"] - Y
        losses[j] = float(np.sum(d * d))
        scales.append(s)
    return losses, scales


def aqas_search(X, W, group_size=0):
    losses, scales = aqas_losses(X, W, group_size)
    j = int(np.argmin(losses))          # first minimum
    return dict(j=j, s=scales[j], losses=losses, ax=channel_absmax(X), aw=channel_absmax(W))


def clip_factor(i: int):
    """rho_i = 1 - 0.05 i in binary32 (one multiply, one subtract)."""
    return F32(F32(1.0) - F32(0.05) * F32(i))


def clipped_params(W, s, group_size, rho):
    """(step, zero) [N, K/G] of the ranges of W diag(s) shrunk by rho[n] (float32 [N])."""
    W = np.asarray(W).astype(F32)
    N, K = W.shape
    G = K if group_size in (0, None) else int(group_size)
    wp = W * np.asarray(s, F32)[None, :] if s is not None else W
    g = wp.reshape(N, K // G, G)
    lo = np.minimum(g.min(axis=2), F32(0)).astype(F32)
    hi = np.maximum(g.max(axis=2), F32(0)).astype(F32)
    rho = np.asarray(rho, F32)[:, None]
    lo, hi = (lo * rho).astype(F32), (hi * rho).astype(F32)
    rng = (hi - lo).astype(F32)
    deg = hi == lo
    step = np.where(deg, F32(1), rng / F32(13)).astype(F32)
    istep = (F32(1) / step).astype(F32)
    zf = np.rint(((-lo).astype(F32) * istep).astype(F32))
    zero = np.where(deg, 0, np.clip(zf, 0, 13)).astype(np.uint8)
    return step, zero


def clip_search(X, W, s, group_size=0):
    """Per-output-channel range factor by output error.  Returns dict(index [N], rho [N],
    err [CLIP_STEPS, N] float64, step, zero of the chosen factors)."""
    N = np.asarray(W).shape[0]
    Y = _reference(X, W)
    err = np.empty((CLIP_STEPS, N), np.float64)
    params = []
    for i in range(CLIP_STEPS):
        st, z = clipped_params(W, s, group_size, np.full(N, clip_factor(i), F32))
        d = layer_output(X, W, s, group_size, step=st, zero=z)["Y16"] - Y
        err[i] = np.sum(d * d, axis=0)
        params.append((st, z))
    idx = np.argmin(err, axis=0)        # first minimum = largest rho
    step = np.stack([params[idx[n]][0][n] for n in range(N)])
    zero = np.stack([params[idx[n]][1][n] for n in range(N)])
    rho = np.array([clip_factor(int(i)) for i in idx], F32)
    return dict(index=idx.astype(np.int32), rho=rho, err=err, step=step, zero=zero)
