"""CPU oracle of the weight-format variants the paper compares dINT4 with (App. A.5 / Tables 10-14:
3-bit dINT, plain INT4) and of the error split of Sec. 4.1 (Eq. 4) -- TEST INFRASTRUCTURE ONLY.

Formats (b bits, p uniform steps, Sec. 4.2):
    dint4   b = 4, p = 2^4 - 3 = 13 integer steps plus the two special levels +-step/2     (Eq. 5)
    dint3   b = 3, p = 2^3 - 3 = 5, the same rule                                          (Table 10)
    int4    b = 4, p = 2^4 - 1 = 15, no special levels: the ordinary asymmetric integer format
Codes live in one 4-bit code space so that the same packing and the same GEMM serve all three:
integer level k is code k, the special levels are codes 14 (+step/2) and 15 (-step/2) for the dINT
formats (dint3 uses codes 0..5, 14, 15); for int4 codes 14 and 15 are ordinary levels.  A 3-bit
storage form of dint3 (codes 0..5, 6 = +step/2, 7 = -step/2; eight codes in three bytes, code i of a
group of eight at bits 3i..3i+2 of the little-endian 24-bit word) is given by pack3 / unpack3.

Every step that decides a code is one IEEE binary32 operation (numpy float32 arithmetic), in the
order of the definition: w' = w * s; lo = min(0, min w'), hi = max(0, max w'); step = (hi - lo) / p;
istep = 1 / step; z = clamp(rne(-lo * istep), 0, p); u = w' * istep; dINT: 0.25 < u <= 0.75 -> +step/2,
-0.75 <= u < -0.25 -> -step/2; else clamp(rne(u) + z, 0, p).  The integer GEMM is numpy's int64 matmul.
"""
from __future__ import annotations

import numpy as np

F32 = np.float32
FORMATS = {"dint4": (13, True), "int4": (15, False), "dint3": (5, True)}
FORMAT_IDS = {"dint4": 0, "int4": 1, "dint3": 2}
C1, C2 = 14, 15

__all__ = ["FORMATS", "FORMAT_IDS", "quantize_weight", "half_steps", "dequant", "int_gemm",
           "layer_output64", "pack3", "unpack3", "error_split", "output_error_terms"]


def _groups(K, group_size):
    G = K if group_size in (0, None) else int(group_size)
    if G <= 0 or K % G:
        raise ValueError("bad group size")
    return G


def quantize_weight(W, s=None, group_size=0, fmt="dint4"):
    """Returns (codes u8 [N,K] in the 4-bit code space, step f32 [N,K/G], zero u8 [N,K/G])."""
    p, special = FORMATS[fmt]
    W = np.asarray(W).astype(F32)
    N, K = W.shape
    G = _groups(K, group_size)
    wp = (W * np.asarray(s, F32)[None, :]).astype(F32) if s is not None else W
    g = wp.reshape(N, K // G, G)
    lo = np.minimum(g.min(axis=2), F32(0)).astype(F32)
    hi = np.maximum(g.max(axis=2), F32(0)).astype(F32)
    deg = hi == lo
    step = np.where(deg, F32(1), ((hi - lo).astype(F32) / F32(p)).astype(F32)).astype(F32)
    istep = (F32(1) / step).astype(F32)
    zf = np.rint(((-lo).astype(F32) * istep).astype(F32))
    zero = np.where(deg, 0, np.clip(zf, 0, p)).astype(np.int32)
    u = (g * istep[:, :, None]).astype(F32)
    codes = np.clip(np.rint(u).astype(np.int32) + zero[:, :, None], 0, p)
    if special:
        codes = np.where((u > F32(0.25)) & (u <= F32(0.75)), C1, codes)
        codes = np.where((u >= F32(-0.75)) & (u < F32(-0.25)), C2, codes)
    return codes.reshape(N, K).astype(np.uint8), step, zero.astype(np.uint8)


def half_steps(codes, zero, group_size=0, fmt="dint4"):
    """Weights in units of step/2 (int64 [N,K]): 2 (code - z), or +-1 for the special codes."""
    _, special = FORMATS[fmt]
    codes = np.asarray(codes).astype(np.int64)
    N, K = codes.shape
    G = _groups(K, group_size)
    z = np.repeat(np.asarray(zero).astype(np.int64).reshape(N, K // G), G, axis=1)
    d = 2 * (codes - z)
    if special:
        d = np.where(codes == C1, 1, np.where(codes == C2, -1, d))
    return d


def dequant(codes, step, zero, group_size=0, fmt="dint4"):
    """float64 values of the codes."""
    N, K = np.asarray(codes).shape
    G = _groups(K, group_size)
    st = np.repeat(np.asarray(step, np.float64).reshape(N, K // G), G, axis=1)
    return half_steps(codes, zero, group_size, fmt) * (0.5 * st)


def int_gemm(Xq, codes, zero, group_size=0, fmt="dint4"):
    """acc[m,n,g] = sum_{k in g} Xq[m,k] d[n,k] (int64 matmul per group, returned as int32)."""
    Xq = np.asarray(Xq).astype(np.int64)
    d = half_steps(codes, zero, group_size, fmt)
    M, K = Xq.shape
    N = d.shape[0]
    G = _groups(K, group_size)
    acc = np.empty((M, N, K // G), np.int64)
    for g in range(K // G):
        acc[:, :, g] = Xq[:, g * G:(g + 1) * G] @ d[:, g * G:(g + 1) * G].T
    return acc.astype(np.int32)


def layer_output64(Xq, sx, codes, step, zero, group_size=0, fmt="dint4"):
    """sx[m] * sum_g (step/2) acc[m,n,g] in float64."""
    acc = int_gemm(Xq, codes, zero, group_size, fmt).astype(np.float64)
    half = 0.5 * np.asarray(step, np.float64)
    return np.asarray(sx, np.float64)[:, None] * np.einsum("mng,ng->mn", acc, half)


def pack3(codes3):
    """3-bit codes (0..7) [N,K], K % 8 == 0 -> bytes [N, 3K/8]."""
    c = np.asarray(codes3).astype(np.uint32)
    N, K = c.shape
    if K % 8 or c.max(initial=0) > 7:
        raise ValueError("pack3: K % 8 != 0 or a code above 7")
    g = c.reshape(N, K // 8, 8)
    word = np.zeros((N, K // 8), np.uint32)
    for i in range(8):
        word |= g[:, :, i] << np.uint32(3 * i)
    out = np.stack([(word >> np.uint32(8 * b)) & np.uint32(0xFF) for b in range(3)], axis=2)
    return out.reshape(N, 3 * K // 8).astype(np.uint8)


def unpack3(packed):
    p = np.asarray(packed).astype(np.uint32)
    N, B = p.shape
    t = p.reshape(N, B // 3, 3)
    word = t[:, :, 0] | (t[:, :, 1] << np.uint32(8)) | (t[:, :, 2] << np.uint32(16))
    out = np.stack([(word >> np.uint32(3 * i)) & np.uint32(7) for i in range(8)], axis=2)
    return out.reshape(N, 8 * (B // 3)).astype(np.uint8)


def error_split(W, s, group_size=0, fmt="dint4"):
    """The split of Sec. 4.1: with W' = W diag(s) and Wq its dequantized codes, the error Wq - W' on
    the weights whose quantized value is zero (underflow, Delta_u) and on the others (rounding,
    Delta_r).  Returns (Delta_u, Delta_r) in float64; they have disjoint supports and add up to the
    total error."""
    W = np.asarray(W).astype(F32)
    wp = (W * np.asarray(s, F32)[None, :]).astype(F32) if s is not None else W
    codes, step, zero = quantize_weight(W, s, group_size, fmt)
    wq = dequant(codes, step, zero, group_size, fmt)
    delta = wq - wp.astype(np.float64)
    under = wq == 0.0
    return np.where(under, delta, 0.0), np.where(under, 0.0, delta)


def output_error_terms(X, W, s, group_size=0, fmt="dint4"):
    """The three terms of Eq. 4 on activations X [M,K] (unquantized, X' = X diag(s)^-1 in float64):
    sum (Delta_u X')^2, sum (Delta_r X')^2, sum 2 (Delta_u X')(Delta_r X'); their sum is the squared
    output error of weight quantization alone."""
    du, dr = error_split(W, s, group_size, fmt)
    Xs = np.asarray(X, np.float64)
    if s is not None:
        Xs = Xs * (F32(1) / np.asarray(s, F32)).astype(np.float64)[None, :]
    pu, pr = Xs @ du.T, Xs @ dr.T
    return float(np.sum(pu * pu)), float(np.sum(pr * pr)), float(np.sum(2.0 * pu * pr))
