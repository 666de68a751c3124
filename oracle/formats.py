"""CPU oracle of the weight-format variants the paper compares dINT4 with (App. A.5 / Tables 9-14:
other special values, 3-bit dINT, plain INT4) and of the error split of Sec. 4.1 (Eq. 4) -- TEST
INFRASTRUCTURE ONLY.

Formats (b bits, p uniform steps, Sec. 4.2):
    dint4   b = 4, p = 2^4 - 3 = 13 integer steps plus the two special levels +-step/2     (Eq. 5)
    dint3   b = 3, p = 2^3 - 3 = 5, the same rule                                          (Table 10)
    int4    b = 4, p = 2^4 - 1 = 15, no special levels: the ordinary asymmetric integer format
Codes live in one 4-bit code space so that the same packing and the same GEMM serve all three:
integer level k is code k, the special levels are codes 14 (+step/2) and 15 (-step/2) for the dINT
formats (dint3 uses codes 0..5, 14, 15); for int4 codes 14 and 15 are ordinary levels.  A 3-bit
storage form of dint3 (codes 0..5, 6 = +step/2, 7 = -step/2; eight codes in three bytes, code i of a
group of eight at bits 3i..3i+2 of the little-endian 24-bit word) is given by pack3 / unpack3.

Special value (App. A.5, Table 9): the paper also tries c = step/4 and step/8 in place of step/2.
With c = step / 2^t (t = special_shift = 1, 2, 3) the codes keep their meaning (14 = +c, 15 = -c)
and the rule stays "nearest level": the band of +c runs from the midpoint between 0 and c to the
midpoint between c and one step, c/2 < w' <= (step + c)/2, i.e. 2^-(t+1) < u <= 1/2 + 2^-(t+1) in
units of the step (both bounds exact in binary32), with the same open / closed ends as Eq. 5; the
band of -c is its mirror image.  The paper prints no rule for t > 1; this is the reading taken.
The integer GEMM then counts in units of step / 2^t: 2^t (code - z), or +-1 for the special codes.
expand_special rewrites such a matrix as an ordinary dINT4 matrix of twice the width (see there).

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

__all__ = ["FORMATS", "FORMAT_IDS", "quantize_weight", "half_steps", "level_units", "dequant",
           "int_gemm", "layer_output64", "pack3", "unpack3", "error_split", "output_error_terms",
           "expand_special"]


def _groups(K, group_size):
    G = K if group_size in (0, None) else int(group_size)
    if G <= 0 or K % G:
        raise ValueError("bad group size")
    return G


def _shift(special_shift):
    t = int(special_shift)
    if t not in (1, 2, 3):
        raise ValueError("special_shift must be 1, 2 or 3")
    return t


def quantize_weight(W, s=None, group_size=0, fmt="dint4", special_shift=1):
    """Returns (codes u8 [N,K] in the 4-bit code space, step f32 [N,K/G], zero u8 [N,K/G])."""
    p, special = FORMATS[fmt]
    t = _shift(special_shift)
    lo_t = F32(2.0 ** -(t + 1))          # midpoint between 0 and c, in steps
    hi_t = F32(0.5 + 2.0 ** -(t + 1))    # midpoint between c and one step
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
        codes = np.where((u > lo_t) & (u <= hi_t), C1, codes)
        codes = np.where((u >= -hi_t) & (u < -lo_t), C2, codes)
    return codes.reshape(N, K).astype(np.uint8), step, zero.astype(np.uint8)


def level_units(codes, zero, group_size=0, fmt="dint4", special_shift=1):
    """Weights in units of step / 2^t (int64 [N,K]): 2^t (code - z), or +-1 for the special codes."""
    _, special = FORMATS[fmt]
    t = _shift(special_shift)
    codes = np.asarray(codes).astype(np.int64)
    N, K = codes.shape
    G = _groups(K, group_size)
    z = np.repeat(np.asarray(zero).astype(np.int64).reshape(N, K // G), G, axis=1)
    d = (1 << t) * (codes - z)
    if special:
        d = np.where(codes == C1, 1, np.where(codes == C2, -1, d))
    return d


def half_steps(codes, zero, group_size=0, fmt="dint4"):
    """Weights in units of step/2 (int64 [N,K]): 2 (code - z), or +-1 for the special codes."""
    return level_units(codes, zero, group_size, fmt, 1)


def dequant(codes, step, zero, group_size=0, fmt="dint4", special_shift=1):
    """float64 values of the codes."""
    N, K = np.asarray(codes).shape
    G = _groups(K, group_size)
    st = np.repeat(np.asarray(step, np.float64).reshape(N, K // G), G, axis=1)
    return level_units(codes, zero, group_size, fmt, special_shift) * (st / (1 << _shift(special_shift)))


def int_gemm(Xq, codes, zero, group_size=0, fmt="dint4", special_shift=1):
    """acc[m,n,g] = sum_{k in g} Xq[m,k] d[n,k], d in units of step / 2^t (int64 matmul per group,
    returned as int32)."""
    Xq = np.asarray(Xq).astype(np.int64)
    d = level_units(codes, zero, group_size, fmt, special_shift)
    M, K = Xq.shape
    N = d.shape[0]
    G = _groups(K, group_size)
    acc = np.empty((M, N, K // G), np.int64)
    for g in range(K // G):
        acc[:, :, g] = Xq[:, g * G:(g + 1) * G] @ d[:, g * G:(g + 1) * G].T
    return acc.astype(np.int32)


def layer_output64(Xq, sx, codes, step, zero, group_size=0, fmt="dint4", special_shift=1):
    """sx[m] * sum_g (step / 2^t) acc[m,n,g] in float64."""
    acc = int_gemm(Xq, codes, zero, group_size, fmt, special_shift).astype(np.float64)
    unit = np.asarray(step, np.float64) / (1 << _shift(special_shift))
    return np.asarray(sx, np.float64)[:, None] * np.einsum("mng,ng->mn", acc, unit)


def expand_special(codes, step, zero, group_size=0, special_shift=2):
    """A dINT4 matrix whose special value is c = step / 2^t, t > 1, as an ordinary dINT4 matrix
    (special value step / 2) of twice the width, for a GEMM that only knows the ordinary format:
        +-c = +-step/2 -+ (1 - 2^(1-t)) step/2,
    so columns K .. 2K-1 repeat the groups with step' = (1 - 2^(1-t)) step (one binary32 multiply; 1/2
    and 3/4 are exact factors, the product is rounded for t = 3), the same zero-points, the special
    codes with their signs exchanged and every other code replaced by the zero level z (value 0).
    Multiplied with the activations repeated, [Xq | Xq], the sums of the two halves of a group are
    A1 (ordinary half steps) and A2; in units of step / 2^t the true sum is
        2^(t-1) A1 + (2^(t-1) - 1) A2.
    Returns (codes' u8 [N,2K], step' f32 [N,2K/G], zero' u8 [N,2K/G])."""
    t = _shift(special_shift)
    codes = np.asarray(codes).astype(np.uint8)
    N, K = codes.shape
    G = _groups(K, group_size)
    step = np.asarray(step, F32).reshape(N, K // G)
    zero = np.asarray(zero).astype(np.uint8).reshape(N, K // G)
    zfull = np.repeat(zero, G, axis=1)
    corr = np.where(codes == C1, C2, np.where(codes == C2, C1, zfull)).astype(np.uint8)
    factor = F32(1.0 - 2.0 ** (1 - t))
    step2 = (step * factor).astype(F32)
    return (np.concatenate([codes, corr], axis=1), np.concatenate([step, step2], axis=1),
            np.concatenate([zero, zero], axis=1))


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


def error_split(W, s, group_size=0, fmt="dint4", special_shift=1):
    """The split of Sec. 4.1: with W' = W diag(s) and Wq its dequantized codes, the error Wq - W' on
    the weights whose quantized value is zero (underflow, Delta_u) and on the others (rounding,
    Delta_r).  Returns (Delta_u, Delta_r) in float64; they have disjoint supports and add up to the
    total error."""
    W = np.asarray(W).astype(F32)
    wp = (W * np.asarray(s, F32)[None, :]).astype(F32) if s is not None else W
    codes, step, zero = quantize_weight(W, s, group_size, fmt, special_shift)
    wq = dequant(codes, step, zero, group_size, fmt, special_shift)
    delta = wq - wp.astype(np.float64)
    under = wq == 0.0
    return np.where(under, delta, 0.0), np.where(under, 0.0, delta)


def output_error_terms(X, W, s, group_size=0, fmt="dint4", special_shift=1):
    """The three terms of Eq. 4 on activations X [M,K] (unquantized, X' = X diag(s)^-1 in float64):
    sum (Delta_u X')^2, sum (Delta_r X')^2, sum 2 (Delta_u X')(Delta_r X'); their sum is the squared
    output error of weight quantization alone."""
    du, dr = error_split(W, s, group_size, fmt, special_shift)
    Xs = np.asarray(X, np.float64)
    if s is not None:
        Xs = Xs * (F32(1) / np.asarray(s, F32)).astype(np.float64)[None, :]
    pu, pr = Xs @ du.T, Xs @ dr.T
    return float(np.sum(pu * pu)), float(np.sum(pr * pr)), float(np.sum(2.0 * pu * pr))
