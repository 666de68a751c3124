"""ctypes front end of the plain-C oracle (``w4a8_oracle.c``) -- TEST INFRASTRUCTURE ONLY.

Marshals numpy arrays to the C functions; holds no arithmetic of the method
beyond exact widening casts (fp16 -> fp32) and the final output cast.
The shared object is compiled with gcc on first use if it is not there.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "w4a8_oracle.c")
_LIB = os.path.join(_HERE, "libw4a8_oracle.so")
_lib = None

__all__ = [
    "build", "num_threads", "quantize_act_int8", "quantize_weight_dint4", "pack_dint4",
    "unpack_dint4", "decode_dint4", "dequant_dint4", "int_gemm", "int_gemm_sampled",
    "dequant_epilogue", "cast_output", "linear_w4a8",
    "quantize_act_uint8_asym", "int_gemm_asym", "int_gemm_asym_sampled", "weight_sums",
    "linear_w4a8_asym", "quantize_value_dint4", "attention_value_w4a8",
]


def build(force: bool = False) -> str:
    """Compile the oracle: one IEEE binary32 operation per source operation (no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, vp = ctypes.c_int64, ctypes.c_void_p
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_quantize_act_int8.argtypes = [vp, i64, i64, i64, vp, vp, vp, vp]
        lib.oracle_quantize_weight_dint4.argtypes = [vp, i64, i64, i64, vp, i64, ctypes.c_int,
                                                     vp, vp, vp]
        lib.oracle_pack_dint4.argtypes = [vp, i64, i64, vp]
        lib.oracle_unpack_dint4.argtypes = [vp, i64, i64, vp]
        lib.oracle_decode_dint4.argtypes = [ctypes.c_int, ctypes.c_int]
        lib.oracle_decode_dint4.restype = ctypes.c_int
        lib.oracle_dequant_dint4.argtypes = [vp, i64, i64, i64, vp, vp, vp]
        lib.oracle_int_gemm.argtypes = [vp, i64, vp, vp, i64, i64, i64, vp]
        lib.oracle_int_gemm_sampled.argtypes = [vp, i64, vp, vp, i64, i64, i64, vp, vp, i64, vp]
        lib.oracle_dequant_epilogue.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp]
        lib.oracle_quantize_act_uint8_asym.argtypes = [vp, i64, i64, i64, vp, vp, vp, vp, vp]
        lib.oracle_int_gemm_asym.argtypes = [vp, vp, i64, vp, vp, i64, i64, i64, vp]
        lib.oracle_int_gemm_asym_sampled.argtypes = [vp, vp, i64, vp, vp, i64, i64, i64, vp, vp,
                                                     i64, vp]
        lib.oracle_weight_sums.argtypes = [vp, vp, i64, i64, i64, i64, vp]
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what}: bad arguments")


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _as_f32(a):
    """Exact widening of fp16 / fp32 input to contiguous fp32 rows."""
    a = np.asarray(a)
    if a.dtype not in (np.float16, np.float32):
        raise TypeError(f"unsupported input dtype {a.dtype}")
    return np.ascontiguousarray(a.astype(np.float32))


def quantize_act_int8(X, s=None):
    """Per-token absmax INT8 of X diag(s)^-1.  Returns (Xq int8 [M,K], sx float32 [M])."""
    X = _as_f32(X)
    M, K = X.shape
    s32 = None if s is None else np.ascontiguousarray(s, dtype=np.float32)
    Xq = np.empty((M, K), np.int8)
    sx = np.empty((M,), np.float32)
    rbuf = np.empty((K,), np.float32)
    _check(_load().oracle_quantize_act_int8(_p(X), M, K, K, _p(s32), _p(Xq), _p(sx), _p(rbuf)),
           "quantize_act_int8")
    return Xq, sx


def quantize_weight_dint4(W, s=None, group_size=0, step=None, zero=None):
    """dINT4 codes of W diag(s).  Returns (codes u8 [N,K], step f32 [N,K/G], zero u8 [N,K/G]).

    With ``step`` and ``zero`` given they are used as the quantization parameters.
    """
    W = _as_f32(W)
    N, K = W.shape
    G = K if group_size in (0, None) else int(group_size)
    if G <= 0 or K % G:
        raise ValueError("oracle quantize_weight_dint4: bad arguments")
    s32 = None if s is None else np.ascontiguousarray(s, dtype=np.float32)
    use_given = step is not None
    if use_given:
        step_a = np.ascontiguousarray(step, dtype=np.float32).reshape(N, K // G).copy()
        zero_a = np.ascontiguousarray(zero, dtype=np.uint8).reshape(N, K // G).copy()
    else:
        step_a = np.empty((N, K // G), np.float32)
        zero_a = np.empty((N, K // G), np.uint8)
    codes = np.empty((N, K), np.uint8)
    _check(_load().oracle_quantize_weight_dint4(_p(W), N, K, K, _p(s32), G, int(use_given),
                                                _p(codes), _p(step_a), _p(zero_a)),
           "quantize_weight_dint4")
    return codes, step_a, zero_a


def pack_dint4(codes):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, K = codes.shape
    packed = np.empty((N, K // 2), np.uint8)
    _check(_load().oracle_pack_dint4(_p(codes), N, K, _p(packed)), "pack_dint4")
    return packed


def unpack_dint4(packed):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    N, K2 = packed.shape
    codes = np.empty((N, 2 * K2), np.uint8)
    _check(_load().oracle_unpack_dint4(_p(packed), N, 2 * K2, _p(codes)), "unpack_dint4")
    return codes


def decode_dint4(code: int, z: int) -> int:
    """Value of one code in half-step units."""
    return int(_load().oracle_decode_dint4(int(code), int(z)))


def dequant_dint4(codes, step, zero, group_size=0):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, K = codes.shape
    G = K if group_size in (0, None) else int(group_size)
    step = np.ascontiguousarray(step, dtype=np.float32).reshape(N, K // G)
    zero = np.ascontiguousarray(zero, dtype=np.uint8).reshape(N, K // G)
    out = np.empty((N, K), np.float32)
    _check(_load().oracle_dequant_dint4(_p(codes), N, K, G, _p(step), _p(zero), _p(out)),
           "dequant_dint4")
    return out


def int_gemm(Xq, packed, zero, group_size=0):
    """acc[m,n,g] int32 from int8 activations and canonically packed dINT4 weights."""
    Xq = np.ascontiguousarray(Xq, dtype=np.int8)
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    M, K = Xq.shape
    N = packed.shape[0]
    if packed.shape[1] * 2 != K:
        raise ValueError("oracle int_gemm: K mismatch")
    G = K if group_size in (0, None) else int(group_size)
    zero = np.ascontiguousarray(zero, dtype=np.uint8).reshape(N, K // G)
    acc = np.empty((M, N, K // G), np.int32)
    _check(_load().oracle_int_gemm(_p(Xq), M, _p(packed), _p(zero), N, K, G, _p(acc)), "int_gemm")
    return acc


def int_gemm_sampled(Xq, packed, zero, group_size, mi, ni):
    """acc[i,g] for the output coordinates (mi[i], ni[i])."""
    Xq = np.ascontiguousarray(Xq, dtype=np.int8)
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    M, K = Xq.shape
    N = packed.shape[0]
    G = K if group_size in (0, None) else int(group_size)
    zero = np.ascontiguousarray(zero, dtype=np.uint8).reshape(N, K // G)
    mi = np.ascontiguousarray(mi, dtype=np.int64)
    ni = np.ascontiguousarray(ni, dtype=np.int64)
    acc = np.empty((mi.size, K // G), np.int32)
    _check(_load().oracle_int_gemm_sampled(_p(Xq), M, _p(packed), _p(zero), N, K, G,
                                           _p(mi), _p(ni), mi.size, _p(acc)), "int_gemm_sampled")
    return acc


def dequant_epilogue(acc, sx, step):
    """Returns (Y32, Y64): binary32 sequence and binary64 evaluation of sx * sum_g (step/2) acc."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    M, N, ng = acc.shape
    sx = np.ascontiguousarray(sx, dtype=np.float32)
    step = np.ascontiguousarray(step, dtype=np.float32).reshape(N, ng)
    y32 = np.empty((M, N), np.float32)
    y64 = np.empty((M, N), np.float64)
    _check(_load().oracle_dequant_epilogue(_p(acc), _p(sx), _p(step), M, N, ng, _p(y32), _p(y64)),
           "dequant_epilogue")
    return y32, y64


def cast_output(Y32, dtype: str):
    """Round fp32 results to the output type (round to nearest even) and widen back to fp32."""
    Y32 = np.asarray(Y32, dtype=np.float32)
    if dtype == "f16":
        return Y32.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        bits = Y32.view(np.uint32).astype(np.uint64)
        rounded = ((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16) << 16
        return rounded.astype(np.uint32).view(np.float32).reshape(Y32.shape)
    if dtype == "f32":
        return Y32
    raise ValueError(dtype)


def linear_w4a8(X, W, s=None, group_size=0):
    """Whole path on the CPU.  Returns a dict of every intermediate."""
    Xq, sx = quantize_act_int8(X, s)
    codes, step, zero = quantize_weight_dint4(W, s, group_size)
    packed = pack_dint4(codes)
    acc = int_gemm(Xq, packed, zero, group_size)
    y32, y64 = dequant_epilogue(acc, sx, step)
    return dict(Xq=Xq, sx=sx, codes=codes, step=step, zero=zero, packed=packed, acc=acc,
                Y32=y32, Y64=y64)


# ---- asymmetric (min-max, token zero-point) activations: App. A.1 ------------------------------
def quantize_act_uint8_asym(X, s=None):
    """Per-token min-max asymmetric 8-bit codes of X diag(s)^-1.
    Returns (Q uint8 [M,K], sx float32 [M], zx int32 [M]); value = (Q - zx) * sx."""
    X = _as_f32(X)
    M, K = X.shape
    s32 = None if s is None else np.ascontiguousarray(s, dtype=np.float32)
    Q = np.empty((M, K), np.uint8)
    sx = np.empty((M,), np.float32)
    zx = np.empty((M,), np.int32)
    rbuf = np.empty((K,), np.float32)
    _check(_load().oracle_quantize_act_uint8_asym(_p(X), M, K, K, _p(s32), _p(Q), _p(sx), _p(zx),
                                                  _p(rbuf)), "quantize_act_uint8_asym")
    return Q, sx, zx


def int_gemm_asym(Q, zx, packed, zero, group_size=0):
    """acc[m,n,g] = sum_k (Q - zx) * d from uint8 codes with a token zero-point."""
    Q = np.ascontiguousarray(Q, dtype=np.uint8)
    zx = np.ascontiguousarray(zx, dtype=np.int32)
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    M, K = Q.shape
    N = packed.shape[0]
    if packed.shape[1] * 2 != K or zx.shape != (M,):
        raise ValueError("oracle int_gemm_asym: shape mismatch")
    G = K if group_size in (0, None) else int(group_size)
    zero = np.ascontiguousarray(zero, dtype=np.uint8).reshape(N, K // G)
    acc = np.empty((M, N, K // G), np.int32)
    _check(_load().oracle_int_gemm_asym(_p(Q), _p(zx), M, _p(packed), _p(zero), N, K, G, _p(acc)),
           "int_gemm_asym")
    return acc


def int_gemm_asym_sampled(Q, zx, packed, zero, group_size, mi, ni):
    """acc[i,g] for the output coordinates (mi[i], ni[i])."""
    Q = np.ascontiguousarray(Q, dtype=np.uint8)
    zx = np.ascontiguousarray(zx, dtype=np.int32)
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    M, K = Q.shape
    N = packed.shape[0]
    G = K if group_size in (0, None) else int(group_size)
    zero = np.ascontiguousarray(zero, dtype=np.uint8).reshape(N, K // G)
    mi = np.ascontiguousarray(mi, dtype=np.int64)
    ni = np.ascontiguousarray(ni, dtype=np.int64)
    acc = np.empty((mi.size, K // G), np.int32)
    _check(_load().oracle_int_gemm_asym_sampled(_p(Q), _p(zx), M, _p(packed), _p(zero), N, K, G,
                                                _p(mi), _p(ni), mi.size, _p(acc)),
           "int_gemm_asym_sampled")
    return acc


def weight_sums(packed, zero, group_size=0, block=0):
    """wsum int32 [N, K/block]: sums of the weights in half steps over blocks of `block` input
    channels (default: the quantization group)."""
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    N, K = packed.shape[0], packed.shape[1] * 2
    G = K if group_size in (0, None) else int(group_size)
    T = G if block in (0, None) else int(block)
    zero = np.ascontiguousarray(zero, dtype=np.uint8).reshape(N, K // G)
    wsum = np.empty((N, K // T), np.int32)
    _check(_load().oracle_weight_sums(_p(packed), _p(zero), N, K, G, T, _p(wsum)), "weight_sums")
    return wsum


def linear_w4a8_asym(X, W, s=None, group_size=0):
    """Whole path with asymmetric activations on the CPU."""
    Q, sx, zx = quantize_act_uint8_asym(X, s)
    codes, step, zero = quantize_weight_dint4(W, s, group_size)
    packed = pack_dint4(codes)
    acc = int_gemm_asym(Q, zx, packed, zero, group_size)
    y32, y64 = dequant_epilogue(acc, sx, step)
    wsum = weight_sums(packed, zero, group_size)
    return dict(Q=Q, sx=sx, zx=zx, codes=codes, step=step, zero=zero, packed=packed, acc=acc,
                wsum=wsum, Y32=y32, Y64=y64)


# ---- 4-bit Value cache: attention probabilities times Value (Sec. 5.1, App. A.1) ----------------
def quantize_value_dint4(V, group_size=0):
    """Channel-wise dINT4 of the cached Value tensor V [B, T, D] (B heads, T tokens, D channels).

    The product P.V accumulates over the tokens, so one (step, zero) belongs to a channel d (or to
    a group of `group_size` consecutive tokens of it) and is shared along the accumulation
    dimension: V^T [D, T] of every head is quantized exactly like a weight matrix with one output
    channel per row.  Returns (codes u8 [B, D, T], step f32 [B, D, T/G], zero u8 [B, D, T/G])."""
    V = np.asarray(V)
    B, T, D = V.shape
    G = T if group_size in (0, None) else int(group_size)
    codes = np.empty((B, D, T), np.uint8)
    step = np.empty((B, D, T // G), np.float32)
    zero = np.empty((B, D, T // G), np.uint8)
    for b in range(B):
        Vt = np.ascontiguousarray(V[b].T)            # [D, T]: accumulation dimension last
        codes[b], step[b], zero[b] = quantize_weight_dint4(Vt, None, G)
    return codes, step, zero


def attention_value_w4a8(P, V, group_size=0, asym=False):
    """O[b] = dequant( Q8(P[b]) . dINT4(V[b]) ) for every head b.

    P [B, M, T]: attention probabilities of M query tokens, 8-bit token-wise (absmax form, or the
    min-max form with a zero-point when ``asym``); V [B, T, D] as in quantize_value_dint4.
    Returns a dict of every intermediate, stacked over b."""
    P = np.asarray(P)
    B, M, T = P.shape
    D = V.shape[2]
    G = T if group_size in (0, None) else int(group_size)
    codes, step, zero = quantize_value_dint4(V, G)
    out = dict(codes=codes, step=step, zero=zero,
               Q=np.empty((B, M, T), np.uint8 if asym else np.int8), sx=np.empty((B, M), np.float32),
               zx=np.zeros((B, M), np.int32), acc=np.empty((B, M, D, T // G), np.int32),
               Y32=np.empty((B, M, D), np.float32), Y64=np.empty((B, M, D), np.float64))
    for b in range(B):
        packed = pack_dint4(codes[b])
        if asym:
            out["Q"][b], out["sx"][b], out["zx"][b] = quantize_act_uint8_asym(P[b])
            out["acc"][b] = int_gemm_asym(out["Q"][b], out["zx"][b], packed, zero[b], G)
        else:
            out["Q"][b], out["sx"][b] = quantize_act_int8(P[b])
            out["acc"][b] = int_gemm(out["Q"][b], packed, zero[b], G)
        out["Y32"][b], out["Y64"][b] = dequant_epilogue(out["acc"][b], out["sx"][b], step[b])
    return out
