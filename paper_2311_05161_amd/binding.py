"""Thin ctypes binding of libw4a8.so (the C ABI declared in include/w4a8.h).

Argument marshalling only: every step of the layer runs in the HIP kernels.  PyTorch supplies
device memory (``tensor.data_ptr()``) and the current HIP stream, nothing else.  There is no CPU
fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libw4a8.so")

OK, ERR_NULL, ERR_SHAPE, ERR_DTYPE, ERR_WORKSPACE, ERR_HIP = range(6)
F32, F16, BF16 = 0, 1, 2
LAYOUT_CANONICAL, LAYOUT_TILED = 0, 1

_DTYPES = {torch.float32: F32, torch.float16: F16, torch.bfloat16: BF16}

EXPORTS = (
    "quantize_act_int8", "quantize_weight_dint4", "pack_dint4", "unpack_dint4",
    "w4a8_gemm_workspace_bytes", "w4a8_gemm", "w4a8_status_string",
    "w4a8_gemm_static", "w4a8_gemm_static_scratch_bytes", "w4a8_linear", "w4a8_linear_workspace_bytes",
    "quantize_act_int8_asym", "dint4_weight_sums", "w4a8_gemm_asym", "w4a8_gemm_batched",
    "quantize_value_dint4",
    "aqas_search_workspace_bytes", "aqas_channel_absmax", "aqas_scale", "aqas_search",
    "dint4_clipped_params", "aqas_clip_search",
    "quantize_weight_format", "w4a8_gemm_format", "pack_dint3", "unpack_dint3", "pack_format",
    "unpack_format",
    "dint_error_terms_workspace_bytes", "dint_error_terms",
    "expand_special_value", "w4a8_gemm_special_workspace_bytes", "w4a8_gemm_special",
    "w4a8_measure_stream_read", "w4a8_measure_mfma_i8", "w4a8_measure_ktile_mix",
)
FMT_DINT4, FMT_INT4, FMT_DINT3, FMT_DINT4_C4, FMT_DINT4_C8 = 0, 1, 2, 3, 4

_lib = None


class W4A8Error(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def load_library(path: str | None = None) -> ctypes.CDLL:
    """Load libw4a8.so; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} not found: build it with `python -m paper_2311_05161_amd.build`")
    lib = ctypes.CDLL(path)
    i64, vp, ci, sz = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.quantize_act_int8.argtypes = [vp, ci, i64, i64, i64, vp, vp, vp, vp]
    lib.quantize_act_int8.restype = ci
    lib.quantize_weight_dint4.argtypes = [vp, ci, i64, i64, i64, vp, i64, ci, vp, vp, vp, vp]
    lib.quantize_weight_dint4.restype = ci
    lib.pack_dint4.argtypes = [vp, i64, i64, vp, ci, vp]
    lib.pack_dint4.restype = ci
    lib.unpack_dint4.argtypes = [vp, i64, i64, vp, ci, vp]
    lib.unpack_dint4.restype = ci
    lib.w4a8_gemm_workspace_bytes.argtypes = [i64, i64, i64, i64, ci]
    lib.w4a8_gemm_workspace_bytes.restype = sz
    lib.w4a8_gemm.argtypes = [vp, vp, i64, vp, ci, vp, vp, i64, i64, i64, vp, ci, i64, vp, vp, sz, vp]
    lib.w4a8_gemm.restype = ci
    lib.w4a8_gemm_static.argtypes = [vp, vp, i64, vp, ci, vp, vp, i64, i64, i64, vp, ci, i64, vp, vp]
    lib.w4a8_gemm_static.restype = ci
    lib.w4a8_linear_workspace_bytes.argtypes = [i64, i64, i64, i64, ci]
    lib.w4a8_linear_workspace_bytes.restype = sz
    lib.w4a8_linear.argtypes = [vp, ci, i64, i64, i64, vp, vp, ci, vp, vp, i64, i64, vp, ci, i64, vp, vp, vp,
                                vp, sz, vp]
    lib.w4a8_linear.restype = ci
    lib.w4a8_gemm_static_scratch_bytes.argtypes = []
    lib.w4a8_gemm_static_scratch_bytes.restype = sz
    lib.quantize_act_int8_asym.argtypes = [vp, ci, i64, i64, i64, vp, vp, vp, vp, vp]
    lib.quantize_act_int8_asym.restype = ci
    lib.dint4_weight_sums.argtypes = [vp, vp, i64, i64, i64, vp, vp, vp]
    lib.dint4_weight_sums.restype = ci
    lib.w4a8_gemm_asym.argtypes = [vp, vp, vp, i64, vp, ci, vp, vp, vp, vp, i64, i64, i64, vp, ci,
                                   i64, vp, vp, sz, vp]
    lib.w4a8_gemm_asym.restype = ci
    lib.w4a8_gemm_batched.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, vp, i64, i64, i64, vp, ci,
                                      i64, i64, vp]
    lib.w4a8_gemm_batched.restype = ci
    lib.quantize_value_dint4.argtypes = [vp, ci, i64, i64, i64, i64, i64, i64, vp, vp, vp, vp]
    lib.quantize_value_dint4.restype = ci
    lib.aqas_search_workspace_bytes.argtypes = [i64, i64, i64, i64]
    lib.aqas_search_workspace_bytes.restype = sz
    lib.aqas_channel_absmax.argtypes = [vp, ci, i64, i64, i64, vp, vp]
    lib.aqas_channel_absmax.restype = ci
    lib.aqas_scale.argtypes = [vp, vp, i64, ci, vp, vp]
    lib.aqas_scale.restype = ci
    lib.aqas_search.argtypes = [vp, vp, ci, i64, i64, i64, i64, i64, i64, vp, vp, vp, vp, sz, vp]
    lib.aqas_search.restype = ci
    lib.dint4_clipped_params.argtypes = [vp, ci, i64, i64, i64, vp, i64, vp, ci, vp, vp, vp]
    lib.dint4_clipped_params.restype = ci
    lib.aqas_clip_search.argtypes = [vp, vp, ci, i64, i64, i64, i64, i64, vp, i64, vp, vp, vp, vp, vp,
                                     sz, vp]
    lib.aqas_clip_search.restype = ci
    lib.quantize_weight_format.argtypes = [vp, ci, i64, i64, i64, vp, i64, ci, ci, vp, vp, vp, vp]
    lib.quantize_weight_format.restype = ci
    lib.w4a8_gemm_format.argtypes = [vp, vp, i64, vp, ci, vp, vp, i64, i64, i64, ci, vp, ci, i64, vp, vp,
                                     sz, vp]
    lib.w4a8_gemm_format.restype = ci
    lib.pack_format.argtypes = [vp, i64, i64, vp, ci, ci, vp]
    lib.pack_format.restype = ci
    lib.unpack_format.argtypes = [vp, i64, i64, vp, ci, ci, vp]
    lib.unpack_format.restype = ci
    lib.expand_special_value.argtypes = [vp, vp, vp, i64, i64, i64, ci, vp, vp, vp, vp]
    lib.expand_special_value.restype = ci
    lib.w4a8_gemm_special_workspace_bytes.argtypes = [i64, i64, i64, i64, ci]
    lib.w4a8_gemm_special_workspace_bytes.restype = sz
    lib.w4a8_gemm_special.argtypes = [vp, vp, i64, vp, ci, vp, vp, i64, i64, i64, vp, ci, i64, vp, vp, sz, vp]
    lib.w4a8_gemm_special.restype = ci
    lib.w4a8_measure_stream_read.argtypes = [vp, i64, vp, vp]
    lib.w4a8_measure_stream_read.restype = ci
    lib.w4a8_measure_mfma_i8.argtypes = [i64, vp, vp, vp]
    lib.w4a8_measure_mfma_i8.restype = ci
    lib.w4a8_measure_ktile_mix.argtypes = [i64, ci, vp, vp]
    lib.w4a8_measure_ktile_mix.restype = ci
    lib.pack_dint3.argtypes = [vp, i64, i64, vp, vp]
    lib.pack_dint3.restype = ci
    lib.unpack_dint3.argtypes = [vp, i64, i64, vp, vp]
    lib.unpack_dint3.restype = ci
    lib.dint_error_terms_workspace_bytes.argtypes = [i64, i64, i64, i64]
    lib.dint_error_terms_workspace_bytes.restype = sz
    lib.dint_error_terms.argtypes = [vp, ci, i64, i64, i64, vp, ci, i64, i64, vp, i64, ci, vp, vp, sz, vp]
    lib.dint_error_terms.restype = ci
    lib.w4a8_status_string.argtypes = [ci]
    lib.w4a8_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().w4a8_status_string(int(status)).decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status: int, where: str):
    if status != OK:
        raise W4A8Error(status, where)


def _rows(t: torch.Tensor, what: str):
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError(f"{what} must be 2-D with contiguous rows")
    return t.shape[0], t.shape[1], t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])


def quantize_act_int8(X: torch.Tensor, s: torch.Tensor | None = None, Xq=None, sx=None):
    """Xq int8 [M,K], sx float32 [M] = per-token absmax INT8 of X diag(s)^-1."""
    M, K, ldx = _rows(X, "X")
    if Xq is None:
        Xq = torch.empty((M, K), dtype=torch.int8, device=X.device)
    if sx is None:
        sx = torch.empty((M,), dtype=torch.float32, device=X.device)
    _check(load_library().quantize_act_int8(_ptr(X), _DTYPES[X.dtype], M, K, ldx, _ptr(s),
                                            _ptr(Xq), _ptr(sx), _stream()), "quantize_act_int8")
    return Xq, sx


def quantize_weight_dint4(W: torch.Tensor, s: torch.Tensor | None = None, group_size: int = 0,
                          step: torch.Tensor | None = None, zero: torch.Tensor | None = None):
    """codes u8 [N,K], step f32 [N,K/G], zero u8 [N,K/G] = dINT4 quantization of W diag(s).

    With ``step`` and ``zero`` given they are used as the quantization parameters.
    """
    N, K, ldw = _rows(W, "W")
    G = K if group_size in (0, None) else int(group_size)
    use_given = step is not None
    ngr = K // G if G > 0 and K % G == 0 else 1
    if not use_given:
        step = torch.empty((N, ngr), dtype=torch.float32, device=W.device)
        zero = torch.empty((N, ngr), dtype=torch.uint8, device=W.device)
    codes = torch.empty((N, K), dtype=torch.uint8, device=W.device)
    _check(load_library().quantize_weight_dint4(_ptr(W), _DTYPES[W.dtype], N, K, ldw, _ptr(s),
                                                int(group_size or 0), int(use_given), _ptr(codes),
                                                _ptr(step), _ptr(zero), _stream()),
           "quantize_weight_dint4")
    return codes, step, zero


def pack_dint4(codes: torch.Tensor, layout: int = LAYOUT_TILED, out=None):
    N, K = codes.shape
    packed = out if out is not None else torch.empty((N * K // 2,), dtype=torch.uint8,
                                                     device=codes.device)
    _check(load_library().pack_dint4(_ptr(codes), N, K, _ptr(packed), int(layout), _stream()),
           "pack_dint4")
    return packed.view(N, K // 2) if layout == LAYOUT_CANONICAL and out is None else packed


def unpack_dint4(packed: torch.Tensor, N: int, K: int, layout: int = LAYOUT_TILED):
    codes = torch.empty((N, K), dtype=torch.uint8, device=packed.device)
    _check(load_library().unpack_dint4(_ptr(packed), N, K, _ptr(codes), int(layout), _stream()),
           "unpack_dint4")
    return codes


def gemm_workspace_bytes(M: int, N: int, K: int, group_size: int = 0,
                         layout: int = LAYOUT_TILED) -> int:
    return int(load_library().w4a8_gemm_workspace_bytes(M, N, K, int(group_size or 0), int(layout)))


def w4a8_gemm(Xq: torch.Tensor, sx: torch.Tensor, Wp: torch.Tensor, step: torch.Tensor,
              zero: torch.Tensor, N: int, K: int, group_size: int = 0, layout: int = LAYOUT_TILED,
              out_dtype=torch.float16, Y=None, acc_out=None, workspace=None, want_acc=False):
    """Y [M,N] = dequant(Xq . dINT4(Wp)^T); optionally also the exact int32 accumulators."""
    M = Xq.shape[0]
    if Y is None:
        Y = torch.empty((M, N), dtype=out_dtype, device=Xq.device)
    G = K if group_size in (0, None) else int(group_size)
    if want_acc and acc_out is None:
        acc_out = torch.empty((M, N, K // G), dtype=torch.int32, device=Xq.device)
    need = gemm_workspace_bytes(M, N, K, group_size, layout)
    if workspace is None and need > 0:
        workspace = torch.empty((need,), dtype=torch.uint8, device=Xq.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    ldy = Y.stride(0) if M > 1 else max(Y.stride(0), N)
    _check(load_library().w4a8_gemm(_ptr(Xq), _ptr(sx), M, _ptr(Wp), int(layout), _ptr(step),
                                    _ptr(zero), N, K, int(group_size or 0), _ptr(Y),
                                    _DTYPES[Y.dtype], ldy, _ptr(acc_out), _ptr(workspace), ws_bytes,
                                    _stream()), "w4a8_gemm")
    return (Y, acc_out) if want_acc else Y


def w4a8_linear(X: torch.Tensor, s, Wp: torch.Tensor, step: torch.Tensor, zero: torch.Tensor, N: int,
                group_size: int = 0, layout: int = LAYOUT_TILED, out_dtype=torch.float16, Y=None,
                want_quantized=False, want_acc=False, workspace=None):
    """The whole layer in one call (one launch for up to 16 tokens of fp16 activations).
    Returns Y, or (Y, Xq, sx[, acc]) with want_quantized / want_acc."""
    M, K, ldx = _rows(X, "X")
    if Y is None:
        Y = torch.empty((M, N), dtype=out_dtype, device=X.device)
    G = K if group_size in (0, None) else int(group_size)
    Xq = torch.empty((M, K), dtype=torch.int8, device=X.device) if want_quantized else None
    sx = torch.empty((M,), dtype=torch.float32, device=X.device) if want_quantized else None
    acc = torch.empty((M, N, K // G), dtype=torch.int32, device=X.device) if want_acc else None
    need = int(load_library().w4a8_linear_workspace_bytes(M, N, K, int(group_size or 0), int(layout)))
    if workspace is None and need > 0:
        workspace = torch.empty((need,), dtype=torch.uint8, device=X.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    ldy = Y.stride(0) if M > 1 else max(Y.stride(0), N)
    _check(load_library().w4a8_linear(_ptr(X), _DTYPES[X.dtype], M, K, ldx, _ptr(s), _ptr(Wp), int(layout),
                                      _ptr(step), _ptr(zero), N, int(group_size or 0), _ptr(Y),
                                      _DTYPES[Y.dtype], ldy, _ptr(Xq), _ptr(sx), _ptr(acc), _ptr(workspace),
                                      ws_bytes, _stream()), "w4a8_linear")
    out = (Y,)
    if want_quantized:
        out += (Xq, sx)
    if want_acc:
        out += (acc,)
    return out[0] if len(out) == 1 else out


def w4a8_gemm_static(Xq: torch.Tensor, sx: torch.Tensor, Wp: torch.Tensor, step: torch.Tensor,
                     zero: torch.Tensor, N: int, K: int, group_size: int = 0, layout: int = LAYOUT_TILED,
                     Y=None, acc_out=None):
    """w4a8_gemm on the library's static scratch: Y and acc_out come from the caller (this wrapper
    allocates nothing either)."""
    M = Xq.shape[0]
    ldy = Y.stride(0) if M > 1 else max(Y.stride(0), N)
    _check(load_library().w4a8_gemm_static(_ptr(Xq), _ptr(sx), M, _ptr(Wp), int(layout), _ptr(step),
                                           _ptr(zero), N, K, int(group_size or 0), _ptr(Y),
                                           _DTYPES[Y.dtype], ldy, _ptr(acc_out), _stream()),
           "w4a8_gemm_static")
    return Y


def quantize_act_int8_asym(X: torch.Tensor, s: torch.Tensor | None = None, Xq=None, sx=None,
                           zx=None):
    """Token-wise min-max asymmetric 8-bit quantization of X diag(s)^-1.
    Returns (Xq int8 = code - 128, sx float32 [M], zx int32 [M] = zero-point - 128)."""
    M, K, ldx = _rows(X, "X")
    if Xq is None:
        Xq = torch.empty((M, K), dtype=torch.int8, device=X.device)
    if sx is None:
        sx = torch.empty((M,), dtype=torch.float32, device=X.device)
    if zx is None:
        zx = torch.empty((M,), dtype=torch.int32, device=X.device)
    _check(load_library().quantize_act_int8_asym(_ptr(X), _DTYPES[X.dtype], M, K, ldx, _ptr(s),
                                                 _ptr(Xq), _ptr(sx), _ptr(zx), _stream()),
           "quantize_act_int8_asym")
    return Xq, sx, zx


def dint4_weight_sums(codes: torch.Tensor, zero: torch.Tensor, group_size: int = 0):
    """(wsum int32 [N,K/G], tsum int32 [N,K/128]) of a quantized weight matrix (offline)."""
    N, K = codes.shape
    G = K if group_size in (0, None) else int(group_size)
    ngr = K // G if G > 0 and K % G == 0 else 1
    wsum = torch.empty((N, ngr), dtype=torch.int32, device=codes.device)
    tsum = torch.empty((N, max(1, K // 128)), dtype=torch.int32, device=codes.device)
    _check(load_library().dint4_weight_sums(_ptr(codes), _ptr(zero), N, K, int(group_size or 0),
                                            _ptr(wsum), _ptr(tsum), _stream()),
           "dint4_weight_sums")
    return wsum, tsum


def w4a8_gemm_asym(Xq: torch.Tensor, sx: torch.Tensor, zx: torch.Tensor, Wp: torch.Tensor,
                   step: torch.Tensor, zero: torch.Tensor, wsum: torch.Tensor, tsum: torch.Tensor,
                   N: int, K: int, group_size: int = 0, layout: int = LAYOUT_TILED,
                   out_dtype=torch.float16, Y=None, acc_out=None, workspace=None, want_acc=False):
    """w4a8_gemm for activations with a token zero-point (quantize_act_int8_asym)."""
    M = Xq.shape[0]
    if Y is None:
        Y = torch.empty((M, N), dtype=out_dtype, device=Xq.device)
    G = K if group_size in (0, None) else int(group_size)
    if want_acc and acc_out is None:
        acc_out = torch.empty((M, N, K // G), dtype=torch.int32, device=Xq.device)
    need = gemm_workspace_bytes(M, N, K, group_size, layout)
    if workspace is None and need > 0:
        workspace = torch.empty((need,), dtype=torch.uint8, device=Xq.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    ldy = Y.stride(0) if M > 1 else max(Y.stride(0), N)
    _check(load_library().w4a8_gemm_asym(_ptr(Xq), _ptr(sx), _ptr(zx), M, _ptr(Wp), int(layout),
                                         _ptr(step), _ptr(zero), _ptr(wsum), _ptr(tsum), N, K,
                                         int(group_size or 0), _ptr(Y), _DTYPES[Y.dtype], ldy,
                                         _ptr(acc_out), _ptr(workspace), ws_bytes, _stream()),
           "w4a8_gemm_asym")
    return (Y, acc_out) if want_acc else Y


def w4a8_gemm_batched(Xq: torch.Tensor, sx: torch.Tensor, Wp: torch.Tensor, step: torch.Tensor,
                      zero: torch.Tensor, batch: int, M: int, N: int, K: int, group_size: int = 0,
                      zx=None, wsum=None, tsum=None, out_dtype=torch.float16, Y=None):
    """`batch` decode products (M <= 16) of one shape in one launch; operands densely stacked:
    Xq [batch*M, K], Wp tiled [batch*N*K/2], step/zero [batch*N, K/G], Y [batch*M, N]."""
    if Y is None:
        Y = torch.empty((batch * M, N), dtype=out_dtype, device=Xq.device)
    _check(load_library().w4a8_gemm_batched(_ptr(Xq), _ptr(sx), _ptr(zx), M, _ptr(Wp), _ptr(step),
                                            _ptr(zero), _ptr(wsum), _ptr(tsum), N, K,
                                            int(group_size or 0), _ptr(Y), _DTYPES[Y.dtype],
                                            Y.stride(0), batch, _stream()), "w4a8_gemm_batched")
    return Y


def quantize_value_dint4(V: torch.Tensor, group_size: int = 0):
    """V [batch, T, D] (last dimension contiguous) -> (codes u8 [batch*D, T], step f32
    [batch*D, T/G], zero u8 [batch*D, T/G]): channel-wise dINT4 along the tokens, stored as V^T."""
    B, T, D = V.shape
    if V.stride(2) != 1 and D > 1:
        raise ValueError("the channel dimension of V must be contiguous")
    G = T if not group_size else int(group_size)
    ng = T // G if G > 0 and T % G == 0 else 1
    codes = torch.empty((B * D, T), dtype=torch.uint8, device=V.device)
    step = torch.empty((B * D, ng), dtype=torch.float32, device=V.device)
    zero = torch.empty((B * D, ng), dtype=torch.uint8, device=V.device)
    _check(load_library().quantize_value_dint4(_ptr(V), _DTYPES[V.dtype], B, T, D, V.stride(1),
                                               V.stride(0), int(group_size or 0), _ptr(codes),
                                               _ptr(step), _ptr(zero), _stream()),
           "quantize_value_dint4")
    return codes, step, zero


# ---- AQAS scale search and weight clipping (offline calibration) ---------------------------------
def aqas_channel_absmax(A: torch.Tensor) -> torch.Tensor:
    R, K, lda = _rows(A, "A")
    out = torch.empty((K,), dtype=torch.float32, device=A.device)
    _check(load_library().aqas_channel_absmax(_ptr(A), _DTYPES[A.dtype], R, K, lda, _ptr(out), _stream()),
           "aqas_channel_absmax")
    return out


def aqas_scale(ax: torch.Tensor, aw: torch.Tensor, j: int) -> torch.Tensor:
    s = torch.empty_like(ax)
    _check(load_library().aqas_scale(_ptr(ax), _ptr(aw), ax.numel(), int(j), _ptr(s), _stream()),
           "aqas_scale")
    return s


def _aqas_ws(M, N, K, group_size, device):
    need = int(load_library().aqas_search_workspace_bytes(M, N, K, int(group_size or 0)))
    return torch.empty((max(need, 1),), dtype=torch.uint8, device=device), need


def aqas_search(X: torch.Tensor, W: torch.Tensor, group_size: int = 0):
    """Grid search of the AQAS scale on calibration activations X [M,K] for weights W [N,K].
    Returns (s float32 [K], best_j int32 [1], losses float64 [17]), all on the device."""
    M, K, ldx = _rows(X, "X")
    N, _, ldw = _rows(W, "W")
    ws, need = _aqas_ws(M, N, K, group_size, X.device)
    s = torch.empty((K,), dtype=torch.float32, device=X.device)
    best = torch.empty((1,), dtype=torch.int32, device=X.device)
    losses = torch.empty((17,), dtype=torch.float64, device=X.device)
    _check(load_library().aqas_search(_ptr(X), _ptr(W), _DTYPES[X.dtype], M, N, K, ldx, ldw,
                                      int(group_size or 0), _ptr(s), _ptr(best), _ptr(losses),
                                      _ptr(ws), need, _stream()), "aqas_search")
    return s, best, losses


def dint4_clipped_params(W: torch.Tensor, s, group_size: int = 0, index=None, uniform_index: int = 0):
    N, K, ldw = _rows(W, "W")
    G = K if not group_size else int(group_size)
    ng = K // G if G > 0 and K % G == 0 else 1
    step = torch.empty((N, ng), dtype=torch.float32, device=W.device)
    zero = torch.empty((N, ng), dtype=torch.uint8, device=W.device)
    _check(load_library().dint4_clipped_params(_ptr(W), _DTYPES[W.dtype], N, K, ldw, _ptr(s),
                                               int(group_size or 0), _ptr(index), int(uniform_index),
                                               _ptr(step), _ptr(zero), _stream()), "dint4_clipped_params")
    return step, zero


def aqas_clip_search(X: torch.Tensor, W: torch.Tensor, s: torch.Tensor, group_size: int = 0,
                     want_table: bool = False):
    """Per-output-channel range factor by output error.  Returns (index int32 [N], step, zero[, err])."""
    M, K, ldx = _rows(X, "X")
    N, _, ldw = _rows(W, "W")
    G = K if not group_size else int(group_size)
    ng = K // G if G > 0 and K % G == 0 else 1
    ws, need = _aqas_ws(M, N, K, group_size, X.device)
    idx = torch.empty((N,), dtype=torch.int32, device=X.device)
    step = torch.empty((N, ng), dtype=torch.float32, device=X.device)
    zero = torch.empty((N, ng), dtype=torch.uint8, device=X.device)
    table = torch.empty((11, N), dtype=torch.float64, device=X.device) if want_table else None
    _check(load_library().aqas_clip_search(_ptr(X), _ptr(W), _DTYPES[X.dtype], M, N, K, ldx, ldw, _ptr(s),
                                           int(group_size or 0), _ptr(idx), _ptr(step), _ptr(zero),
                                           _ptr(table), _ptr(ws), need, _stream()), "aqas_clip_search")
    return (idx, step, zero, table) if want_table else (idx, step, zero)


# ---- weight-format variants and the error split -----------------------------------------------------
def quantize_weight_format(W: torch.Tensor, s=None, group_size: int = 0, fmt: int = FMT_DINT4):
    N, K, ldw = _rows(W, "W")
    G = K if not group_size else int(group_size)
    ngr = K // G if G > 0 and K % G == 0 else 1
    step = torch.empty((N, ngr), dtype=torch.float32, device=W.device)
    zero = torch.empty((N, ngr), dtype=torch.uint8, device=W.device)
    codes = torch.empty((N, K), dtype=torch.uint8, device=W.device)
    _check(load_library().quantize_weight_format(_ptr(W), _DTYPES[W.dtype], N, K, ldw, _ptr(s),
                                                 int(group_size or 0), int(fmt), 0, _ptr(codes), _ptr(step),
                                                 _ptr(zero), _stream()), "quantize_weight_format")
    return codes, step, zero


def w4a8_gemm_format(Xq, sx, Wp, step, zero, N: int, K: int, group_size: int = 0, fmt: int = FMT_DINT4,
                     out_dtype=torch.float16, want_acc=False):
    M = Xq.shape[0]
    Y = torch.empty((M, N), dtype=out_dtype, device=Xq.device)
    G = K if not group_size else int(group_size)
    acc = torch.empty((M, N, K // G), dtype=torch.int32, device=Xq.device) if want_acc else None
    need = gemm_workspace_bytes(M, N, K, group_size, LAYOUT_TILED)
    ws = torch.empty((max(need, 1),), dtype=torch.uint8, device=Xq.device)
    _check(load_library().w4a8_gemm_format(_ptr(Xq), _ptr(sx), M, _ptr(Wp), LAYOUT_TILED, _ptr(step),
                                           _ptr(zero), N, K, int(group_size or 0), int(fmt), _ptr(Y),
                                           _DTYPES[Y.dtype], N, _ptr(acc), _ptr(ws), need, _stream()),
           "w4a8_gemm_format")
    return (Y, acc) if want_acc else Y


def pack_format(codes: torch.Tensor, layout: int = LAYOUT_TILED, fmt: int = FMT_DINT4) -> torch.Tensor:
    N, K = codes.shape
    out = torch.empty((N * K // 2,), dtype=torch.uint8, device=codes.device)
    _check(load_library().pack_format(_ptr(codes), N, K, _ptr(out), int(layout), int(fmt), _stream()),
           "pack_format")
    return out


def unpack_format(packed: torch.Tensor, N: int, K: int, layout: int = LAYOUT_TILED,
                  fmt: int = FMT_DINT4) -> torch.Tensor:
    out = torch.empty((N, K), dtype=torch.uint8, device=packed.device)
    _check(load_library().unpack_format(_ptr(packed), N, K, _ptr(out), int(layout), int(fmt), _stream()),
           "unpack_format")
    return out


def expand_special_value(codes, step, zero, group_size: int = 0, fmt: int = FMT_DINT4_C4):
    """dINT4 codes with special value step/4 or step/8 -> ordinary dINT4 operands of twice the width."""
    N, K = codes.shape
    ng = step.shape[1]
    codes2 = torch.empty((N, 2 * K), dtype=torch.uint8, device=codes.device)
    step2 = torch.empty((N, 2 * ng), dtype=torch.float32, device=codes.device)
    zero2 = torch.empty((N, 2 * ng), dtype=torch.uint8, device=codes.device)
    _check(load_library().expand_special_value(_ptr(codes), _ptr(step), _ptr(zero), N, K, int(group_size or 0),
                                               int(fmt), _ptr(codes2), _ptr(step2), _ptr(zero2), _stream()),
           "expand_special_value")
    return codes2, step2, zero2


def w4a8_gemm_special(Xq, sx, Wp2, step2, zero2, N: int, K: int, group_size: int = 0,
                      out_dtype=torch.float16, want_acc=False):
    """The GEMM on the operands of expand_special_value (packed N x 2K); acc [M, N, 2K/G] if asked for."""
    M = Xq.shape[0]
    Y = torch.empty((M, N), dtype=out_dtype, device=Xq.device)
    G = K if not group_size else int(group_size)
    acc = torch.empty((M, N, 2 * K // G), dtype=torch.int32, device=Xq.device) if want_acc else None
    need = load_library().w4a8_gemm_special_workspace_bytes(M, N, K, int(group_size or 0), LAYOUT_TILED)
    ws = torch.empty((max(need, 1),), dtype=torch.uint8, device=Xq.device)
    _check(load_library().w4a8_gemm_special(_ptr(Xq), _ptr(sx), M, _ptr(Wp2), LAYOUT_TILED, _ptr(step2),
                                            _ptr(zero2), N, K, int(group_size or 0), _ptr(Y), _DTYPES[Y.dtype],
                                            N, _ptr(acc), _ptr(ws), need, _stream()), "w4a8_gemm_special")
    return (Y, acc) if want_acc else Y


def pack_dint3(codes: torch.Tensor) -> torch.Tensor:
    N, K = codes.shape
    out = torch.empty((N, 3 * K // 8), dtype=torch.uint8, device=codes.device)
    _check(load_library().pack_dint3(_ptr(codes), N, K, _ptr(out), _stream()), "pack_dint3")
    return out


def unpack_dint3(packed: torch.Tensor, N: int, K: int) -> torch.Tensor:
    out = torch.empty((N, K), dtype=torch.uint8, device=packed.device)
    _check(load_library().unpack_dint3(_ptr(packed), N, K, _ptr(out), _stream()), "unpack_dint3")
    return out


def dint_error_terms(X: torch.Tensor, W: torch.Tensor, s=None, group_size: int = 0, fmt: int = FMT_DINT4):
    """The three terms of the underflow / rounding split of the output error and the number of
    underflowing weights, float64 [4] on the device."""
    M, K, ldx = _rows(X, "X")
    N, _, ldw = _rows(W, "W")
    need = int(load_library().dint_error_terms_workspace_bytes(M, N, K, int(group_size or 0)))
    ws = torch.empty((max(need, 1),), dtype=torch.uint8, device=X.device)
    terms = torch.empty((4,), dtype=torch.float64, device=X.device)
    _check(load_library().dint_error_terms(_ptr(X), _DTYPES[X.dtype], M, K, ldx, _ptr(W), _DTYPES[W.dtype],
                                           N, ldw, _ptr(s), int(group_size or 0), int(fmt), _ptr(terms),
                                           _ptr(ws), need, _stream()), "dint_error_terms")
    return terms
