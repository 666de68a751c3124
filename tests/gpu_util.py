"""Helpers shared by the GPU parity tests (device transfer, tolerance, the tiled layout in numpy)."""
import numpy as np
import torch


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def host(t):
    torch.cuda.synchronize()
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy()
    return t.cpu().numpy()


def tiled_layout_np(codes):
    """The tiled packed layout written out from its definition in include/w4a8.h (numpy only)."""
    codes = np.asarray(codes, np.uint8)
    N, K = codes.shape
    assert N % 16 == 0 and K % 128 == 0
    e = np.where(codes <= 13, (codes >> 1) | ((codes & 1) << 3), np.where(codes == 14, 15, 7))
    e = e.astype(np.uint8).reshape(N // 16, 16, K // 128, 4, 4, 2, 4)  # nt, ln, kt, kb, q, hl, b
    byte = e[:, :, :, :, :, 0, :] | (e[:, :, :, :, :, 1, :] << 4)       # nt, ln, kt, kb, q, b
    return np.ascontiguousarray(byte.transpose(0, 2, 3, 1, 4, 5)).reshape(-1)  # nt, kt, kb, ln, q, b


def assert_y_close(y_gpu, y64, out_dtype="f16"):
    """|Y - Yref| <= tol * max(|Yref|, 1e-3 * row rms); tol = 1e-3 for fp16, 2^-8 for bf16.

    fp16 rounding alone is 2^-11 ~ 4.9e-4 relative, the fp32 epilogue adds ~1e-6; bf16 keeps 8
    significant bits, so its own rounding (2^-9) sets the bound there.
    """
    y_gpu = np.asarray(y_gpu, np.float64)
    tol = 1e-3 if out_dtype == "f16" else 2.0 ** -8
    rms = np.sqrt(np.mean(y64 * y64, axis=1, keepdims=True))
    floor = 1e-3 * rms + 1e-30
    bound = tol * np.maximum(np.abs(y64), floor)
    err = np.abs(y_gpu - y64)
    bad = err > bound
    assert not bad.any(), (f"{bad.sum()} of {bad.size} outputs off; worst rel "
                           f"{(err / np.maximum(np.abs(y64), floor)).max():.3e}")


def decode_table_np(codes, zero, G):
    """Weights in half steps from the closed form of Eq. 5's second half, in numpy only:
    2 (code - z) for the integer codes 0..13, +1 for code 14, -1 for code 15."""
    codes = np.asarray(codes)
    N, K = codes.shape
    G = G or K
    z = np.repeat(np.asarray(zero).reshape(N, K // G).astype(np.int16), G, axis=1)
    c = codes.astype(np.int16)
    return np.where(c <= 13, 2 * (c - z), np.where(c == 14, 1, -1)).astype(np.int16)


def acc_by_float64_matmul(Xq, d, G):
    """acc[m, n, g] = sum_{k in g} Xq[m,k] d[n,k] as a float64 library matmul of the integer-valued
    operands.  Exact: every partial sum is an integer far below 2^53, so the result is the integer
    product of Eq. 1 whatever order the library adds in.  Returns float64 [M, n, K/G]."""
    Xq = np.asarray(Xq)
    M, K = Xq.shape
    G = G or K
    ng = K // G
    X3 = Xq.astype(np.float64).reshape(M, ng, G).transpose(1, 0, 2)            # [ng, M, G]
    D3 = np.asarray(d).astype(np.float64).reshape(-1, ng, G).transpose(1, 2, 0)  # [ng, G, n]
    return np.matmul(X3, D3).transpose(1, 2, 0)                                   # [M, n, ng]
