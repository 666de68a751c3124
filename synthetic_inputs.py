"""Seeded synthetic inputs shaped like the OPT / LLaMA linear layers the paper quantizes.

The models and datasets the paper measures on are not available, so these tensors
stand in for them: activations ~N(0,1) with a few fixed large-magnitude outlier
channels (the structure the paper describes for OPT/LLaMA activations, Sec. 3.1),
narrow-range weights ~N(0, 0.02), and an AQAS scale vector s that is an *input* of
the layer (Eq. 1).  This module serves both the CPU oracle and the GPU library and
holds none of the method's arithmetic.

All tensors come from numpy's PCG64 with seed 20231105 + 1000*config + tensor index.
"""
from __future__ import annotations

import math

import numpy as np

BASE_SEED = 20231105

# name -> (config index, x dtype, group size (0 = per output channel), outlier recipe)
CONFIGS = {
    "C1": dict(index=1, x_dtype="f32", group_size=0, M=16, K=768, N=768),
    "C2": dict(index=2, x_dtype="f16", group_size=128, M=16, K=4096, N=4096),
    "C3_up": dict(index=3, x_dtype="f16", group_size=0, M=2048, K=4096, N=11008),
    "C3_down": dict(index=3, x_dtype="f16", group_size=0, M=2048, K=11008, N=4096),
    "C4_5120x5120": dict(index=4, x_dtype="f16", group_size=128, M=2048, K=5120, N=5120),
    "C4_5120x13824": dict(index=4, x_dtype="f16", group_size=128, M=2048, K=5120, N=13824),
    "C4_13824x5120": dict(index=4, x_dtype="f16", group_size=128, M=2048, K=13824, N=5120),
    "C5": dict(index=5, x_dtype="f16", group_size=0, M=4096, K=9216, N=36864),
}


def _rng(config_index: int, tensor_index: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * config_index + tensor_index))


def _normal(rng, shape, std, dtype, chunk_rows=2048):
    """N(0, std) generated in row chunks to bound peak memory."""
    out = np.empty(shape, dtype=dtype)
    for r0 in range(0, shape[0], chunk_rows):
        r1 = min(shape[0], r0 + chunk_rows)
        out[r0:r1] = (rng.standard_normal((r1 - r0, shape[1]), dtype=np.float32) * std).astype(dtype)
    return out


def make_layer(name: str, M: int | None = None, K: int | None = None, N: int | None = None,
               group_size: int | None = None, variant: int = 0):
    """Build (X, W, s, group_size) for a named configuration.

    M / K / N / group_size override the configuration's sizes (reduced shapes for tests keep the
    distribution and outlier structure).  ``variant`` shifts the seeds (distinct weight copies).
    """
    cfg = dict(CONFIGS[name])
    M = cfg["M"] if M is None else M
    K = cfg["K"] if K is None else K
    N = cfg["N"] if N is None else N
    G = cfg["group_size"] if group_size is None else group_size
    ci = cfg["index"] + 100 * variant
    xdt = np.float32 if cfg["x_dtype"] == "f32" else np.float16
    fam = name.split("_")[0]

    rng_x, rng_w, rng_s, rng_o = _rng(ci, 0), _rng(ci, 1), _rng(ci, 2), _rng(ci, 3)
    X = rng_x.standard_normal((M, K), dtype=np.float32)
    if fam == "C1":
        ch = rng_o.choice(K, size=min(4, K), replace=False)
        X[:, ch] *= 30.0
    elif fam in ("C2", "C3"):
        ch = rng_o.choice(K, size=max(1, math.ceil(0.005 * K)), replace=False)
        X[:, ch] *= 50.0
    elif fam == "C4":
        ch = rng_o.choice(K, size=max(1, math.ceil(0.005 * K)), replace=False)
        X[:, ch] = 50.0 * rng_o.standard_t(3.0, size=(M, ch.size)).astype(np.float32)
    elif fam == "C5":
        ch = rng_o.choice(K, size=max(1, round(0.01 * K)), replace=False)
        X[:, ch] *= 100.0
    X = np.clip(X, -65504.0, 65504.0).astype(xdt)

    W = _normal(rng_w, (N, K), 0.02, xdt)

    if fam == "C1":
        s = np.ones((K,), np.float32)
    elif fam == "C5":
        # the alpha = 0.5 point of a max-magnitude scale search space (App. A.4); an input here
        ax = np.abs(X.astype(np.float32)).max(axis=0)
        aw = np.zeros((K,), np.float32)
        for r0 in range(0, N, 2048):
            aw = np.maximum(aw, np.abs(W[r0:r0 + 2048].astype(np.float32)).max(axis=0))
        s = (np.sqrt(np.maximum(ax, 1e-5)) / np.sqrt(np.maximum(aw, 1e-5))).astype(np.float32)
    else:
        s = rng_s.uniform(0.5, 2.0, size=K).astype(np.float32)
    return X, W, s, G


def random_layer(seed: int, M: int, K: int, N: int, x_dtype="f16", outlier_frac=0.005,
                 outlier_gain=50.0, s_range=(0.5, 2.0)):
    """Free-form seeded layer for edge-case tests (same distribution family)."""
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 7919 * seed))
    xdt = np.float32 if x_dtype == "f32" else np.float16
    X = rng.standard_normal((M, K), dtype=np.float32)
    if K > 0 and outlier_frac > 0:
        ch = rng.choice(K, size=max(1, math.ceil(outlier_frac * K)), replace=False)
        X[:, ch] *= outlier_gain
    X = np.clip(X, -65504.0, 65504.0).astype(xdt)
    W = (rng.standard_normal((N, K), dtype=np.float32) * 0.02).astype(xdt)
    s = rng.uniform(s_range[0], s_range[1], size=K).astype(np.float32)
    return X, W, s


def attention_value(seed: int, B: int, M: int, T: int, D: int, v_dtype="f16"):
    """Attention probabilities P [B, M, T] (fp32 rows that sum to 1: a softmax over seeded scores
    with a heavily attended first token and a few peaked positions, the usual shape of decoder
    attention maps) and a cached Value tensor V [B, T, D] ~ N(0, 1) whose channels have seeded
    gains in [0.25, 4] plus two 8x outlier channels per head.  Stands in for the attention maps and
    Value caches of the OPT / LLaMA runs the paper quantizes (Sec. 5.1); values only."""
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 104729 * seed + 17))
    sc = rng.standard_normal((B, M, T), dtype=np.float32) * 2.0
    if T > 0:
        sc[:, :, 0] += 4.0
        hot = rng.integers(0, T, size=(B, M, min(3, T)))
        np.put_along_axis(sc, hot, np.take_along_axis(sc, hot, 2) + 5.0, 2)
        sc -= sc.max(axis=2, keepdims=True)
    P = np.exp(sc)
    P /= np.maximum(P.sum(axis=2, keepdims=True), 1e-30)
    gain = np.exp2(rng.uniform(-2.0, 2.0, size=(B, 1, D))).astype(np.float32)
    if D >= 2:
        for b in range(B):
            gain[b, 0, rng.choice(D, size=2, replace=False)] *= 8.0
    V = rng.standard_normal((B, T, D), dtype=np.float32) * gain
    vdt = np.float32 if v_dtype == "f32" else np.float16
    return P.astype(np.float32), np.clip(V, -65504.0, 65504.0).astype(vdt)
