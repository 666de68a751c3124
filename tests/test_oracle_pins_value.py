"""Pins of the oracle's 4-bit Value-cache functions (Sec. 5.1 "W4A8V4"; App. A.1: Value is
quantized channel-wise, along the dimension the product with the attention map accumulates over).

No expectation below comes from the function it checks: closed-form invariances that only hold for
the right quantization axis, a brute-force nearest-level search in float64, float64 products of
operands rebuilt in numpy, a pure-Python evaluation on a tiny case."""
import numpy as np
import pytest

import synthetic_inputs as syn

P = 13


def levels64(step, z):
    """The 16 dINT4 levels of a (step, zero-point): 14 integer levels and +-step/2 (Eq. 5)."""
    return np.array([(c - z) * step for c in range(P + 1)] + [0.5 * step, -0.5 * step], np.float64)


def dequant64(codes, step, zero):
    """float64 values of codes [B, D, T] with parameters [B, D, T/G], from the level set."""
    B, D, T = codes.shape
    G = T // step.shape[2]
    out = np.empty((B, D, T), np.float64)
    for b in range(B):
        for d in range(D):
            for g in range(T // G):
                lv = levels64(float(step[b, d, g]), int(zero[b, d, g]))
                out[b, d, g * G:(g + 1) * G] = lv[codes[b, d, g * G:(g + 1) * G]]
    return out


def test_parameters_belong_to_channels_not_tokens(oracle):
    """Scale channel d of one base pattern by 2^d: with per-channel ranges over the tokens every
    channel gets the same codes and zero-point and a step scaled by exactly 2^d.  (Ranges taken
    per token instead would mix the channels and change the codes.)"""
    rng = np.random.default_rng(11)
    T, D = 96, 7
    base = rng.standard_normal(T).astype(np.float32)
    V = (base[:, None] * np.exp2(np.arange(D, dtype=np.float32))[None, :])[None]   # [1, T, D]
    codes, step, zero = oracle.quantize_value_dint4(V)
    assert codes.shape == (1, D, T) and step.shape == (1, D, 1) and zero.shape == (1, D, 1)
    for d in range(1, D):
        np.testing.assert_array_equal(codes[0, d], codes[0, 0])
        assert zero[0, d, 0] == zero[0, 0, 0]
        assert step[0, d, 0] == step[0, 0, 0] * np.float32(2.0 ** d)
    # the one step of a channel is its range over ALL tokens divided by p = 13
    lo, hi = min(0.0, float(base.min())), max(0.0, float(base.max()))
    assert step[0, 0, 0] == np.float32(np.float32(hi - lo) / np.float32(13.0))


def test_token_groups_split_the_token_axis(oracle):
    """group_size G: tokens [gG, (g+1)G) of a channel share parameters; scaling one token group of
    every channel by 4 scales exactly that group's steps by 4 and leaves all codes unchanged."""
    rng = np.random.default_rng(12)
    B, T, D, G = 2, 64, 5, 16
    V = rng.standard_normal((B, T, D)).astype(np.float32)
    V2 = V.copy()
    V2[:, G:2 * G, :] *= 4.0
    c1, s1, z1 = oracle.quantize_value_dint4(V, G)
    c2, s2, z2 = oracle.quantize_value_dint4(V2, G)
    np.testing.assert_array_equal(c1, c2)
    np.testing.assert_array_equal(z1, z2)
    want = s1.copy()
    want[:, :, 1] *= 4.0
    np.testing.assert_array_equal(s2, want)


@pytest.mark.parametrize("G", [0, 32])
def test_value_codes_are_nearest_levels_per_channel(oracle, G):
    """Every cached value maps to the nearest of its channel's 16 levels (float64 search), so the
    error is at most step/2, and step/4 within one step of zero; heads are independent."""
    _, V = syn.attention_value(3, 3, 1, 128, 24)
    codes, step, zero = oracle.quantize_value_dint4(V, G)
    dq = dequant64(codes, step, zero)
    Vt = V.astype(np.float64).transpose(0, 2, 1)              # [B, D, T]
    g = V.shape[1] if G == 0 else G
    for b in range(V.shape[0]):
        for d in range(V.shape[2]):
            for k in range(V.shape[1] // g):
                st, z = float(step[b, d, k]), int(zero[b, d, k])
                lv = levels64(st, z)
                x = Vt[b, d, k * g:(k + 1) * g]
                best = np.abs(x[:, None] - lv[None, :]).min(axis=1)
                err = np.abs(x - dq[b, d, k * g:(k + 1) * g])
                assert np.all(err <= best + 1e-5 * st)
                assert np.all(err <= 0.5 * st * (1 + 1e-5))
                near0 = np.abs(x) <= st
                assert np.all(err[near0] <= 0.25 * st * (1 + 1e-5))
    # head b's result does not depend on the other heads
    c0, s0, z0 = oracle.quantize_value_dint4(V[1:2], G)
    np.testing.assert_array_equal(c0[0], codes[1])
    np.testing.assert_array_equal(s0[0], step[1])


@pytest.mark.parametrize("asym", [False, True])
@pytest.mark.parametrize("G", [0, 64])
def test_attention_value_equals_float64_product_of_dequantized_operands(oracle, asym, G):
    B, M, T, D = 3, 5, 192, 16
    Pm, V = syn.attention_value(4, B, M, T, D)
    r = oracle.attention_value_w4a8(Pm, V, G, asym)
    Vdq = dequant64(r["codes"], r["step"], r["zero"])        # [B, D, T]
    q = r["Q"].astype(np.float64) - r["zx"].astype(np.float64)[:, :, None]
    Pdq = q * r["sx"].astype(np.float64)[:, :, None]         # [B, M, T]
    want = np.einsum("bmt,bdt->bmd", Pdq, Vdq)
    np.testing.assert_allclose(r["Y64"], want, rtol=1e-12, atol=1e-12 * np.abs(want).max())
    # the 8-bit probabilities are token-wise: row maxima hit the top code, rows are non-negative
    if asym:
        assert np.all(r["zx"] == 0) and np.all(r["Q"].max(axis=2) == 255)
    else:
        assert np.all(r["Q"].max(axis=2) == 127) and np.all(r["Q"] >= 0)
    # int32 accumulators against an integer product rebuilt in numpy (float64 matmul is exact here)
    g = T if G == 0 else G
    hs = np.where(r["codes"] <= P, 2 * (r["codes"].astype(np.int64) - np.repeat(r["zero"], g, axis=2)),
                  np.where(r["codes"] == 14, 1, -1)).astype(np.float64)
    for k in range(T // g):
        acc = np.einsum("bmt,bdt->bmd", q[:, :, k * g:(k + 1) * g], hs[:, :, k * g:(k + 1) * g])
        np.testing.assert_array_equal(r["acc"][:, :, :, k], acc.astype(np.int64))
    # and the quantized product approximates the unquantized one
    exact = np.einsum("bmt,btd->bmd", Pm.astype(np.float64), V.astype(np.float64))
    scale = np.abs(V.astype(np.float64)).max(axis=1)[:, None, :]          # per channel
    assert np.all(np.abs(r["Y64"] - exact) <= 0.08 * scale)


def test_brute_force_tiny_attention_value(oracle):
    """Pure-Python evaluation: per channel range over the tokens, Eq. 5 codes, absmax 8-bit rows."""
    P_ = np.array([[[0.5, 0.25, 0.125, 0.125], [0.0, 1.0, 0.0, 0.0]]], np.float32)      # [1, 2, 4]
    V = np.array([[[1.0, -8.0], [0.25, 4.0], [-0.5, 0.5], [2.25, 5.0]]], np.float32)    # [1, 4, 2]
    r = oracle.attention_value_w4a8(P_, V)
    # channel 0: tokens (1, .25, -.5, 2.25): range [-0.5, 2.25], step 2.75/13; channel 1: [-8, 5], step 1
    want_codes = []
    for d in range(2):
        col = [float(V[0, t, d]) for t in range(4)]
        lo, hi = min(0.0, min(col)), max(0.0, max(col))
        st = np.float32(np.float32(hi - lo) / np.float32(13))
        ist = np.float32(1) / st
        z = int(min(13, max(0, round(float(np.float32(-lo) * ist)))))
        assert r["step"][0, d, 0] == st and r["zero"][0, d, 0] == z
        row = []
        for x in col:
            u = float(np.float32(x) * ist)
            if 0.25 < u <= 0.75:
                row.append(14)
            elif -0.75 <= u < -0.25:
                row.append(15)
            else:
                row.append(min(13, max(0, int(np.rint(u)) + z)))
        want_codes.append(row)
    assert r["codes"][0].tolist() == want_codes
    assert r["step"][0, 1, 0] == 1.0 and r["zero"][0, 1, 0] == 8
    assert want_codes[1] == [0, 12, 14, 13]               # -8, 4, +step/2, 5 with z = 8
    assert r["Q"][0].tolist() == [[127, 64, 32, 32], [0, 127, 0, 0]]    # 63.5 ties to even 64
    hs1 = [2 * (c - 8) if c <= 13 else (1 if c == 14 else -1) for c in want_codes[1]]
    assert r["acc"][0, 0, 1, 0] == sum(q * h for q, h in zip([127, 64, 32, 32], hs1))
    assert r["acc"][0, 1, 1, 0] == 127 * hs1[1]
    # second query token attends to token 1 only: output = its dequantized Value
    assert abs(r["Y64"][0, 1, 1] - 4.0) < 1e-6
