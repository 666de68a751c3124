"""Pins of the oracle's asymmetric-activation functions (token-wise min-max 8-bit, App. A.1).

None of the expectations below is produced by the function it checks: hand-worked fixture,
closed forms and bounds, float64 matmuls of independently rebuilt operands, brute force."""
import os

import numpy as np
import pytest

from conftest import GOLDEN

P = 13


def half_steps(codes, z):
    codes = codes.astype(np.int64)
    return np.where(codes <= P, 2 * (codes - z), np.where(codes == 14, 1, -1))


def read_tokens():
    tok, rows = {}, []
    with open(os.path.join(GOLDEN, "act_uint8_asym_worked_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            p = line.split()
            if p[0] == "T":
                tok[int(p[1])] = [float(v) for v in p[2:]]
            else:
                rows.append([float(v) for v in p])
    return tok, np.array(rows)


def test_golden_asym_worked_example(oracle):
    tok, rows = read_tokens()
    for t, (lo, hi, sx_want, zx_want) in tok.items():
        r = rows[rows[:, 0] == t]
        x = r[:, 1].astype(np.float32)[None, :]
        s = r[:, 2].astype(np.float32)
        # the fixture's own t column is x / s, and its extremes are the stated range
        np.testing.assert_array_equal((x[0] / s).astype(np.float32), r[:, 3].astype(np.float32))
        assert min(0.0, r[:, 3].min()) == lo and max(0.0, r[:, 3].max()) == hi
        q, sx, zx = oracle.quantize_act_uint8_asym(x, s)
        assert sx[0] == np.float32(sx_want) and zx[0] == int(zx_want)
        assert q[0].tolist() == r[:, 4].astype(int).tolist()


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_asym_properties(oracle, seed):
    rng = np.random.default_rng(500 + seed)
    M, K = 37, 200
    x = (rng.standard_normal((M, K)) * rng.uniform(0.1, 30, (M, 1)) +
         rng.uniform(-20, 20, (M, 1))).astype(np.float32)
    x[3] = np.abs(x[3])          # all positive
    x[4] = -np.abs(x[4])         # all negative
    x[5] = 0                     # zero token
    s = rng.uniform(0.5, 2.0, K).astype(np.float32)
    q, sx, zx = oracle.quantize_act_uint8_asym(x, s)
    t = x.astype(np.float64) / s.astype(np.float64)   # float64 evaluation of the fold
    lo = np.minimum(0, t.min(1))
    hi = np.maximum(0, t.max(1))
    # zero token
    assert sx[5] == 1.0 and zx[5] == 0 and not q[5].any()
    live = hi > lo
    # scale = range / 255 up to binary32 rounding of the fold, the subtraction and the division
    np.testing.assert_allclose(sx[live], ((hi - lo) / 255)[live], rtol=4e-7)
    # zero-point: the real value 0 is a level; it sits at -lo / sx rounded, within the code range
    assert ((zx >= 0) & (zx <= 255)).all()
    assert np.all(np.abs(zx[live] - (-lo[live] / sx[live])) <= 0.5 + 1e-3)
    assert zx[3] == 0 and zx[4] == 255
    # reconstruction error is at most half a step (plus the zero-point's own rounding at the
    # clamped ends) for every element, and the extremes map to the end codes
    rec = (q.astype(np.float64) - zx[:, None]) * sx[:, None]
    err = np.abs(rec - t)
    assert np.all(err[live] <= (0.5 + 0.5 + 1e-3) * sx[live, None])
    inner = (q > 0) & (q < 255)
    assert np.all(err[inner] <= ((0.5 + 2e-3) * sx[:, None] * np.ones_like(err))[inner])
    for m in np.nonzero(live)[0]:
        # rne(lo / sx) + rne(-lo / sx) = 0; rne(hi / sx) + rne(-lo / sx) is 255 up to one rounding
        if lo[m] < 0:
            assert q[m, t[m].argmin()] == 0
        if hi[m] > 0:
            assert q[m, t[m].argmax()] in (254, 255)
    # exact zeros of the input land exactly on the zero-point
    x2 = x.copy()
    x2[:, ::7] = 0
    q2, sx2, zx2 = oracle.quantize_act_uint8_asym(x2, s)
    assert np.all(q2[:, ::7] == zx2[:, None].astype(np.uint8))


def test_asym_matches_textbook_formula_away_from_ties(oracle):
    """The textbook asymmetric quantizer in float64, compared wherever float64 and binary32 cannot
    disagree about the rounding (u farther than 1e-3 from a half-integer)."""
    rng = np.random.default_rng(77)
    x = (rng.standard_normal((64, 512)) * 3 + 1.5).astype(np.float32)
    q, sx, zx = oracle.quantize_act_uint8_asym(x, None)
    t = x.astype(np.float64)
    lo = np.minimum(0, t.min(1, keepdims=True))
    hi = np.maximum(0, t.max(1, keepdims=True))
    st = (hi - lo) / 255
    z = np.clip(np.rint(-lo / st), 0, 255)
    u = t / st
    safe = np.abs(u - np.floor(u) - 0.5) > 1e-3
    want = np.clip(np.rint(u) + z, 0, 255)
    assert (zx == z[:, 0]).all()
    assert np.array_equal(q[safe], want[safe].astype(np.uint8))
    assert safe.mean() > 0.99


def test_asym_power_of_two_row_scaling(oracle):
    """Scaling a token by 2^k scales sx by 2^k and changes no code or zero-point."""
    rng = np.random.default_rng(78)
    x = (rng.standard_normal((8, 96)) + 0.3).astype(np.float32)
    q, sx, zx = oracle.quantize_act_uint8_asym(x, None)
    q8, sx8, zx8 = oracle.quantize_act_uint8_asym(x * np.float32(8.0), None)
    assert np.array_equal(q, q8) and np.array_equal(zx, zx8)
    assert np.array_equal(sx8, sx * np.float32(8.0))


def test_symmetric_range_reduces_to_a_plain_uniform_quantizer(oracle):
    """With lo = -hi = -255/64 the step is exactly 1/32 and the zero-point 128 (127.5 ties to
    even): the codes are those of a plain uniform quantizer with that step."""
    x = np.array([[-3.984375, 3.984375, 1.0, -1.0, 0.0, 3.9, -0.3]], np.float32)
    q, sx, zx = oracle.quantize_act_uint8_asym(x, None)
    assert zx[0] == 128 and sx[0] == np.float32(0.03125)
    want = np.clip(np.rint(x[0].astype(np.float64) * 32) + 128, 0, 255)
    assert q[0].tolist() == want.astype(int).tolist()


@pytest.mark.parametrize("G", [0, 32])
def test_int_gemm_asym_equals_float64_matmul(oracle, G):
    """acc = (Q - zx) @ d^T exactly: float64 BLAS on independently rebuilt integer operands."""
    rng = np.random.default_rng(79)
    M, N, K = 9, 24, 128
    X = (rng.standard_normal((M, K)) * 2 + 1).astype(np.float32)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    r = oracle.linear_w4a8_asym(X, W, None, G)
    g = K if G == 0 else G
    ng = K // g
    d = half_steps(r["codes"].reshape(N, ng, g), r["zero"].reshape(N, ng, 1)).astype(np.float64)
    xa = (r["Q"].astype(np.float64) - r["zx"][:, None]).reshape(M, ng, g)
    want = np.einsum("mgk,ngk->mng", xa, d)
    assert np.array_equal(r["acc"].astype(np.float64), want)
    # the product of the dequantized operands, in float64
    Xd = (r["Q"].astype(np.float64) - r["zx"][:, None]) * r["sx"].astype(np.float64)[:, None]
    Wd = (d * (0.5 * r["step"].astype(np.float64)).reshape(N, ng, 1)).reshape(N, K)
    np.testing.assert_allclose(r["Y64"], Xd @ Wd.T, rtol=1e-12, atol=1e-12)
    # the decomposition an implementation on codes may use: sum (Q - zx) d = sum Q d - zx * wsum
    qd = np.einsum("mgk,ngk->mng", r["Q"].astype(np.float64).reshape(M, ng, g), d)
    assert np.array_equal(want, qd - r["zx"][:, None, None] * r["wsum"][None].astype(np.float64))
    # and in the offset-128 storage a signed-int8 kernel uses: (Q - 128) and (zx - 128)
    q128 = (r["Q"].astype(np.int64) - 128).reshape(M, ng, g).astype(np.float64)
    assert np.array_equal(
        want, np.einsum("mgk,ngk->mng", q128, d)
        - (r["zx"] - 128)[:, None, None] * r["wsum"][None].astype(np.float64))


def test_weight_sums_closed_form(oracle):
    rng = np.random.default_rng(80)
    N, K, G = 12, 256, 64
    codes = rng.integers(0, 16, (N, K)).astype(np.uint8)
    zero = rng.integers(0, 14, (N, K // G)).astype(np.uint8)
    packed = oracle.pack_dint4(codes)
    d = half_steps(codes.reshape(N, K // G, G), zero.reshape(N, K // G, 1))
    assert np.array_equal(oracle.weight_sums(packed, zero, G), d.sum(2))
    # finer blocks inside a group use the group's zero-point and add up to the group sums
    fine = oracle.weight_sums(packed, zero, G, 16)
    assert np.array_equal(fine, d.reshape(N, K // 16, 16).sum(2))
    assert np.array_equal(fine.reshape(N, K // G, G // 16).sum(2), d.sum(2))
    # all codes equal to the zero-point: every sum is zero
    codes0 = np.repeat(zero, G, axis=1)
    assert not oracle.weight_sums(oracle.pack_dint4(codes0), zero, G).any()
    # the two denormal codes are +1 and -1 half steps whatever the zero-point
    c14 = np.full((1, 32), 14, np.uint8); c15 = np.full((1, 32), 15, np.uint8)
    for z in (0, 7, 13):
        zz = np.array([[z]], np.uint8)
        assert oracle.weight_sums(oracle.pack_dint4(c14), zz, 0)[0, 0] == 32
        assert oracle.weight_sums(oracle.pack_dint4(c15), zz, 0)[0, 0] == -32


def test_brute_force_tiny_asym(oracle):
    """Pure-Python evaluation of the whole asymmetric path on a tiny case."""
    rng = np.random.default_rng(81)
    M, N, K = 3, 4, 8
    X = (rng.standard_normal((M, K)) + 0.5).astype(np.float32)
    W = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    r = oracle.linear_w4a8_asym(X, W, None, 0)
    for m in range(M):
        for n in range(N):
            z = int(r["zero"][n, 0])
            tot = 0
            for k in range(K):
                c = int(r["codes"][n, k])
                dd = 2 * (c - z) if c <= 13 else (1 if c == 14 else -1)
                tot += (int(r["Q"][m, k]) - int(r["zx"][m])) * dd
            assert tot == int(r["acc"][m, n, 0])
            y = float(r["sx"][m]) * (0.5 * float(r["step"][n, 0])) * tot
            assert abs(y - r["Y64"][m, n]) <= 1e-12 * max(1.0, abs(y))


def test_asym_sampled_gemm_agrees_with_full(oracle):
    rng = np.random.default_rng(82)
    M, N, K, G = 6, 16, 64, 32
    X = (rng.standard_normal((M, K)) + 1).astype(np.float32)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    r = oracle.linear_w4a8_asym(X, W, None, G)
    mi = np.array([0, 5, 3, 3]); ni = np.array([15, 0, 7, 8])
    acc = oracle.int_gemm_asym_sampled(r["Q"], r["zx"], r["packed"], r["zero"], G, mi, ni)
    assert np.array_equal(acc, r["acc"][mi, ni])
