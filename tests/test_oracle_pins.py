"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU needed).

Every expectation here is computed WITHOUT the oracle: closed forms from Sec. 4.2 / Eq. 5,
hand-worked fixtures under tests/golden/, brute-force search in float64, numpy's float64
matmul, or pure-Python enumeration.  A dropped term, a wrong sign or index, a transposed
operand or a wrong tie direction in the oracle fails at least one test.
"""
import itertools

import numpy as np
import pytest

from conftest import read_golden_table

P = 13  # uniform steps of dINT4: 2^4 - 3 (Sec. 4.2)


def levels64(step, z):
    """The 16 representable values indexed by code (Sec. 4.2 / Eq. 5 second half), float64."""
    step = float(step)
    return np.array([(c - z) * step for c in range(P + 1)] + [step / 2, -step / 2], np.float64)


def half_step_table(z):
    """Integer value of each code in units of step/2 (integer codes are even, specials +-1)."""
    return np.array([2 * (c - z) for c in range(P + 1)] + [1, -1], np.int64)


# ------------------------------------------------------------------ golden, hand-worked
def test_golden_eq5_worked_example(oracle):
    rows = np.array(read_golden_table("dint4_eq5_worked_example.txt"))
    w = rows[:, 0].astype(np.float32)[None, :]
    codes, step, zero = oracle.quantize_weight_dint4(w)
    assert step[0, 0] == np.float32(0.5) and zero[0, 0] == 5
    assert codes[0].tolist() == rows[:, 2].astype(int).tolist()
    dq = oracle.dequant_dint4(codes, step, zero)
    assert dq[0].tolist() == rows[:, 3].tolist()


def test_golden_act_worked_example(oracle):
    rows = np.array(read_golden_table("act_int8_worked_example.txt"))
    x = rows[:, 0].astype(np.float32)[None, :]
    s = np.full((x.shape[1],), 2.0, np.float32)
    xq, sx = oracle.quantize_act_int8(x, s)
    assert sx[0] == np.float32(1.0)
    assert xq[0].tolist() == rows[:, 2].astype(int).tolist()


# ------------------------------------------------------------------ P1 level set
def test_level_set_closed_form(oracle):
    rng = np.random.default_rng(1)
    all16 = np.arange(16, dtype=np.uint8)[None, :]
    for z in range(P + 1):
        for step in [1.0, 0.5, 0.0131, float(rng.uniform(1e-3, 3.0))]:
            st = np.array([[step]], np.float32)
            dq = oracle.dequant_dint4(all16, st, np.array([[z]], np.uint8))[0].astype(np.float64)
            want = levels64(np.float32(step), z)
            np.testing.assert_allclose(dq, want, rtol=3e-7, atol=0)
            assert len(set(dq.tolist())) == 16  # 14 integer levels + 2 denormals, all distinct
            assert [oracle.decode_dint4(c, z) for c in range(16)] == half_step_table(z).tolist()


# ------------------------------------------------------------------ P2 nearest level
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_quantizer_picks_nearest_level(oracle, seed):
    rng = np.random.default_rng(100 + seed)
    N, K = 64, 512
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    W[:, :8] *= rng.uniform(0.0, 0.2, size=(N, 8)).astype(np.float32)  # crowd the band near 0
    codes, step, zero = oracle.quantize_weight_dint4(W)
    for n in range(N):
        lv = levels64(step[n, 0], int(zero[n, 0]))
        w = W[n].astype(np.float64)
        dist = np.abs(w[:, None] - lv[None, :])
        best = dist.min(axis=1)
        got = dist[np.arange(K), codes[n]]
        st = float(step[n, 0])
        # the chosen level is a nearest one, up to fp32 rounding of u at a midpoint
        assert np.all(got <= best + 1e-5 * st)
        # error bounds that follow from the thresholds being midpoints of {0, s/2, s}
        inner = np.abs(w) <= st
        assert np.all(got[inner] <= st / 4 * (1 + 1e-5))
        assert np.all(got <= st / 2 * (1 + 1e-5))


# ------------------------------------------------------------------ P3 ties, P4 underflow band
def test_tie_directions_exact(oracle):
    step = np.float32(0.25)  # power of two: u = w / step is exact
    z = 6
    us = np.array([0.25, -0.25, 0.75, -0.75, 0.5, -0.5, 1.5, -1.5, 2.5, -2.5, 0.0,
                   np.nextafter(np.float32(0.25), np.float32(1)),
                   np.nextafter(np.float32(-0.25), np.float32(-1)),
                   np.nextafter(np.float32(0.75), np.float32(1)),
                   np.nextafter(np.float32(-0.75), np.float32(-1))], np.float32)
    want_halfsteps = [0, 0, 1, -1, 1, -1, 4, -4, 4, -4, 0, 1, -1, 2, -2]
    W = (us * step)[None, :].astype(np.float32)
    st = np.array([[step]], np.float32)
    zz = np.array([[z]], np.uint8)
    codes, _, _ = oracle.quantize_weight_dint4(W, step=st, zero=zz)
    tab = half_step_table(z)
    assert [int(tab[c]) for c in codes[0]] == want_halfsteps


def test_underflow_band(oracle):
    rng = np.random.default_rng(5)
    step = np.float32(0.037)
    for z in (0, 4, 13):
        u = rng.uniform(-3, 3, size=4000)
        w = (u * float(step)).astype(np.float32)[None, :]
        codes, _, _ = oracle.quantize_weight_dint4(w, step=np.array([[step]], np.float32),
                                                   zero=np.array([[z]], np.uint8))
        ur = w[0].astype(np.float64) / float(step)
        is_zero = codes[0] == z
        clear = np.abs(np.abs(ur) - 0.25) > 1e-5
        assert np.all(is_zero[clear & (np.abs(ur) < 0.25)])
        # inside the representable range [-z, 13 - z] steps nothing beyond the band underflows
        # (outside it the clamp to code 0 / 13 lands on z only when z itself is 0 / 13)
        in_range = (ur >= -z) & (ur <= P - z)
        assert not np.any(is_zero[clear & (np.abs(ur) > 0.25) & in_range])


# ------------------------------------------------------------------ P5 idempotence
def test_quantize_dequantize_idempotent(oracle):
    rng = np.random.default_rng(7)
    all16 = np.arange(16, dtype=np.uint8)[None, :]
    for z in range(P + 1):
        for _ in range(25):
            st = np.array([[rng.uniform(1e-4, 10.0)]], np.float32)
            zz = np.array([[z]], np.uint8)
            dq = oracle.dequant_dint4(all16, st, zz)
            codes2, _, _ = oracle.quantize_weight_dint4(dq, step=st, zero=zz)
            assert codes2[0].tolist() == list(range(16))
            dq2 = oracle.dequant_dint4(codes2, st, zz)
            assert np.array_equal(dq, dq2)
    W = (rng.standard_normal((32, 256)) * 0.02).astype(np.float32)
    codes, step, zero = oracle.quantize_weight_dint4(W, group_size=128)
    dq = oracle.dequant_dint4(codes, step, zero, 128)
    codes2, _, _ = oracle.quantize_weight_dint4(dq, group_size=128, step=step, zero=zero)
    assert np.array_equal(codes, codes2)


# ------------------------------------------------------------------ P6 range mapping
def test_range_mapping(oracle):
    rng = np.random.default_rng(11)
    W = (rng.standard_normal((200, 128)) * 0.02).astype(np.float32)
    W[:50] += 0.03   # mostly positive rows -> small z
    W[50:100] -= 0.03
    W[100:110] = np.abs(W[100:110])  # all-positive rows: range extended down to 0, z = 0
    W[110:120] = -np.abs(W[110:120])
    W[:, 7] = 0.0
    codes, step, zero = oracle.quantize_weight_dint4(W)
    w64 = W.astype(np.float64)
    lo = np.minimum(w64.min(axis=1), 0.0)
    hi = np.maximum(w64.max(axis=1), 0.0)
    np.testing.assert_allclose(step[:, 0], (hi - lo) / P, rtol=3e-7)
    assert zero.min() >= 0 and zero.max() <= P
    zr = -lo / ((hi - lo) / P)
    assert np.all(np.abs(zero[:, 0] - zr) <= 0.5 + 1e-4)
    assert np.all(zero[100:110, 0] == 0) and np.all(zero[110:120, 0] == P)
    assert np.array_equal(codes[:, 7], zero[:, 0])  # real zero is exactly the level "z"
    amax = w64.argmax(axis=1)
    amin = w64.argmin(axis=1)
    rows = np.arange(W.shape[0])
    pos = hi > 0.75 * step[:, 0]
    assert np.all(codes[rows, amax][pos] == P)
    neg = -lo > 0.76 * step[:, 0].astype(np.float64)
    assert np.all(codes[rows, amin][neg] == 0)
    # a group whose minimum lies in the denormal band: it maps to c2, not to code 0
    w = np.zeros((1, 128), np.float32)
    w[0, 0] = 1.3
    w[0, 1] = -0.05          # step = 1.35/13 ~ 0.1038, u ~ -0.48
    c, st, zz = oracle.quantize_weight_dint4(w)
    assert zz[0, 0] == 0 and c[0, 1] == 15 and c[0, 0] == P


def test_degenerate_group(oracle):
    w = np.zeros((3, 256), np.float32)
    codes, step, zero = oracle.quantize_weight_dint4(w, group_size=128)
    assert np.all(codes == 0) and np.all(step == 1.0) and np.all(zero == 0)


# ------------------------------------------------------------------ P7 textbook special case
def test_reduces_to_uniform_asymmetric_outside_band(oracle):
    """Without values in (step/4, 3step/4], dINT4 is the standard 14-level asymmetric quantizer."""
    rng = np.random.default_rng(13)
    N, K = 48, 256
    step = 0.125  # power of two so the band test below is exact
    z_true = rng.integers(0, P + 1, size=N)
    W = np.empty((N, K), np.float32)
    for n in range(N):
        lo, hi = -z_true[n] * step, (P - z_true[n]) * step
        u = rng.uniform(lo / step, hi / step, size=K)
        frac = np.abs(u)
        bad = (frac > 0.2) & (frac < 0.8)
        u[bad] = np.sign(u[bad]) * rng.choice([0.1, 0.9, 1.2], size=bad.sum())
        u = np.clip(u, lo / step, hi / step)
        u[0], u[1] = lo / step, hi / step
        W[n] = (u * step).astype(np.float32)
    codes, st, zero = oracle.quantize_weight_dint4(W)
    assert np.all(st[:, 0] == np.float32(step)) and np.array_equal(zero[:, 0], z_true)
    uniform = np.clip(np.rint(W.astype(np.float64) / step) + z_true[:, None], 0, P)
    assert np.array_equal(codes, uniform.astype(np.uint8))


# ------------------------------------------------------------------ P8 activations
def test_activation_properties(oracle):
    rng = np.random.default_rng(17)
    M, K = 37, 300
    X = rng.standard_normal((M, K)).astype(np.float32)
    X[:, [3, 77]] *= 40.0
    X[5] = 0.0
    s = rng.uniform(0.5, 2.0, size=K).astype(np.float32)
    Xq, sx = oracle.quantize_act_int8(X, s)
    assert Xq.dtype == np.int8 and Xq.min() >= -127 and Xq.max() <= 127
    t = X.astype(np.float64) / s.astype(np.float64)
    amax = np.abs(t).max(axis=1)
    nz = amax > 0
    assert np.all(np.abs(Xq[nz]).max(axis=1) == 127)
    np.testing.assert_allclose(sx[nz], amax[nz] / 127.0, rtol=4e-7)
    assert sx[5] == 1.0 and not Xq[5].any()
    err = np.abs(t - Xq.astype(np.float64) * sx[:, None].astype(np.float64))
    assert np.all(err <= 0.5 * sx[:, None] * (1 + 1e-4) + 1e-12)
    # the argmax element carries the sign of the extreme value
    j = np.abs(t).argmax(axis=1)
    assert np.array_equal(np.sign(Xq[np.arange(M), j])[nz], np.sign(t[np.arange(M), j])[nz])
    # scaling a row by a power of two changes only its scale
    X2 = X.copy()
    X2[2] *= 8.0
    Xq2, sx2 = oracle.quantize_act_int8(X2, s)
    assert np.array_equal(Xq2, Xq) and sx2[2] == sx[2] * 8 and np.array_equal(sx2[3:], sx[3:])
    # s = None means s = 1
    Xq3, sx3 = oracle.quantize_act_int8(X, None)
    Xq4, sx4 = oracle.quantize_act_int8(X, np.ones(K, np.float32))
    assert np.array_equal(Xq3, Xq4) and np.array_equal(sx3, sx4)
    # fp16 input is widened exactly
    Xh = X.astype(np.float16)
    a, b = oracle.quantize_act_int8(Xh, s)
    c, d = oracle.quantize_act_int8(Xh.astype(np.float32), s)
    assert np.array_equal(a, c) and np.array_equal(b, d)


def test_activation_rounding_is_two_binary32_steps_then_ties_to_even(oracle):
    """The precision of the decision (a reading of the token-wise 8-bit quantizer, App. A.1): the code is
    rne(fl32(t * fl32(127 / a))).  With x = a / 2 the exact product is 63.5 - eps whenever fl32(127 / a)
    was rounded down and its rounded value is the tie 63.5 itself, which goes to the even code 64; a
    version that rounds the exact product (one fused step) would give 63.  Checked against exact
    rational arithmetic on the float64 product (35 significant bits: exact)."""
    a = np.arange(0x3c00, 0x7800, dtype=np.uint16).view(np.float16).astype(np.float32)
    inv = np.float32(127.0) / a
    half = (a * np.float32(0.5)).astype(np.float32)
    exact = half.astype(np.float64) * inv.astype(np.float64)
    below = a[((half * inv).astype(np.float32) == np.float32(63.5)) & (exact < 63.5)]
    above = a[((half * inv).astype(np.float32) == np.float32(63.5)) & (exact > 63.5)]
    assert below.size > 1000 and above.size > 1000
    for arr, fused in ((below[:200], 63), (above[:200], 64)):
        X = np.stack([arr, 0.5 * arr, -0.5 * arr], axis=1).astype(np.float32)
        Xq, sx = oracle.quantize_act_int8(X, None)
        assert np.array_equal(Xq[:, 0], np.full(arr.size, 127, np.int8))
        assert np.all(Xq[:, 1] == 64) and np.all(Xq[:, 2] == -64)          # ties to even, both signs
        assert np.all(np.rint(0.5 * arr.astype(np.float64) * (np.float32(127.0) / arr).astype(np.float64)) == fused)
    # a tie that goes DOWN to even: x = a * 125 / 254 would be 62.5 -> 62; use exact small integers instead
    X = np.array([[127.0, 62.5, 61.5, -62.5, 0.5, 1.5, 2.5]], np.float32)   # a = 127: inv = 1 exactly
    Xq, _ = oracle.quantize_act_int8(X, None)
    assert Xq[0].tolist() == [127, 62, 62, -62, 0, 2, 2]


def test_vanishing_token_counts_as_all_zero(oracle):
    """A reading for a case the paper does not treat: when 127 / max|t| is not a finite binary32 number
    (max|t| = 0, or below 127 / FLT_MAX ~ 3.7e-37) the products t * inv would be inf or nan; such a token
    is quantized like the all-zero token (scale 1, codes 0).  Just above the threshold the ordinary rule
    applies; subnormal scales a / 127 are kept."""
    thr = np.float32(127.0) / np.finfo(np.float32).max            # 3.73e-37
    K = 64
    X = np.zeros((6, K), np.float32)
    X[0, :3] = [1e-38, -3e-39, 2e-40]                             # max below the threshold
    X[1, :3] = [np.float32(thr) * np.float32(0.999), 1e-40, 0]    # just below
    X[2, :3] = [np.float32(thr) * np.float32(1.01), -np.float32(thr) * np.float32(0.505), 1e-39]   # just above
    X[3, :3] = [1e-30, -5e-31, 2.6e-31]                           # small but ordinary: sx = 7.9e-33
    X[4, :2] = [1e-45, -1e-45]                                    # the smallest subnormals
    Xq, sx = oracle.quantize_act_int8(X, None)
    for m in (0, 1, 4, 5):
        assert sx[m] == 1.0 and not Xq[m].any()
    assert sx[2] == np.float32(X[2, 0]) / np.float32(127.0) and Xq[2, :3].tolist() == [127, -64, 0]
    assert sx[3] == np.float32(1e-30) / np.float32(127.0) and Xq[3, :3].tolist() == [127, -64, 33]
    # the asymmetric form: the same rule on 255 / (hi - lo)
    Q, sa, zx = oracle.quantize_act_uint8_asym(X, None)
    for m in (0, 1, 4, 5):
        assert sa[m] == 1.0 and zx[m] == 0 and not Q[m].any()
    assert sa[3] == (np.float32(1e-30) + np.float32(5e-31)) / np.float32(255.0) and 0 < zx[3] < 255


# ------------------------------------------------------------------ P9 GEMM identities
@pytest.mark.parametrize("G", [0, 128])
def test_int_gemm_equals_float64_matmul(oracle, G):
    rng = np.random.default_rng(19)
    M, K, N = 23, 384, 40
    X = rng.standard_normal((M, K)).astype(np.float32)
    X[:, 11] *= 50
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    s = rng.uniform(0.5, 2.0, size=K).astype(np.float32)
    r = oracle.linear_w4a8(X, W, s, G)
    ng = r["step"].shape[1]
    Gs = K // ng
    # integer operands rebuilt here from the codes with the closed-form table
    d = np.empty((N, K), np.int64)
    for n in range(N):
        for g in range(ng):
            tab = half_step_table(int(r["zero"][n, g]))
            d[n, g * Gs:(g + 1) * Gs] = tab[r["codes"][n, g * Gs:(g + 1) * Gs]]
    xq = r["Xq"].astype(np.float64)
    for g in range(ng):
        ref = xq[:, g * Gs:(g + 1) * Gs] @ d[:, g * Gs:(g + 1) * Gs].astype(np.float64).T
        assert np.array_equal(r["acc"][:, :, g].astype(np.float64), ref)  # exact: integers < 2^53
    # float matmul of the dequantized operands (Eq. 1 product)
    wdq = np.empty((N, K), np.float64)
    for n in range(N):
        for g in range(ng):
            lv = levels64(r["step"][n, g], int(r["zero"][n, g]))
            wdq[n, g * Gs:(g + 1) * Gs] = lv[r["codes"][n, g * Gs:(g + 1) * Gs]]
    xdq = xq * r["sx"].astype(np.float64)[:, None]
    yref = xdq @ wdq.T
    np.testing.assert_allclose(r["Y64"], yref, rtol=1e-11, atol=1e-12 * np.abs(yref).max())
    np.testing.assert_allclose(r["Y32"], yref, rtol=2e-5, atol=2e-5 * np.abs(yref).max())
    # and the quantized layer approximates the unquantized one (4-bit round-to-nearest noise, statistical)
    ytrue = X.astype(np.float64) @ W.astype(np.float64).T
    rel = np.linalg.norm(r["Y64"] - ytrue) / np.linalg.norm(ytrue)
    assert rel < 0.35


def test_sampled_gemm_matches_full(oracle):
    rng = np.random.default_rng(23)
    M, K, N = 9, 256, 12
    Xq = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    codes = rng.integers(0, 16, size=(N, K)).astype(np.uint8)
    zero = rng.integers(0, P + 1, size=(N, 2)).astype(np.uint8)
    packed = oracle.pack_dint4(codes)
    full = oracle.int_gemm(Xq, packed, zero, 128)
    mi = rng.integers(0, M, size=30)
    ni = rng.integers(0, N, size=30)
    samp = oracle.int_gemm_sampled(Xq, packed, zero, 128, mi, ni)
    assert np.array_equal(samp, full[mi, ni])


# ------------------------------------------------------------------ P10 brute force
def test_bruteforce_tiny_shapes(oracle):
    rng = np.random.default_rng(29)
    for M, N, K, G in [(1, 1, 2, 0), (3, 2, 4, 2), (8, 8, 8, 4), (5, 7, 6, 0), (2, 3, 8, 2)]:
        Xq = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
        codes = rng.integers(0, 16, size=(N, K)).astype(np.uint8)
        Gs = K if G == 0 else G
        ng = K // Gs
        zero = rng.integers(0, P + 1, size=(N, ng)).astype(np.uint8)
        step = rng.uniform(0.01, 1.0, size=(N, ng)).astype(np.float32)
        sx = rng.uniform(0.01, 1.0, size=M).astype(np.float32)
        acc = oracle.int_gemm(Xq, oracle.pack_dint4(codes), zero, G)
        y32, y64 = oracle.dequant_epilogue(acc, sx, step)
        for m, n in itertools.product(range(M), range(N)):
            ytot = 0.0
            for g in range(ng):
                tot = 0
                for k in range(g * Gs, (g + 1) * Gs):
                    c, z = int(codes[n, k]), int(zero[n, g])
                    hs = 1 if c == 14 else (-1 if c == 15 else 2 * (c - z))
                    tot += int(Xq[m, k]) * hs
                assert acc[m, n, g] == tot
                ytot += tot * float(step[n, g]) / 2.0
            assert y64[m, n] == pytest.approx(float(sx[m]) * ytot, rel=1e-13, abs=1e-300)
            assert y32[m, n] == pytest.approx(float(sx[m]) * ytot, rel=1e-5, abs=1e-9)


def test_product_table_exhaustive(oracle):
    """All 16 codes x 14 zero-points x 255 activation values through the GEMM (K = 2)."""
    xs = np.arange(-127, 128, dtype=np.int8)
    Xq = np.stack([xs, np.zeros_like(xs)], axis=1)
    for z in range(P + 1):
        codes = np.stack([np.arange(16, dtype=np.uint8), np.full(16, z, np.uint8)], axis=1)
        zero = np.full((16, 1), z, np.uint8)
        acc = oracle.int_gemm(Xq, oracle.pack_dint4(codes), zero, 0)[:, :, 0]
        want = xs.astype(np.int64)[:, None] * half_step_table(z)[None, :]
        assert np.array_equal(acc, want)


def test_pack_layout_and_roundtrip(oracle):
    pairs = np.array([(lo, hi) for hi in range(16) for lo in range(16)], np.uint8)
    codes = pairs.reshape(1, -1)
    packed = oracle.pack_dint4(codes)
    assert packed[0].tolist() == list(range(256))  # byte = low | high << 4, even k in the low nibble
    assert np.array_equal(oracle.unpack_dint4(packed), codes)
    rng = np.random.default_rng(31)
    c = rng.integers(0, 16, size=(5, 64)).astype(np.uint8)
    assert np.array_equal(oracle.pack_dint4(c), c[:, 0::2] | (c[:, 1::2] << 4))
    assert np.array_equal(oracle.unpack_dint4(oracle.pack_dint4(c)), c)


# ------------------------------------------------------------------ P11 AQAS invariance
@pytest.mark.parametrize("j", [-2, 1, 3])
def test_power_of_two_scale_invariance(oracle, j):
    rng = np.random.default_rng(37)
    M, K, N = 6, 256, 10
    X = rng.standard_normal((M, K)).astype(np.float32)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    base = oracle.linear_w4a8(X, W, np.ones(K, np.float32), 128)
    scl = oracle.linear_w4a8(X, W, np.full(K, 2.0 ** j, np.float32), 128)
    assert np.array_equal(base["Xq"], scl["Xq"]) and np.array_equal(base["codes"], scl["codes"])
    assert np.array_equal(base["zero"], scl["zero"]) and np.array_equal(base["acc"], scl["acc"])
    assert np.array_equal(scl["sx"], base["sx"] * np.float32(2.0 ** -j))
    assert np.array_equal(scl["step"], base["step"] * np.float32(2.0 ** j))
    assert np.array_equal(base["Y32"], scl["Y32"])


def test_scale_fold_direction(oracle):
    """Weights are multiplied by s and activations divided by s (Eq. 1), not the reverse."""
    K = 128
    X = np.ones((1, K), np.float32)
    W = np.full((1, K), 0.01, np.float32)
    s = np.ones(K, np.float32)
    s[5] = 4.0
    Xq, sx = oracle.quantize_act_int8(X, s)
    assert Xq[0, 5] == 32 and Xq[0, 4] == 127 and sx[0] == np.float32(1 / 127)
    codes, step, zero = oracle.quantize_weight_dint4(W, s)
    assert step[0, 0] == np.float32(np.float32(0.04) / np.float32(13)) and codes[0, 5] == P
    assert codes[0, 4] == 3 and zero[0, 0] == 0  # 0.01 / (0.04/13) = 3.25 -> 3


# ------------------------------------------------------------------ statistical sanity (Fig. 4c)
def test_dint4_underflows_less_than_int4(oracle):
    rng = np.random.default_rng(41)
    W = (rng.standard_normal((64, 1024)) * 0.02).astype(np.float32)
    codes, step, zero = oracle.quantize_weight_dint4(W)
    dint_zero = np.mean((codes == zero) & (W != 0))
    w64 = W.astype(np.float64)
    lo, hi = w64.min(axis=1, keepdims=True), w64.max(axis=1, keepdims=True)
    st15 = (hi - lo) / 15.0  # plain 16-level INT4 min-max
    z15 = np.rint(-lo / st15)
    q15 = np.clip(np.rint(w64 / st15) + z15, 0, 15)
    int_zero = np.mean((q15 == z15) & (W != 0))
    assert dint_zero < 0.7 * int_zero


def test_bad_arguments_raise(oracle):
    with pytest.raises(ValueError):
        oracle.quantize_weight_dint4(np.zeros((2, 100), np.float32), group_size=64)
    with pytest.raises(ValueError):
        oracle.pack_dint4(np.zeros((2, 3), np.uint8))
