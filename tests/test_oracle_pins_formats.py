"""Pins of the oracle's weight-format variants (3-bit dINT, plain INT4; App. A.5, Tables 10-14) and
of the error split of Sec. 4.1 (Eq. 4).  Expectations come from the pinned dINT4 quantizer, closed
forms, a float64 nearest-level search, hand-worked values and brute force -- never from the function
under test."""
import numpy as np
import pytest

import synthetic_inputs as syn


def levels64(step, z, fmt):
    p = {"dint4": 13, "int4": 15, "dint3": 5}[fmt]
    lv = [(k - z) * step for k in range(p + 1)]
    if fmt != "int4":
        lv += [0.5 * step, -0.5 * step]
    return np.array(lv, np.float64)


def test_dint4_variant_is_the_pinned_quantizer(oracle):
    X, W, s = syn.random_layer(3, 4, 512, 40)
    for G in (0, 128):
        c, st, z = oracle.formats.quantize_weight(W, s, G, "dint4")
        c0, st0, z0 = oracle.quantize_weight_dint4(W, s, G)
        np.testing.assert_array_equal(c, c0)
        np.testing.assert_array_equal(st, st0)
        np.testing.assert_array_equal(z, z0)
        Xq, sx = oracle.quantize_act_int8(X, s)
        acc0 = oracle.int_gemm(Xq, oracle.pack_dint4(c0), z0, G)
        np.testing.assert_array_equal(oracle.formats.int_gemm(Xq, c, z, G, "dint4"), acc0)


@pytest.mark.parametrize("fmt", ["dint3", "int4"])
@pytest.mark.parametrize("G", [0, 64])
def test_codes_are_nearest_levels_of_the_format(oracle, fmt, G):
    f = oracle.formats
    _, W, s = syn.random_layer(5, 1, 256, 24)
    W = W.astype(np.float32)
    W[0, :64] = np.abs(W[0, :64])        # an all-positive group: zero-point 0
    W[1, :64] = 0                        # a degenerate group
    codes, step, zero = f.quantize_weight(W, s, G, fmt)
    p = f.FORMATS[fmt][0]
    g = 256 if G == 0 else G
    assert zero.max() <= p and (step[1, 0] == 1.0 if G else True)
    used = set(np.unique(codes).tolist())
    assert used <= (set(range(p + 1)) | ({14, 15} if fmt != "int4" else set()))
    wp = (W * s[None, :]).astype(np.float32).astype(np.float64)
    dq = f.dequant(codes, step, zero, G, fmt)
    for n in range(W.shape[0]):
        for k in range(256 // g):
            st, z = float(step[n, k]), int(zero[n, k])
            lv = levels64(st, z, fmt)
            x = wp[n, k * g:(k + 1) * g]
            best = np.abs(x[:, None] - lv[None, :]).min(axis=1)
            err = np.abs(x - dq[n, k * g:(k + 1) * g])
            assert np.all(err <= best + 1e-5 * st)          # nearest level (up to exact ties)
            assert np.all(err <= 0.5 * st * (1 + 1e-5))
            if fmt == "int4":                                # textbook: clamp(round(w/step) + z, 0, 15)
                away = np.abs(x / st - np.rint(x / st)) < 0.49
                want = np.clip(np.rint(x / st) + z, 0, 15)
                np.testing.assert_array_equal(codes[n, k * g:(k + 1) * g][away], want[away])
            else:                                            # no value beyond step/4 underflows to zero
                assert np.all(dq[n, k * g:(k + 1) * g][np.abs(x) > 0.2500001 * st] != 0)


def test_hand_worked_dint3_and_int4_rows(oracle):
    f = oracle.formats
    # range [-2, 3]: dint3 step 1, z = 2; values at the band edges and beyond
    w = np.array([[-2.0, 3.0, 0.25, 0.26, 0.75, 0.76, -0.25, -0.26, -0.75, -0.76, 1.5, 2.5, 0.0, 1.0, -1.0, 2.0]],
                 np.float32)
    c, st, z = f.quantize_weight(w, None, 0, "dint3")
    assert st[0, 0] == 1.0 and z[0, 0] == 2
    assert c[0].tolist() == [0, 5, 2, 14, 14, 3, 2, 15, 15, 1, 4, 4, 2, 3, 1, 4]   # 1.5, 2.5 tie to even
    np.testing.assert_array_equal(f.half_steps(c, z, 0, "dint3")[0],
                                  [-4, 6, 0, 1, 1, 2, 0, -1, -1, -2, 4, 4, 0, 2, -2, 4])
    # int4 on [-5, 10]: step 1, z = 5, no special band: 0.26 and 0.5 go to zero / tie to even
    w4 = np.array([[-5.0, 10.0, 0.26, 0.5, 1.5, -0.75, 9.0, 9.6] + [0.0] * 8], np.float32)
    c4, st4, z4 = f.quantize_weight(w4, None, 0, "int4")
    assert st4[0, 0] == 1.0 and z4[0, 0] == 5
    assert c4[0, :8].tolist() == [0, 15, 5, 5, 7, 4, 14, 15]
    # codes 14 and 15 are ordinary levels for int4 (9 and 10 steps above -5), special for the dINTs
    np.testing.assert_array_equal(f.half_steps(c4, z4, 0, "int4")[0, :8], [-10, 20, 0, 0, 4, -2, 18, 20])


def test_int_gemm_and_output_against_brute_force(oracle):
    f = oracle.formats
    rng = np.random.default_rng(2)
    for fmt in ("dint3", "int4"):
        W = rng.standard_normal((6, 16)).astype(np.float32)
        Xq = rng.integers(-127, 128, (3, 16)).astype(np.int8)
        sx = rng.uniform(0.1, 1, 3).astype(np.float32)
        c, st, z = f.quantize_weight(W, None, 8, fmt)
        acc = f.int_gemm(Xq, c, z, 8, fmt)
        p, special = f.FORMATS[fmt]
        for m in range(3):
            for n in range(6):
                for g in range(2):
                    tot = 0
                    for k in range(8 * g, 8 * g + 8):
                        code = int(c[n, k])
                        d = (1 if code == 14 else -1) if (special and code >= 14) else 2 * (code - int(z[n, g]))
                        tot += int(Xq[m, k]) * d
                    assert acc[m, n, g] == tot
        y = f.layer_output64(Xq, sx, c, st, z, 8, fmt)
        want = (Xq.astype(np.float64) * sx[:, None]) @ f.dequant(c, st, z, 8, fmt).T
        np.testing.assert_allclose(y, want, rtol=1e-12, atol=1e-12)


def test_pack3_layout_and_round_trip(oracle):
    f = oracle.formats
    codes = np.array([[1, 2, 3, 4, 5, 6, 7, 0]], np.uint8)
    # 24-bit word: sum code_i << 3i = 1 + 2*8 + 3*64 + 4*512 + 5*4096 + 6*32768 + 7*262144
    word = sum(int(c) << (3 * i) for i, c in enumerate(codes[0]))
    assert f.pack3(codes)[0].tolist() == [word & 255, (word >> 8) & 255, word >> 16]
    rng = np.random.default_rng(0)
    big = rng.integers(0, 8, (5, 64)).astype(np.uint8)
    np.testing.assert_array_equal(f.unpack3(f.pack3(big)), big)
    assert f.pack3(big).shape == (5, 24)
    with pytest.raises(ValueError):
        f.pack3(np.full((1, 8), 9, np.uint8))


@pytest.mark.parametrize("fmt", ["dint4", "int4", "dint3"])
def test_error_split_of_eq4(oracle, fmt):
    f = oracle.formats
    X, W, s = syn.random_layer(7, 12, 256, 32)
    du, dr = f.error_split(W, s, 0, fmt)
    assert not np.any((du != 0) & (dr != 0))                     # disjoint supports
    codes, step, zero = f.quantize_weight(W, s, 0, fmt)
    wp = (W.astype(np.float32) * s[None, :]).astype(np.float64)
    total = f.dequant(codes, step, zero, 0, fmt) - wp
    np.testing.assert_allclose(du + dr, total, rtol=0, atol=0)
    # underflow entries are exactly the non-zero weights that quantize to zero: error = -w'
    under = du != 0
    np.testing.assert_array_equal(du[under], -wp[under])
    tu, tr, tc = f.output_error_terms(X, W, s, 0, fmt)
    Xs = X.astype(np.float64) * (np.float32(1) / s).astype(np.float64)[None, :]
    want = np.sum((Xs @ total.T) ** 2)
    assert abs((tu + tr + tc) - want) <= 1e-9 * want
    assert tu >= 0 and tr >= 0


def test_dint4_trades_underflow_for_rounding_against_int4(oracle):
    """Sec. 4.1 / Fig. 4(d) on synthetic N(0, 0.02) weights: dINT4's zero band is step/4 wide instead of
    INT4's step/2 (in wider steps), so far fewer weights underflow and the underflow term of the output
    error shrinks by a large factor; the rounding term grows a little (steps 15/13 wider)."""
    f = oracle.formats
    X, W, s = syn.random_layer(9, 32, 1024, 64)
    u4, r4, _ = f.output_error_terms(X, W, s, 0, "int4")
    ud, rd, _ = f.output_error_terms(X, W, s, 0, "dint4")
    assert ud < 0.35 * u4
    assert r4 < rd < 1.6 * r4
    n4 = np.count_nonzero(f.error_split(W, s, 0, "int4")[0])
    nd = np.count_nonzero(f.error_split(W, s, 0, "dint4")[0])
    assert nd < 0.6 * n4


# ---- special value c = step / 2^t (App. A.5, Table 9) ---------------------------------------------

def levels64_special(step, z, t):
    return np.array([(k - z) * step for k in range(14)] + [step / 2 ** t, -step / 2 ** t], np.float64)


def test_special_shift_one_is_the_dint4_rule(oracle):
    _, W, s = syn.random_layer(11, 1, 512, 24)
    for G in (0, 128):
        c, st, z = oracle.formats.quantize_weight(W, s, G, "dint4", special_shift=1)
        c0, st0, z0 = oracle.quantize_weight_dint4(W, s, G)
        np.testing.assert_array_equal(c, c0)
        np.testing.assert_array_equal(st, st0)
        np.testing.assert_array_equal(z, z0)
    with pytest.raises(ValueError):
        oracle.formats.quantize_weight(W, s, 0, "dint4", special_shift=4)


@pytest.mark.parametrize("t", [2, 3])
@pytest.mark.parametrize("G", [0, 64])
def test_special_value_codes_are_nearest_levels(oracle, t, G):
    f = oracle.formats
    _, W, s = syn.random_layer(12 + t, 1, 256, 24)
    W = W.astype(np.float32)
    W[0, :64] = np.abs(W[0, :64])
    codes, step, zero = f.quantize_weight(W, s, G, "dint4", special_shift=t)
    c1, step1, zero1 = f.quantize_weight(W, s, G, "dint4", special_shift=1)
    np.testing.assert_array_equal(step, step1)          # the range rule does not depend on c
    np.testing.assert_array_equal(zero, zero1)
    g = 256 if G == 0 else G
    wp = (W * s[None, :]).astype(np.float32).astype(np.float64)
    dq = f.dequant(codes, step, zero, G, "dint4", special_shift=t)
    units = f.level_units(codes, zero, G, "dint4", special_shift=t)
    n_special = 0
    for n in range(W.shape[0]):
        for k in range(256 // g):
            st, z = float(step[n, k]), int(zero[n, k])
            lv = levels64_special(st, z, t)
            x = wp[n, k * g:(k + 1) * g]
            d = np.abs(x[:, None] - lv[None, :])
            best = d.min(axis=1)
            got = dq[n, k * g:(k + 1) * g]
            assert np.all(np.abs(x - got) <= best + 1e-5 * st)            # nearest level (up to exact ties)
            srt = np.sort(d, axis=1)
            clear = srt[:, 1] - srt[:, 0] > 1e-4 * st                     # away from ties: the level itself
            np.testing.assert_allclose(got[clear], lv[np.argmin(d, axis=1)][clear], rtol=0, atol=1e-9 * st)
            # nothing larger than c/2 underflows to zero any more
            assert np.all(got[np.abs(x) > st * 2.0 ** -(t + 1) * 1.00001] != 0)
            u = units[n, k * g:(k + 1) * g]
            np.testing.assert_allclose(u * (st / 2 ** t), got, rtol=0, atol=0)
            n_special += int(np.sum(np.abs(u) == 1))
    assert n_special > 20                                                  # the bands are exercised


def test_hand_worked_special_value_rows(oracle):
    f = oracle.formats
    # range [-2, 11]: step 1, z = 2.  t = 2: c = 1/4, bands (1/8, 5/8];  t = 3: c = 1/8, bands (1/16, 9/16]
    w2 = np.array([[-2.0, 11.0, 0.125, 0.13, 0.625, 0.63, -0.125, -0.13, -0.625, -0.63, 0.5, 0.3, 1.4, -1.5, 0.0, 3.0]],
                  np.float32)
    c, st, z = f.quantize_weight(w2, None, 0, "dint4", special_shift=2)
    assert st[0, 0] == 1.0 and z[0, 0] == 2
    assert c[0].tolist() == [0, 13, 2, 14, 14, 3, 2, 15, 15, 1, 14, 14, 3, 0, 2, 5]    # -1.5 ties to even: -2
    np.testing.assert_array_equal(f.level_units(c, z, 0, "dint4", 2)[0],
                                  [-8, 44, 0, 1, 1, 4, 0, -1, -1, -4, 1, 1, 4, -8, 0, 12])
    np.testing.assert_array_equal(f.dequant(c, st, z, 0, "dint4", 2)[0],
                                  [-2, 11, 0, .25, .25, 1, 0, -.25, -.25, -1, .25, .25, 1, -2, 0, 3])
    w3 = np.array([[-2.0, 11.0, 0.0625, 0.07, 0.5625, 0.57, -0.0625, -0.07, -0.5625, -0.57, 0.5, 0.3, 0.05, 1.0, -1.0, 2.0]],
                  np.float32)
    c, st, z = f.quantize_weight(w3, None, 0, "dint4", special_shift=3)
    assert c[0].tolist() == [0, 13, 2, 14, 14, 3, 2, 15, 15, 1, 14, 14, 2, 3, 1, 4]
    np.testing.assert_array_equal(f.level_units(c, z, 0, "dint4", 3)[0],
                                  [-16, 88, 0, 1, 1, 8, 0, -1, -1, -8, 1, 1, 0, 8, -8, 16])


@pytest.mark.parametrize("t", [2, 3])
def test_expand_special_is_the_same_product(oracle, t):
    """The double-width rewriting against the definition, through the pinned ordinary dINT4 GEMM."""
    f = oracle.formats
    X, W, s = syn.random_layer(20 + t, 5, 256, 12)
    Xq, sx = oracle.quantize_act_int8(X, s)
    for G in (0, 128):
        codes, step, zero = f.quantize_weight(W, s, G, "dint4", special_shift=t)
        want = f.int_gemm(Xq, codes, zero, G, "dint4", special_shift=t).astype(np.int64)
        c2, st2, z2 = f.expand_special(codes, step, zero, G, t)
        g = 256 if G == 0 else G
        ng = 256 // g
        assert c2.shape == (12, 512) and st2.shape == (12, 2 * ng) and z2.shape == (12, 2 * ng)
        np.testing.assert_array_equal(c2[:, :256], codes)
        np.testing.assert_array_equal(st2[:, :ng], step)
        np.testing.assert_array_equal(st2[:, ng:], (step * np.float32(1 - 2.0 ** (1 - t))).astype(np.float32))
        both = oracle.int_gemm(np.concatenate([Xq, Xq], axis=1), oracle.pack_dint4(c2), z2, g).astype(np.int64)
        a1, a2 = both[:, :, :ng], both[:, :, ng:]
        np.testing.assert_array_equal(2 ** (t - 1) * a1 + (2 ** (t - 1) - 1) * a2, want)
        # brute force of the definition on a few outputs
        d = f.level_units(codes, zero, G, "dint4", t)
        for (m, n, k) in [(0, 0, 0), (4, 11, ng - 1), (2, 5, 0)]:
            assert want[m, n, k] == sum(int(Xq[m, j]) * int(d[n, j]) for j in range(k * g, (k + 1) * g))
        # and the float outputs: the ordinary epilogue on the expanded operands is the variant's output
        y = f.layer_output64(Xq, sx, codes, step, zero, G, "dint4", t)
        y2 = f.layer_output64(np.concatenate([Xq, Xq], axis=1), sx, c2, st2, z2, g, "dint4", 1)
        np.testing.assert_allclose(y2, y, rtol=1e-6, atol=1e-6 * np.abs(y).max())


@pytest.mark.parametrize("t", [2, 3])
def test_error_split_with_special_values(oracle, t):
    f = oracle.formats
    X, W, s = syn.random_layer(31, 9, 256, 20)
    du, dr = f.error_split(W, s, 64, "dint4", special_shift=t)
    codes, step, zero = f.quantize_weight(W, s, 64, "dint4", special_shift=t)
    wq = f.dequant(codes, step, zero, 64, "dint4", t)
    wp = (W.astype(np.float32) * s[None, :]).astype(np.float32).astype(np.float64)
    np.testing.assert_array_equal(du + dr, wq - wp)
    assert not np.any((du != 0) & (dr != 0))
    assert np.all(np.abs(wp[du != 0]) <= np.repeat(step, 64, axis=1)[du != 0] * 2.0 ** -(t + 1) * 1.00001)
    tu, tr, tc = f.output_error_terms(X, W, s, 64, "dint4", special_shift=t)
    xs = X.astype(np.float64) * (np.float32(1) / s.astype(np.float32)).astype(np.float64)[None, :]
    total = np.sum((xs @ (wq - wp).T) ** 2)
    np.testing.assert_allclose(tu + tr + tc, total, rtol=1e-10)
