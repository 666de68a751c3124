"""Pins of the oracle's AQAS scale search (Sec. 3.2, Eq. 1; App. A.4): the scale family at its
closed-form points, the loss against a float64 evaluation from independently rebuilt operands,
exact invariances, and planted cases whose answer is known."""
import numpy as np
import pytest

import synthetic_inputs as syn

P = 13


def dequant64(codes, step, zero, G):
    N, K = codes.shape
    z = np.repeat(zero.astype(np.int64), G, axis=1)
    st = np.repeat(step.astype(np.float64), G, axis=1)
    c = codes.astype(np.int64)
    return np.where(c <= P, (c - z) * st, np.where(c == 14, 0.5 * st, -0.5 * st))


def test_sixteenth_powers(oracle):
    aq = oracle.aqas_search
    x = np.array([0.0, 1.0, 2.0 ** 16, 2.0 ** -32, 3.7, 0.02, 65504.0, 1e-3], np.float32)
    for j in range(17):
        got = aq.pow_sixteenths(x, j)
        want = np.power(x.astype(np.float64), j / 16.0)
        if j == 0:
            want = np.ones_like(want)            # x^0 = 1 also for x = 0
        assert got.dtype == np.float32
        np.testing.assert_allclose(got, want, rtol=6e-7)       # a few binary32 roundings
        # exact for perfect sixteenth powers of two
        assert got[2] == np.float32(2.0 ** j) and got[3] == np.float32(2.0 ** (-2 * j))
    np.testing.assert_array_equal(aq.pow_sixteenths(x, 16), x)
    np.testing.assert_array_equal(aq.pow_sixteenths(x, 8), np.sqrt(x))
    np.testing.assert_array_equal(aq.pow_sixteenths(x, 4), np.sqrt(np.sqrt(x)))
    np.testing.assert_array_equal(aq.pow_sixteenths(x, 12), np.sqrt(x) * np.sqrt(np.sqrt(x)))


def test_scale_family_end_points_and_direction(oracle):
    aq = oracle.aqas_search
    ax = np.array([4.0, 100.0, 0.5, 0.0, 9.0], np.float32)
    aw = np.array([0.25, 0.01, 2.0, 1.0, 0.0], np.float32)
    s0, s8, s16 = aq.aqas_scale(ax, aw, 0), aq.aqas_scale(ax, aw, 8), aq.aqas_scale(ax, aw, 16)
    # alpha = 0: weights alone are equalized (1 / max|W|); alpha = 1: activations alone (max|X|);
    # alpha = 1/2: sqrt(max|X|) / sqrt(max|W|)
    np.testing.assert_array_equal(s0[:3], np.float32(1) / aw[:3])
    np.testing.assert_array_equal(s16[:3], ax[:3])
    np.testing.assert_array_equal(s8[:3], np.sqrt(ax[:3]) / np.sqrt(aw[:3]))
    assert s8[0] == 4.0 and s8[1] == 100.0                      # sqrt(4)/sqrt(.25), sqrt(100)/sqrt(.01)
    for s in (s0, s8, s16):
        assert s[3] == 1.0 and s[4] == 1.0                      # dead channels keep s = 1
    # dividing the activations by s flattens an outlier channel, multiplying the weights keeps W s X
    big = aq.aqas_scale(np.array([1e9], np.float32), np.array([1e-9], np.float32), 16)
    assert big[0] == np.float32(1e4)                            # clamp


@pytest.mark.parametrize("G", [0, 64])
def test_losses_equal_float64_evaluation_of_rebuilt_operands(oracle, G):
    aq = oracle.aqas_search
    X, W, _ = syn.random_layer(41, 24, 128, 20, outlier_frac=0.03, outlier_gain=40.0)
    losses, scales = aq.aqas_losses(X, W, G)
    g = 128 if G == 0 else G
    Y = X.astype(np.float64) @ W.astype(np.float64).T
    ax = np.abs(X.astype(np.float32)).max(axis=0)
    np.testing.assert_array_equal(aq.channel_absmax(X), ax)
    for j in (0, 5, 8, 16):
        s = scales[j]
        r = oracle.linear_w4a8(X, W, s, G)
        Wdq = dequant64(r["codes"], r["step"], r["zero"], g)
        Xdq = r["Xq"].astype(np.float64) * r["sx"].astype(np.float64)[:, None]
        Yq = Xdq @ Wdq.T                                        # float64, before the fp16 cast
        y16 = Yq.astype(np.float32).astype(np.float16).astype(np.float64)
        want = np.sum((y16 - Y) ** 2)
        # the oracle rounds its binary32 epilogue result to fp16; Yq here is float64: a few outputs
        # may fall on the other side of an fp16 rounding boundary
        assert abs(losses[j] - want) <= 2e-3 * want
    # scaling X by 2^3 and W by 2^2 (exact in fp16 here) rescales the whole problem: the same codes,
    # every output times 2^5, every loss times 2^10 (up to fp16 subnormal outputs); s at alpha = 1
    # follows the activations (x 8), at alpha = 0 the weights (x 1/4)
    l2, s2 = aq.aqas_losses((X.astype(np.float32) * 8).astype(np.float16),
                            (W.astype(np.float32) * 4).astype(np.float16), G)
    np.testing.assert_allclose(l2[[0, 16]], losses[[0, 16]] * 2.0 ** 10, rtol=1e-6)
    np.testing.assert_array_equal(s2[16], scales[16] * np.float32(8))
    np.testing.assert_array_equal(s2[0], scales[0] * np.float32(0.25))


def test_search_picks_first_minimum_and_beats_the_end_points(oracle):
    aq = oracle.aqas_search
    # activations with strong outlier channels, narrow weights: neither pure weight equalization
    # (alpha = 0) nor pure activation smoothing (alpha = 1) is best
    X, W, _ = syn.random_layer(43, 32, 256, 48, outlier_frac=0.03, outlier_gain=60.0)
    r = aq.aqas_search(X, W, 0)
    assert r["losses"][r["j"]] == r["losses"].min()
    assert np.all(r["losses"][:r["j"]] > r["losses"][r["j"]])   # first minimum
    assert 0 < r["j"] < 16
    assert r["losses"][r["j"]] < 0.8 * min(r["losses"][0], r["losses"][16])
    np.testing.assert_array_equal(r["s"], aq.aqas_scale(r["ax"], r["aw"], r["j"]))
    # and the searched scale beats no scaling at all (s = 1)
    base = aq.layer_output(X, W, np.ones(256, np.float32), 0)["Y16"] - X.astype(np.float64) @ W.astype(np.float64).T
    assert r["losses"][r["j"]] < np.sum(base * base)


def test_clip_factors_and_parameters(oracle):
    aq = oracle.aqas_search
    assert [float(aq.clip_factor(i)) for i in (0, 1, 10)] == [1.0, float(np.float32(1) - np.float32(0.05)),
                                                              float(np.float32(1) - np.float32(0.05) * np.float32(10))]
    W = np.array([[-4.0, 9.0, 1.0, 0.5], [2.0, 6.5, 0.0, 1.0]], np.float32)
    step, zero = aq.clipped_params(W, None, 0, np.array([1.0, 0.5], np.float32))
    assert step[0, 0] == 1.0 and zero[0, 0] == 4                # range [-4, 9] / 13
    assert step[1, 0] == np.float32(3.25) / np.float32(13) and zero[1, 0] == 0   # [0, 6.5] * 0.5
    # rho = 1 reproduces the quantizer's own parameters
    _, st, z = oracle.quantize_weight_dint4(W, None, 0)
    s1, z1 = aq.clipped_params(W, None, 0, np.ones(2, np.float32))
    np.testing.assert_array_equal(s1, st)
    np.testing.assert_array_equal(z1, z)


def test_clipping_helps_exactly_where_an_unused_outlier_widens_the_range(oracle):
    aq = oracle.aqas_search
    rng = np.random.default_rng(5)
    T, K, N = 40, 128, 6
    X = rng.standard_normal((T, K)).astype(np.float16)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    X[:, 7] = 0                       # input channel 7 is never excited ...
    W[2, 7] = 0.4                     # ... so this 20-sigma weight only wastes row 2's range
    s = np.ones(K, np.float32)
    r = aq.clip_search(X, W, s, 0)
    assert r["err"].shape == (aq.CLIP_STEPS, N)
    i2 = int(r["index"][2])
    assert i2 >= 4 and r["rho"][2] == aq.clip_factor(i2)        # range cut by 20 % or more
    assert r["err"][i2, 2] < 0.6 * r["err"][0, 2]
    others = [n for n in range(N) if n != 2]
    assert np.all(r["index"][others] <= 3)                       # ordinary rows keep (nearly) their range
    # every channel ends at its own best factor, never worse than no clipping, first minimum
    for n in range(N):
        i = r["index"][n]
        assert r["err"][i, n] == r["err"][:, n].min() and np.all(r["err"][:i, n] > r["err"][i, n])
    st, z = aq.clipped_params(W, s, 0, r["rho"])
    np.testing.assert_array_equal(r["step"], st)
    np.testing.assert_array_equal(r["zero"], z)
    # the error table against a float64 evaluation from rebuilt operands (row 2, its chosen factor)
    st5, z5 = aq.clipped_params(W, s, 0, np.full(N, aq.clip_factor(i2), np.float32))
    out = aq.layer_output(X, W, s, 0, step=st5, zero=z5)
    Wdq = dequant64(out["codes"], st5, z5, K)
    Yq = (out["Xq"].astype(np.float64) * out["sx"].astype(np.float64)[:, None]) @ Wdq.T
    Y = X.astype(np.float64) @ W.astype(np.float64).T
    want = np.sum((Yq[:, 2].astype(np.float32).astype(np.float16).astype(np.float64) - Y[:, 2]) ** 2)
    assert abs(r["err"][i2, 2] - want) <= 2e-3 * want
    # clipped weights saturate at the ends of the shrunk range
    assert out["codes"][2, 7] == 13
