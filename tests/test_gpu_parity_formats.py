"""GPU parity of the weight-format variants (3-bit dINT, plain INT4; App. A.5, Tables 10-14) and of the
error split of Sec. 4.1 (Eq. 4) against the CPU oracle: codes / steps / zero-points / int32 accumulators /
3-bit packed bytes bit-identical, Y within 1e-3, the three error terms within 1e-4 relative."""
import numpy as np
import pytest
import torch

import synthetic_inputs as syn
from gpu_util import assert_y_close, dev, host

pytestmark = pytest.mark.gpu
FMT = {"dint4": 0, "int4": 1, "dint3": 2}


@pytest.fixture(scope="module")
def lib():
    import paper_2311_05161_amd as w
    w.load_library()
    assert torch.cuda.is_available()
    return w


CASES = [
    # name, M, K, N, G
    ("decode_grouped", 16, 1024, 528, 128),
    ("decode_per_channel", 5, 1152, 272, 0),
    ("decode_k_split", 3, 9216, 48, 128),
    ("prefill_per_channel", 300, 768, 1040, 0),
    ("prefill_grouped", 130, 1024, 304, 256),
    ("prefill_grouped_128_k_phases", 130, 1408, 80, 128),   # the kernel that cuts K into phases inside the workgroup
    ("prefill_64_rows", 40, 512, 256, 128),
]


@pytest.mark.parametrize("fmt", ["int4", "dint3", "dint4"])
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_format_layer_matches_oracle(lib, oracle, case, fmt):
    name, M, K, N, G = case
    f = oracle.formats
    X, W, s = syn.random_layer(sum(name.encode()) % 971, M, K, N)
    W = W.copy()
    W[1, :] = np.abs(W[1, :])                    # an all-positive row: zero-point 0
    W[2, : min(K, 256)] = -np.abs(W[2, : min(K, 256)])
    Xq_h, sx_h = oracle.quantize_act_int8(X, s)
    codes_h, step_h, zero_h = f.quantize_weight(W, s, G, fmt)
    codes, step, zero = lib.quantize_weight_format(dev(W), dev(s), G, FMT[fmt])
    np.testing.assert_array_equal(host(step), step_h)
    np.testing.assert_array_equal(host(zero), zero_h)
    np.testing.assert_array_equal(host(codes), codes_h)
    if fmt == "int4":
        assert host(zero).max() > 13 or host(codes).max() == 15      # the two extra integer levels are in use
    Xq, sx = lib.quantize_act_int8(dev(X), dev(s))
    Wp = lib.pack_format(codes, lib.LAYOUT_TILED, FMT[fmt])
    np.testing.assert_array_equal(host(lib.unpack_format(Wp, N, K, lib.LAYOUT_TILED, FMT[fmt])), codes_h)
    Y, acc = lib.w4a8_gemm_format(Xq, sx, Wp, step, zero, N, K, G, FMT[fmt], want_acc=True)
    np.testing.assert_array_equal(host(acc), f.int_gemm(Xq_h, codes_h, zero_h, G, fmt))
    assert_y_close(host(Y), f.layer_output64(Xq_h, sx_h, codes_h, step_h, zero_h, G, fmt), "f16")
    Y2 = lib.w4a8_gemm_format(Xq, sx, Wp, step, zero, N, K, G, FMT[fmt])
    assert torch.equal(Y, Y2)


def test_int4_every_code_and_zero_point(lib, oracle):
    """All 16 codes x 16 zero-points of the plain INT4 table through both GEMM kernels."""
    f = oracle.formats
    rng = np.random.default_rng(1)
    N, K = 256, 256
    codes = rng.integers(0, 16, (N, K)).astype(np.uint8)
    zero = (np.arange(N) % 16).astype(np.uint8)[:, None]
    step = rng.uniform(0.01, 0.1, (N, 1)).astype(np.float32)
    for M in (7, 48):
        Xq = rng.integers(-127, 128, (M, K)).astype(np.int8)
        sx = rng.uniform(0.01, 0.1, M).astype(np.float32)
        for G, z, st in ((0, zero, step), (128, np.repeat(zero, 2, 1), np.repeat(step, 2, 1))):
            Wp = lib.pack_format(dev(codes), lib.LAYOUT_TILED, FMT["int4"])
            Y, acc = lib.w4a8_gemm_format(dev(Xq), dev(sx), Wp, dev(st), dev(z), N, K, G, FMT["int4"], want_acc=True)
            np.testing.assert_array_equal(host(acc), f.int_gemm(Xq, codes, z, G, "int4"))
            assert_y_close(host(Y), f.layer_output64(Xq, sx, codes, st, z, G, "int4"), "f16")


def test_dint3_three_bit_storage(lib, oracle):
    f = oracle.formats
    _, W, s = syn.random_layer(17, 1, 1024, 304)
    codes, step, zero = lib.quantize_weight_format(dev(W), dev(s), 128, FMT["dint3"])
    c4 = host(codes)
    assert set(np.unique(c4).tolist()) <= {0, 1, 2, 3, 4, 5, 14, 15}
    packed = lib.pack_dint3(codes)
    c3 = np.where(c4 >= 14, c4 - 8, c4).astype(np.uint8)
    np.testing.assert_array_equal(host(packed), f.pack3(c3))            # 3 bits per weight at rest
    assert packed.numel() * 8 == c4.size * 3
    back = lib.unpack_dint3(packed, *c4.shape)
    np.testing.assert_array_equal(host(back), c4)                       # and back, ready for pack_dint4 + GEMM
    np.testing.assert_array_equal(f.unpack3(host(packed)), c3)


@pytest.mark.parametrize("fmt", ["dint4", "int4", "dint3"])
@pytest.mark.parametrize("G", [0, 128])
def test_error_split_terms(lib, oracle, fmt, G):
    f = oracle.formats
    X, W, s = syn.random_layer(23, 70, 512, 100)
    t = host(lib.dint_error_terms(dev(X), dev(W), dev(s), G, FMT[fmt]))
    tu, tr, tc = f.output_error_terms(X, W, s, G, fmt)
    np.testing.assert_allclose(t[0], tu, rtol=1e-4)
    np.testing.assert_allclose(t[1], tr, rtol=1e-4)
    assert abs(t[2] - tc) <= 1e-4 * (tu + tr)
    assert int(t[3]) == np.count_nonzero(f.error_split(W, s, G, fmt)[0])


@pytest.mark.parametrize("t", [2, 3])
def test_error_split_terms_of_the_special_values(lib, oracle, t):
    f = oracle.formats
    X, W, s = syn.random_layer(29, 70, 512, 100)
    fmt_id = {2: lib.FMT_DINT4_C4, 3: lib.FMT_DINT4_C8}[t]
    for G in (0, 128):
        got = host(lib.dint_error_terms(dev(X), dev(W), dev(s), G, fmt_id))
        tu, tr, tc = f.output_error_terms(X, W, s, G, "dint4", special_shift=t)
        np.testing.assert_allclose(got[0], tu, rtol=1e-4)
        np.testing.assert_allclose(got[1], tr, rtol=1e-4)
        assert abs(got[2] - tc) <= 1e-4 * (tu + tr)
        assert int(got[3]) == np.count_nonzero(f.error_split(W, s, G, "dint4", t)[0])
        # a smaller special value narrows the band that underflows to zero
        assert int(got[3]) < np.count_nonzero(f.error_split(W, s, G, "dint4", 1)[0])


def test_dint4_reduces_the_underflow_term_on_the_gpu(lib):
    """Sec. 4.1 / Fig. 4(d) with the library's own kernels on a synthetic LLaMA-sized layer."""
    X, W, s, G = syn.make_layer("C2", M=64)
    i4 = host(lib.dint_error_terms(dev(X), dev(W), dev(s), G, FMT["int4"]))
    d4 = host(lib.dint_error_terms(dev(X), dev(W), dev(s), G, FMT["dint4"]))
    assert d4[0] < 0.35 * i4[0] and d4[3] < 0.6 * i4[3]          # underflow term, underflowing weights
    assert 0.7 * i4[1] < d4[1] < 1.6 * i4[1]                     # rounding term: about the same
    assert d4[:3].sum() < i4[:3].sum()                           # and the output error as a whole is lower


# ---- special value c = step / 2^t (App. A.5, Table 9) ---------------------------------------------
SPECIAL_CASES = [
    # name, M, K, N, G
    ("decode_grouped", 16, 1024, 528, 128),
    ("decode_per_channel", 5, 1152, 272, 0),
    ("decode_k_split", 3, 4096, 48, 128),          # 2K = 8192: two K ranges per workgroup row
    ("prefill_per_channel", 300, 768, 1040, 0),
    ("prefill_grouped", 130, 1024, 304, 256),
]


@pytest.mark.parametrize("t", [2, 3])
@pytest.mark.parametrize("case", SPECIAL_CASES, ids=[c[0] for c in SPECIAL_CASES])
def test_special_value_layer_matches_oracle(lib, oracle, case, t):
    name, M, K, N, G = case
    f = oracle.formats
    fmt_id = {2: lib.FMT_DINT4_C4, 3: lib.FMT_DINT4_C8}[t]
    X, W, s = syn.random_layer(sum(name.encode()) % 977 + t, M, K, N)
    W = W.copy()
    W[1, :] = np.abs(W[1, :])
    Xq_h, sx_h = oracle.quantize_act_int8(X, s)
    codes_h, step_h, zero_h = f.quantize_weight(W, s, G, "dint4", special_shift=t)
    codes, step, zero = lib.quantize_weight_format(dev(W), dev(s), G, fmt_id)
    np.testing.assert_array_equal(host(step), step_h)
    np.testing.assert_array_equal(host(zero), zero_h)
    np.testing.assert_array_equal(host(codes), codes_h)
    c1_h = f.quantize_weight(W, s, G, "dint4", special_shift=1)[0]
    assert np.count_nonzero(codes_h != c1_h) > 0                      # the bands really moved
    c2_h, st2_h, z2_h = f.expand_special(codes_h, step_h, zero_h, G, t)
    c2, st2, z2 = lib.expand_special_value(codes, step, zero, G, fmt_id)
    np.testing.assert_array_equal(host(c2), c2_h)
    np.testing.assert_array_equal(host(st2).view(np.uint32), st2_h.view(np.uint32))
    np.testing.assert_array_equal(host(z2), z2_h)
    Xq, sx = lib.quantize_act_int8(dev(X), dev(s))
    Wp2 = lib.pack_dint4(c2, lib.LAYOUT_TILED)
    Y, acc = lib.w4a8_gemm_special(Xq, sx, Wp2, st2, z2, N, K, G, want_acc=True)
    acc = host(acc).astype(np.int64)
    ng = acc.shape[2] // 2
    got = 2 ** (t - 1) * acc[:, :, :ng] + (2 ** (t - 1) - 1) * acc[:, :, ng:]
    np.testing.assert_array_equal(got, f.int_gemm(Xq_h, codes_h, zero_h, G, "dint4", special_shift=t))
    assert_y_close(host(Y), f.layer_output64(Xq_h, sx_h, codes_h, step_h, zero_h, G, "dint4", t), "f16")
    Y2 = lib.w4a8_gemm_special(Xq, sx, Wp2, st2, z2, N, K, G)
    assert torch.equal(Y, Y2)


def test_special_value_band_edges_on_the_gpu(lib, oracle):
    """Weights placed on and next to the band edges of both special values (steps of exactly 1)."""
    f = oracle.formats
    row = np.array([-2.0, 11.0, 0.125, 0.13, 0.625, 0.63, -0.125, -0.13, -0.625, -0.63, 0.0625, 0.07, 0.5625,
                    0.57, -0.0625, -0.07, -0.5625, -0.57, 0.5, 0.3, 0.25, 0.75, -0.25, -0.75, 1.5, -1.5, 2.5,
                    0.0, 1.0, -1.0, 10.4, 10.6], np.float32)
    W = np.tile(row, (16, 4)).astype(np.float32)                      # [16, 128]
    for t, fmt_id in ((2, lib.FMT_DINT4_C4), (3, lib.FMT_DINT4_C8)):
        c_h, st_h, z_h = f.quantize_weight(W, None, 32, "dint4", special_shift=t)
        assert np.all(st_h == 1.0) and np.all(z_h == 2)
        c, st, z = lib.quantize_weight_format(dev(W), None, 32, fmt_id)
        np.testing.assert_array_equal(host(c), c_h)
        np.testing.assert_array_equal(host(st), st_h)
        np.testing.assert_array_equal(host(z), z_h)
