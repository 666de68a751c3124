"""GPU parity of the asymmetric-activation path (token-wise min-max 8-bit with a zero-point,
App. A.1) against the CPU oracle: codes, zero-points, token scales, weight sums and int32
accumulators bit-identical; Y within 1e-3 relative (fp16) of the oracle's float64 evaluation."""
import numpy as np
import pytest
import torch

import synthetic_inputs as syn
from gpu_util import assert_y_close, dev, host

pytestmark = pytest.mark.gpu

TORCH_DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


@pytest.fixture(scope="module")
def lib():
    import paper_2311_05161_amd as w
    w.load_library()
    assert torch.cuda.is_available()
    return w


def _shifted(X, seed):
    """Activations with a per-token offset, so that ranges are lopsided (what the zero-point is for)."""
    rng = np.random.default_rng(seed)
    X = X.astype(np.float32) + rng.uniform(-3, 3, (X.shape[0], 1)).astype(np.float32)
    if X.shape[0] > 3:
        X[1] = 0.0                      # all-zero token
        X[2] = np.abs(X[2])             # all positive: zero-point 0
        X[3] = -np.abs(X[3])            # all negative: zero-point 255
    return X


ACT_CASES = [
    ("c2_decode", 16, 4096, "f16", True, 0),
    ("one_row", 1, 4096, "f16", True, 0),
    ("ragged_rows", 37, 5120, "f16", True, 0),
    ("wide", 130, 13824, "f16", False, 0),
    ("many_rows", 2100, 1024, "f16", True, 0),
    ("bf16", 33, 2048, "bf16", True, 0),
    ("f32_tiny", 16, 768, "f32", False, 0),
    ("odd_k_generic", 19, 1001, "f16", True, 0),
    ("strided_unaligned", 5, 264, "f16", True, 3),
]


@pytest.mark.parametrize("case", ACT_CASES, ids=[c[0] for c in ACT_CASES])
def test_act_quant_asym_bit_exact(lib, oracle, case):
    name, M, K, dtype, use_s, pad = case
    X, _, s = syn.random_layer(sum(name.encode()) % 1000, M, K, 1, x_dtype="f32")
    X = _shifted(X, 3)
    if dtype == "bf16":
        t = torch.from_numpy(X).to(torch.bfloat16)
        Xh = t.float().numpy()
    else:
        Xh = X.astype(np.float16 if dtype == "f16" else np.float32)
    buf = torch.zeros((M, K + pad), dtype=TORCH_DT[dtype], device="cuda")
    buf[:, :K] = torch.from_numpy(Xh.astype(np.float32)).to(TORCH_DT[dtype]).cuda()
    Xq, sx, zx = lib.quantize_act_int8_asym(buf[:, :K], dev(s) if use_s else None)
    q_ref, sx_ref, zx_ref = oracle.quantize_act_uint8_asym(Xh.astype(np.float32),
                                                           s if use_s else None)
    assert np.array_equal(host(sx).view(np.uint32), sx_ref.view(np.uint32))
    assert np.array_equal(host(zx) + 128, zx_ref)                       # stored minus 128
    assert np.array_equal(host(Xq).astype(np.int32) + 128, q_ref.astype(np.int32))


def test_weight_sums_bit_exact(lib, oracle):
    for seed, (N, K, G) in enumerate([(48, 384, 128), (768, 768, 0), (4096, 4096, 128), (32, 1024, 256)]):
        _, W, s = syn.random_layer(40 + seed, 1, K, N)
        codes, step, zero = lib.quantize_weight_dint4(dev(W), dev(s), G)
        wsum, tsum = lib.dint4_weight_sums(codes, zero, G)
        c_ref, st_ref, z_ref = oracle.quantize_weight_dint4(W, s, G)
        assert np.array_equal(host(codes), c_ref)
        packed = oracle.pack_dint4(c_ref)
        assert np.array_equal(host(wsum), oracle.weight_sums(packed, z_ref, G))
        assert np.array_equal(host(tsum), oracle.weight_sums(packed, z_ref, G, 128))


def _gemm_asym_case(lib, oracle, seed, M, K, N, G, out_dtype="f16", layout=1):
    X, W, s = syn.random_layer(seed, M, K, N)
    X = _shifted(X, seed).astype(np.float16)
    r = oracle.linear_w4a8_asym(X, W, s, G)
    Xq, sx, zx = lib.quantize_act_int8_asym(dev(X), dev(s))
    codes, step, zero = lib.quantize_weight_dint4(dev(W), dev(s), G)
    assert np.array_equal(host(Xq).astype(np.int32) + 128, r["Q"].astype(np.int32))
    assert np.array_equal(host(zx) + 128, r["zx"]) and np.array_equal(host(codes), r["codes"])
    wsum, tsum = lib.dint4_weight_sums(codes, zero, G)
    Wp = lib.pack_dint4(codes, layout)
    Y, acc = lib.w4a8_gemm_asym(Xq, sx, zx, Wp, step, zero, wsum, tsum, N, K, G, layout=layout,
                                out_dtype=TORCH_DT[out_dtype], want_acc=True)
    assert np.array_equal(host(acc), r["acc"]), "int32 accumulators differ"
    assert_y_close(host(Y), r["Y64"], out_dtype)
    Y2 = lib.w4a8_gemm_asym(Xq, sx, zx, Wp, step, zero, wsum, tsum, N, K, G, layout=layout,
                            out_dtype=TORCH_DT[out_dtype])
    assert torch.equal(Y, Y2)


GEMM_CASES = [
    # name, M, K, N, G : decode, K-split decode, prefill, K-split prefill, grouped / per-channel
    ("decode_c2_m16", 16, 4096, 4096, 128),
    ("decode_m1", 1, 4096, 1024, 128),
    ("decode_per_channel_tail", 7, 1152, 272, 0),
    ("decode_k_split_g128", 16, 9216, 48, 128),
    ("decode_k_split_per_channel", 5, 11008, 32, 0),
    ("decode_per_channel_9_tiles_per_wave", 16, 9216, 272, 0),
    ("decode_per_channel_7_tiles_ragged", 5, 6784, 48, 0),
    ("decode_many_n_tiles", 16, 512, 9232, 128),
    ("prefill_m17", 17, 384, 272, 0),
    ("blocks_m33_g128", 33, 1280, 400, 128),
    ("blocks_m50_per_channel", 50, 2304, 272, 0),
    ("blocks_m20_k_ranges_per_channel", 20, 11008, 32, 0),
    ("blocks_m36_k_ranges_g128", 36, 9216, 48, 128),
    ("prefill_m64_g128", 64, 512, 256, 128),
    ("prefill_m130_g128_ksplit", 130, 1024, 304, 128),
    ("prefill_m300", 300, 768, 1040, 0),
    ("prefill_two_workgroups_per_cu_ragged", 1030, 256, 7440, 0),
    ("prefill_m300_g256", 300, 768, 512, 256),
    ("prefill_m600_multi_block", 600, 1024, 784, 0),
    ("prefill_m128_ksplit_per_channel", 128, 2048, 512, 0),
]


@pytest.mark.parametrize("case", GEMM_CASES, ids=[c[0] for c in GEMM_CASES])
def test_gemm_asym_parity(lib, oracle, case):
    name, M, K, N, G = case
    _gemm_asym_case(lib, oracle, 31 + len(name), M, K, N, G)


def test_gemm_asym_bf16_and_canonical(lib, oracle):
    _gemm_asym_case(lib, oracle, 6, 12, 512, 64, 128, out_dtype="bf16")
    _gemm_asym_case(lib, oracle, 7, 40, 256, 48, 0, layout=0)
    # the tile kernel: bf16 output per-channel and group-wise, canonical weights
    _gemm_asym_case(lib, oracle, 8, 200, 512, 272, 0, out_dtype="bf16")
    _gemm_asym_case(lib, oracle, 9, 150, 384, 256, 128, out_dtype="bf16", layout=0)


def test_asym_with_symmetric_tokens_matches_dequantized_product(lib, oracle):
    """Y of the asymmetric path equals the float64 product of its own dequantized operands."""
    X, W, s = syn.random_layer(9, 24, 1024, 256)
    Xq, sx, zx = lib.quantize_act_int8_asym(dev(X), dev(s))
    codes, step, zero = lib.quantize_weight_dint4(dev(W), dev(s), 128)
    wsum, tsum = lib.dint4_weight_sums(codes, zero, 128)
    Y = lib.w4a8_gemm_asym(Xq, sx, zx, lib.pack_dint4(codes), step, zero, wsum, tsum, 256, 1024, 128)
    Xd = (host(Xq).astype(np.float64) - host(zx)[:, None]) * host(sx).astype(np.float64)[:, None]
    Wd = oracle.dequant_dint4(host(codes), host(step), host(zero), 128).astype(np.float64)
    assert_y_close(host(Y), Xd @ Wd.T)


def test_full_size_c2_and_c4_asym(lib, oracle):
    """Full-size decode and prefill shapes in the timed launch configuration, sampled outputs."""
    for name, M, seed in [("C2", 16, 1), ("C4_5120x13824", 512, 2), ("C3_down", 2048, 3)]:
        X, W, s, G = syn.make_layer(name, M=M)
        X = _shifted(X, seed).astype(np.float16)
        Mq, K = X.shape
        N = W.shape[0]
        Xq, sx, zx = lib.quantize_act_int8_asym(dev(X), dev(s))
        q_ref, sx_ref, zx_ref = oracle.quantize_act_uint8_asym(X, s)
        assert np.array_equal(host(Xq).astype(np.int32) + 128, q_ref.astype(np.int32))
        assert np.array_equal(host(sx), sx_ref) and np.array_equal(host(zx) + 128, zx_ref)
        codes, step, zero = lib.quantize_weight_dint4(dev(W), dev(s), G)
        c_ref, st_ref, z_ref = oracle.quantize_weight_dint4(W, s, G)
        assert np.array_equal(host(codes), c_ref)
        wsum, tsum = lib.dint4_weight_sums(codes, zero, G)
        Wp = lib.pack_dint4(codes)
        Y, acc = lib.w4a8_gemm_asym(Xq, sx, zx, Wp, step, zero, wsum, tsum, N, K, G, want_acc=True)
        rng = np.random.default_rng(seed)
        mi = rng.integers(0, Mq, size=64)
        ni = rng.integers(0, N, size=64)
        mi[:4] = [0, Mq - 1, 0, Mq - 1]
        ni[:4] = [0, 0, N - 1, N - 1]
        acc_ref = oracle.int_gemm_asym_sampled(q_ref, zx_ref, oracle.pack_dint4(c_ref), z_ref, G, mi, ni)
        tm, tn = torch.from_numpy(mi).cuda(), torch.from_numpy(ni).cuda()
        assert np.array_equal(host(acc[tm, tn]), acc_ref)
        y64 = sx_ref[mi].astype(np.float64) * np.sum(
            0.5 * st_ref[ni].astype(np.float64) * acc_ref.astype(np.float64), axis=1)
        y_gpu = host(Y[tm, tn]).astype(np.float64)
        rms = np.sqrt(np.mean(host(Y[mi[0]]).astype(np.float64) ** 2))
        assert np.all(np.abs(y_gpu - y64) <= 1e-3 * np.maximum(np.abs(y64), 1e-3 * rms))
