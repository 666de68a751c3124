"""w4a8_linear -- the whole layer in one call, one launch for up to 16 tokens -- against the CPU oracle
and against the two-call path (quantize_act_int8 + w4a8_gemm), through the C ABI.

The one-launch instances quantize the activations inside the streaming kernel; what they make (Xq, sx,
through the entry point's check outputs), the int32 accumulators and Y must be what the two kernels
give: bit for bit, Y included (the same reduction order from the same operands).
"""
import numpy as np
import pytest
import torch

import synthetic_inputs as syn
from gpu_util import assert_y_close, dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import paper_2311_05161_amd as w
    w.load_library()  # raises if the HIP library has not been built: no fallback
    assert torch.cuda.is_available()
    return w


def _case(lib, oracle, seed, M, K, N, G, x_dtype="f16", use_s=True, pad=0, layout=1, zero_row=True):
    X, W, s = syn.random_layer(seed, M, K, N, x_dtype="f32" if x_dtype == "f32" else "f16")
    if zero_row and M > 2:
        X[1] = 0          # an all-zero token
    if x_dtype == "bf16":
        Xt = torch.from_numpy(X.astype(np.float32)).to(torch.bfloat16)
        Xh = Xt.float().numpy()
    else:
        Xt = torch.from_numpy(X)
        Xh = X
    buf = torch.zeros((M, K + pad), dtype=Xt.dtype, device="cuda")
    buf[:, :K] = Xt.cuda()
    Xd = buf[:, :K]
    sd = dev(s) if use_s else None
    r = oracle.linear_w4a8(Xh.astype(np.float32), W, s if use_s else None, G)
    codes, step, zero = lib.quantize_weight_dint4(dev(W), sd, G)
    assert np.array_equal(host(codes), r["codes"])
    Wp = lib.pack_dint4(codes, layout)
    Y, Xq, sx, acc = lib.w4a8_linear(Xd, sd, Wp, step, zero, N, G, layout=layout, want_quantized=True,
                                     want_acc=True)
    assert np.array_equal(host(sx).view(np.uint32), r["sx"].view(np.uint32)), "token scales differ"
    assert np.array_equal(host(Xq), r["Xq"]), "int8 activations differ"
    assert np.array_equal(host(acc), r["acc"]), "int32 accumulators differ"
    assert_y_close(host(Y), r["Y64"])
    # the production form (no check outputs, no hook) and the two-call path: the same Y, bit for bit
    Y1 = lib.w4a8_linear(Xd, sd, Wp, step, zero, N, G, layout=layout)
    Xq2, sx2 = lib.quantize_act_int8(Xd, sd)
    Y2 = lib.w4a8_gemm(Xq2, sx2, Wp, step, zero, N, K, G, layout=layout)
    assert torch.equal(Y1, Y) and torch.equal(Y2, Y)
    return r


ONE_LAUNCH = [
    # name, M, K, N, G -- all fp16, tiled weights, K in one range of the streaming kernel
    ("c2_m16", 16, 4096, 4096, 128),
    ("c2_m1", 1, 4096, 4096, 128),
    ("c2_m5", 5, 4096, 4096, 128),
    ("one_tile", 3, 128, 16, 128),
    ("ring_one_ktile_per_wave", 16, 512, 9232, 128),
    ("ring_five_ktiles_per_wave", 16, 5120, 5136, 128),
    ("group256_ragged", 7, 1280, 400, 256),
    ("per_channel_k_tail", 16, 1152, 272, 0),
    ("per_channel_three_ktiles_ring", 9, 3072, 8208, 0),
    ("per_channel_seven_ktiles_ragged", 16, 6784, 48, 0),
    ("per_channel_seven_ktiles_ring", 2, 7168, 4640, 0),
    ("c1_shape_fp16", 16, 768, 768, 0),
]


@pytest.mark.parametrize("case", ONE_LAUNCH, ids=[c[0] for c in ONE_LAUNCH])
def test_linear_one_launch(lib, oracle, case):
    name, M, K, N, G = case
    assert lib.load_library().w4a8_linear_workspace_bytes(M, N, K, G, 1) >= M * K + 4 * M
    _case(lib, oracle, 40 + len(name), M, K, N, G)


def test_linear_one_launch_variants(lib, oracle):
    _case(lib, oracle, 1, 16, 1024, 272, 128, use_s=False)           # s = NULL
    _case(lib, oracle, 2, 11, 1024, 272, 0, pad=8)                   # rows 16-byte aligned in a wider buffer
    _case(lib, oracle, 3, 2, 512, 64, 128, zero_row=False)


TWO_STEP = [
    # name, M, K, N, G, x_dtype, pad, layout -- what the one-launch instances do not take
    ("bf16_activations", 16, 1024, 272, 128, "bf16", 0, 1),
    ("fp32_activations_c1", 16, 768, 768, 0, "f32", 0, 1),
    ("nine_ktiles_per_wave", 9, 9216, 272, 0, "f16", 0, 1),
    ("k_in_two_ranges", 16, 9216, 48, 128, "f16", 0, 1),
    ("unaligned_rows", 5, 512, 64, 128, "f16", 3, 1),
    ("canonical_layout", 9, 256, 32, 128, "f16", 0, 0),
    ("token_blocks_m40", 40, 512, 256, 128, "f16", 0, 1),
    ("tile_kernel_m300", 300, 768, 1040, 0, "f16", 0, 1),
    ("tile_kernel_k_ranges", 130, 1024, 304, 128, "f16", 0, 1),
]


@pytest.mark.parametrize("case", TWO_STEP, ids=[c[0] for c in TWO_STEP])
def test_linear_two_steps(lib, oracle, case):
    name, M, K, N, G, x_dtype, pad, layout = case
    _case(lib, oracle, 60 + len(name), M, K, N, G, x_dtype=x_dtype, pad=pad, layout=layout)


def test_linear_full_size_c4_up_projection(lib, oracle):
    """The decode object of bench.py at its real size: LLaMA-13B up-projection, 16 tokens, one launch."""
    X, W, s, G = syn.make_layer("C4_5120x13824", M=16)
    K, N = X.shape[1], W.shape[0]
    r = oracle.linear_w4a8(X, W, s, G)
    codes, step, zero = lib.quantize_weight_dint4(dev(W), dev(s), G)
    Wp = lib.pack_dint4(codes, lib.LAYOUT_TILED)
    Y, Xq, sx, acc = lib.w4a8_linear(dev(X), dev(s), Wp, step, zero, N, G, want_quantized=True, want_acc=True)
    assert np.array_equal(host(Xq), r["Xq"]) and np.array_equal(host(sx), r["sx"])
    assert np.array_equal(host(acc), r["acc"])
    assert_y_close(host(Y), r["Y64"])
    assert torch.equal(lib.w4a8_linear(dev(X), dev(s), Wp, step, zero, N, G), Y)


def test_linear_exact_output_of_the_plain_one_launch_instances(lib, oracle):
    """Bit-exact Y without any hook (see test_gpu_parity_exact.py for the construction): the activations
    are small integers whose row maximum is exactly 127, so the quantizer reproduces them (scale 1)."""
    from test_gpu_parity_exact import _exact_operands
    for (M, K, N, G) in ((16, 4096, 4096, 128), (16, 5120, 5136, 128), (9, 3072, 8208, 0), (7, 6656, 48, 0)):
        Xq, _, codes, zero, step = _exact_operands(300 + M + N, M, K, N, G)
        Xq[:, 0], Xq[:, K // 2] = 127, -127       # a mirrored pair: it cancels like every other column
        sx = np.ones(M, np.float32)
        acc = oracle.int_gemm(Xq, oracle.pack_dint4(codes), zero, G)
        y32, y64 = oracle.dequant_epilogue(acc, sx, step)
        assert np.array_equal(y32.astype(np.float64), y64) and np.array_equal(y32.astype(np.float16), y32)
        ref_q, ref_sx = oracle.quantize_act_int8(Xq.astype(np.float32), None)
        assert np.array_equal(ref_q, Xq) and np.array_equal(ref_sx, sx)      # premise: the quantizer is the identity here
        Wp = lib.pack_dint4(dev(codes), lib.LAYOUT_TILED)
        Y = lib.w4a8_linear(dev(Xq.astype(np.float16)), None, Wp, dev(step), dev(zero), N, G)
        got = host(Y).astype(np.float32)
        assert np.array_equal(got, y32), f"{(got != y32).sum()} outputs differ from the exact result"


def test_product_is_rounded_before_the_tie_break(lib, oracle):
    """Per-token INT8 rounding is rne(fl32(t * fl32(127 / a))): two binary32 roundings, then the tie
    break.  For a token whose maximum is a and that also holds a / 2, the exact product is 63.5 - eps
    for about half of all a (127 / a rounded down), the rounded product is the tie 63.5 itself: the
    definition gives 64, a multiply-add fused with the rounding step would give 63.  Both GPU paths
    (quantize_act_int8 and the one-launch w4a8_linear, which rounds inside the streaming kernel) must
    give the definition's value."""
    halves = np.arange(0x3c00, 0x7800, dtype=np.uint16).view(np.float16).astype(np.float32)   # fp16 in [1, 32768)
    inv = np.float32(127.0) / halves
    t = (halves * np.float32(0.5)).astype(np.float32)              # a / 2: exact in fp16 (normal range)
    y32 = (t * inv).astype(np.float32)
    exact = t.astype(np.float64) * inv.astype(np.float64)
    witness = halves[(y32 == np.float32(63.5)) & (exact < 63.5)]
    assert witness.size > 1000                                     # the premise: such maxima are common
    rng = np.random.default_rng(5)
    M, K, N, G = 16, 1024, 272, 128
    X = (rng.standard_normal((M, K)) * 0.25).astype(np.float16).astype(np.float32)
    a = rng.choice(witness[witness < 2048], size=M, replace=False)
    cols = rng.choice(np.arange(1, K), size=(M, 24), replace=True)
    for m in range(M):
        X[m, 0] = a[m]
        X[m, cols[m]] = np.where(rng.random(24) < 0.5, 0.5, -0.5) * a[m]
    X16 = X.astype(np.float16)
    assert np.array_equal(X16.astype(np.float32), X)
    ref_q, ref_sx = oracle.quantize_act_int8(X, None)
    for m in range(M):
        assert set(np.abs(ref_q[m, cols[m]]).tolist()) == {64}     # the definition: ties to even
        fused = np.rint(X[m, cols[m]].astype(np.float64) * np.float64(np.float32(127.0) / np.float32(a[m])))
        assert set(np.abs(fused).tolist()) == {63}                 # what a fused multiply-add would give
    Xd = dev(X16)
    q2, sx2 = lib.quantize_act_int8(Xd, None)
    assert np.array_equal(host(q2), ref_q) and np.array_equal(host(sx2), ref_sx)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    codes, step, zero = lib.quantize_weight_dint4(dev(W), None, G)
    Wp = lib.pack_dint4(codes, lib.LAYOUT_TILED)
    Y, Xq, sx, acc = lib.w4a8_linear(Xd, None, Wp, step, zero, N, G, want_quantized=True, want_acc=True)
    assert np.array_equal(host(sx), ref_sx)
    bad = host(Xq) != ref_q
    assert not bad.any(), f"{bad.sum()} int8 activations differ from the definition, first at {np.argwhere(bad)[0]}"
    Y1 = lib.w4a8_linear(Xd, None, Wp, step, zero, N, G)
    Y2 = lib.w4a8_gemm(q2, sx2, Wp, step, zero, N, K, G)
    assert torch.equal(Y1, Y2)


def test_vanishing_tokens_are_quantized_as_all_zero(lib, oracle):
    """Tokens whose 127 / max|t| (255 / range for the asymmetric form) overflows binary32 -- below about 3.7e-37,
    reachable from fp32 activations or through a huge AQAS scale -- take the all-zero rule on both sides: scale 1,
    codes 0; subnormal scales just above that are kept bit for bit."""
    rng = np.random.default_rng(11)
    M, K, N, G = 16, 1024, 272, 128
    scale = np.array([1e-38, 3e-39, 1e-41, 1e-44, 1.0, 1e-30, 6e-8, 1e-45, 1.2e-37, 3.8e-37, 1e-36, 1e-35,
                      0.0, 2.0, 1e-20, 5e-37], np.float32)
    X32 = (rng.standard_normal((M, K)).astype(np.float32) * scale[:, None]).astype(np.float32)
    s = rng.uniform(0.5, 2.0, K).astype(np.float32)
    ref_q, ref_sx = oracle.quantize_act_int8(X32, s)
    assert (ref_sx == 1.0).sum() >= 6 and (ref_sx < np.finfo(np.float32).tiny).sum() >= 1   # dead rows, and a subnormal scale that is kept
    q, sx = lib.quantize_act_int8(dev(X32), dev(s))
    assert np.array_equal(host(sx).view(np.uint32), ref_sx.view(np.uint32)) and np.array_equal(host(q), ref_q)
    Q, sa, zx = oracle.quantize_act_uint8_asym(X32, s)
    qa, sxa, zxa = lib.quantize_act_int8_asym(dev(X32), dev(s))
    assert np.array_equal(host(sxa).view(np.uint32), sa.view(np.uint32))
    assert np.array_equal(host(zxa).astype(np.int64) + 128, zx.astype(np.int64))
    assert np.array_equal(host(qa).astype(np.int16) + 128, Q.astype(np.int16))
    # fp16 activations with a huge AQAS scale: through both quantizer paths of the layer
    Xh = (rng.standard_normal((M, K)) * np.where(np.arange(M)[:, None] % 2, 1.0, 1e-3)).astype(np.float16)
    s_big = np.full(K, 3e38, np.float32)
    s_big[::3] = 1e35
    ref_q, ref_sx = oracle.quantize_act_int8(Xh.astype(np.float32), s_big)
    assert 0 < (ref_sx == 1.0).sum() < M
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    codes, step, zero = lib.quantize_weight_dint4(dev(W), None, G)
    Wp = lib.pack_dint4(codes, lib.LAYOUT_TILED)
    Y, Xq, sxl, acc = lib.w4a8_linear(dev(Xh), dev(s_big), Wp, step, zero, N, G, want_quantized=True, want_acc=True)
    assert np.array_equal(host(sxl).view(np.uint32), ref_sx.view(np.uint32)) and np.array_equal(host(Xq), ref_q)
    q2, sx2 = lib.quantize_act_int8(dev(Xh), dev(s_big))
    assert np.array_equal(host(sx2).view(np.uint32), ref_sx.view(np.uint32)) and np.array_equal(host(q2), ref_q)
    assert torch.isfinite(Y.float()).all()
