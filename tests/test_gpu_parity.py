"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Integer results (int8 activations, 4-bit codes, packed bytes, zero-points, int32 accumulators)
and the fp32 quantization parameters (token scales, steps) must be bit-identical; Y must lie
within 1e-3 relative (fp16) of the oracle's float64 evaluation.
"""
import numpy as np
import pytest
import torch

import synthetic_inputs as syn
from gpu_util import acc_by_float64_matmul, assert_y_close, decode_table_np, dev, host, tiled_layout_np

pytestmark = pytest.mark.gpu

TORCH_DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


@pytest.fixture(scope="module")
def lib():
    import paper_2311_05161_amd as w
    w.load_library()  # raises if the HIP library has not been built: no fallback
    assert torch.cuda.is_available()
    return w


def _x_for(dtype, X):
    """Host array widened exactly the way the device sees it, plus the device tensor."""
    if dtype == "bf16":
        t = torch.from_numpy(X.astype(np.float32)).to(torch.bfloat16)
        return t.float().numpy(), t.cuda()
    a = X.astype(np.float16 if dtype == "f16" else np.float32)
    return a, dev(a)


# --------------------------------------------------------------------------- activations
ACT_CASES = [
    # name, M, K, dtype, use_s, ld_pad
    ("c1_tiny", 16, 768, "f32", False, 0),
    ("c2_decode", 16, 4096, "f16", True, 0),
    ("one_row", 1, 4096, "f16", True, 0),
    ("ragged_rows", 37, 5120, "f16", True, 0),
    ("wide", 130, 13824, "f16", True, 0),
    ("many_rows", 2100, 1024, "f16", True, 0),
    ("bf16", 33, 2048, "bf16", True, 0),
    ("odd_k_generic", 19, 1001, "f16", True, 0),
    ("strided", 21, 512, "f32", True, 24),
    ("strided_unaligned", 5, 264, "f16", True, 3),
    ("very_wide_generic", 3, 16392, "f16", False, 0),
]


@pytest.mark.parametrize("case", ACT_CASES, ids=[c[0] for c in ACT_CASES])
def test_act_quant_bit_exact(lib, oracle, case):
    name, M, K, dtype, use_s, pad = case
    X, _, s = syn.random_layer(sum(name.encode()) % 1000, M, K, 1, x_dtype="f32")
    if M > 2:
        X[1] = 0.0  # an all-zero token
    Xh, _ = _x_for(dtype, X)
    buf = torch.zeros((M, K + pad), dtype=TORCH_DT[dtype], device="cuda")
    buf[:, :K] = torch.from_numpy(Xh).to(TORCH_DT[dtype]).cuda()
    Xd = buf[:, :K]
    sd = dev(s) if use_s else None
    Xq, sx = lib.quantize_act_int8(Xd, sd)
    ref_q, ref_s = oracle.quantize_act_int8(Xh.astype(np.float32), s if use_s else None)
    assert np.array_equal(host(sx).view(np.uint32), ref_s.view(np.uint32))
    assert np.array_equal(host(Xq), ref_q)


def test_act_quant_empty(lib):
    X = torch.zeros((0, 256), dtype=torch.float16, device="cuda")
    Xq, sx = lib.quantize_act_int8(X)
    assert Xq.shape == (0, 256) and sx.shape == (0,)


# --------------------------------------------------------------------------- weights
WQ_CASES = [
    # name, N, K, G, dtype, use_s
    ("c1_per_channel", 768, 768, 0, "f32", False),
    ("c2_group128", 512, 4096, 128, "f16", True),
    ("per_channel_wide", 100, 11008, 0, "f16", True),
    ("group256_bf16", 48, 1024, 256, "bf16", True),
    ("group50_pairs", 7, 100, 50, "f16", True),
    ("group33_scalar", 5, 99, 33, "f32", True),
    ("one_row", 1, 128, 128, "f16", False),
]


@pytest.mark.parametrize("case", WQ_CASES, ids=[c[0] for c in WQ_CASES])
def test_weight_quant_bit_exact(lib, oracle, case):
    name, N, K, G, dtype, use_s = case
    _, W, s = syn.random_layer(sum(name.encode()) % 1000 + 1, 1, K, N, x_dtype="f32")
    if N > 3:
        W[2] = 0.0                 # degenerate group: step 1, z 0
        W[3] = np.abs(W[3])        # all positive: range extended to 0
    Wh, Wd = _x_for(dtype, W)
    sd = dev(s) if use_s else None
    codes, step, zero = lib.quantize_weight_dint4(Wd, sd, G)
    rc, rs, rz = oracle.quantize_weight_dint4(Wh.astype(np.float32), s if use_s else None, G)
    assert np.array_equal(host(step).view(np.uint32), rs.view(np.uint32))
    assert np.array_equal(host(zero), rz)
    assert np.array_equal(host(codes), rc)
    # externally given parameters (clipped ranges): only the per-element rule runs
    st2 = (rs * np.float32(0.8)).astype(np.float32)
    codes2, _, _ = lib.quantize_weight_dint4(Wd, sd, G, step=dev(st2), zero=dev(rz))
    rc2, _, _ = oracle.quantize_weight_dint4(Wh.astype(np.float32), s if use_s else None, G,
                                             step=st2, zero=rz)
    assert np.array_equal(host(codes2), rc2)


# --------------------------------------------------------------------------- packing
@pytest.mark.parametrize("N,K", [(16, 128), (48, 384), (768, 768), (4096, 4096)])
def test_pack_layouts_bit_exact(lib, oracle, N, K):
    rng = np.random.default_rng(N + K)
    codes = rng.integers(0, 16, size=(N, K)).astype(np.uint8)
    cd = dev(codes)
    p0 = lib.pack_dint4(cd, lib.LAYOUT_CANONICAL)
    assert np.array_equal(host(p0), oracle.pack_dint4(codes))
    p1 = lib.pack_dint4(cd, lib.LAYOUT_TILED)
    assert np.array_equal(host(p1).reshape(-1), tiled_layout_np(codes))
    assert np.array_equal(host(lib.unpack_dint4(p0, N, K, lib.LAYOUT_CANONICAL)), codes)
    assert np.array_equal(host(lib.unpack_dint4(p1, N, K, lib.LAYOUT_TILED)), codes)


def test_pack_canonical_small_even_k(lib, oracle):
    codes = np.arange(16, dtype=np.uint8).repeat(2).reshape(1, 32)[:, :30]
    codes = np.ascontiguousarray(np.tile(codes, (3, 1)))
    p0 = lib.pack_dint4(dev(codes), lib.LAYOUT_CANONICAL)
    assert np.array_equal(host(p0), oracle.pack_dint4(codes))


# --------------------------------------------------------------------------- GEMM
def _gemm_case(lib, oracle, seed, M, K, N, G, out_dtype="f16", layout=1, x_dtype="f16"):
    X, W, s = syn.random_layer(seed, M, K, N, x_dtype=x_dtype)
    r = oracle.linear_w4a8(X, W, s, G)
    Xq, sx = lib.quantize_act_int8(dev(X), dev(s))
    codes, step, zero = lib.quantize_weight_dint4(dev(W), dev(s), G)
    assert np.array_equal(host(Xq), r["Xq"]) and np.array_equal(host(codes), r["codes"])
    Wp = lib.pack_dint4(codes, layout)
    Y, acc = lib.w4a8_gemm(Xq, sx, Wp, step, zero, N, K, G, layout=layout,
                           out_dtype=TORCH_DT[out_dtype], want_acc=True)
    assert np.array_equal(host(acc), r["acc"]), "int32 accumulators differ"
    assert_y_close(host(Y), r["Y64"], out_dtype)
    # without the accumulator hook the same Y comes out (bitwise: fixed reduction order)
    Y2 = lib.w4a8_gemm(Xq, sx, Wp, step, zero, N, K, G, layout=layout,
                       out_dtype=TORCH_DT[out_dtype])
    assert torch.equal(Y, Y2)
    return r, Y


DECODE_CASES = [
    # name, M, K, N, G
    ("c1_tiny", 16, 768, 768, 0),
    ("c2_m1", 1, 4096, 4096, 128),
    ("c2_m5", 5, 4096, 4096, 128),
    ("c2_m16", 16, 4096, 4096, 128),
    ("g256_ragged", 7, 1280, 400, 256),
    ("per_channel_k_tail", 16, 1152, 272, 0),
    ("one_tile", 3, 128, 16, 128),
    ("k_split_2_g128", 16, 9216, 48, 128),        # K > 8192: two K-ranges + deterministic combine
    ("k_split_2_per_channel", 5, 11008, 32, 0),
    ("k_split_3_ragged", 9, 16512, 16, 384),
    ("per_channel_6_tiles_per_wave", 16, 6144, 272, 0),   # K <= 9216 per channel: one K-range, 6..9 k-tiles per wave
    ("per_channel_7_tiles_ragged", 3, 6784, 48, 0),
    ("per_channel_8_tiles_per_wave", 16, 8192, 528, 0),
    ("per_channel_9_tiles_per_wave", 9, 9216, 1040, 0),
    ("per_channel_9_tiles_ragged", 16, 8576, 32, 0),
    ("many_n_tiles_per_block", 16, 512, 9232, 128),  # 577 n-tiles: several per workgroup, ragged
    ("many_n_tiles_per_channel", 2, 1024, 4640, 0),
    # 1285 n-tiles x 40 groups: six n-tiles and 3840 decode records per workgroup (eight parameter
    # stages per thread), workgroups with five and with six n-tiles
    ("many_records_per_block", 2, 5120, 20560, 128),
]


@pytest.mark.parametrize("case", DECODE_CASES, ids=[c[0] for c in DECODE_CASES])
def test_gemm_decode_parity(lib, oracle, case):
    name, M, K, N, G = case
    _gemm_case(lib, oracle, 11 + len(name), M, K, N, G, x_dtype="f32" if "c1" in name else "f16")


PREFILL_CASES = [
    # 17 .. 64 tokens with K in one range run as 16-token blocks of the streaming kernel
    ("m17", 17, 384, 272, 0),
    ("m64_g128", 64, 512, 256, 128),
    ("m33_three_blocks_last_of_one_row_g128", 33, 1280, 400, 128),
    ("m50_blocks_per_channel_9_tiles_per_wave", 50, 9216, 272, 0),
    ("m64_blocks_many_n_tiles", 64, 512, 4112, 128),
    ("m40_blocks_with_k_in_two_ranges_g128", 40, 5248, 272, 128),
    ("m24_blocks_with_k_in_two_ranges_per_channel", 24, 11008, 48, 0),
    ("m113_eight_blocks_small_layer", 113, 640, 528, 128),
    ("m100_ragged", 100, 640, 528, 0),
    ("m130_g128", 130, 1024, 304, 128),
    # group-128 weights, 129 .. 256 tokens, few output tiles: the kernel that cuts K into four phases
    # inside the workgroup -- super-steps of four k-tiles with a ragged last one (11, 18 k-tiles), exactly
    # two super-steps, a ragged 64-channel tile, one and two token tiles
    ("m130_k_phases_11_ktiles_g128", 130, 1408, 80, 128),
    ("m256_k_phases_18_ktiles_g128", 256, 2304, 1040, 128),
    ("m129_k_phases_two_super_steps_g128", 129, 1024, 64, 128),
    ("m200_k_phases_40_ktiles_g128", 200, 5120, 336, 128),
    # the same decomposition for per-channel weights (int32 phase sums, bias removal with the row-sums)
    ("m130_k_phases_11_ktiles_per_channel", 130, 1408, 80, 0),
    ("m256_k_phases_18_ktiles_per_channel", 256, 2304, 1040, 0),
    ("m129_k_phases_two_super_steps_per_channel", 129, 1024, 64, 0),
    ("m200_k_phases_86_ktiles_per_channel", 200, 11008, 336, 0),
    ("m300", 300, 768, 1040, 0),
    ("m300_g256", 300, 768, 512, 256),
    ("m600_multi_block", 600, 1024, 784, 0),
    # 5 x 30 tiles of 256 tokens with a ragged last token tile and a 16-channel last column
    ("m1030_256_row_tiles_ragged", 1030, 256, 7440, 0),
    # 16 x 44 = 704 tiles of 128 tokens against 352 of 256 (two rounds of the CUs): the tile-height rule
    # takes the per-channel instance that runs two workgroups to a CU; ragged last token tile (10 rows)
    # and a 16-channel last column
    ("m1930_two_per_cu_ragged", 1930, 256, 11024, 0),
]


@pytest.mark.parametrize("case", PREFILL_CASES, ids=[c[0] for c in PREFILL_CASES])
def test_gemm_prefill_parity(lib, oracle, case):
    name, M, K, N, G = case
    _gemm_case(lib, oracle, 23 + len(name), M, K, N, G)


# The K-phase kernel's edges: 65 / 128 / 129 / 256 tokens (above the token blocks' reach only where the
# layer is large or M > 128: the small ones here run M > 128), every residue of the k-tile count modulo
# the four phases and modulo the four weight register sets (8 .. 15 k-tiles: one to four super-steps, ragged
# and full), one 64-channel tile, a ragged one, and -- on layers beyond the token blocks' 48 Mi weights -- 65 and
# 128 tokens with a grid of 128 / 129 workgroups and 50 k-tiles (the other arm of the dispatch rule).
K_PHASE_EDGES = [(129 + 9 * kt, 128 * kt, 16 * (1 + kt % 7)) for kt in range(8, 16)] + [
    (256, 1024, 64), (255, 1152, 4096 + 16), (129, 6144, 48), (65, 6400, 8192), (128, 6400, 8192 + 64)]


@pytest.mark.parametrize("G", [128, 0])
@pytest.mark.parametrize("M,K,N", K_PHASE_EDGES)
def test_gemm_k_phase_kernel_edges(lib, oracle, M, K, N, G):
    _gemm_case(lib, oracle, M + K + N + G, M, K, N, G)


def test_gemm_bf16_output_and_canonical_layout(lib, oracle):
    _gemm_case(lib, oracle, 5, 12, 512, 64, 128, out_dtype="bf16")
    _gemm_case(lib, oracle, 6, 40, 512, 64, 0, out_dtype="bf16")
    _gemm_case(lib, oracle, 7, 9, 256, 32, 128, layout=0)
    _gemm_case(lib, oracle, 8, 70, 256, 48, 0, layout=0)
    # the tile kernel's bf16 epilogue: staged whole-row stores, direct stores of a ragged tile,
    # group-wise sums, K cut into ranges, and its canonical-layout repack
    _gemm_case(lib, oracle, 9, 300, 512, 512, 0, out_dtype="bf16")
    _gemm_case(lib, oracle, 10, 150, 384, 272, 128, out_dtype="bf16")
    _gemm_case(lib, oracle, 11, 200, 1024, 304, 0, out_dtype="bf16", layout=0)


@pytest.mark.parametrize("M,K,N,G", [(16, 512, 272, 128), (5, 1152, 48, 0), (3, 9216, 32, 128), (40, 512, 256, 0),
                                     (130, 256, 304, 128)])
def test_gemm_output_views(lib, oracle, M, K, N, G):
    """Y as a view of a wider buffer: a leading dimension that allows 8-byte stores, and one (with an
    odd element offset) that does not; the columns outside the view stay untouched."""
    X, W, s = syn.random_layer(77 + M, M, K, N)
    Xq, sx = lib.quantize_act_int8(dev(X), dev(s))
    codes, step, zero = lib.quantize_weight_dint4(dev(W), dev(s), G)
    Wp = lib.pack_dint4(codes, lib.LAYOUT_TILED)
    ref = lib.w4a8_gemm(Xq, sx, Wp, step, zero, N, K, G)
    for pad_l, pad_r in ((4, 4), (1, 5), (3, 2)):
        big = torch.full((M, pad_l + N + pad_r), -7.0, dtype=torch.float16, device=ref.device)
        view = big[:, pad_l:pad_l + N]
        out = lib.w4a8_gemm(Xq, sx, Wp, step, zero, N, K, G, Y=view)
        assert out.data_ptr() == view.data_ptr()
        assert torch.equal(view, ref)
        assert bool((big[:, :pad_l] == -7.0).all()) and bool((big[:, pad_l + N:] == -7.0).all())


def test_gemm_every_code_and_zero_point(lib, oracle):
    """Random codes / zero-points / extreme activations straight into the GEMM (no quantizer)."""
    rng = np.random.default_rng(77)
    for M in (4, 48):
        K, N, G = 512, 64, 128
        Xq = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
        Xq[0] = 127
        Xq[1] = -127
        codes = rng.integers(0, 16, size=(N, K)).astype(np.uint8)
        codes[0] = 13
        codes[1] = 0
        zero = rng.integers(0, 14, size=(N, K // G)).astype(np.uint8)
        zero[0] = 0
        zero[1] = 13
        step = rng.uniform(0.001, 0.1, size=(N, K // G)).astype(np.float32)
        sx = rng.uniform(0.01, 1.0, size=M).astype(np.float32)
        acc_ref = oracle.int_gemm(Xq, oracle.pack_dint4(codes), zero, G)
        _, y64 = oracle.dequant_epilogue(acc_ref, sx, step)
        Wp = lib.pack_dint4(dev(codes), lib.LAYOUT_TILED)
        Y, acc = lib.w4a8_gemm(dev(Xq), dev(sx), Wp, dev(step), dev(zero), N, K, G, want_acc=True)
        assert np.array_equal(host(acc), acc_ref)
        assert_y_close(host(Y), y64)


def test_gemm_empty_batch(lib):
    N, K = 32, 128
    Xq = torch.zeros((0, K), dtype=torch.int8, device="cuda")
    sx = torch.zeros((0,), dtype=torch.float32, device="cuda")
    Wp = torch.zeros((N * K // 2,), dtype=torch.uint8, device="cuda")
    step = torch.ones((N, 1), dtype=torch.float32, device="cuda")
    zero = torch.zeros((N, 1), dtype=torch.uint8, device="cuda")
    Y = lib.w4a8_gemm(Xq, sx, Wp, step, zero, N, K, 0)
    assert Y.shape == (0, N)


def test_aqas_power_of_two_invariance_on_gpu(lib, oracle):
    """s = 2^j for every channel rescales sx and step exactly and leaves Y unchanged (Eq. 1)."""
    X, W, _ = syn.random_layer(3, 8, 512, 64)
    outs = []
    for j in (0, 2):
        s = dev(np.full(512, 2.0 ** j, np.float32))
        Xq, sx = lib.quantize_act_int8(dev(X), s)
        codes, step, zero = lib.quantize_weight_dint4(dev(W), s, 128)
        Y = lib.w4a8_gemm(Xq, sx, lib.pack_dint4(codes), step, zero, 64, 512, 128)
        outs.append((host(Xq), host(sx), host(codes), host(step), host(Y)))
    a, b = outs
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[2], b[2])
    assert np.array_equal(a[1], b[1] * 4) and np.array_equal(a[3] * 4, b[3])
    assert np.array_equal(a[4], b[4])


# --------------------------------------------------------------------------- full-size configurations
def _full_size_case(lib, oracle, name, M=None, seed=0, N=None, whole=True, n_samples=4096):
    """A BASELINE configuration at its real size, in the launch configuration bench.py times.

    Quantizers: compared with the oracle in full, bit for bit.  Accumulators: the WHOLE [M, N, K/G]
    array against Eq. 1's integer product evaluated on the CPU as a float64 library matmul of the
    oracle's int8 activations and of its codes decoded by the closed form (exact: all partial sums
    are integers below 2^53; chunked over N) -- plus outputs that the oracle's own plain loop
    computes one by one.  Y: the whole matrix against the float64 evaluation of the epilogue on
    those accumulators.  `whole` = False (the OPT-66B layer, 1.4e12 multiply-accumulates): 32 full
    output rows, 32 full output columns and `n_samples` single entries instead of everything."""
    X, W, s, G = syn.make_layer(name, M=M, N=N)
    Mq, K = X.shape
    N = W.shape[0]
    Gs = G or K
    Xd, Wd, sd = dev(X), dev(W), dev(s)
    Xq, sx = lib.quantize_act_int8(Xd, sd)
    codes, step, zero = lib.quantize_weight_dint4(Wd, sd, G)
    del Wd
    ref_q, ref_sx = oracle.quantize_act_int8(X, s)
    assert np.array_equal(host(Xq), ref_q) and np.array_equal(host(sx), ref_sx)
    ref_codes, ref_step, ref_zero = oracle.quantize_weight_dint4(W, s, G)
    assert np.array_equal(host(step), ref_step) and np.array_equal(host(zero), ref_zero)
    assert np.array_equal(host(codes), ref_codes)
    Wp = lib.pack_dint4(codes, lib.LAYOUT_TILED)
    del codes
    ws = torch.empty((max(1, lib.gemm_workspace_bytes(Mq, N, K, G)),), dtype=torch.uint8, device="cuda")
    Y = lib.w4a8_gemm(Xq, sx, Wp, step, zero, N, K, G, workspace=ws)     # the timed configuration
    Y2, acc = lib.w4a8_gemm(Xq, sx, Wp, step, zero, N, K, G, workspace=ws, want_acc=True)
    assert torch.equal(Y, Y2)
    assert int(acc.abs().max()) <= 127 * 26 * Gs

    d = decode_table_np(ref_codes, ref_zero, G)              # [N, K] int16, half steps
    sx64 = ref_sx.astype(np.float64)
    hs64 = 0.5 * ref_step.astype(np.float64)                 # [N, ng]

    def check_block(rows, cols):
        """GPU accumulators and Y of the block rows x cols (index arrays) against the float64 matmul."""
        a64 = acc_by_float64_matmul(ref_q[rows], d[cols], G)                 # [r, c, ng]
        rt, ct = torch.from_numpy(rows).cuda(), torch.from_numpy(cols).cuda()
        a_gpu = host(acc.index_select(0, rt).index_select(1, ct))
        assert np.array_equal(a_gpu, a64), "int32 accumulators differ from the exact product"
        y64 = sx64[rows, None] * np.einsum("mng,ng->mn", a64, hs64[cols])
        y_gpu = host(Y.index_select(0, rt).index_select(1, ct)).astype(np.float64)
        return y_gpu, y64

    rms_rows = host(Y.float().square().mean(1).sqrt()).astype(np.float64)   # per token, of the GPU's own Y
    def check_y(y_gpu, y64, row_rms):
        bound = 1e-3 * np.maximum(np.abs(y64), 1e-3 * row_rms[:, None] + 1e-30)
        assert np.all(np.abs(y_gpu - y64) <= bound), "Y out of tolerance"

    rng = np.random.default_rng(seed)
    if whole:
        nc = max(16, min(N, (1 << 27) // max(1, Mq * (K // Gs)) // 16 * 16))   # ~1 GiB of float64 per chunk
        y_all = np.empty((Mq, N), np.float64)
        for n0 in range(0, N, nc):
            cols = np.arange(n0, min(N, n0 + nc))
            y_gpu, y64 = check_block(np.arange(Mq), cols)
            y_all[:, cols] = y64
            check_y(y_gpu, y64, rms_rows)
        # the row rms used above is the GPU's: it must agree with the reference's
        assert np.allclose(rms_rows, np.sqrt(np.mean(y_all ** 2, axis=1)), rtol=1e-2)
    else:
        rows = np.unique(np.concatenate([[0, Mq - 1], rng.integers(0, Mq, size=30)]))
        cols = np.unique(np.concatenate([[0, N - 1], rng.integers(0, N, size=30)]))
        nc = 4096
        for n0 in range(0, N, nc):                       # full rows, chunked over N
            cs = np.arange(n0, min(N, n0 + nc))
            y_gpu, y64 = check_block(rows, cs)
            check_y(y_gpu, y64, rms_rows[rows])
        y_gpu, y64 = check_block(np.arange(Mq), cols)    # full columns
        check_y(y_gpu, y64, rms_rows)
    # single outputs by the oracle's own plain loop (the corners among them)
    ns = min(n_samples, 256) if whole else n_samples
    mi = rng.integers(0, Mq, size=ns)
    ni = rng.integers(0, N, size=ns)
    mi[:4] = [0, Mq - 1, 0, Mq - 1]
    ni[:4] = [0, 0, N - 1, N - 1]
    acc_ref = oracle.int_gemm_sampled(ref_q, oracle.pack_dint4(ref_codes), ref_zero, G, mi, ni)
    acc_gpu = acc[torch.from_numpy(mi).cuda(), torch.from_numpy(ni).cuda()]
    assert np.array_equal(host(acc_gpu), acc_ref), "sampled int32 accumulators differ"
    y64 = sx64[mi] * np.sum(hs64[ni] * acc_ref.astype(np.float64), axis=1)
    y_gpu = host(Y[torch.from_numpy(mi).cuda(), torch.from_numpy(ni).cuda()]).astype(np.float64)
    assert np.all(np.abs(y_gpu - y64) <= 1e-3 * np.maximum(np.abs(y64), 1e-3 * rms_rows[mi]))


def test_full_size_c2_decode_all_m(lib, oracle):
    for M in (1, 2, 4, 8, 16):
        _full_size_case(lib, oracle, "C2", M=M, seed=M)


# the whole LLaMA-13B sweep: three layers x five token counts
@pytest.mark.parametrize("name", ["C4_5120x5120", "C4_5120x13824", "C4_13824x5120"])
@pytest.mark.parametrize("M", [1, 16, 128, 512, 2048])
def test_full_size_llama13b_sweep(lib, oracle, name, M):
    _full_size_case(lib, oracle, name, M=M, seed=M)


@pytest.mark.parametrize("name,M", [("C3_up", 2048), ("C3_down", 2048), ("C4_5120x13824", 64)])
def test_full_size_llama_shapes(lib, oracle, name, M):
    _full_size_case(lib, oracle, name, M=M, seed=M)


@pytest.mark.parametrize("M", [130, 256])
def test_k_phase_kernel_per_channel_on_a_full_size_layer(lib, oracle, M):
    """65 .. 256 tokens on the per-channel 11008 -> 4096 layer (LLaMA-7B down-projection): 64-token x 64-channel
    workgroups with K in four phases (at most one per CU), whole-matrix accumulators and Y."""
    _full_size_case(lib, oracle, "C3_down", M=M, seed=300 + M)


def test_64_token_tiles_on_a_layer_too_large_for_token_blocks(lib, oracle):
    """64 tokens on 24832 x 5120 group-128 weights: four 16-token blocks would need more than two
    generations of workgroups, so this runs on the tile kernel's 64-row instance."""
    # (the workspace tells: two K-ranges of fp32 partial sums, which only the tile kernel asks for here)
    assert lib.gemm_workspace_bytes(64, 24832, 5120, 128, lib.LAYOUT_TILED) == 2 * 64 * 24832 * 4
    _full_size_case(lib, oracle, "C4_5120x13824", M=64, N=24832, seed=64)


def test_last_round_of_group_wise_tiles_runs_with_k_in_ranges(lib, oracle):
    """More than one round of 512 resident 128 x 128 group-wise tiles with a nearly empty last round (here 9 x 61
    tiles, ragged in both directions): the channels of the last round run as a launch of their own with K cut
    into ranges, and a combine pass over that slice of Y.  (The 2048-token cells of the LLaMA-13B sweep on the
    5120-channel layers take the same path.)"""
    # (the workspace tells: four K-ranges of fp32 partial sums for the last 528 channels)
    assert lib.gemm_workspace_bytes(1100, 7696, 5120, 128, lib.LAYOUT_TILED) == 4 * 1100 * 528 * 4
    _full_size_case(lib, oracle, "C4_5120x5120", M=1100, N=7696, seed=61)


def test_full_size_c5_opt66b_end_to_end(lib, oracle):
    """OPT-66B-shaped layer: activation quantization and GEMM back to back on one stream."""
    _full_size_case(lib, oracle, "C5", whole=False, n_samples=4096, seed=5)


def test_measurement_aids_run_and_count_their_work(lib):
    """The streaming read and the MFMA loop that bench.py times as measured ceilings: both run,
    write nothing (the sink stays as it was) and the loop reports its operation count."""
    import ctypes
    L = lib.load_library()
    buf = torch.randint(0, 256, (1 << 20,), dtype=torch.uint8, device="cuda")
    sink = torch.full((4,), 7, dtype=torch.int32, device="cuda")
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert L.w4a8_measure_stream_read(buf.data_ptr(), buf.numel(), sink.data_ptr(), st) == 0
    assert L.w4a8_measure_stream_read(buf.data_ptr() + 16, 4096 + 16, sink.data_ptr(), st) == 0   # ragged tail
    ops = ctypes.c_int64(0)
    assert L.w4a8_measure_mfma_i8(3, sink.data_ptr(), ctypes.byref(ops), st) == 0
    # the k-tile instruction mix, with its operands in registers and with the fragment reads from LDS
    assert L.w4a8_measure_ktile_mix(5, 0, sink.data_ptr(), st) == 0
    assert L.w4a8_measure_ktile_mix(5, 1, sink.data_ptr(), st) == 0
    torch.cuda.synchronize()
    assert ops.value == 512 * 4 * 8 * 3 * 2 * 32 ** 3
    assert sink.tolist() == [7, 7, 7, 7]
