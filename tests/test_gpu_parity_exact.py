"""Exact outputs of the GEMM instances that run WITHOUT the accumulator hook (the ones that are timed).

The hook instances return their int32 accumulators, which the other parity tests compare bit for
bit; the plain instances only return fp16 / bf16 Y, where a wrong unit in an accumulator of 1e5
would disappear in the rounding.  Here the operands are built so that every output is a small
integer times a power of two -- exactly representable in fp16 -- while the individual products and
per-group accumulators stay large:

  * the second half of K repeats the first half's weight columns (codes, zero-points, steps), and
    the activations of the second half are the NEGATED first half plus a sparse +-1 pattern e, so
    acc(first half) + acc(second half) = sum_k e[m,k] d[n,k]: at most 30 non-zeros of e per token,
    |d| <= 26, hence |total| <= 1560 per step exponent;
  * steps are 2^(e_n + b_g) with b_g in {0, 1}, token scales are powers of two: every fp32
    operation of the epilogue (Eq. 5 second half) is exact in any order, the total is below 2^11 in
    units of the smallest step, and the cast to fp16 rounds nothing.

So Y must equal the oracle's binary32 evaluation BIT FOR BIT, whatever order the kernel adds in; any
wrong, missing or doubled contribution of any k-tile, wave or K range changes an output.
"""
import numpy as np
import pytest
import torch

from gpu_util import dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import paper_2311_05161_amd as w
    w.load_library()  # raises if the HIP library has not been built: no fallback
    assert torch.cuda.is_available()
    return w


def _exact_operands(seed, M, K, N, G, amax=15, nnz=30):
    rng = np.random.default_rng(seed)
    Gs = G or K
    K2 = K // 2
    assert K % 256 == 0 and (G == 0 or K2 % G == 0)
    ng2 = max(1, K2 // Gs)                                   # groups in one half (per channel: one for all of K)
    a = rng.integers(-amax, amax + 1, size=(M, K2)).astype(np.int16)
    e = np.zeros((M, K2), np.int16)
    for m in range(M):
        pos = rng.choice(K2, size=min(nnz, K2), replace=False)
        e[m, pos] = rng.choice(np.array([-1, 1], np.int16), size=pos.size)
    Xq = np.concatenate([a, e - a], axis=1).astype(np.int8)
    c_half = rng.integers(0, 16, size=(N, K2)).astype(np.uint8)
    codes = np.concatenate([c_half, c_half], axis=1)
    z_half = rng.integers(0, 14, size=(N, ng2)).astype(np.uint8)
    expo = -(4 + (np.arange(N) % 5))[:, None] + rng.integers(0, 2, size=(N, ng2))
    s_half = np.exp2(expo).astype(np.float32)
    if G == 0:
        zero, step = z_half, s_half
    else:
        zero, step = np.concatenate([z_half, z_half], axis=1), np.concatenate([s_half, s_half], axis=1)
    sx = np.exp2(-(np.arange(M) % 4)).astype(np.float32)
    return Xq, sx, codes, np.ascontiguousarray(zero), np.ascontiguousarray(step)


def _exact_case(lib, oracle, seed, M, K, N, G, out_dtype=torch.float16):
    Xq, sx, codes, zero, step = _exact_operands(seed, M, K, N, G)
    acc = oracle.int_gemm(Xq, oracle.pack_dint4(codes), zero, G)
    y32, y64 = oracle.dequant_epilogue(acc, sx, step)
    # the premises: the binary32 evaluation is exact and the result needs at most 11 bits
    assert np.array_equal(y32.astype(np.float64), y64)
    units = y64 / (sx.astype(np.float64)[:, None] * 0.5 * step.min(axis=1).astype(np.float64)[None, :])
    assert np.array_equal(units, np.rint(units)) and np.abs(units).max() < 2048
    # large inside (group-wise: the group accumulators themselves; per channel the one accumulator is
    # the small total, the partial sums of waves, k-tiles and K ranges inside the kernel are not), not
    # trivial outside
    assert G == 0 or np.abs(acc).max() > 2000
    assert np.count_nonzero(y64) > 0.9 * y64.size
    want = oracle.cast_output(y32, "f16" if out_dtype == torch.float16 else "bf16")
    if out_dtype == torch.bfloat16:   # 8 significant bits: the cast may round; both sides round to nearest even
        pass
    else:
        assert np.array_equal(want, y32)
    Wp = lib.pack_dint4(dev(codes), lib.LAYOUT_TILED)
    Y = lib.w4a8_gemm(dev(Xq), dev(sx), Wp, dev(step), dev(zero), N, K, G, out_dtype=out_dtype)   # no hook
    got = host(Y).astype(np.float32)
    bad = got != want
    assert not bad.any(), (f"{bad.sum()} of {bad.size} outputs differ from the exact result; first at "
                           f"{np.argwhere(bad)[0]}: {got[bad][0]} != {want[bad][0]}")


# name, M, K, N, G -- with the kernel instance the shape is dispatched to
EXACT_CASES = [
    # streaming kernel (M <= 16)
    ("c2_m16_one_ntile_per_workgroup_no_ring", 16, 4096, 4096, 128),
    ("c2_m1", 1, 4096, 4096, 128),
    ("ring_group128_one_ktile_per_wave", 16, 512, 9232, 128),
    ("ring_group128_five_ktiles_per_wave", 16, 5120, 5120, 128),
    ("ring_group256_ragged_tokens", 7, 2560, 4400, 256),
    ("per_channel_no_ring_nine_ktiles_per_wave", 9, 9216, 1040, 0),
    ("per_channel_ring_nine_ktiles_per_wave", 16, 9216, 4640, 0),
    ("per_channel_ring_three_ktiles_per_wave", 5, 3072, 8208, 0),
    ("k_in_two_ranges_group128", 16, 9216, 48, 128),
    ("k_in_two_ranges_per_channel", 5, 11008, 32, 0),
    ("k_in_three_ranges_many_ntiles", 16, 13824, 5120, 128),
    # 16-token blocks of the streaming kernel
    ("token_blocks_m40_group128", 40, 512, 256, 128),
    ("token_blocks_m128_small_layer", 128, 1024, 528, 128),
    ("token_blocks_m50_per_channel", 50, 9216, 272, 0),
    ("token_blocks_k_in_two_ranges", 40, 5376, 272, 128),
    # tile kernel
    ("tile_256_rows_per_channel", 1024, 512, 8448, 0),
    ("tile_128_rows_per_channel_one_per_cu", 300, 768, 1040, 0),
    ("tile_128_rows_per_channel_two_per_cu", 2048, 256, 11008, 0),
    ("tile_128_rows_group128", 300, 768, 512, 128),
    ("tile_128_rows_group256_ragged", 270, 1024, 400, 256),
    ("tile_128_rows_group128_many_tiles", 1100, 512, 4112, 128),
    ("tile_128_rows_group128_last_round_k_ranges", 1100, 5120, 7696, 128),
    ("tile_k_ranges_group256", 130, 2048, 304, 256),
    ("tile_k_ranges_per_channel", 300, 2048, 304, 0),
    # K in four phases inside the workgroup (group-128, 129 .. 256 tokens, few output tiles)
    ("k_phases_group128", 130, 2048, 304, 128),
    ("k_phases_group128_ragged_last_super_step", 256, 2816, 1040, 128),
    ("k_phases_group128_40_ktiles", 130, 5120, 1040, 128),
    ("k_phases_per_channel", 130, 2048, 304, 0),
    ("k_phases_per_channel_ragged_last_super_step", 256, 2816, 1040, 0),
    ("k_phases_per_channel_86_ktiles", 200, 11008, 336, 0),
]


@pytest.mark.parametrize("case", EXACT_CASES, ids=[c[0] for c in EXACT_CASES])
def test_plain_instances_give_the_exact_result(lib, oracle, case):
    name, M, K, N, G = case
    _exact_case(lib, oracle, 100 + len(name), M, K, N, G)


def test_plain_instances_bf16_output(lib, oracle):
    """bf16 keeps 8 bits: the exact fp32 result is rounded once, to nearest even, on both sides."""
    _exact_case(lib, oracle, 7, 16, 4096, 4096, 128, out_dtype=torch.bfloat16)
    _exact_case(lib, oracle, 8, 300, 768, 1040, 0, out_dtype=torch.bfloat16)
    _exact_case(lib, oracle, 9, 300, 768, 512, 128, out_dtype=torch.bfloat16)
