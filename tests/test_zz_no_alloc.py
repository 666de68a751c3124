"""w4a8_gemm_static -- the GEMM entry point that allocates nothing (its workspace is a static device
array inside the library) -- against w4a8_gemm, through the C ABI.

Both run the same kernels, so Y and the int32 accumulators must be bit-identical.  Every case makes
two calls in a row on the shared array, the second with a smaller input: what the first call left
behind must not leak into the second.
"""
import ctypes

import numpy as np
import pytest
import torch

import synthetic_inputs as syn
from gpu_util import dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import paper_2311_05161_amd as w
    w.load_library()  # raises if the HIP library has not been built: no fallback
    assert torch.cuda.is_available()
    return w


def _operands(lib, seed, M, K, N, G, layout):
    X, W, s = syn.random_layer(seed, M, K, N)
    Xq, sx = lib.quantize_act_int8(dev(X), dev(s))
    codes, step, zero = lib.quantize_weight_dint4(dev(W), dev(s), G)
    return Xq, sx, lib.pack_dint4(codes, layout), step, zero


def _static_call(lib, ops, M, K, N, G, layout, out_dtype, want_acc):
    """One call of the C entry point itself; outputs pre-filled so that untouched elements show."""
    Xq, sx, Wp, step, zero = ops
    Gs = G or K
    Y = torch.full((M, N), -3.0, dtype=out_dtype, device="cuda")
    acc = torch.full((M, N, K // Gs), 12345, dtype=torch.int32, device="cuda") if want_acc else None
    P = lambda t: None if t is None else ctypes.c_void_p(t.data_ptr())
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    dt = {torch.float16: lib.F16, torch.bfloat16: lib.BF16}[out_dtype]
    rc = lib.load_library().w4a8_gemm_static(P(Xq), P(sx), M, P(Wp), layout, P(step), P(zero), N, K, G,
                                             P(Y), dt, N, P(acc), st)
    assert rc == 0, lib.status_string(rc)
    return Y, acc


# (name, first call, second smaller call); a call = (M, K, N, G, layout).  What each pair keeps in the
# scratch array is named; the last pair needs none (the array is never asked for).
PAIRS = [
    ("decode_k_ranges_fp32_partials", (16, 9216, 48, 128, 1), (5, 5248, 32, 128, 1)),
    ("decode_k_ranges_int32_partials_per_channel", (9, 11008, 64, 0, 1), (3, 9344, 16, 0, 1)),
    ("token_blocks_k_ranges", (40, 5248, 272, 128, 1), (24, 5248, 48, 128, 1)),
    ("tile_kernel_row_sums", (300, 768, 1040, 0, 1), (150, 512, 272, 0, 1)),
    ("tile_kernel_k_ranges_and_row_sums", (200, 2048, 304, 0, 1), (129, 1024, 64, 0, 1)),
    ("tile_kernel_k_ranges_group_wise", (130, 1024, 304, 128, 1), (129, 1024, 48, 128, 1)),
    ("canonical_weights_retiled", (9, 512, 64, 128, 0), (70, 256, 48, 0, 0)),
    ("large_then_tiny", (256, 11008, 4096, 0, 1), (1, 128, 16, 128, 0)),
    ("no_scratch_needed", (16, 4096, 4096, 128, 1), (7, 1280, 400, 256, 1)),
]


@pytest.mark.parametrize("pair", PAIRS, ids=[p[0] for p in PAIRS])
@pytest.mark.parametrize("out_dtype", [torch.float16, torch.bfloat16], ids=["f16", "bf16"])
def test_static_scratch_gemm_matches_w4a8_gemm(lib, pair, out_dtype):
    name, first, second = pair
    need = [lib.gemm_workspace_bytes(M, N, K, G, layout) for (M, K, N, G, layout) in (first, second)]
    assert (need[0] > 0) == (name != "no_scratch_needed")
    assert max(need) <= lib.load_library().w4a8_gemm_static_scratch_bytes()
    ops = [_operands(lib, 900 + i + len(name), M, K, N, G, layout)
           for i, (M, K, N, G, layout) in enumerate((first, second))]
    for want_acc in (False, True):
        # the two calls back to back on the stream, nothing in between
        got = [_static_call(lib, o, M, K, N, G, layout, out_dtype, want_acc)
               for o, (M, K, N, G, layout) in zip(ops, (first, second))]
        for (Y, acc), o, (M, K, N, G, layout) in zip(got, ops, (first, second)):
            Xq, sx, Wp, step, zero = o
            ref = lib.w4a8_gemm(Xq, sx, Wp, step, zero, N, K, G, layout=layout, out_dtype=out_dtype,
                                want_acc=want_acc)
            Yr, accr = ref if want_acc else (ref, None)
            torch.cuda.synchronize()
            assert torch.equal(Y, Yr), f"{name}: Y differs (M={M} K={K} N={N} G={G})"
            if want_acc:
                assert torch.equal(acc, accr), f"{name}: accumulators differ"


def test_static_scratch_gemm_against_the_oracle(lib, oracle):
    """Not only equal to w4a8_gemm: a K-range shape against the CPU oracle itself, second call smaller."""
    from gpu_util import assert_y_close, host
    for (M, K, N, G) in ((16, 9216, 48, 128), (5, 5248, 32, 128)):
        X, W, s = syn.random_layer(31 + M, M, K, N)
        r = oracle.linear_w4a8(X, W, s, G)
        ops = _operands(lib, 31 + M, M, K, N, G, 1)
        Y, acc = _static_call(lib, ops, M, K, N, G, 1, torch.float16, True)
        assert np.array_equal(host(acc), r["acc"])
        assert_y_close(host(Y), r["Y64"])


def test_static_scratch_gemm_empty_and_view(lib):
    """M == 0 is a no-op; Y may be a view of a wider buffer (columns outside stay untouched)."""
    L = lib.load_library()
    assert L.w4a8_gemm_static(None, None, 0, None, 1, None, None, 32, 128, 0, None, lib.F16, 32, None, None) == 0
    M, K, N, G = 16, 9216, 48, 128
    ops = _operands(lib, 5, M, K, N, G, 1)
    Xq, sx, Wp, step, zero = ops
    ref = lib.w4a8_gemm(Xq, sx, Wp, step, zero, N, K, G)
    big = torch.full((M, N + 8), -7.0, dtype=torch.float16, device="cuda")
    view = big[:, 4:4 + N]
    out = lib.w4a8_gemm_static(Xq, sx, Wp, step, zero, N, K, G, Y=view)
    torch.cuda.synchronize()
    assert out.data_ptr() == view.data_ptr() and torch.equal(view, ref)
    assert bool((big[:, :4] == -7.0).all()) and bool((big[:, 4 + N:] == -7.0).all())
