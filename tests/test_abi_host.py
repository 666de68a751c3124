"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INCLUDE = os.path.join(ROOT, "include")


@pytest.fixture(scope="module")
def lib():
    import paper_2311_05161_amd as w
    if not os.path.exists(w.LIB_PATH):
        from paper_2311_05161_amd.build import build
        build()
    return w


def declared_functions():
    """Every function that any header under include/ declares."""
    names = set()
    for fn in sorted(os.listdir(INCLUDE)):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(INCLUDE, fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b([a-z_0-9]+)\s*\([^;{]*\)\s*;", text))
    return sorted(names)


def test_library_exports_every_declared_symbol(lib):
    names = declared_functions()
    assert {"quantize_act_int8", "quantize_weight_dint4", "pack_dint4", "unpack_dint4",
            "w4a8_gemm", "w4a8_gemm_workspace_bytes", "w4a8_status_string"} <= set(names)
    cdll = lib.load_library()
    for n in names:
        assert hasattr(cdll, n), f"{n} declared in w4a8.h but not exported"
    assert set(lib.EXPORTS) == set(names)


def test_status_strings(lib):
    seen = {lib.status_string(i) for i in range(6)}
    assert len(seen) == 6 and lib.status_string(0) == "ok"
    assert lib.status_string(99) == "unknown status"


def test_workspace_sizes(lib):
    # decode needs none with the tiled layout; per-channel prefill needs one row-sum per token
    assert lib.gemm_workspace_bytes(16, 4096, 4096, 128, lib.LAYOUT_TILED) == 0
    assert lib.gemm_workspace_bytes(2048, 4096, 4096, 128, lib.LAYOUT_TILED) == 0
    assert lib.gemm_workspace_bytes(2048, 4096, 4096, 0, lib.LAYOUT_TILED) == 2048 * 4
    need = lib.gemm_workspace_bytes(16, 4096, 4096, 128, lib.LAYOUT_CANONICAL)
    assert need == 4096 * 4096 // 2
    assert lib.gemm_workspace_bytes(16, 4096, 4096, 100, lib.LAYOUT_TILED) == 0  # invalid group
    # K > 5120 at decode is split over workgroups: fp32 partial sums [splits][M][N]
    assert lib.gemm_workspace_bytes(16, 5120, 13824, 128, lib.LAYOUT_TILED) == 3 * 16 * 5120 * 4
    assert lib.gemm_workspace_bytes(16, 13824, 5120, 128, lib.LAYOUT_TILED) == 0
    # per-channel weights: a workgroup covers up to 9216 columns, no split below that
    assert lib.gemm_workspace_bytes(16, 36864, 9216, 0, lib.LAYOUT_TILED) == 0
    assert lib.gemm_workspace_bytes(16, 4096, 11008, 0, lib.LAYOUT_TILED) == 2 * 16 * 4096 * 4
    # mid-size M with few output tiles: K is split as well (here 9 ranges of 12 k-tiles), and the
    # per-channel variant adds one row-sum per (range, token), 256-byte aligned before the partials
    part = 9 * 128 * 5120 * 4
    assert lib.gemm_workspace_bytes(128, 5120, 13824, 128, lib.LAYOUT_TILED) == part
    assert lib.gemm_workspace_bytes(128, 5120, 13824, 0, lib.LAYOUT_TILED) == 9 * 128 * 4 + part
    # 17 .. 64 tokens (.. 128 on small layers) run as 16-token blocks of the streaming kernel where K fits
    # one range: nothing needed
    assert lib.gemm_workspace_bytes(64, 5120, 5120, 128, lib.LAYOUT_TILED) == 0
    assert lib.gemm_workspace_bytes(17, 36864, 9216, 0, lib.LAYOUT_TILED) == 0
    # K in three ranges: fp32 partial sums of all 64 token rows
    assert lib.gemm_workspace_bytes(64, 5120, 13824, 128, lib.LAYOUT_TILED) == 3 * 64 * 5120 * 4
    assert lib.gemm_workspace_bytes(128, 4096, 4096, 128, lib.LAYOUT_TILED) == 0
    assert lib.gemm_workspace_bytes(128, 4096, 4096, 0, lib.LAYOUT_TILED) == 0
    # group-wise tiles of 128 x 128, 512 resident at a time: 16 x 40 tiles are one round and a quarter, so the
    # last 8 channel tiles (1024 channels) run with K in four ranges: their fp32 partial sums
    assert lib.gemm_workspace_bytes(2048, 5120, 5120, 128, lib.LAYOUT_TILED) == 4 * 2048 * 1024 * 4
    assert lib.gemm_workspace_bytes(2048, 4096, 4096, 128, lib.LAYOUT_TILED) == 0   # exactly one round
    # empty or invalid shapes size to nothing (and divide by nothing): an empty dimension, a K or a
    # group that is no multiple of 128, a channel count that is no multiple of 16
    L = lib.load_library()
    assert lib.gemm_workspace_bytes(32, 0, 1024, 0, lib.LAYOUT_TILED) == 0
    assert lib.gemm_workspace_bytes(0, 4096, 1024, 0, lib.LAYOUT_CANONICAL) == 0
    assert lib.gemm_workspace_bytes(2048, 0, 1024, 128, lib.LAYOUT_CANONICAL) == 0
    assert lib.gemm_workspace_bytes(32, 16, 0, 0, lib.LAYOUT_TILED) == 0
    assert lib.gemm_workspace_bytes(32, 16, 64, 0, lib.LAYOUT_TILED) == 0
    assert lib.gemm_workspace_bytes(32, 16, 65536 + 128, 0, lib.LAYOUT_TILED) == 0
    assert L.w4a8_gemm_special_workspace_bytes(1, 16, 32, 0, 1) == 0
    assert L.w4a8_gemm_special_workspace_bytes(1, 16, 0, 0, 1) == 0
    assert L.w4a8_gemm_special_workspace_bytes(1, 24, 128, 0, 1) == 0
    assert L.w4a8_gemm_special_workspace_bytes(1, 16, 256, 64, 1) == 0
    assert L.w4a8_gemm_special_workspace_bytes(1, 16, 256, 0, 7) == 0
    assert L.w4a8_gemm_special_workspace_bytes(40, 16, 32768 + 128, 0, 1) == 0
    # the no-op GEMM with an empty output and many tokens goes through the binding's workspace query
    assert L.w4a8_gemm(None, None, 32, None, 1, None, None, 0, 1024, 0, None, 1, 16, None, None, 0, None) == 0


def test_argument_errors_are_reported_before_any_launch(lib):
    """Fake non-null pointers are never dereferenced: validation happens on the host."""
    c = lib.load_library()
    P = ctypes.c_void_p(0x1000)  # 16-byte aligned, never touched
    Z = ctypes.c_void_p(0)
    from paper_2311_05161_amd import binding as b
    # activations
    assert c.quantize_act_int8(P, 7, 4, 128, 128, Z, P, P, Z) == b.ERR_DTYPE
    assert c.quantize_act_int8(P, b.F16, 4, 128, 64, Z, P, P, Z) == b.ERR_SHAPE
    assert c.quantize_act_int8(P, b.F16, -1, 128, 128, Z, P, P, Z) == b.ERR_SHAPE
    assert c.quantize_act_int8(P, b.F16, 4, 0, 0, Z, P, P, Z) == b.ERR_SHAPE
    assert c.quantize_act_int8(Z, b.F16, 4, 128, 128, Z, P, P, Z) == b.ERR_NULL
    assert c.quantize_act_int8(Z, b.F16, 0, 128, 128, Z, Z, Z, Z) == b.OK
    # weights
    assert c.quantize_weight_dint4(P, b.F16, 4, 128, 128, Z, 48, 0, P, P, P, Z) == b.ERR_SHAPE
    assert c.quantize_weight_dint4(P, 9, 4, 128, 128, Z, 0, 0, P, P, P, Z) == b.ERR_DTYPE
    assert c.quantize_weight_dint4(P, b.F16, 4, 128, 128, Z, 0, 0, Z, P, P, Z) == b.ERR_NULL
    # packing
    assert c.pack_dint4(P, 4, 127, P, 0, Z) == b.ERR_SHAPE
    assert c.pack_dint4(P, 8, 128, P, 1, Z) == b.ERR_SHAPE       # tiled needs N % 16 == 0
    assert c.pack_dint4(P, 16, 64, P, 1, Z) == b.ERR_SHAPE       # tiled needs K % 128 == 0
    assert c.pack_dint4(P, 16, 128, P, 5, Z) == b.ERR_DTYPE
    assert c.unpack_dint4(Z, 16, 128, P, 1, Z) == b.ERR_NULL
    # gemm
    def gemm(M=4, N=16, K=128, G=0, layout=1, ydt=b.F16, ldy=16, Xq=P, ws=Z, wsb=0, Wp=P):
        return c.w4a8_gemm(Xq, P, M, Wp, layout, P, P, N, K, G, P, ydt, ldy, Z, ws, wsb, Z)
    assert gemm(N=24) == b.ERR_SHAPE
    assert gemm(K=192) == b.ERR_SHAPE
    assert gemm(K=256, G=64) == b.ERR_SHAPE          # groups must be multiples of 128
    assert gemm(K=256, G=100) == b.ERR_SHAPE
    assert gemm(ldy=8) == b.ERR_SHAPE
    assert gemm(K=128 * 2048) == b.ERR_SHAPE         # beyond the int32-safe K
    assert gemm(K=65536 + 128) == b.ERR_SHAPE
    assert gemm(M=1 << 20, K=4096, ws=P, wsb=1 << 40) == b.ERR_SHAPE   # 32-bit offsets into Xq
    assert gemm(N=1 << 20, K=4096, ldy=1 << 20) == b.ERR_SHAPE         # 32-bit offsets into the weights
    assert gemm(ydt=b.F32) == b.ERR_DTYPE
    assert gemm(layout=3) == b.ERR_DTYPE
    assert gemm(Xq=Z) == b.ERR_NULL
    assert gemm(Xq=ctypes.c_void_p(0x1004)) == b.ERR_SHAPE   # int8 rows must be 16-byte aligned
    assert gemm(M=200) == b.ERR_WORKSPACE            # the tile kernel needs the row-sum workspace
    assert gemm(M=200, ws=P, wsb=8) == b.ERR_WORKSPACE
    assert gemm(layout=0) == b.ERR_WORKSPACE         # canonical weights are re-tiled into workspace
    assert gemm(M=0) == b.OK
    # the entry point on static scratch: the same argument errors, and a clear one beyond its limit
    def gemm_static(M=4, N=16, K=128, G=0, layout=1, ydt=b.F16, ldy=16, Xq=P):
        return c.w4a8_gemm_static(Xq, P, M, P, layout, P, P, N, K, G, P, ydt, ldy, Z, Z)
    limit = c.w4a8_gemm_static_scratch_bytes()
    assert limit == 64 << 20
    assert gemm_static(N=24) == b.ERR_SHAPE
    assert gemm_static(K=256, G=64) == b.ERR_SHAPE
    assert gemm_static(ldy=8) == b.ERR_SHAPE
    assert gemm_static(ydt=b.F32) == b.ERR_DTYPE
    assert gemm_static(layout=3) == b.ERR_DTYPE
    assert gemm_static(Xq=Z) == b.ERR_NULL
    assert gemm_static(Xq=ctypes.c_void_p(0x1004)) == b.ERR_SHAPE
    assert gemm_static(M=0) == b.OK
    assert lib.gemm_workspace_bytes(16, 16384, 16384, 0, 0) > limit      # canonical weights of 256 Mi codes
    assert gemm_static(M=16, N=16384, K=16384, ldy=16384, layout=0) == b.ERR_WORKSPACE
    assert lib.gemm_workspace_bytes(16, 800000, 5248, 128, 1) > limit    # two K ranges of a very tall layer
    assert gemm_static(M=16, N=800000, K=5248, G=128, ldy=800000) == b.ERR_WORKSPACE
    # asymmetric activations
    assert c.quantize_act_int8_asym(P, b.F16, 4, 128, 128, Z, P, P, Z, Z) == b.ERR_NULL   # zx missing
    assert c.quantize_act_int8_asym(P, b.F16, 4, 128, 64, Z, P, P, P, Z) == b.ERR_SHAPE
    assert c.quantize_act_int8_asym(P, 5, 4, 128, 128, Z, P, P, P, Z) == b.ERR_DTYPE
    assert c.dint4_weight_sums(P, P, 16, 128, 48, P, P, Z) == b.ERR_SHAPE
    assert c.dint4_weight_sums(P, P, 16, 192, 0, P, P, Z) == b.ERR_SHAPE     # tile sums need K % 128
    assert c.dint4_weight_sums(P, P, 16, 128, 0, Z, P, Z) == b.ERR_NULL

    def gemm_asym(zx=P, wsum=P, tsum=P, N=16):
        return c.w4a8_gemm_asym(P, P, zx, 4, P, 1, P, P, wsum, tsum, N, 128, 0, P, b.F16, 16, Z,
                                Z, 0, Z)
    assert gemm_asym(zx=Z) == b.ERR_NULL
    assert gemm_asym(wsum=Z) == b.ERR_NULL
    assert gemm_asym(tsum=Z) == b.ERR_NULL
    assert gemm_asym(N=24) == b.ERR_SHAPE

    # Value cache and the batched decode product
    def vq(dt=b.F16, B=2, T=256, D=128, ld_t=128, ld_b=256 * 128, G=0, V=P, codes=P):
        return c.quantize_value_dint4(V, dt, B, T, D, ld_t, ld_b, G, codes, P, P, Z)
    assert vq(dt=4) == b.ERR_DTYPE
    assert vq(ld_t=64) == b.ERR_SHAPE                # token stride below D
    assert vq(ld_b=-1) == b.ERR_SHAPE
    assert vq(G=100) == b.ERR_SHAPE                  # groups must divide T
    assert vq(B=1 << 17) == b.ERR_SHAPE
    assert vq(V=Z) == b.ERR_NULL
    assert vq(codes=Z) == b.ERR_NULL
    assert vq(B=0) == b.OK

    def batched(M=4, N=128, K=256, G=0, ydt=b.F16, ldy=128, batch=8, zx=Z, wsum=Z, Xq=P):
        return c.w4a8_gemm_batched(Xq, P, zx, M, P, P, P, wsum, wsum, N, K, G, P, ydt, ldy, batch, Z)
    assert batched(M=17) == b.ERR_SHAPE              # decode shapes only
    assert batched(K=9344) == b.ERR_SHAPE            # a single K-range per workgroup
    assert batched(K=5248, G=128) == b.ERR_SHAPE     # (5120 columns with token groups)
    assert batched(N=120) == b.ERR_SHAPE
    assert batched(K=192) == b.ERR_SHAPE
    assert batched(M=1, K=128, Xq=ctypes.c_void_p(0x1008)) == b.ERR_SHAPE
    assert batched(batch=1 << 16) == b.ERR_SHAPE
    assert batched(ldy=64) == b.ERR_SHAPE
    assert batched(ydt=b.F32) == b.ERR_DTYPE
    assert batched(Xq=Z) == b.ERR_NULL
    assert batched(zx=P, wsum=Z) == b.ERR_NULL       # a zero-point needs the weight sums
    assert batched(batch=0) == b.OK

    # AQAS scale search and clipping
    assert c.aqas_channel_absmax(P, 9, 4, 128, 128, P, Z) == b.ERR_DTYPE
    assert c.aqas_channel_absmax(P, b.F16, 4, 128, 64, P, Z) == b.ERR_SHAPE
    assert c.aqas_channel_absmax(P, b.F16, 4, 128, 128, Z, Z) == b.ERR_NULL
    assert c.aqas_scale(P, P, 128, 17, P, Z) == b.ERR_SHAPE          # grid points 0..16
    assert c.aqas_scale(P, Z, 128, 3, P, Z) == b.ERR_NULL
    need = lib.load_library().aqas_search_workspace_bytes(32, 64, 256, 0)
    assert need > 32 * 256 + 64 * 256 + 64 * 128 + 32 * 64 * 6
    assert lib.load_library().aqas_search_workspace_bytes(32, 60, 256, 0) == 0   # N % 16

    def search(dt=b.F16, M=32, N=64, K=256, ldx=256, G=0, X=P, ws=ctypes.c_void_p(0x10000), wsb=1 << 30,
               s_out=P):
        return c.aqas_search(X, P, dt, M, N, K, ldx, 256, G, s_out, P, P, ws, wsb, Z)
    assert search(dt=7) == b.ERR_DTYPE
    assert search(N=60) == b.ERR_SHAPE
    assert search(K=200) == b.ERR_SHAPE
    assert search(ldx=100) == b.ERR_SHAPE
    assert search(ldx=260) == b.ERR_SHAPE                            # fp16 rows must stay 16-byte aligned
    assert search(M=0) == b.ERR_SHAPE
    assert search(X=Z) == b.ERR_NULL
    assert search(ws=Z) == b.ERR_WORKSPACE
    assert search(wsb=1000) == b.ERR_WORKSPACE
    assert search(s_out=Z) == b.ERR_NULL
    assert c.dint4_clipped_params(P, b.F16, 16, 128, 128, Z, 0, Z, 11, P, P, Z) == b.ERR_SHAPE   # i = 0..10
    assert c.dint4_clipped_params(P, b.F16, 16, 128, 128, Z, 48, Z, 0, P, P, Z) == b.ERR_SHAPE
    assert c.dint4_clipped_params(P, b.F16, 16, 128, 128, Z, 0, Z, 0, Z, P, Z) == b.ERR_NULL
    assert c.aqas_clip_search(P, P, b.F16, 32, 64, 256, 256, 256, P, 0, Z, P, P, Z,
                              ctypes.c_void_p(0x10000), 1 << 30, Z) == b.ERR_NULL
    assert c.aqas_clip_search(P, P, b.F16, 32, 64, 256, 256, 256, P, 0, P, P, P, Z, Z, 0, Z) == b.ERR_WORKSPACE

    # weight-format variants, 3-bit packing, error split
    assert c.quantize_weight_format(P, b.F16, 16, 128, 128, Z, 0, 5, 0, P, P, P, Z) == b.ERR_DTYPE   # format id
    assert c.quantize_weight_format(P, b.F16, 16, 128, 64, Z, 0, 1, 0, P, P, P, Z) == b.ERR_SHAPE
    assert c.quantize_weight_format(P, b.F16, 16, 128, 128, Z, 0, 2, 0, Z, P, P, Z) == b.ERR_NULL
    assert c.w4a8_gemm_format(P, P, 4, P, 1, P, P, 16, 128, 0, 7, P, b.F16, 16, Z, Z, 0, Z) == b.ERR_DTYPE
    assert c.w4a8_gemm_format(P, P, 4, P, 1, P, P, 24, 128, 0, 1, P, b.F16, 24, Z, Z, 0, Z) == b.ERR_SHAPE
    assert c.pack_format(P, 16, 128, P, 1, 5, Z) == b.ERR_DTYPE
    assert c.pack_format(P, 8, 128, P, 1, 1, Z) == b.ERR_SHAPE
    assert c.unpack_format(Z, 16, 128, P, 1, 1, Z) == b.ERR_NULL
    assert c.pack_dint3(P, 4, 12, P, Z) == b.ERR_SHAPE               # eight codes per 24-bit word
    assert c.pack_dint3(Z, 4, 16, P, Z) == b.ERR_NULL
    assert c.unpack_dint3(P, 4, 16, Z, Z) == b.ERR_NULL
    assert c.unpack_dint3(P, 0, 16, Z, Z) == b.OK
    # special value step/4, step/8: expansion to double width and the GEMM on it
    assert c.expand_special_value(P, P, P, 16, 128, 0, 0, P, P, P, Z) == b.ERR_DTYPE     # only formats 3, 4
    assert c.expand_special_value(P, P, P, 16, 128, 48, 3, P, P, P, Z) == b.ERR_SHAPE
    assert c.expand_special_value(P, P, P, 16, 128, 0, 3, P, Z, P, Z) == b.ERR_NULL
    assert c.expand_special_value(P, P, P, 0, 128, 0, 4, Z, Z, Z, Z) == b.OK
    L = lib.load_library()
    assert L.w4a8_gemm_special_workspace_bytes(4, 16, 256, 128, 1) >= 4 * 512
    assert (L.w4a8_gemm_special_workspace_bytes(4, 16, 256, 128, 1)
            == 2048 + L.w4a8_gemm_workspace_bytes(4, 16, 512, 128, 1))
    assert L.w4a8_gemm_special_workspace_bytes(4, 16, 256, 100, 1) == 0
    WS = ctypes.c_void_p(0x10000)

    def special(M=4, N=16, K=256, G=128, X=ctypes.c_void_p(0x2000), ws=WS, wsb=1 << 30, Y=P, yd=b.F16, ldy=16):
        return c.w4a8_gemm_special(X, P, M, P, 1, P, P, N, K, G, Y, yd, ldy, Z, ws, wsb, Z)
    assert special(K=200) == b.ERR_SHAPE
    assert special(K=32768 + 128) == b.ERR_SHAPE                     # 2K <= 65536
    assert special(N=24) == b.ERR_SHAPE
    assert special(ldy=8) == b.ERR_SHAPE
    assert special(yd=b.F32) == b.ERR_DTYPE
    assert special(X=Z) == b.ERR_NULL
    assert special(X=ctypes.c_void_p(0x2004)) == b.ERR_SHAPE
    assert special(Y=Z) == b.ERR_NULL
    assert special(ws=Z) == b.ERR_WORKSPACE
    assert special(wsb=100) == b.ERR_WORKSPACE
    assert special(M=0) == b.OK
    need = lib.load_library().dint_error_terms_workspace_bytes(8, 16, 128, 0)
    assert need >= 16 * 128 * 9 + 8 * 128 * 4 + 2 * 8 * 16 * 4
    W0 = ctypes.c_void_p(0x10000)
    assert c.dint_error_terms(P, b.F16, 8, 128, 128, P, b.F16, 16, 128, Z, 0, 9, P, W0, 1 << 30, Z) == b.ERR_DTYPE
    assert c.dint_error_terms(P, b.F16, 8, 128, 100, P, b.F16, 16, 128, Z, 0, 0, P, W0, 1 << 30, Z) == b.ERR_SHAPE
    assert c.dint_error_terms(P, b.F16, 8, 128, 128, P, b.F16, 16, 128, Z, 0, 0, Z, W0, 1 << 30, Z) == b.ERR_NULL
    assert c.dint_error_terms(P, b.F16, 8, 128, 128, P, b.F16, 16, 128, Z, 0, 0, P, W0, 100, Z) == b.ERR_WORKSPACE
    # the two measurement aids
    assert c.w4a8_measure_stream_read(Z, 1024, Z, Z) == b.ERR_NULL
    assert c.w4a8_measure_stream_read(P, 1000, Z, Z) == b.ERR_SHAPE
    assert c.w4a8_measure_stream_read(ctypes.c_void_p(0x1008), 1024, Z, Z) == b.ERR_SHAPE
    assert c.w4a8_measure_stream_read(P, 0, Z, Z) == b.OK
    assert c.w4a8_measure_mfma_i8(-1, Z, Z, Z) == b.ERR_SHAPE
    assert c.w4a8_measure_mfma_i8((1 << 24) + 1, Z, Z, Z) == b.ERR_SHAPE
    assert c.w4a8_measure_ktile_mix(-1, 0, Z, Z) == b.ERR_SHAPE
    assert c.w4a8_measure_ktile_mix((1 << 24) + 1, 1, Z, Z) == b.ERR_SHAPE


def test_linear_argument_errors_before_any_launch(lib):
    """w4a8_linear: every call here is rejected (or is a no-op) on the host; nothing is launched."""
    import ctypes
    L = lib.load_library()
    P, Z = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    F16 = lib.F16
    def call(X=P, dt=F16, M=4, K=128, ldx=128, N=16, G=0, layout=1, Y=P, ydt=F16, ldy=16, ws=Z, wsb=0, Xq=Z):
        return L.w4a8_linear(X, dt, M, K, ldx, Z, P, layout, P, P, N, G, Y, ydt, ldy, Xq, Z, Z, ws, wsb, Z)
    assert call(M=0) == 0
    assert call(dt=7) == 3 and call(ydt=lib.F32) == 3 and call(layout=5) == 3
    assert call(N=24) == 2 and call(K=192) == 2 and call(ldx=64) == 2 and call(ldy=8) == 2
    assert call(X=Z) == 1 and call(Y=Z) == 1
    assert call(Xq=ctypes.c_void_p(0x1004)) == 2
    assert call(M=40) == 4                       # two steps: workspace needed
    assert call(dt=lib.BF16) == 4
    assert call(M=40, ws=ctypes.c_void_p(0x10000), wsb=100) == 4


def test_product_path_has_no_cpu_fallback(lib, tmp_path):
    with pytest.raises(FileNotFoundError):
        lib.load_library(str(tmp_path / "missing_libw4a8.so"))
