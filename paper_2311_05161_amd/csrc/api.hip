// The C ABI of w4a8.h: host-side argument validation and dispatch.  No allocation, no state,
// no synchronization; every error is reported before anything is launched.
#include "w4a8_common.hpp"

using namespace w4a8;

namespace {

constexpr int64_t MAX_K = 65536;   // keeps the biased int32 accumulators far below 2^31
constexpr size_t WS_ALIGN = 256;

inline size_t align_up(size_t v) { return (v + WS_ALIGN - 1) / WS_ALIGN * WS_ALIGN; }
inline bool valid_dtype(int d) { return d == W4A8_F32 || d == W4A8_F16 || d == W4A8_BF16; }
inline bool valid_layout(int l) { return l == W4A8_LAYOUT_CANONICAL || l == W4A8_LAYOUT_TILED; }

// group_size 0 means "per output channel"
inline bool resolve_group(int64_t K, int64_t &G)
{
    if (G == 0) G = K;
    return G > 0 && K > 0 && K % G == 0;
}

// the shape limits of the GEMM entry points (G already resolved): what the kernels' tiles, 32-bit
// offsets and launch plans assume.  Everything that sizes a workspace or plans a launch checks
// this first, so no plan ever sees an empty dimension.
inline bool gemm_shape_ok(int64_t M, int64_t N, int64_t K, int64_t G)
{
    if (M < 0 || N < 0 || K < TILE_K || G < TILE_K || K % G != 0) return false;
    if (N % TILE_N != 0 || K % TILE_K != 0 || G % TILE_K != 0 || K > MAX_K) return false;
    if (M > 0x7fffffffLL || N * K / 2 > 0x7fffffffLL) return false;   // 32-bit byte offsets into the weights
    // the tile kernel addresses Xq with 32-bit byte offsets and numbers its tiles in 32 bits
    if (M > 16 && (M * K > 0x7fffffffLL || (M + 63) / 64 * ((N + 255) / 256) > 0x1ffffLL)) return false;
    return true;
}

struct WsPlan {
    size_t repack_off, repack_bytes;  // canonical -> tiled copy of the weights
    size_t rs_off, rs_bytes;          // per-token row-sums (M > 16, per-channel weights only)
    size_t part_off, part_bytes;      // fp32 partial sums [splits][M][N] of a launch that splits K
    size_t total;
};

WsPlan plan_workspace(int64_t M, int64_t N, int64_t K, int64_t G, int layout)
{
    WsPlan w{0, 0, 0, 0, 0, 0, 0};
    size_t off = 0;
    if (layout == W4A8_LAYOUT_CANONICAL) {
        w.repack_off = off;
        w.repack_bytes = (size_t)(N * K / 2);
        off = align_up(off + w.repack_bytes);
    }
    if (M > 16 && gemv_token_blocks(M, N, K, G) == 0) {
        const GemmPlan gp = plan_gemm(M, N, K, G);
        w.rs_off = off;            // per-channel weights: bias removal needs row-sums per token
        w.rs_bytes = gp.rs_bytes;
        off = align_up(off + w.rs_bytes);
        w.part_off = off;          // few output tiles: K is split, fp32 partial sums
        w.part_bytes = gp.partial_bytes;
        off = align_up(off + w.part_bytes);
    } else if (M > 0 && N > 0) {
        // the streaming kernel (M <= 16, or a few 16-token blocks): fp32 partial sums when K is cut
        const int nb = M > 16 ? gemv_token_blocks(M, N, K, G) : 1;
        const GemvPlan gp = plan_gemv(M > 16 ? 16 : M, N, K, G, nb);
        w.part_off = off;
        w.part_bytes = gp.splits > 1 ? (size_t)gp.splits * M * N * sizeof(float) : 0;
        off = align_up(off + w.part_bytes);
    }
    w.total = off;
    return w;
}

// w4a8_gemm and w4a8_gemm_asym (zx, wsum, tsum null for the former)
int gemm_common(const int8_t *Xq, const float *sx, const int32_t *zx, int64_t M,
                const uint8_t *Wp, int layout, const float *step, const uint8_t *zero,
                const int32_t *wsum, const int32_t *tsum, int64_t N, int64_t K, int64_t group_size,
                void *Y, int y_dtype, int64_t ldy,
                int32_t *acc_out, void *workspace, size_t workspace_bytes, void *stream,
                int format = W4A8_FMT_DINT4, bool validate_only = false)
{
    if (!valid_layout(layout)) return W4A8_ERR_DTYPE;
    if (format != W4A8_FMT_DINT4 && format != W4A8_FMT_INT4 && format != W4A8_FMT_DINT3) return W4A8_ERR_DTYPE;
    const int plain = format == W4A8_FMT_INT4;   // dINT3 lives in dINT4's code space: nothing to change
    if (y_dtype != W4A8_F16 && y_dtype != W4A8_BF16) return W4A8_ERR_DTYPE;
    int64_t G = group_size;
    if (M < 0 || N < 0 || !resolve_group(K, G)) return W4A8_ERR_SHAPE;
    if (!gemm_shape_ok(M, N, K, G) || ldy < N) return W4A8_ERR_SHAPE;
    if (M == 0 || N == 0) return W4A8_OK;
    if (!Xq || !sx || !Wp || !step || !zero || !Y) return W4A8_ERR_NULL;
    if ((uintptr_t)Xq % 16 != 0 || (uintptr_t)Wp % 16 != 0 || (uintptr_t)Y % 2 != 0 ||
        (acc_out && (uintptr_t)acc_out % 4 != 0))
        return W4A8_ERR_SHAPE;

    const WsPlan ws = plan_workspace(M, N, K, G, layout);
    if (ws.total > 0) {
        if (!workspace || workspace_bytes < ws.total) return W4A8_ERR_WORKSPACE;
        if ((uintptr_t)workspace % WS_ALIGN != 0) return W4A8_ERR_WORKSPACE;
    }
    if (validate_only) return W4A8_OK;
    hipStream_t st = (hipStream_t)stream;
    uint8_t *wsb = (uint8_t *)workspace;
    const ZeroPoint zp = {zx, wsum, tsum};

    const uint8_t *Wt = Wp;
    if (layout == W4A8_LAYOUT_CANONICAL) {
        uint8_t *tiled = wsb + ws.repack_off;
        const int rc = launch_repack_canonical_to_tiled(Wp, N, K, tiled, st, plain);
        if (rc != W4A8_OK) return rc;
        Wt = tiled;
    }
    if (M <= 16 || gemv_token_blocks(M, N, K, G) > 0) {   // the streaming kernel, also for a few 16-token blocks
        if (acc_out) {  // the split-K waves add exact partial sums into it
            const int rc = launch_fill_i32(acc_out, M * N * (K / G), 0, st);
            if (rc != W4A8_OK) return rc;
        }
        const int rc = launch_gemv(Xq, sx, zp, M, Wt, step, zero, N, K, G, Y, y_dtype, ldy,
                                   acc_out, (float *)(wsb + ws.part_off), 1, st, plain);
        if (rc != W4A8_OK || !zx || !acc_out) return rc;
        return launch_acc_zero_point(acc_out, zx, wsum, M, N * (K / G), st);
    }
    if (acc_out && ws.part_bytes > 0 && G == K) {  // K-split workgroups add exact partial sums
        const int rc = launch_fill_i32(acc_out, M * N, 0, st);
        if (rc != W4A8_OK) return rc;
    }
    const int rc = launch_gemm(Xq, sx, zp, (int32_t *)(wsb + ws.rs_off), M, Wt, step, zero, N,
                               K, G, Y, y_dtype, ldy, acc_out, (float *)(wsb + ws.part_off), st, plain);
    if (rc != W4A8_OK || !zx || !acc_out) return rc;
    return launch_acc_zero_point(acc_out, zx, wsum, M, N * (K / G), st);
}

}  // namespace

extern "C" {

int w4a8_measure_stream_read(const void *buf, int64_t bytes, uint32_t *sink, void *stream)
{
    if (buf == nullptr) return W4A8_ERR_NULL;
    if (bytes < 0 || bytes % 16 != 0 || (uintptr_t)buf % 16 != 0) return W4A8_ERR_SHAPE;
    if (bytes == 0) return W4A8_OK;
    return launch_stream_read(buf, bytes, sink, (hipStream_t)stream);
}

int w4a8_measure_mfma_i8(int64_t iters, uint32_t *sink, int64_t *ops, void *stream)
{
    if (iters < 0 || iters > (1LL << 24)) return W4A8_ERR_SHAPE;
    return launch_mfma_i8_loop(iters, sink, ops, (hipStream_t)stream);
}

int w4a8_measure_ktile_mix(int64_t iters, int fragment_reads, uint32_t *sink, void *stream)
{
    if (iters < 0 || iters > (1LL << 24)) return W4A8_ERR_SHAPE;
    return launch_ktile_mix(iters, fragment_reads, sink, (hipStream_t)stream);
}

const char *w4a8_status_string(int status)
{
    switch (status) {
        case W4A8_OK: return "ok";
        case W4A8_ERR_NULL: return "null pointer";
        case W4A8_ERR_SHAPE: return "invalid shape, leading dimension, group size or alignment";
        case W4A8_ERR_DTYPE: return "unsupported element type or layout";
        case W4A8_ERR_WORKSPACE: return "workspace missing or too small";
        case W4A8_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

int quantize_act_int8(const void *X, int x_dtype, int64_t M, int64_t K, int64_t ldx,
                      const float *s, int8_t *Xq, float *sx, void *stream)
{
    if (!valid_dtype(x_dtype)) return W4A8_ERR_DTYPE;
    if (M < 0 || K < 1 || ldx < K || M > 0x7fffffffLL) return W4A8_ERR_SHAPE;
    if (M == 0) return W4A8_OK;
    if (!X || !Xq || !sx) return W4A8_ERR_NULL;
    return launch_act_quant(X, x_dtype, M, K, ldx, s, Xq, sx, nullptr, (hipStream_t)stream);
}

int quantize_act_int8_asym(const void *X, int x_dtype, int64_t M, int64_t K, int64_t ldx,
                           const float *s, int8_t *Xq, float *sx, int32_t *zx, void *stream)
{
    if (!valid_dtype(x_dtype)) return W4A8_ERR_DTYPE;
    if (M < 0 || K < 1 || ldx < K || M > 0x7fffffffLL) return W4A8_ERR_SHAPE;
    if (M == 0) return W4A8_OK;
    if (!X || !Xq || !sx || !zx) return W4A8_ERR_NULL;
    return launch_act_quant(X, x_dtype, M, K, ldx, s, Xq, sx, zx, (hipStream_t)stream);
}

int dint4_weight_sums(const uint8_t *codes, const uint8_t *zero, int64_t N, int64_t K,
                      int64_t group_size, int32_t *wsum, int32_t *tsum, void *stream)
{
    int64_t G = group_size;
    if (N < 0 || K < 1 || !resolve_group(K, G)) return W4A8_ERR_SHAPE;
    if (tsum && (K % TILE_K != 0 || G % TILE_K != 0)) return W4A8_ERR_SHAPE;
    if (N == 0) return W4A8_OK;
    if (!codes || !zero || !wsum) return W4A8_ERR_NULL;
    int rc = launch_weight_sums(codes, zero, N, K, G, G, wsum, (hipStream_t)stream);
    if (rc != W4A8_OK || !tsum) return rc;
    return launch_weight_sums(codes, zero, N, K, G, TILE_K, tsum, (hipStream_t)stream);
}

int quantize_weight_dint4(const void *W, int w_dtype, int64_t N, int64_t K, int64_t ldw,
                          const float *s, int64_t group_size, int use_given_params,
                          uint8_t *codes, float *step, uint8_t *zero, void *stream)
{
    if (!valid_dtype(w_dtype)) return W4A8_ERR_DTYPE;
    int64_t G = group_size;
    if (N < 0 || K < 1 || ldw < K || !resolve_group(K, G)) return W4A8_ERR_SHAPE;
    if (N == 0) return W4A8_OK;
    if (!W || !codes || !step || !zero) return W4A8_ERR_NULL;
    return launch_weight_quant(W, w_dtype, N, K, ldw, s, G, use_given_params, codes, step, zero,
                               W4A8_FMT_DINT4, (hipStream_t)stream);
}

int quantize_value_dint4(const void *V, int v_dtype, int64_t batch, int64_t T, int64_t D,
                         int64_t ld_t, int64_t ld_b, int64_t group_size, uint8_t *codes,
                         float *step, uint8_t *zero, void *stream)
{
    if (!valid_dtype(v_dtype)) return W4A8_ERR_DTYPE;
    int64_t G = group_size;
    if (batch < 0 || D < 0 || T < 1 || ld_t < D || !resolve_group(T, G)) return W4A8_ERR_SHAPE;
    if (ld_b < 0) return W4A8_ERR_SHAPE;
    if (batch > 65535 || T / G > 65535 || batch * D * T > 0x3fffffffffffLL) return W4A8_ERR_SHAPE;
    if (batch == 0 || D == 0) return W4A8_OK;
    if (!V || !codes || !step || !zero) return W4A8_ERR_NULL;
    return launch_value_quant(V, v_dtype, batch, T, D, ld_t, ld_b, G, codes, step, zero,
                              (hipStream_t)stream);
}

static int check_pack_shape(int64_t N, int64_t K, int layout)
{
    if (!valid_layout(layout)) return W4A8_ERR_DTYPE;
    if (N < 0 || K < 1) return W4A8_ERR_SHAPE;
    if (layout == W4A8_LAYOUT_CANONICAL ? (K % 2 != 0) : (N % TILE_N != 0 || K % TILE_K != 0))
        return W4A8_ERR_SHAPE;
    return W4A8_OK;
}

int pack_dint4(const uint8_t *codes, int64_t N, int64_t K, uint8_t *packed, int layout,
               void *stream)
{
    const int rc = check_pack_shape(N, K, layout);
    if (rc != W4A8_OK) return rc;
    if (N == 0) return W4A8_OK;
    if (!codes || !packed) return W4A8_ERR_NULL;
    if (layout == W4A8_LAYOUT_TILED && (uintptr_t)packed % 4 != 0) return W4A8_ERR_SHAPE;
    return launch_pack(codes, N, K, packed, layout, (hipStream_t)stream);
}

int unpack_dint4(const uint8_t *packed, int64_t N, int64_t K, uint8_t *codes, int layout,
                 void *stream)
{
    const int rc = check_pack_shape(N, K, layout);
    if (rc != W4A8_OK) return rc;
    if (N == 0) return W4A8_OK;
    if (!codes || !packed) return W4A8_ERR_NULL;
    if (layout == W4A8_LAYOUT_TILED && (uintptr_t)packed % 4 != 0) return W4A8_ERR_SHAPE;
    return launch_unpack(packed, N, K, codes, layout, (hipStream_t)stream);
}

size_t w4a8_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t group_size, int layout)
{
    int64_t G = group_size;
    if (!resolve_group(K, G) || !gemm_shape_ok(M, N, K, G) || !valid_layout(layout) || M == 0 || N == 0)
        return 0;
    return plan_workspace(M, N, K, G, layout).total;
}

int w4a8_gemm(const int8_t *Xq, const float *sx, int64_t M,
              const uint8_t *Wp, int layout, const float *step, const uint8_t *zero,
              int64_t N, int64_t K, int64_t group_size,
              void *Y, int y_dtype, int64_t ldy,
              int32_t *acc_out, void *workspace, size_t workspace_bytes, void *stream)
{
    return gemm_common(Xq, sx, nullptr, M, Wp, layout, step, zero, nullptr, nullptr, N, K,
                       group_size, Y, y_dtype, ldy, acc_out, workspace, workspace_bytes, stream);
}

int w4a8_gemm_asym(const int8_t *Xq, const float *sx, const int32_t *zx, int64_t M,
                   const uint8_t *Wp, int layout, const float *step, const uint8_t *zero,
                   const int32_t *wsum, const int32_t *tsum,
                   int64_t N, int64_t K, int64_t group_size,
                   void *Y, int y_dtype, int64_t ldy,
                   int32_t *acc_out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (M > 0 && N > 0 && (!zx || !wsum || !tsum)) return W4A8_ERR_NULL;
    return gemm_common(Xq, sx, zx, M, Wp, layout, step, zero, wsum, tsum, N, K, group_size, Y,
                       y_dtype, ldy, acc_out, workspace, workspace_bytes, stream);
}

int w4a8_gemm_batched(const int8_t *Xq, const float *sx, const int32_t *zx, int64_t M,
                      const uint8_t *Wp, const float *step, const uint8_t *zero,
                      const int32_t *wsum, const int32_t *tsum,
                      int64_t N, int64_t K, int64_t group_size,
                      void *Y, int y_dtype, int64_t ldy, int64_t batch, void *stream)
{
    if (y_dtype != W4A8_F16 && y_dtype != W4A8_BF16) return W4A8_ERR_DTYPE;
    int64_t G = group_size;
    if (M < 0 || N < 0 || batch < 0 || !resolve_group(K, G)) return W4A8_ERR_SHAPE;
    // the decode kernel only, one K-range per workgroup, 32-bit offsets inside one problem
    if (M > 16 || N % TILE_N != 0 || K % TILE_K != 0 || G % TILE_K != 0 || K > (G == K ? 9216 : 5120) || ldy < N ||
        N * K / 2 > 0x7fffffffLL || batch > 65535)
        return W4A8_ERR_SHAPE;
    if (M == 0 || N == 0 || batch == 0) return W4A8_OK;
    if (!Xq || !sx || !Wp || !step || !zero || !Y) return W4A8_ERR_NULL;
    if (zx && (!wsum || !tsum)) return W4A8_ERR_NULL;
    if ((uintptr_t)Xq % 16 != 0 || (M * K) % 16 != 0 || (uintptr_t)Wp % 16 != 0 ||
        (uintptr_t)Y % 2 != 0)
        return W4A8_ERR_SHAPE;
    const ZeroPoint zp = {zx, zx ? wsum : nullptr, zx ? tsum : nullptr};
    return launch_gemv(Xq, sx, zp, M, Wp, step, zero, N, K, G, Y, y_dtype, ldy, nullptr, nullptr,
                       batch, (hipStream_t)stream);
}


// ---- the whole layer in one call -----------------------------------------------------------------
}  // extern "C"

namespace {

struct LinearWs {
    size_t xq, sx, gemm, gemm_bytes, total;
};
LinearWs plan_linear(int64_t M, int64_t N, int64_t K, int64_t G, int layout)
{
    LinearWs w{};
    size_t off = 0;
    w.xq = off;
    off = align_up(off + (size_t)(M * K));
    w.sx = off;
    off = align_up(off + (size_t)M * sizeof(float));
    w.gemm = off;
    w.gemm_bytes = plan_workspace(M, N, K, G, layout).total;
    w.total = off + w.gemm_bytes;
    return w;
}

}  // namespace

extern "C" {

size_t w4a8_linear_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t group_size, int layout)
{
    int64_t G = group_size;
    if (!resolve_group(K, G) || !gemm_shape_ok(M, N, K, G) || !valid_layout(layout) || M == 0 || N == 0)
        return 0;
    return plan_linear(M, N, K, G, layout).total;
}

int w4a8_linear(const void *X, int x_dtype, int64_t M, int64_t K, int64_t ldx, const float *s,
                const uint8_t *Wp, int layout, const float *step, const uint8_t *zero,
                int64_t N, int64_t group_size, void *Y, int y_dtype, int64_t ldy,
                int8_t *Xq_out, float *sx_out, int32_t *acc_out,
                void *workspace, size_t workspace_bytes, void *stream)
{
    if (!valid_dtype(x_dtype) || !valid_layout(layout)) return W4A8_ERR_DTYPE;
    if (y_dtype != W4A8_F16 && y_dtype != W4A8_BF16) return W4A8_ERR_DTYPE;
    int64_t G = group_size;
    if (M < 0 || N < 0 || !resolve_group(K, G)) return W4A8_ERR_SHAPE;
    if (!gemm_shape_ok(M, N, K, G) || ldy < N || ldx < K) return W4A8_ERR_SHAPE;
    if (M == 0 || N == 0) return W4A8_OK;
    if (!X || !Wp || !step || !zero || !Y) return W4A8_ERR_NULL;
    if ((uintptr_t)Wp % 16 != 0 || (uintptr_t)Y % 2 != 0 || (acc_out && (uintptr_t)acc_out % 4 != 0) ||
        (Xq_out && (uintptr_t)Xq_out % 16 != 0))
        return W4A8_ERR_SHAPE;
    hipStream_t st = (hipStream_t)stream;

    // At most 16 tokens of fp16 activations on tiled weights whose K the streaming kernel takes in one
    // range: ONE launch, the activations are quantized inside it.
    const bool one_launch = M <= 16 && x_dtype == W4A8_F16 && layout == W4A8_LAYOUT_TILED &&
                            (uintptr_t)X % 16 == 0 && ldx % 8 == 0 && ldx <= (1LL << 24) &&
                            gemv_can_fuse(M, N, K, G);
    if (one_launch) {
        if (acc_out) {  // the compute waves add exact partial sums into it
            const int rc = launch_fill_i32(acc_out, M * N * (K / G), 0, st);
            if (rc != W4A8_OK) return rc;
        }
        const FusedAct fa = {X, ldx, s, Xq_out, sx_out};
        return launch_gemv(nullptr, nullptr, ZeroPoint{nullptr, nullptr, nullptr}, M, Wp, step, zero, N, K, G,
                           Y, y_dtype, ldy, acc_out, nullptr, 1, st, 0, &fa);
    }
    // Otherwise the two steps one after the other, the int8 activations and token scales in the workspace
    // (or where the caller wants to see them).
    const LinearWs w = plan_linear(M, N, K, G, layout);
    if (!workspace || workspace_bytes < w.total || (uintptr_t)workspace % WS_ALIGN != 0) return W4A8_ERR_WORKSPACE;
    uint8_t *wsb = (uint8_t *)workspace;
    int8_t *Xq = Xq_out ? Xq_out : (int8_t *)(wsb + w.xq);
    float *sx = sx_out ? sx_out : (float *)(wsb + w.sx);
    // (all of the GEMM's own checks before anything is launched)
    int rc = gemm_common(Xq, sx, nullptr, M, Wp, layout, step, zero, nullptr, nullptr, N, K, group_size, Y,
                         y_dtype, ldy, acc_out, w.gemm_bytes ? wsb + w.gemm : nullptr, w.gemm_bytes, stream,
                         W4A8_FMT_DINT4, true);
    if (rc != W4A8_OK) return rc;
    rc = launch_act_quant(X, x_dtype, M, K, ldx, s, Xq, sx, nullptr, st);
    if (rc != W4A8_OK) return rc;
    return gemm_common(Xq, sx, nullptr, M, Wp, layout, step, zero, nullptr, nullptr, N, K, group_size, Y,
                       y_dtype, ldy, acc_out, w.gemm_bytes ? wsb + w.gemm : nullptr, w.gemm_bytes, stream);
}

// ---- w4a8_gemm for callers that cannot allocate: the workspace is a static device array ----------
}  // extern "C"

// The scratch memory of w4a8_gemm_static: every GPU the library runs on holds its own copy of this
// array, at its own address, until the process ends.  In host code the array's NAME is only a
// stand-in for the symbol (not a device address): the address on the current device comes from
// hipGetSymbolAddress, once per device, and only that pointer is ever handed to a kernel.
static __device__ __align__(256) uint8_t scratch[W4A8_STATIC_SCRATCH_BYTES];

namespace {

constexpr int SCRATCH_MAX_DEVICES = 64;
std::atomic<uint8_t *> scratch_ptr[SCRATCH_MAX_DEVICES];   // per device ordinal; null = not asked yet

// Address of `scratch` on the current device (nullptr with *status set on failure).  Racing first
// calls on one device both ask the runtime and store the same answer.
uint8_t *scratch_on_current_device(int *status)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        *status = W4A8_ERR_HIP;
        return nullptr;
    }
    const bool cached = dev >= 0 && dev < SCRATCH_MAX_DEVICES;
    if (cached) {
        uint8_t *known = scratch_ptr[dev].load(std::memory_order_acquire);
        if (known != nullptr) return known;
    }
    uint8_t *ptr = nullptr;
    if (hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
        (void)hipGetLastError();   // reported through the status; leave no sticky error behind
        *status = W4A8_ERR_HIP;
        return nullptr;
    }
    if (cached) scratch_ptr[dev].store(ptr, std::memory_order_release);
    return ptr;
}

}  // namespace

extern "C" {

size_t w4a8_gemm_static_scratch_bytes(void) { return W4A8_STATIC_SCRATCH_BYTES; }

int w4a8_gemm_static(const int8_t *Xq, const float *sx, int64_t M,
                     const uint8_t *Wp, int layout, const float *step, const uint8_t *zero,
                     int64_t N, int64_t K, int64_t group_size,
                     void *Y, int y_dtype, int64_t ldy, int32_t *acc_out, void *stream)
{
    // every check of w4a8_gemm first (with a workspace that is certainly large enough), so that
    // argument errors come back exactly as they do there and before the size limit is looked at
    static_assert(W4A8_STATIC_SCRATCH_BYTES % WS_ALIGN == 0, "scratch size keeps the workspace alignment");
    void *const probe = (void *)(uintptr_t)WS_ALIGN;   // never dereferenced: validate_only launches nothing
    int rc = gemm_common(Xq, sx, nullptr, M, Wp, layout, step, zero, nullptr, nullptr, N, K, group_size, Y,
                         y_dtype, ldy, acc_out, probe, SIZE_MAX, stream, W4A8_FMT_DINT4, true);
    if (rc != W4A8_OK || M == 0 || N == 0) return rc;
    int64_t G = group_size;
    resolve_group(K, G);
    const size_t need = plan_workspace(M, N, K, G, layout).total;
    if (need > W4A8_STATIC_SCRATCH_BYTES) return W4A8_ERR_WORKSPACE;
    uint8_t *ws = nullptr;
    if (need > 0 && (ws = scratch_on_current_device(&rc)) == nullptr) return rc;
    // Nothing in the workspace has to start at zero: the re-tiled weights, the row-sums and the
    // partial sums of the K ranges are all written in full before they are read, so what the last
    // call left there does not matter.
    return gemm_common(Xq, sx, nullptr, M, Wp, layout, step, zero, nullptr, nullptr, N, K, group_size, Y,
                       y_dtype, ldy, acc_out, ws, need, stream);
}

}  // extern "C"

// ---- AQAS scale search and weight clipping (Sec. 3.2, Eq. 1; App. A.4) ---------------------------
namespace {

constexpr int AQ_GRID = 16, AQ_CLIP_STEPS = 11;

struct AqasWs {
    size_t ax, aw, s, Xq, sx, codes, step, zero, Wp, Y, Yref, err, best_err, gemm, gemm_bytes, total;
};

AqasWs plan_aqas(int64_t M, int64_t N, int64_t K, int64_t G)
{
    AqasWs w{};
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = align_up(off + bytes);
        return at;
    };
    const size_t ng = (size_t)(K / G);
    w.ax = take((size_t)K * 4);
    w.aw = take((size_t)K * 4);
    w.s = take((size_t)K * 4);
    w.Xq = take((size_t)M * K);
    w.sx = take((size_t)M * 4);
    w.codes = take((size_t)N * K);
    w.step = take((size_t)N * ng * 4);
    w.zero = take((size_t)N * ng);
    w.Wp = take((size_t)N * K / 2);
    w.Y = take((size_t)M * N * 2);
    w.Yref = take((size_t)M * N * 4);
    w.err = take((size_t)N * 8);
    w.best_err = take((size_t)N * 8);
    w.gemm_bytes = plan_workspace(M, N, K, G, W4A8_LAYOUT_TILED).total;
    w.gemm = take(w.gemm_bytes);
    w.total = off;
    return w;
}

int aqas_check(const void *X, const void *W, int dtype, int64_t M, int64_t N, int64_t K, int64_t ldx,
               int64_t ldw, int64_t &G, const void *workspace, size_t workspace_bytes)
{
    if (!valid_dtype(dtype)) return W4A8_ERR_DTYPE;
    if (M < 1 || N < 1 || !resolve_group(K, G)) return W4A8_ERR_SHAPE;
    if (N % TILE_N != 0 || K % TILE_K != 0 || G % TILE_K != 0 || K > MAX_K || ldx < K || ldw < K ||
        M > 0x7fffffffLL || N * K / 2 > 0x7fffffffLL || M * K > 0x7fffffffLL)
        return W4A8_ERR_SHAPE;
    if (!X || !W) return W4A8_ERR_NULL;
    // the reference product fetches 16 bytes per lane from fp16 rows
    if (dtype == W4A8_F16 && ((uintptr_t)X % 16 != 0 || (uintptr_t)W % 16 != 0 || ldx % 8 != 0 || ldw % 8 != 0))
        return W4A8_ERR_SHAPE;
    if (!workspace || (uintptr_t)workspace % WS_ALIGN != 0 || workspace_bytes < plan_aqas(M, N, K, G).total)
        return W4A8_ERR_WORKSPACE;
    return W4A8_OK;
}

// One evaluation of the layer with scale s: err[n] = sum_m (Yq[m,n] - Yref[m,n])^2.
// clip_uniform >= 0: the weight ranges are shrunk by that clipping index first.
int aqas_evaluate(const void *X, const void *W, int dtype, int64_t M, int64_t N, int64_t K, int64_t ldx,
                  int64_t ldw, int64_t G, const float *s, int clip_uniform, uint8_t *ws, const AqasWs &w,
                  void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    int8_t *Xq = (int8_t *)(ws + w.Xq);
    float *sx = (float *)(ws + w.sx), *step = (float *)(ws + w.step);
    uint8_t *codes = ws + w.codes, *zero = ws + w.zero, *Wp = ws + w.Wp;
    int rc = quantize_act_int8(X, dtype, M, K, ldx, s, Xq, sx, stream);
    if (rc != W4A8_OK) return rc;
    if (clip_uniform >= 0) {
        rc = launch_clip_params(W, dtype, N, K, ldw, s, G, nullptr, clip_uniform, step, zero, st);
        if (rc != W4A8_OK) return rc;
    }
    rc = quantize_weight_dint4(W, dtype, N, K, ldw, s, G, clip_uniform >= 0 ? 1 : 0, codes, step, zero, stream);
    if (rc != W4A8_OK) return rc;
    rc = pack_dint4(codes, N, K, Wp, W4A8_LAYOUT_TILED, stream);
    if (rc != W4A8_OK) return rc;
    rc = w4a8_gemm(Xq, sx, M, Wp, W4A8_LAYOUT_TILED, step, zero, N, K, G, ws + w.Y, W4A8_F16, N, nullptr,
                   w.gemm_bytes ? ws + w.gemm : nullptr, w.gemm_bytes, stream);
    if (rc != W4A8_OK) return rc;
    return launch_output_sq_error(ws + w.Y, W4A8_F16, N, (const float *)(ws + w.Yref), M, N,
                                  (double *)(ws + w.err), st);
}

}  // namespace

extern "C" {

size_t aqas_search_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t group_size)
{
    int64_t G = group_size;
    if (M < 1 || N < 1 || !resolve_group(K, G) || K % TILE_K != 0 || G % TILE_K != 0 || N % TILE_N != 0)
        return 0;
    return plan_aqas(M, N, K, G).total;
}

int aqas_channel_absmax(const void *A, int dtype, int64_t R, int64_t K, int64_t lda, float *out,
                        void *stream)
{
    if (!valid_dtype(dtype)) return W4A8_ERR_DTYPE;
    if (R < 0 || K < 1 || lda < K || (R + 255) / 256 > 65535) return W4A8_ERR_SHAPE;
    if (!out || (R > 0 && !A)) return W4A8_ERR_NULL;
    return launch_channel_absmax(A, dtype, R, K, lda, out, (hipStream_t)stream);
}

int aqas_scale(const float *ax, const float *aw, int64_t K, int j, float *s, void *stream)
{
    if (K < 1 || j < 0 || j > AQ_GRID) return W4A8_ERR_SHAPE;
    if (!ax || !aw || !s) return W4A8_ERR_NULL;
    return launch_aqas_scale(ax, aw, K, j, nullptr, s, (hipStream_t)stream);
}

int aqas_search(const void *X, const void *W, int dtype, int64_t M, int64_t N, int64_t K, int64_t ldx,
                int64_t ldw, int64_t group_size, float *s_out, int32_t *best_j, double *losses,
                void *workspace, size_t workspace_bytes, void *stream)
{
    int64_t G = group_size;
    int rc = aqas_check(X, W, dtype, M, N, K, ldx, ldw, G, workspace, workspace_bytes);
    if (rc != W4A8_OK) return rc;
    if (!s_out || !best_j || !losses) return W4A8_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    uint8_t *ws = (uint8_t *)workspace;
    const AqasWs w = plan_aqas(M, N, K, G);
    float *ax = (float *)(ws + w.ax), *aw = (float *)(ws + w.aw), *s = (float *)(ws + w.s);
    if ((rc = launch_channel_absmax(X, dtype, M, K, ldx, ax, st)) != W4A8_OK) return rc;
    if ((rc = launch_channel_absmax(W, dtype, N, K, ldw, aw, st)) != W4A8_OK) return rc;
    if ((rc = launch_ref_gemm(X, W, dtype, M, N, K, ldx, ldw, (float *)(ws + w.Yref), st)) != W4A8_OK) return rc;
    for (int j = 0; j <= AQ_GRID; ++j) {
        if ((rc = launch_aqas_scale(ax, aw, K, j, nullptr, s, st)) != W4A8_OK) return rc;
        if ((rc = aqas_evaluate(X, W, dtype, M, N, K, ldx, ldw, G, s, -1, ws, w, stream)) != W4A8_OK) return rc;
        if ((rc = launch_loss_sum((const double *)(ws + w.err), N, losses, j, st)) != W4A8_OK) return rc;
    }
    if ((rc = launch_argmin(losses, AQ_GRID + 1, best_j, st)) != W4A8_OK) return rc;
    return launch_aqas_scale(ax, aw, K, 0, best_j, s_out, st);
}

int dint4_clipped_params(const void *W, int w_dtype, int64_t N, int64_t K, int64_t ldw, const float *s,
                         int64_t group_size, const int32_t *index, int uniform_index, float *step,
                         uint8_t *zero, void *stream)
{
    if (!valid_dtype(w_dtype)) return W4A8_ERR_DTYPE;
    int64_t G = group_size;
    if (N < 0 || K < 1 || ldw < K || !resolve_group(K, G)) return W4A8_ERR_SHAPE;
    if (!index && (uniform_index < 0 || uniform_index >= AQ_CLIP_STEPS)) return W4A8_ERR_SHAPE;
    if (N == 0) return W4A8_OK;
    if (!W || !step || !zero) return W4A8_ERR_NULL;
    return launch_clip_params(W, w_dtype, N, K, ldw, s, G, index, uniform_index, step, zero,
                              (hipStream_t)stream);
}

int aqas_clip_search(const void *X, const void *W, int dtype, int64_t M, int64_t N, int64_t K,
                     int64_t ldx, int64_t ldw, const float *s, int64_t group_size, int32_t *index_out,
                     float *step_out, uint8_t *zero_out, double *err_table, void *workspace,
                     size_t workspace_bytes, void *stream)
{
    int64_t G = group_size;
    int rc = aqas_check(X, W, dtype, M, N, K, ldx, ldw, G, workspace, workspace_bytes);
    if (rc != W4A8_OK) return rc;
    if (!index_out || !step_out || !zero_out) return W4A8_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    uint8_t *ws = (uint8_t *)workspace;
    const AqasWs w = plan_aqas(M, N, K, G);
    if ((rc = launch_ref_gemm(X, W, dtype, M, N, K, ldx, ldw, (float *)(ws + w.Yref), st)) != W4A8_OK) return rc;
    for (int i = 0; i < AQ_CLIP_STEPS; ++i) {
        if ((rc = aqas_evaluate(X, W, dtype, M, N, K, ldx, ldw, G, s, i, ws, w, stream)) != W4A8_OK) return rc;
        if ((rc = launch_clip_select((const double *)(ws + w.err), N, i, (double *)(ws + w.best_err),
                                     index_out, err_table, st)) != W4A8_OK)
            return rc;
    }
    return launch_clip_params(W, dtype, N, K, ldw, s, G, index_out, 0, step_out, zero_out, st);
}

}  // extern "C"


// ---- weight-format variants (App. A.5, Tables 10-14) and the error split of Sec. 4.1 -------------
namespace {

struct ErrWs {
    size_t codes, step, zero, du, dr, xs, pu, pr, total;
};
ErrWs plan_err(int64_t M, int64_t N, int64_t K, int64_t G)
{
    ErrWs w{};
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = align_up(off + bytes);
        return at;
    };
    w.codes = take((size_t)N * K);
    w.step = take((size_t)N * (K / G) * 4);
    w.zero = take((size_t)N * (K / G));
    w.du = take((size_t)N * K * 4);
    w.dr = take((size_t)N * K * 4);
    w.xs = take((size_t)M * K * 4);
    w.pu = take((size_t)M * N * 4);
    w.pr = take((size_t)M * N * 4);
    w.total = off;
    return w;
}

}  // namespace

extern "C" {

int quantize_weight_format(const void *W, int w_dtype, int64_t N, int64_t K, int64_t ldw, const float *s,
                           int64_t group_size, int format, int use_given_params, uint8_t *codes,
                           float *step, uint8_t *zero, void *stream)
{
    if (!valid_dtype(w_dtype)) return W4A8_ERR_DTYPE;
    if (format < W4A8_FMT_DINT4 || format > W4A8_FMT_DINT4_C8) return W4A8_ERR_DTYPE;
    int64_t G = group_size;
    if (N < 0 || K < 1 || ldw < K || !resolve_group(K, G)) return W4A8_ERR_SHAPE;
    if (N == 0) return W4A8_OK;
    if (!W || !codes || !step || !zero) return W4A8_ERR_NULL;
    return launch_weight_quant(W, w_dtype, N, K, ldw, s, G, use_given_params, codes, step, zero, format,
                               (hipStream_t)stream);
}

int w4a8_gemm_format(const int8_t *Xq, const float *sx, int64_t M, const uint8_t *Wp, int layout,
                     const float *step, const uint8_t *zero, int64_t N, int64_t K, int64_t group_size,
                     int format, void *Y, int y_dtype, int64_t ldy, int32_t *acc_out, void *workspace,
                     size_t workspace_bytes, void *stream)
{
    return gemm_common(Xq, sx, nullptr, M, Wp, layout, step, zero, nullptr, nullptr, N, K, group_size, Y,
                       y_dtype, ldy, acc_out, workspace, workspace_bytes, stream, format);
}

int pack_format(const uint8_t *codes, int64_t N, int64_t K, uint8_t *packed, int layout, int format,
                void *stream)
{
    if (format != W4A8_FMT_DINT4 && format != W4A8_FMT_INT4 && format != W4A8_FMT_DINT3) return W4A8_ERR_DTYPE;
    const int rc = check_pack_shape(N, K, layout);
    if (rc != W4A8_OK) return rc;
    if (N == 0) return W4A8_OK;
    if (!codes || !packed) return W4A8_ERR_NULL;
    if (layout == W4A8_LAYOUT_TILED && (uintptr_t)packed % 4 != 0) return W4A8_ERR_SHAPE;
    return launch_pack(codes, N, K, packed, layout, (hipStream_t)stream, format == W4A8_FMT_INT4);
}

int unpack_format(const uint8_t *packed, int64_t N, int64_t K, uint8_t *codes, int layout, int format,
                  void *stream)
{
    if (format != W4A8_FMT_DINT4 && format != W4A8_FMT_INT4 && format != W4A8_FMT_DINT3) return W4A8_ERR_DTYPE;
    const int rc = check_pack_shape(N, K, layout);
    if (rc != W4A8_OK) return rc;
    if (N == 0) return W4A8_OK;
    if (!codes || !packed) return W4A8_ERR_NULL;
    if (layout == W4A8_LAYOUT_TILED && (uintptr_t)packed % 4 != 0) return W4A8_ERR_SHAPE;
    return launch_unpack(packed, N, K, codes, layout, (hipStream_t)stream, format == W4A8_FMT_INT4);
}

int expand_special_value(const uint8_t *codes, const float *step, const uint8_t *zero, int64_t N, int64_t K,
                         int64_t group_size, int format, uint8_t *codes2, float *step2, uint8_t *zero2,
                         void *stream)
{
    if (format != W4A8_FMT_DINT4_C4 && format != W4A8_FMT_DINT4_C8) return W4A8_ERR_DTYPE;
    int64_t G = group_size;
    if (N < 0 || K < 1 || !resolve_group(K, G)) return W4A8_ERR_SHAPE;
    if (N == 0) return W4A8_OK;
    if (!codes || !step || !zero || !codes2 || !step2 || !zero2) return W4A8_ERR_NULL;
    return launch_expand_special(codes, step, zero, N, K, G, format == W4A8_FMT_DINT4_C4 ? 2 : 3, codes2,
                                 step2, zero2, (hipStream_t)stream);
}

size_t w4a8_gemm_special_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t group_size, int layout)
{
    int64_t G = group_size;
    if (M <= 0 || N <= 0 || !resolve_group(K, G) || !gemm_shape_ok(M, N, 2 * K, G) || !valid_layout(layout))
        return 0;
    return align_up((size_t)(M * 2 * K)) + plan_workspace(M, N, 2 * K, G, layout).total;
}

int w4a8_gemm_special(const int8_t *Xq, const float *sx, int64_t M, const uint8_t *Wp2, int layout,
                      const float *step2, const uint8_t *zero2, int64_t N, int64_t K, int64_t group_size,
                      void *Y, int y_dtype, int64_t ldy, int32_t *acc_out, void *workspace,
                      size_t workspace_bytes, void *stream)
{
    int64_t G = group_size;
    if (M < 0 || N < 0 || !resolve_group(K, G) || K % TILE_K != 0 || 2 * K > MAX_K) return W4A8_ERR_SHAPE;
    if (M == 0 || N == 0) return W4A8_OK;
    if (!Xq) return W4A8_ERR_NULL;
    if ((uintptr_t)Xq % 16 != 0) return W4A8_ERR_SHAPE;
    const size_t xx_bytes = align_up((size_t)(M * 2 * K));
    if (!workspace || (uintptr_t)workspace % WS_ALIGN != 0 || workspace_bytes < xx_bytes)
        return W4A8_ERR_WORKSPACE;
    int8_t *xx = (int8_t *)workspace;
    uint8_t *rest = (uint8_t *)workspace + xx_bytes;
    // all of the GEMM's own checks first: nothing is launched when an argument is wrong
    int rc = gemm_common(xx, sx, nullptr, M, Wp2, layout, step2, zero2, nullptr, nullptr, N, 2 * K, G, Y,
                         y_dtype, ldy, acc_out, rest, workspace_bytes - xx_bytes, stream, W4A8_FMT_DINT4,
                         true);
    if (rc != W4A8_OK) return rc;
    rc = launch_repeat_activations(Xq, M, K, xx, (hipStream_t)stream);
    if (rc != W4A8_OK) return rc;
    return gemm_common(xx, sx, nullptr, M, Wp2, layout, step2, zero2, nullptr, nullptr, N, 2 * K, G, Y,
                       y_dtype, ldy, acc_out, rest, workspace_bytes - xx_bytes, stream, W4A8_FMT_DINT4);
}

int pack_dint3(const uint8_t *codes, int64_t N, int64_t K, uint8_t *packed, void *stream)
{
    if (N < 0 || K < 1 || K % 8 != 0) return W4A8_ERR_SHAPE;
    if (N == 0) return W4A8_OK;
    if (!codes || !packed) return W4A8_ERR_NULL;
    return launch_pack3(codes, N, K, packed, (hipStream_t)stream);
}

int unpack_dint3(const uint8_t *packed, int64_t N, int64_t K, uint8_t *codes, void *stream)
{
    if (N < 0 || K < 1 || K % 8 != 0) return W4A8_ERR_SHAPE;
    if (N == 0) return W4A8_OK;
    if (!codes || !packed) return W4A8_ERR_NULL;
    return launch_unpack3(packed, N, K, codes, (hipStream_t)stream);
}

size_t dint_error_terms_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t group_size)
{
    int64_t G = group_size;
    if (M < 1 || N < 1 || !resolve_group(K, G) || K % 2 != 0) return 0;
    return plan_err(M, N, K, G).total;
}

int dint_error_terms(const void *X, int x_dtype, int64_t M, int64_t K, int64_t ldx, const void *W,
                     int w_dtype, int64_t N, int64_t ldw, const float *s, int64_t group_size, int format,
                     double *terms, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!valid_dtype(x_dtype) || !valid_dtype(w_dtype)) return W4A8_ERR_DTYPE;
    if (format < W4A8_FMT_DINT4 || format > W4A8_FMT_DINT4_C8) return W4A8_ERR_DTYPE;
    const int special = format == W4A8_FMT_INT4 ? 0 : (format == W4A8_FMT_DINT4_C4 ? 2 : (format == W4A8_FMT_DINT4_C8 ? 3 : 1));
    int64_t G = group_size;
    if (M < 1 || N < 1 || !resolve_group(K, G) || K % 2 != 0 || ldx < K || ldw < K) return W4A8_ERR_SHAPE;
    if (!X || !W || !terms) return W4A8_ERR_NULL;
    const ErrWs w = plan_err(M, N, K, G);
    if (!workspace || (uintptr_t)workspace % WS_ALIGN != 0 || workspace_bytes < w.total) return W4A8_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    uint8_t *ws = (uint8_t *)workspace;
    float *du = (float *)(ws + w.du), *dr = (float *)(ws + w.dr), *xs = (float *)(ws + w.xs);
    float *pu = (float *)(ws + w.pu), *pr = (float *)(ws + w.pr);
    int rc = launch_weight_quant(W, w_dtype, N, K, ldw, s, G, 0, ws + w.codes, (float *)(ws + w.step),
                                 ws + w.zero, format, st);
    if (rc != W4A8_OK) return rc;
    if ((rc = launch_error_split(W, w_dtype, N, K, ldw, s, G, special, ws + w.codes,
                                 (const float *)(ws + w.step), ws + w.zero, du, dr, st)) != W4A8_OK)
        return rc;
    if ((rc = launch_scale_activations(X, x_dtype, M, K, ldx, s, xs, st)) != W4A8_OK) return rc;
    if ((rc = launch_ref_gemm(xs, du, W4A8_F32, M, N, K, K, K, pu, st)) != W4A8_OK) return rc;
    if ((rc = launch_ref_gemm(xs, dr, W4A8_F32, M, N, K, K, K, pr, st)) != W4A8_OK) return rc;
    return launch_error_terms(pu, pr, M * N, du, N * K, terms, st);
}

}  // extern "C"
