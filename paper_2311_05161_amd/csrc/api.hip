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
    if (M > 16) {
        const GemmPlan gp = plan_gemm(M, N, K, G);
        w.rs_off = off;            // per-channel weights: bias removal needs row-sums per token
        w.rs_bytes = gp.rs_bytes;
        off = align_up(off + w.rs_bytes);
        w.part_off = off;          // few output tiles: K is split, fp32 partial sums
        w.part_bytes = gp.partial_bytes;
        off = align_up(off + w.part_bytes);
    } else if (M > 0 && N > 0) {
        w.part_off = off;
        w.part_bytes = plan_gemv(M, N, K, G).partial_bytes;
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
                int32_t *acc_out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!valid_layout(layout)) return W4A8_ERR_DTYPE;
    if (y_dtype != W4A8_F16 && y_dtype != W4A8_BF16) return W4A8_ERR_DTYPE;
    int64_t G = group_size;
    if (M < 0 || N < 0 || !resolve_group(K, G)) return W4A8_ERR_SHAPE;
    if (N % TILE_N != 0 || K % TILE_K != 0 || G % TILE_K != 0 || K > MAX_K || ldy < N ||
        M > 0x7fffffffLL || N * K / 2 > 0x7fffffffLL)  // 32-bit byte offsets into the weights
        return W4A8_ERR_SHAPE;
    // the tile kernel addresses Xq with 32-bit byte offsets and numbers its tiles in 32 bits
    if (M > 16 && (M * K > 0x7fffffffLL || (M + 63) / 64 * ((N + 255) / 256) > 0x1ffffLL))
        return W4A8_ERR_SHAPE;
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
    hipStream_t st = (hipStream_t)stream;
    uint8_t *wsb = (uint8_t *)workspace;
    const ZeroPoint zp = {zx, wsum, tsum};

    const uint8_t *Wt = Wp;
    if (layout == W4A8_LAYOUT_CANONICAL) {
        uint8_t *tiled = wsb + ws.repack_off;
        const int rc = launch_repack_canonical_to_tiled(Wp, N, K, tiled, st);
        if (rc != W4A8_OK) return rc;
        Wt = tiled;
    }
    if (M <= 16) {
        if (acc_out) {  // the split-K waves add exact partial sums into it
            const int rc = launch_fill_i32(acc_out, M * N * (K / G), 0, st);
            if (rc != W4A8_OK) return rc;
        }
        const int rc = launch_gemv(Xq, sx, zp, M, Wt, step, zero, N, K, G, Y, y_dtype, ldy,
                                   acc_out, (float *)(wsb + ws.part_off), 1, st);
        if (rc != W4A8_OK || !zx || !acc_out) return rc;
        return launch_acc_zero_point(acc_out, zx, wsum, M, N * (K / G), st);
    }
    if (acc_out && ws.part_bytes > 0 && G == K) {  // K-split workgroups add exact partial sums
        const int rc = launch_fill_i32(acc_out, M * N, 0, st);
        if (rc != W4A8_OK) return rc;
    }
    const int rc = launch_gemm(Xq, sx, zp, (int32_t *)(wsb + ws.rs_off), M, Wt, step, zero, N,
                               K, G, Y, y_dtype, ldy, acc_out, (float *)(wsb + ws.part_off), st);
    if (rc != W4A8_OK || !zx || !acc_out) return rc;
    return launch_acc_zero_point(acc_out, zx, wsum, M, N * (K / G), st);
}

}  // namespace

extern "C" {

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
                               (hipStream_t)stream);
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
    if (M < 0 || N < 0 || !resolve_group(K, G) || !valid_layout(layout) || K % TILE_K != 0 ||
        G % TILE_K != 0 || N % TILE_N != 0)
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

}  // extern "C"
