// dINT4 x INT8 GEMM, prefill shape (M > 16): a compute-bound tile kernel on the int8 matrix cores
// (Eq. 1 product on the integer operands with int32 accumulation; Eq. 5 second half fused as the
// dequantizing epilogue; the dINT4 x INT8 multiply-accumulate of Sec. 4.3).
//
// A workgroup of 4 wavefronts computes a BM x 256 output tile; wave w owns all BM token rows of
// 64 output channels, so each packed-weight tile is decoded by exactly one wave: the wave reads
// its four 1 KB weight tiles per 128 columns of K straight from global memory (16 bytes per lane,
// prefetched one step ahead), decodes them in registers through the per-(row, group) LUT and
// reuses every decoded operand for all BM / 16 token sub-tiles.  The int8 activations are staged
// through LDS (double buffered, 16-byte chunks XOR-swizzled by row so that both the staging
// writes and the ds_read_b128 operand reads are bank-conflict free) and shared by the 4 waves.
// The decode bias is removed with per-token group row-sums computed by a small pre-pass.
#include "w4a8_common.hpp"

namespace w4a8 {

constexpr int GM_THREADS = 256;
constexpr int GM_BN = 256;       // output channels per workgroup
constexpr int GM_NS = 4;         // 16-channel sub-tiles per wave

// ---- per-token group row-sums of Xq: rs[m,g] = sum_{k in g} Xq[m,k] -------------------------
__global__ __launch_bounds__(256) void group_rowsum_kernel(const int8_t *__restrict__ Xq, int64_t M,
                                                           int K, int G, int32_t *__restrict__ rs)
{
    const int lane = threadIdx.x & 63;
    const int ng = K / G;
    const int64_t seg = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (seg >= M * ng) return;
    const int64_t m = seg / ng;
    const int g = (int)(seg % ng);
    const int *x = reinterpret_cast<const int *>(Xq + m * K + (int64_t)g * G);
    int sum = 0;
    for (int i = lane; i < G / 4; i += WAVE) sum = __builtin_amdgcn_sdot4(x[i], 0x01010101, sum, false);
    sum = wave_sum_i32(sum);
    if (lane == 0) rs[seg] = sum;
}

int launch_group_rowsum(const int8_t *Xq, int64_t M, int64_t K, int64_t G, int32_t *rs,
                        hipStream_t st)
{
    const int64_t segs = M * (K / G);
    if (segs == 0) return W4A8_OK;
    hipLaunchKernelGGL(group_rowsum_kernel, dim3((unsigned)((segs + 3) / 4)), dim3(256), 0, st, Xq,
                       M, (int)K, (int)G, rs);
    return hip_status(hipGetLastError());
}

// ---- the tile kernel ------------------------------------------------------------------------
template <int BM, bool GROUPED>
__global__ __launch_bounds__(GM_THREADS) void gemm_kernel(
    const int8_t *__restrict__ Xq, const float *__restrict__ sx, const int32_t *__restrict__ rs,
    int M, const v4u *__restrict__ Wt, const float *__restrict__ step,
    const uint8_t *__restrict__ zero, int N, int K, int tiles_per_group, int ng,
    uint16_t *__restrict__ Y, int y_dtype, int64_t ldy, int vec_store,
    int32_t *__restrict__ acc_out, int grid_m, int grid_n)
{
    constexpr int MS = BM / 16;               // token sub-tiles, all owned by every wave
    constexpr int LD_ITERS = BM * 8 / GM_THREADS;  // 16-byte chunks of the A tile per thread
    __shared__ __attribute__((aligned(16))) uint8_t lds[2][BM * TILE_K];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int ln = lane & 15;
    const int kb = lane >> 4;
    const int KT = K / TILE_K;

    // Workgroups are handed to the 8 XCDs round-robin; renumber so that each XCD works on a
    // contiguous range of tiles (token tiles fastest) and its private L2 sees the reuse.
    int bid = blockIdx.x;
    {
        const int total = grid_m * grid_n;
        const int per = total / 8;
        if (bid < per * 8) bid = (bid & 7) * per + (bid >> 3);
    }
    const int bm = bid % grid_m;
    const int bn = bid / grid_m;
    const int m0 = bm * BM;
    const int n0 = bn * GM_BN + wave * (GM_NS * TILE_N);  // first output channel of this wave

    bool ns_valid[GM_NS];
    const v4u *wp[GM_NS];
#pragma unroll
    for (int ns = 0; ns < GM_NS; ++ns) {
        const int nn = n0 + ns * TILE_N;
        ns_valid[ns] = nn < N;
        wp[ns] = Wt + (int64_t)(ns_valid[ns] ? nn / TILE_N : 0) * KT * WAVE + lane;
    }

    v4i acc[MS][GM_NS];
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int ns = 0; ns < GM_NS; ++ns) acc[ms][ns] = v4i{0, 0, 0, 0};

    constexpr int YS = GROUPED ? MS : 1;
    v4f y[YS][GM_NS];
#pragma unroll
    for (int ms = 0; ms < YS; ++ms)
#pragma unroll
        for (int ns = 0; ns < GM_NS; ++ns) y[ms][ns] = v4f{0.f, 0.f, 0.f, 0.f};

    // A-tile staging: chunk c (16 bytes) of row r lives at r*128 + ((c ^ (r & 7)) * 16)
    v4i areg[LD_ITERS];
    auto load_a = [&](int kt) {
#pragma unroll
        for (int i = 0; i < LD_ITERS; ++i) {
            const int idx = tid + i * GM_THREADS;
            const int row = idx >> 3, ch = idx & 7;
            areg[i] = v4i{0, 0, 0, 0};
            if (m0 + row < M)
                areg[i] = *reinterpret_cast<const v4i *>(Xq + (int64_t)(m0 + row) * K +
                                                         (int64_t)kt * TILE_K + ch * 16);
        }
    };
    auto store_a = [&](int buf) {
#pragma unroll
        for (int i = 0; i < LD_ITERS; ++i) {
            const int idx = tid + i * GM_THREADS;
            const int row = idx >> 3, ch = idx & 7;
            *reinterpret_cast<v4i *>(&lds[buf][row * TILE_K + ((ch ^ (row & 7)) << 4)]) = areg[i];
        }
    };

    v4u p[GM_NS], pn[GM_NS];
    auto load_b = [&](int kt, v4u(&dst)[GM_NS]) {
#pragma unroll
        for (int ns = 0; ns < GM_NS; ++ns) dst[ns] = wp[ns][(int64_t)kt * WAVE];
    };

    DecodeLut lut[GM_NS];
    auto load_luts = [&](int g) {
#pragma unroll
        for (int ns = 0; ns < GM_NS; ++ns) {
            const int nn = ns_valid[ns] ? n0 + ns * TILE_N + ln : 0;
            lut[ns] = make_decode_lut(zero[(int64_t)nn * ng + g]);
        }
    };

    // Lane owns, per (ms, ns): token m = m0 + 16 ms + ln, channels n = n0 + 16 ns + 4 kb + r.
    auto flush_group = [&](int g) {
        int rsv[MS];
#pragma unroll
        for (int ms = 0; ms < MS; ++ms) {
            const int m = m0 + ms * 16 + ln;
            rsv[ms] = (m < M) ? rs[(int64_t)m * ng + g] : 0;
        }
#pragma unroll
        for (int ns = 0; ns < GM_NS; ++ns) {
            float es[4];
            int bq[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int nn = ns_valid[ns] ? n0 + ns * TILE_N + 4 * kb + r : 0;
                const int z = zero[(int64_t)nn * ng + g];
                es[r] = step[(int64_t)nn * ng + g] * 0.125f;
                bq[r] = 8 * z + ((~z & 1) << 2);
            }
#pragma unroll
            for (int ms = 0; ms < MS; ++ms) {
                const int m = m0 + ms * 16 + ln;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int v = acc[ms][ns][r] - bq[r] * rsv[ms];
                    if (GROUPED) y[ms][ns][r] += es[r] * (float)v;
                    else acc[ms][ns][r] = v;  // kept for the epilogue
                    if (acc_out != nullptr && m < M && ns_valid[ns]) {
                        const int nn = n0 + ns * TILE_N + 4 * kb + r;
                        acc_out[((int64_t)m * N + nn) * ng + g] = v >> 2;
                    }
                    if (GROUPED) acc[ms][ns][r] = 0;
                }
            }
        }
    };

    load_a(0);
    load_b(0, p);
    store_a(0);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < KT;
        if (more) {
            load_a(kt + 1);
            load_b(kt + 1, pn);
        }
        if (kt % tiles_per_group == 0) load_luts(kt / tiles_per_group);

        v4i w0[GM_NS], w1[GM_NS];
#pragma unroll
        for (int ns = 0; ns < GM_NS; ++ns) decode_lane(p[ns], lut[ns], w0[ns], w1[ns]);

#pragma unroll
        for (int ms = 0; ms < MS; ++ms) {
            const int row = ms * 16 + ln;
            const uint8_t *base = &lds[cur][row * TILE_K];
            const v4i a0 = *reinterpret_cast<const v4i *>(base + (((2 * kb) ^ (row & 7)) << 4));
            const v4i a1 = *reinterpret_cast<const v4i *>(base + (((2 * kb + 1) ^ (row & 7)) << 4));
#pragma unroll
            for (int ns = 0; ns < GM_NS; ++ns) {
                // D[i][j]: rows i = output channels (weights operand), columns j = tokens
                acc[ms][ns] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w0[ns], a0, acc[ms][ns], 0, 0, 0);
                acc[ms][ns] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w1[ns], a1, acc[ms][ns], 0, 0, 0);
            }
        }
        if (GROUPED && (kt + 1) % tiles_per_group == 0) flush_group(kt / tiles_per_group);

        if (more) {
            store_a(cur ^ 1);
#pragma unroll
            for (int ns = 0; ns < GM_NS; ++ns) p[ns] = pn[ns];
        }
        __syncthreads();
    }
    if (!GROUPED) flush_group(0);

    // epilogue: Y[m, n..n+3] = cast(sx[m] * y)
    float es[GM_NS][4];
    if (!GROUPED) {
#pragma unroll
        for (int ns = 0; ns < GM_NS; ++ns)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int nn = ns_valid[ns] ? n0 + ns * TILE_N + 4 * kb + r : 0;
                es[ns][r] = step[(int64_t)nn * ng] * 0.125f;
            }
    }
#pragma unroll
    for (int ms = 0; ms < MS; ++ms) {
        const int m = m0 + ms * 16 + ln;
        if (m >= M) continue;
        const float sxm = sx[m];
#pragma unroll
        for (int ns = 0; ns < GM_NS; ++ns) {
            if (!ns_valid[ns]) continue;
            uint16_t h[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float yv = GROUPED ? y[GROUPED ? ms : 0][ns][r] : es[ns][r] * (float)acc[ms][ns][r];
                const float out = sxm * yv;
                h[r] = (y_dtype == W4A8_F16) ? f32_to_f16_bits(out) : f32_to_bf16_bits(out);
            }
            uint16_t *yp = Y + (int64_t)m * ldy + n0 + ns * TILE_N + 4 * kb;
            if (vec_store) {
                *reinterpret_cast<uint2 *>(yp) =
                    make_uint2((uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16));
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) yp[r] = h[r];
            }
        }
    }
}

template <int BM, bool GROUPED>
static int launch_gemm_t(const int8_t *Xq, const float *sx, const int32_t *rs, int64_t M,
                         const uint8_t *Wt, const float *step, const uint8_t *zero, int64_t N,
                         int64_t K, int64_t G, void *Y, int y_dtype, int64_t ldy, int32_t *acc_out,
                         hipStream_t st)
{
    const int grid_m = (int)((M + BM - 1) / BM);
    const int grid_n = (int)((N + GM_BN - 1) / GM_BN);
    const int vec_store = ((uintptr_t)Y % 8 == 0) && (ldy % 4 == 0);
    hipLaunchKernelGGL((gemm_kernel<BM, GROUPED>), dim3((unsigned)(grid_m * grid_n)),
                       dim3(GM_THREADS), 0, st, Xq, sx, rs, (int)M, (const v4u *)Wt, step, zero,
                       (int)N, (int)K, (int)(G / TILE_K), (int)(K / G), (uint16_t *)Y, y_dtype, ldy,
                       vec_store, acc_out, grid_m, grid_n);
    return hip_status(hipGetLastError());
}

int launch_gemm(const int8_t *Xq, const float *sx, const int32_t *rs, int64_t M, const uint8_t *Wt,
                const float *step, const uint8_t *zero, int64_t N, int64_t K, int64_t G, void *Y,
                int y_dtype, int64_t ldy, int32_t *acc_out, hipStream_t st)
{
    const bool grouped = G != K;
    if ((M + 255) / 256 * ((N + 255) / 256) > 0x7fffffLL) return W4A8_ERR_SHAPE;
    if (grouped)  // int32 group accumulators plus fp32 running sums: 64 token rows fill the registers
        return launch_gemm_t<64, true>(Xq, sx, rs, M, Wt, step, zero, N, K, G, Y, y_dtype, ldy,
                                       acc_out, st);
    if (M <= 64)
        return launch_gemm_t<64, false>(Xq, sx, rs, M, Wt, step, zero, N, K, G, Y, y_dtype, ldy,
                                        acc_out, st);
    if (M <= 128)
        return launch_gemm_t<128, false>(Xq, sx, rs, M, Wt, step, zero, N, K, G, Y, y_dtype, ldy,
                                         acc_out, st);
    return launch_gemm_t<256, false>(Xq, sx, rs, M, Wt, step, zero, N, K, G, Y, y_dtype, ldy,
                                     acc_out, st);
}

}  // namespace w4a8
