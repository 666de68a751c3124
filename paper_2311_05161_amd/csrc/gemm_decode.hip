// dINT4 x INT8 GEMM, decode shape (M <= 16): a memory-bound GEMV that streams the packed
// weights exactly once  (Eq. 1 product on the integer operands; Eq. 5 second half fused as the
// epilogue; the dINT4 x INT8 multiply-accumulate of Sec. 4.3 mapped onto the int8 matrix cores).
//
// Work decomposition.  The tiled weight layout cuts W into 1 KB tiles of 16 output channels x
// 128 input channels.  A persistent workgroup owns q consecutive 16-channel "n-tiles" (all of K,
// or one K-split of it) and runs 8 compute wavefronts plus 1 helper wavefront:
//   * compute wave w owns the k-tiles kt = w, w+8, ... (at most AT of them).  Its int8 activation
//     fragments for those k-tiles are loaded once and stay in registers for the workgroup's
//     lifetime, so in steady state the only memory instructions it issues are 16-byte-per-lane
//     buffer loads of weight tiles (the wave reads one contiguous 1 KB tile per instruction).
//     Weight slot u always holds k-tile u of the n-tile one ahead of the one being consumed; every
//     load is issued unconditionally (tiles that do not exist are addressed out of range, which a
//     buffer load answers with zeros and no traffic), so the s_waitcnt counts are static and a
//     wave only ever waits for the one tile it is about to use.
//   * per tile: one ds_read_b128 fetches the precomputed decode record of (channel, k-tile), the
//     nibbles become int8 through the register LUT (w4a8_common.hpp), two MFMAs
//     (v_mfma_i32_16x16x64_i8, the <= 16 token rows are the other operand) accumulate the biased
//     product and two more against a constant "-4 beta" operand remove the decode bias exactly; the
//     int32 group sum is scaled into an fp32 running sum.
//   * the helper wave never touches the weight stream: after each n-tile's barrier it adds the 8
//     waves' partial sums in a fixed order (deterministic), applies the token scale and stores Y
//     (or an fp32 partial for a later combine when K is split across workgroups).
// Per-CU L2->L1 bandwidth (~30 B/clk) is what makes re-reading activations per tile unaffordable:
// at M = 16 they are twice the bytes of the 4-bit weights.
#include "w4a8_common.hpp"

namespace w4a8 {

constexpr int GV_CW = 8;                          // compute waves per workgroup
constexpr int GV_THREADS = (GV_CW + 1) * WAVE;    // + 1 helper wave
constexpr int GV_MAX_AT = 8;                      // k-tiles per compute wave -> K per split <= 8192
constexpr int GV_STAGE = 6;                       // decode records staged per thread (grouped mode)
constexpr int GV_LDS_BUDGET = 48 * 1024;          // bytes of decode records per workgroup
constexpr int GV_OOB = 0x7fff0000;                // buffer offset beyond any buffer: loads return 0

__device__ __forceinline__ void lds_barrier()
{
    // LDS-only barrier: outstanding global loads (the prefetched weight ring) stay in flight
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ v4u decode_record(int z, float st)
{
    const DecodeLut t = make_decode_lut(z);
    const uint32_t nb8 = (uint32_t)(-t.beta_q) & 0xffu;  // -4 beta as an int8
    return v4u{t.lo, t.hi, __float_as_uint(st * 0.125f), __builtin_amdgcn_perm(nb8, nb8, 0u)};
}

__device__ __forceinline__ v4i as_v4i(const v4u &v) { return v4i{(int)v.x, (int)v.y, (int)v.z, (int)v.w}; }

// GROUPED: one (step, zero) per k-tile or coarser group, rescaled per tile.  !GROUPED: per channel.
template <bool GROUPED, int AT, bool ACC_OUT>
__global__ __launch_bounds__(GV_THREADS) void gemv_kernel(
    const int8_t *__restrict__ Xq, const float *__restrict__ sx, int M,
    const uint8_t *__restrict__ Wt, const float *__restrict__ step, const uint8_t *__restrict__ zero,
    int N, int K, int tiles_per_group, int ng, uint16_t *__restrict__ Y, int y_dtype, int64_t ldy,
    float *__restrict__ partial, int32_t *__restrict__ acc_out, int q, int blocks_per_split,
    int kt_per_split)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    float *red = reinterpret_cast<float *>(smem);                        // [2][GV_CW][256]
    v4u *rec = reinterpret_cast<v4u *>(smem + 2 * GV_CW * 256 * 4);      // [q][KTs or 1][16]

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int KT = K >> 7;
    const int NT = N >> 4;
    const int split = blockIdx.x / blocks_per_split;
    const int nt0 = (blockIdx.x - split * blocks_per_split) * q;
    const int my_nt = min(q, NT - nt0);
    const int kt_begin = split * kt_per_split;
    const int KTs = min(kt_per_split, KT - kt_begin);     // k-tiles of this split
    const int recs_per_nt = GROUPED ? KTs : 1;

    // ---- quantization parameters of this workgroup -> decode records in LDS -------------------
    // element e = ((j * recs_per_nt + ktl) * 16 + row); loads first, LUT arithmetic later
    int st_z[GV_STAGE];
    float st_s[GV_STAGE];
    const int n_rec = my_nt * recs_per_nt * 16;
#pragma unroll
    for (int i = 0; i < GV_STAGE; ++i) {
        const int e = threadIdx.x + i * GV_THREADS;
        st_z[i] = 0;
        st_s[i] = 0.f;
        if ((GROUPED || i == 0) && e < n_rec) {
            const int row = e & 15, t = e >> 4;
            const int j = t / recs_per_nt, ktl = t - j * recs_per_nt;
            const int g = GROUPED ? (kt_begin + ktl) / tiles_per_group : 0;
            const int64_t idx = (int64_t)((nt0 + j) * TILE_N + row) * ng + g;
            st_z[i] = zero[idx];
            st_s[i] = step[idx];
        }
    }
    auto write_records = [&]() {
#pragma unroll
        for (int i = 0; i < GV_STAGE; ++i) {
            const int e = threadIdx.x + i * GV_THREADS;
            if ((GROUPED || i == 0) && e < n_rec) rec[e] = decode_record(st_z[i], st_s[i]);
        }
    };

    if (wave == GV_CW) {
        // ================= helper wave: reduction across the compute waves + output ============
        write_records();
        lds_barrier();
        for (int j = 0; j < my_nt; ++j) {
            lds_barrier();  // the compute waves have published their partial sums of n-tile j
            const float *rb = red + (j & 1) * GV_CW * 256;
#pragma unroll
            for (int o4 = 0; o4 < 4; ++o4) {
                const int o = lane + o4 * 64;  // output (token m = o >> 4, channel o & 15)
                const int m = o >> 4;
                float sum = 0.f;
#pragma unroll
                for (int w = 0; w < GV_CW; ++w) sum += rb[w * 256 + o];
                if (m < M) {
                    const int n = (nt0 + j) * TILE_N + (o & 15);
                    if (partial != nullptr) {
                        partial[((int64_t)split * M + m) * N + n] = sum;
                    } else {
                        const float out = sx[m] * sum;
                        Y[(int64_t)m * ldy + n] =
                            (y_dtype == W4A8_F16) ? f32_to_f16_bits(out) : f32_to_bf16_bits(out);
                    }
                }
            }
        }
        return;
    }

    // ================= compute waves ==========================================================
    const int ln = lane & 15;   // weight operand: output channel;  accumulator: output channel
    const int kb = lane >> 4;   // which 32 of the tile's 128 input channels this lane holds
    const int tpw = (KTs - wave + GV_CW - 1) / GV_CW;   // k-tiles of this wave: kt = wave + 8 u
    __amdgpu_buffer_rsrc_t rw =
        __builtin_amdgcn_make_buffer_rsrc((void *)Wt, 0, (int)((int64_t)N * K / 2), 0x00020000);
    __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)Xq, 0, M * K, 0x00020000);
    // activation operand: token row ln, bytes kb*32 .. +32 of the k-tile; rows >= M lie beyond the
    // buffer and read as zero
    const int voff_x = ln * K + kb * 32 + kt_begin * TILE_K;
    const int wt_lane = lane * 16;
    const int tile0 = nt0 * KT + kt_begin + wave;       // first weight tile of this wave

    v4u p[AT], a0[AT], a1[AT];
#pragma unroll
    for (int u = 0; u < AT; ++u)   // weights first: they come from HBM
        p[u] = __builtin_amdgcn_raw_buffer_load_b128(rw, u < tpw ? wt_lane : GV_OOB,
                                                     u < tpw ? (tile0 + u * GV_CW) * TILE_BYTES : 0, 0);
#pragma unroll
    for (int u = 0; u < AT; ++u) {
        const int vo = u < tpw ? voff_x + (wave + u * GV_CW) * TILE_K : GV_OOB;
        a0[u] = __builtin_amdgcn_raw_buffer_load_b128(rx, vo, 0, 0);
        a1[u] = __builtin_amdgcn_raw_buffer_load_b128(rx, vo + 16, 0, 0);
    }
    write_records();
    lds_barrier();

    const v4i zero4 = {0, 0, 0, 0};
    v4i acc = zero4;
    v4f y = {0.f, 0.f, 0.f, 0.f};
    for (int j = 0; j < my_nt; ++j) {
        const bool more = j + 1 < my_nt;
        const v4u *rj = rec + j * recs_per_nt * 16 + ln;
        v4u r = rj[0];   // per-channel record (overwritten per tile when GROUPED)
#pragma unroll
        for (int u = 0; u < AT; ++u) {
            const v4u pc = p[u];
            // refill the slot with the same k-tile of the next n-tile (out of range when none)
            const bool refill = more && u < tpw;
            p[u] = __builtin_amdgcn_raw_buffer_load_b128(
                rw, refill ? wt_lane : GV_OOB, refill ? (tile0 + (j + 1) * KT + u * GV_CW) * TILE_BYTES : 0, 0);
            if (u < tpw) {
                const int ktl = wave + u * GV_CW;
                if (GROUPED) r = rj[ktl * 16];
                const DecodeLut lut = {r.x, r.y, 0};
                const v4i negb = {(int)r.w, (int)r.w, (int)r.w, (int)r.w};
                const v4i c0 = as_v4i(a0[u]), c1 = as_v4i(a1[u]);
                v4i w0, w1;
                decode_lane(pc, lut, w0, w1);
                // D[i][j] = sum_k A[i][k] B[k][j]: rows i = tokens, columns j = output channels.
                // sum Xq 4(d + beta) - 4 beta sum Xq = 4 sum Xq d, exact in int32
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(c0, negb, GROUPED ? zero4 : acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(c1, negb, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(c0, w0, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(c1, w1, acc, 0, 0, 0);
                if (GROUPED) {
                    const float es = __uint_as_float(r.z);
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) y[rr] += es * (float)acc[rr];
                    if (ACC_OUT) {
                        const int g = (kt_begin + ktl) / tiles_per_group;
#pragma unroll
                        for (int rr = 0; rr < 4; ++rr) {
                            const int m = 4 * kb + rr;
                            if (m < M)
                                atomicAdd(&acc_out[((int64_t)m * N + (nt0 + j) * TILE_N + ln) * ng + g],
                                          acc[rr] >> 2);
                        }
                    }
                }
            }
        }
        if (!GROUPED) {
            const float es = __uint_as_float(r.z);
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) y[rr] = es * (float)acc[rr];
            if (ACC_OUT) {
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const int m = 4 * kb + rr;
                    if (m < M && tpw > 0)
                        atomicAdd(&acc_out[(int64_t)m * N + (nt0 + j) * TILE_N + ln], acc[rr] >> 2);
                }
            }
            acc = zero4;
        }
        // accumulator layout: lane holds tokens m = 4 kb + rr of output channel ln
        float *rb = red + ((j & 1) * GV_CW + wave) * 256;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            rb[(4 * kb + rr) * 16 + ln] = y[rr];
            y[rr] = 0.f;
        }
        lds_barrier();
    }
}

// Y[m,n] = cast(sx[m] * sum_s partial[s,m,n]), fixed order over the K-splits.
__global__ __launch_bounds__(256) void gemv_combine_kernel(const float *__restrict__ partial,
                                                           const float *__restrict__ sx, int M, int N,
                                                           int splits, uint16_t *__restrict__ Y,
                                                           int y_dtype, int64_t ldy)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)M * N) return;
    const int m = (int)(i / N), n = (int)(i - (int64_t)m * N);
    float sum = 0.f;
    for (int s = 0; s < splits; ++s) sum += partial[(int64_t)s * M * N + i];
    const float out = sx[m] * sum;
    Y[(int64_t)m * ldy + n] = (y_dtype == W4A8_F16) ? f32_to_f16_bits(out) : f32_to_bf16_bits(out);
}

GemvPlan plan_gemv(int64_t M, int64_t N, int64_t K, int64_t G)
{
    GemvPlan pl;
    const int KT = (int)(K / TILE_K), NT = (int)(N / TILE_N);
    pl.splits = (KT + GV_CW * GV_MAX_AT - 1) / (GV_CW * GV_MAX_AT);
    pl.kt_per_split = (KT + pl.splits - 1) / pl.splits;
    pl.splits = (KT + pl.kt_per_split - 1) / pl.kt_per_split;
    const int tpw = (pl.kt_per_split + GV_CW - 1) / GV_CW;
    pl.at = tpw <= 4 ? 4 : (tpw <= 6 ? 6 : 8);
    const bool grouped = G != K;
    // equal numbers of n-tiles per workgroup, about one workgroup per CU
    // (more, shorter-lived workgroups measured slower: each one reloads its activation fragments)
    int q = (int)(((int64_t)NT * pl.splits + 255) / 256);
    const int recs = grouped ? pl.kt_per_split : 1;
    const int q_lds = GV_LDS_BUDGET / (recs * 16 * 16);
    const int q_stage = grouped ? (GV_STAGE * GV_THREADS) / (recs * 16) : GV_THREADS / 16;
    if (q > q_lds) q = q_lds;
    if (q > q_stage) q = q_stage;
    if (q < 1) q = 1;
    pl.q = q;
    pl.blocks_per_split = (NT + q - 1) / q;
    pl.lds_bytes = 2 * GV_CW * 256 * 4 + q * recs * 16 * 16;
    pl.partial_bytes = pl.splits > 1 ? (size_t)pl.splits * M * N * sizeof(float) : 0;
    return pl;
}

template <bool GROUPED, bool ACC_OUT>
static void launch_gemv_at(const GemvPlan &pl, dim3 grid, hipStream_t st, const int8_t *Xq,
                           const float *sx, int M, const uint8_t *Wt, const float *step,
                           const uint8_t *zero, int N, int K, int tpg, int ng, uint16_t *Y,
                           int y_dtype, int64_t ldy, float *partial, int32_t *acc_out)
{
#define W4A8_GV_LAUNCH(AT_)                                                                      \
    hipLaunchKernelGGL((gemv_kernel<GROUPED, AT_, ACC_OUT>), grid, dim3(GV_THREADS), pl.lds_bytes, \
                       st, Xq, sx, M, Wt, step, zero, N, K, tpg, ng, Y, y_dtype, ldy, partial,   \
                       acc_out, pl.q, pl.blocks_per_split, pl.kt_per_split)
    if (pl.at == 4) W4A8_GV_LAUNCH(4);
    else if (pl.at == 6) W4A8_GV_LAUNCH(6);
    else W4A8_GV_LAUNCH(8);
#undef W4A8_GV_LAUNCH
}

int launch_gemv(const int8_t *Xq, const float *sx, int64_t M, const uint8_t *Wt, const float *step,
                const uint8_t *zero, int64_t N, int64_t K, int64_t G, void *Y, int y_dtype,
                int64_t ldy, int32_t *acc_out, float *partial, hipStream_t st)
{
    const GemvPlan pl = plan_gemv(M, N, K, G);
    const bool grouped = G != K;
    const int ng = (int)(K / G), tpg = (int)(G / TILE_K);
    const dim3 grid((unsigned)(pl.blocks_per_split * pl.splits));
    float *part = pl.splits > 1 ? partial : nullptr;
    uint16_t *y16 = (uint16_t *)Y;
    if (grouped) {
        if (acc_out)
            launch_gemv_at<true, true>(pl, grid, st, Xq, sx, (int)M, Wt, step, zero, (int)N, (int)K,
                                       tpg, ng, y16, y_dtype, ldy, part, acc_out);
        else
            launch_gemv_at<true, false>(pl, grid, st, Xq, sx, (int)M, Wt, step, zero, (int)N, (int)K,
                                        tpg, ng, y16, y_dtype, ldy, part, acc_out);
    } else {
        if (acc_out)
            launch_gemv_at<false, true>(pl, grid, st, Xq, sx, (int)M, Wt, step, zero, (int)N, (int)K,
                                        tpg, ng, y16, y_dtype, ldy, part, acc_out);
        else
            launch_gemv_at<false, false>(pl, grid, st, Xq, sx, (int)M, Wt, step, zero, (int)N,
                                         (int)K, tpg, ng, y16, y_dtype, ldy, part, acc_out);
    }
    int rc = hip_status(hipGetLastError());
    if (rc != W4A8_OK || pl.splits == 1) return rc;
    return launch_gemv_combine(part, sx, M, N, pl.splits, Y, y_dtype, ldy, st);
}

int launch_gemv_combine(const float *partial, const float *sx, int64_t M, int64_t N, int splits, void *Y,
                        int y_dtype, int64_t ldy, hipStream_t st)
{
    const int64_t outs = M * N;
    hipLaunchKernelGGL(gemv_combine_kernel, dim3((unsigned)((outs + 255) / 256)), dim3(256), 0, st,
                       partial, sx, (int)M, (int)N, splits, (uint16_t *)Y, y_dtype, ldy);
    return hip_status(hipGetLastError());
}

}  // namespace w4a8
