// dINT4 x INT8 GEMM, decode shape (M <= 16): a memory-bound GEMV that streams the packed
// weights exactly once  (Eq. 1 product on the integer operands; Eq. 5 second half fused as the
// epilogue; the dINT4 x INT8 multiply-accumulate of Sec. 4.3 mapped onto the int8 matrix cores).
//
// One workgroup owns 16 output channels (one row of 1 KB tiles of the tiled weight layout) and
// its 8 wavefronts split K: wave w takes tiles w, w+8, ...  A lane reads its 16 packed bytes with
// one 16-byte load (the wave reads a contiguous 1 KB tile), decodes the nibbles to int8 through the
// per-(row, group) register LUT, and issues v_mfma_i32_16x16x64_i8 with the <= 16 token rows as
// the other operand.  A second MFMA against an all-ones operand yields the tokens' group row-sums in
// the accumulator layout; they remove the decode bias exactly.  Group partial sums are scaled to
// fp32 per group, the 8 waves are summed through LDS in a fixed order (deterministic), and the
// epilogue applies the token scale and casts to fp16 / bf16.
#include "w4a8_common.hpp"

namespace w4a8 {

constexpr int GV_WAVES = 8;
constexpr int GV_THREADS = GV_WAVES * WAVE;
constexpr int GV_UNROLL = 4;

__global__ __launch_bounds__(GV_THREADS) void gemv_kernel(
    const int8_t *__restrict__ Xq, const float *__restrict__ sx, int M,
    const v4u *__restrict__ Wt, const float *__restrict__ step, const uint8_t *__restrict__ zero,
    int N, int K, int tiles_per_group, int ng, void *__restrict__ Y, int y_dtype, int64_t ldy,
    int32_t *__restrict__ acc_out)
{
    __shared__ float red[GV_WAVES][256];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int ln = lane & 15;   // operand row: output channel (weights) / token (activations)
    const int kb = lane >> 4;   // which 32 columns of the 128-column tile this lane holds
    const int KT = K / TILE_K;
    const int nt = blockIdx.x;
    const int n = nt * TILE_N + ln;

    const v4u *wp = Wt + (int64_t)nt * KT * WAVE + lane;
    const int8_t *xa = Xq + (int64_t)ln * K + kb * 32;
    const bool a_valid = ln < M;
    const float *stp = step + (int64_t)n * ng;
    const uint8_t *zp = zero + (int64_t)n * ng;

    const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
    v4i acc = {0, 0, 0, 0};
    v4i rsum = {0, 0, 0, 0};
    v4f y = {0.f, 0.f, 0.f, 0.f};
    int cur_g = -1;
    DecodeLut lut = make_decode_lut(0);
    float eighth_step = 0.f;

    auto flush = [&]() {
        // acc = sum Xq * 4 (d + beta); remove the bias: 4 sum Xq d = acc - 4 beta * rowsum (exact)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int v = acc[r] - lut.beta_q * rsum[r];
            y[r] += eighth_step * (float)v;
            if (acc_out != nullptr) {
                const int m = 4 * kb + r;
                if (m < M) atomicAdd(&acc_out[((int64_t)m * N + n) * ng + cur_g], v >> 2);
            }
            acc[r] = 0;
            rsum[r] = 0;
        }
    };

    for (int kt0 = wave; kt0 < KT; kt0 += GV_WAVES * GV_UNROLL) {
        v4u p[GV_UNROLL];
        v4i a0[GV_UNROLL], a1[GV_UNROLL];
        int zz[GV_UNROLL];
        float ss[GV_UNROLL];
#pragma unroll
        for (int u = 0; u < GV_UNROLL; ++u) {
            const int kt = kt0 + u * GV_WAVES;
            p[u] = v4u{0, 0, 0, 0};
            a0[u] = v4i{0, 0, 0, 0};
            a1[u] = v4i{0, 0, 0, 0};
            zz[u] = 0;
            ss[u] = 0.f;
            if (kt < KT) {
                p[u] = wp[(int64_t)kt * WAVE];
                const int g = kt / tiles_per_group;
                zz[u] = zp[g];
                ss[u] = stp[g];
                if (a_valid) {
                    a0[u] = *reinterpret_cast<const v4i *>(xa + (int64_t)kt * TILE_K);
                    a1[u] = *reinterpret_cast<const v4i *>(xa + (int64_t)kt * TILE_K + 16);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < GV_UNROLL; ++u) {
            const int kt = kt0 + u * GV_WAVES;
            if (kt < KT) {
                const int g = kt / tiles_per_group;
                if (g != cur_g) {
                    if (cur_g >= 0) flush();
                    cur_g = g;
                    lut = make_decode_lut(zz[u]);
                    eighth_step = ss[u] * 0.125f;
                }
                v4i w0, w1;
                decode_lane(p[u], lut, w0, w1);
                // D[i][j] = sum_k A[i][k] B[k][j]: rows i = tokens, columns j = output channels
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0[u], w0, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1[u], w1, acc, 0, 0, 0);
                rsum = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0[u], ones, rsum, 0, 0, 0);
                rsum = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1[u], ones, rsum, 0, 0, 0);
            }
        }
    }
    if (cur_g >= 0) flush();

    // lane holds tokens m = 4 kb + r of output channel ln
#pragma unroll
    for (int r = 0; r < 4; ++r) red[wave][(4 * kb + r) * 16 + ln] = y[r];
    __syncthreads();
    if (threadIdx.x < 256) {
        const int m = threadIdx.x >> 4, nn = threadIdx.x & 15;
        if (m < M) {
            float sum = 0.f;
#pragma unroll
            for (int w = 0; w < GV_WAVES; ++w) sum += red[w][threadIdx.x];
            const float out = sx[m] * sum;
            uint16_t *yp = reinterpret_cast<uint16_t *>(Y) + (int64_t)m * ldy + nt * TILE_N + nn;
            *yp = (y_dtype == W4A8_F16) ? f32_to_f16_bits(out) : f32_to_bf16_bits(out);
        }
    }
}

int launch_gemv(const int8_t *Xq, const float *sx, int64_t M, const uint8_t *Wt, const float *step,
                const uint8_t *zero, int64_t N, int64_t K, int64_t G, void *Y, int y_dtype,
                int64_t ldy, int32_t *acc_out, hipStream_t st)
{
    const int ng = (int)(K / G);
    hipLaunchKernelGGL(gemv_kernel, dim3((unsigned)(N / TILE_N)), dim3(GV_THREADS), 0, st, Xq, sx,
                       (int)M, (const v4u *)Wt, step, zero, (int)N, (int)K, (int)(G / TILE_K), ng,
                       Y, y_dtype, ldy, acc_out);
    return hip_status(hipGetLastError());
}

}  // namespace w4a8
