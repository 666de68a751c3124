// Per-token absmax INT8 activation quantization of X diag(s)^-1  (Eq. 1, factor
// Q(diag(s)^-1 X); token-wise 8-bit activations, App. A.1).
//
// HBM-bound: one read of X, one write of Xq.  A workgroup of 256 lanes owns a set of token rows.
// Each lane keeps the reciprocal scales r[k] = 1/s[k] of its own columns in registers (true IEEE
// division, done once per workgroup and reused for every row), loads 8 consecutive elements per
// 16-byte access, keeps the scaled row t = x * r in registers between the absmax reduction and the
// rounding pass, and stores 8 int8 per lane.  Every floating-point step is a single binary32
// operation in the order of the definition, so the result is bit-identical to a CPU evaluation.
#include "w4a8_common.hpp"

namespace w4a8 {

constexpr int AQ_THREADS = 256;
constexpr int AQ_VEC = 8;

template <typename T>
__device__ __forceinline__ void load8(const T *p, float (&v)[8]);

template <>
__device__ __forceinline__ void load8<float>(const float *p, float (&v)[8])
{
    const float4 a = *reinterpret_cast<const float4 *>(p);
    const float4 b = *reinterpret_cast<const float4 *>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
template <>
__device__ __forceinline__ void load8<__half>(const __half *p, float (&v)[8])
{
    const uint4 a = *reinterpret_cast<const uint4 *>(p);
    const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = __half2float(__ushort_as_half((uint16_t)(w[i] & 0xffffu)));
        v[2 * i + 1] = __half2float(__ushort_as_half((uint16_t)(w[i] >> 16)));
    }
}
template <>
__device__ __forceinline__ void load8<bf16_t>(const bf16_t *p, float (&v)[8])
{
    const uint4 a = *reinterpret_cast<const uint4 *>(p);
    const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}

__device__ __forceinline__ float block_max(float v, float *red)
{
    v = wave_max(v);
    const int wave = threadIdx.x >> 6;
    __syncthreads();  // `red` may still be read by the previous row
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

__device__ __forceinline__ int quant1(float t, float inv)
{
    float q = __builtin_rintf(t * inv);  // v_rndne_f32: round half to even
    q = fminf(fmaxf(q, -127.0f), 127.0f);
    return (int)q;
}

// Fast path: K % 8 == 0, 16-byte aligned rows, K <= 256 * 8 * NCH.  Rows r0 .. r0+rows_per_block.
template <typename T, int NCH>
__global__ __launch_bounds__(AQ_THREADS) void act_quant_rows_kernel(
    const T *__restrict__ X, int64_t M, int K, int64_t ldx, const float *__restrict__ s,
    int8_t *__restrict__ Xq, float *__restrict__ sx, int rows_per_block)
{
    __shared__ float red[4];
    const int tid = threadIdx.x;
    const int nchunks = K / AQ_VEC;

    float r[NCH][AQ_VEC];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int ch = tid + c * AQ_THREADS;
#pragma unroll
        for (int j = 0; j < AQ_VEC; ++j) r[c][j] = 1.0f;
        if (s != nullptr && ch < nchunks) {
            float sv[8];
            load8<float>(s + (int64_t)ch * AQ_VEC, sv);
#pragma unroll
            for (int j = 0; j < AQ_VEC; ++j) r[c][j] = 1.0f / sv[j];
        }
    }

    const int64_t row0 = (int64_t)blockIdx.x * rows_per_block;
    for (int rr = 0; rr < rows_per_block; ++rr) {
        const int64_t m = row0 + rr;
        if (m >= M) break;  // uniform over the workgroup
        const T *x = X + m * ldx;
        float t[NCH][AQ_VEC];
        float a = 0.0f;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int ch = tid + c * AQ_THREADS;
            if (ch < nchunks) {
                float xv[8];
                load8<T>(x + (int64_t)ch * AQ_VEC, xv);
#pragma unroll
                for (int j = 0; j < AQ_VEC; ++j) {
                    t[c][j] = xv[j] * r[c][j];
                    a = fmaxf(a, fabsf(t[c][j]));
                }
            } else {
#pragma unroll
                for (int j = 0; j < AQ_VEC; ++j) t[c][j] = 0.0f;
            }
        }
        a = block_max(a, red);
        const bool zero_row = (a == 0.0f);
        const float inv = zero_row ? 0.0f : 127.0f / a;
        if (tid == 0) sx[m] = zero_row ? 1.0f : a / 127.0f;
        int8_t *q = Xq + m * (int64_t)K;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int ch = tid + c * AQ_THREADS;
            if (ch < nchunks) {
                uint32_t w0 = 0, w1 = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    w0 |= (uint32_t)(quant1(t[c][j], inv) & 0xff) << (8 * j);
                    w1 |= (uint32_t)(quant1(t[c][j + 4], inv) & 0xff) << (8 * j);
                }
                *reinterpret_cast<uint2 *>(q + (int64_t)ch * AQ_VEC) = make_uint2(w0, w1);
            }
        }
    }
}

// Any K, any alignment: one workgroup per row, scalar accesses, the row is read twice.
template <typename T>
__global__ __launch_bounds__(AQ_THREADS) void act_quant_generic_kernel(
    const T *__restrict__ X, int64_t M, int64_t K, int64_t ldx, const float *__restrict__ s,
    int8_t *__restrict__ Xq, float *__restrict__ sx)
{
    __shared__ float red[4];
    const int64_t m = blockIdx.x;
    const T *x = X + m * ldx;
    float a = 0.0f;
    for (int64_t k = threadIdx.x; k < K; k += AQ_THREADS) {
        const float r = s ? 1.0f / s[k] : 1.0f;
        const float t = to_f32(x[k]) * r;
        a = fmaxf(a, fabsf(t));
    }
    a = block_max(a, red);
    const bool zero_row = (a == 0.0f);
    const float inv = zero_row ? 0.0f : 127.0f / a;
    if (threadIdx.x == 0) sx[m] = zero_row ? 1.0f : a / 127.0f;
    int8_t *q = Xq + m * K;
    for (int64_t k = threadIdx.x; k < K; k += AQ_THREADS) {
        const float r = s ? 1.0f / s[k] : 1.0f;
        const float t = to_f32(x[k]) * r;
        q[k] = (int8_t)quant1(t, inv);
    }
}

template <typename T>
static int launch_act_quant_t(const T *X, int64_t M, int64_t K, int64_t ldx, const float *s,
                              int8_t *Xq, float *sx, hipStream_t st)
{
    const bool aligned = (K % AQ_VEC == 0) && ((ldx * sizeof(T)) % 16 == 0) &&
                         ((uintptr_t)X % 16 == 0) && ((uintptr_t)Xq % 8 == 0) &&
                         (s == nullptr || (uintptr_t)s % 16 == 0) &&
                         K <= (int64_t)AQ_THREADS * AQ_VEC * 8;
    if (!aligned) {
        hipLaunchKernelGGL((act_quant_generic_kernel<T>), dim3((unsigned)M), dim3(AQ_THREADS), 0, st,
                           X, M, K, ldx, s, Xq, sx);
        return hip_status(hipGetLastError());
    }
    // enough workgroups to fill 256 CUs twice; each amortizes its 1/s divisions over its rows
    int rows = (int)((M + 511) / 512);
    if (rows < 1) rows = 1;
    if (rows > 16) rows = 16;
    const unsigned grid = (unsigned)((M + rows - 1) / rows);
    const int nch = (int)((K / AQ_VEC + AQ_THREADS - 1) / AQ_THREADS);
#define W4A8_AQ_CASE(N_)                                                                         \
    case N_:                                                                                     \
        hipLaunchKernelGGL((act_quant_rows_kernel<T, N_>), dim3(grid), dim3(AQ_THREADS), 0, st, \
                           X, M, (int)K, ldx, s, Xq, sx, rows);                                  \
        break;
    switch (nch) {
        W4A8_AQ_CASE(1) W4A8_AQ_CASE(2) W4A8_AQ_CASE(3) W4A8_AQ_CASE(4)
        W4A8_AQ_CASE(5) W4A8_AQ_CASE(6) W4A8_AQ_CASE(7) W4A8_AQ_CASE(8)
        default: return W4A8_ERR_SHAPE;
    }
#undef W4A8_AQ_CASE
    return hip_status(hipGetLastError());
}

int launch_act_quant(const void *X, int x_dtype, int64_t M, int64_t K, int64_t ldx, const float *s,
                     int8_t *Xq, float *sx, hipStream_t st)
{
    switch (x_dtype) {
        case W4A8_F32: return launch_act_quant_t((const float *)X, M, K, ldx, s, Xq, sx, st);
        case W4A8_F16: return launch_act_quant_t((const __half *)X, M, K, ldx, s, Xq, sx, st);
        case W4A8_BF16: return launch_act_quant_t((const bf16_t *)X, M, K, ldx, s, Xq, sx, st);
        default: return W4A8_ERR_DTYPE;
    }
}

}  // namespace w4a8
