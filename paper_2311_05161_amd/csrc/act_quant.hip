// Per-token INT8 activation quantization of X diag(s)^-1  (Eq. 1, factor Q(diag(s)^-1 X);
// token-wise 8-bit activations, App. A.1): symmetric absmax (ASYM = false) or the paper's min-max
// asymmetric form with a token zero-point (ASYM = true; codes 0..255 are stored minus 128 so that
// the signed int8 matrix cores can take them, and so is the zero-point).
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

// both at once: returns max over the workgroup of (a, b)
__device__ __forceinline__ void block_max2(float &a, float &b, float *red)
{
    a = wave_max(a);
    b = wave_max(b);
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
        red[wave] = a;
        red[4 + wave] = b;
    }
    __syncthreads();
    a = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    b = fmaxf(fmaxf(red[4], red[5]), fmaxf(red[6], red[7]));
}

// asymmetric: code = clamp(rne(t * isx) + zx, 0, 255), stored as code - 128
__device__ __forceinline__ int quant1_asym(float t, float isx, float zf)
{
    float q = __builtin_rintf(t * isx) + zf;
    q = fminf(fmaxf(q, 0.0f), 255.0f);
    return (int)q - 128;
}

// Token parameters of the asymmetric form from the extremes of the (zero-extended) range.
struct AsymParams {
    float sx, isx, zf;
};
__device__ __forceinline__ AsymParams asym_params(float lo, float hi)
{
    AsymParams p;
    if (hi == lo) {   // all-zero token
        p.sx = 1.0f; p.isx = 0.0f; p.zf = 0.0f;
        return p;
    }
    const float range = hi - lo;
    p.sx = range / 255.0f;
    p.isx = 1.0f / p.sx;
    p.zf = fminf(fmaxf(__builtin_rintf(-lo * p.isx), 0.0f), 255.0f);
    return p;
}

__device__ __forceinline__ int quant1(float t, float inv)
{
    float q = __builtin_rintf(t * inv);  // v_rndne_f32: round half to even
    q = fminf(fmaxf(q, -127.0f), 127.0f);
    return (int)q;
}

// Fast path: K % 8 == 0, 16-byte aligned rows, K <= 256 * 8 * NCH.  Rows r0 .. r0+rows_per_block.
template <typename T, int NCH, bool ASYM>
__global__ __launch_bounds__(AQ_THREADS) void act_quant_rows_kernel(
    const T *__restrict__ X, int64_t M, int K, int64_t ldx, const float *__restrict__ s,
    int8_t *__restrict__ Xq, float *__restrict__ sx, int32_t *__restrict__ zx, int rows_per_block)
{
    __shared__ float red[8];
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
        float a = 0.0f, b = 0.0f;   // symmetric: a = max |t|;  asymmetric: a = max(0, t), b = max(0, -t)
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int ch = tid + c * AQ_THREADS;
            if (ch < nchunks) {
                float xv[8];
                load8<T>(x + (int64_t)ch * AQ_VEC, xv);
#pragma unroll
                for (int j = 0; j < AQ_VEC; ++j) {
                    t[c][j] = xv[j] * r[c][j];
                    if (ASYM) {
                        a = fmaxf(a, t[c][j]);
                        b = fmaxf(b, -t[c][j]);
                    } else {
                        a = fmaxf(a, fabsf(t[c][j]));
                    }
                }
            } else {
#pragma unroll
                for (int j = 0; j < AQ_VEC; ++j) t[c][j] = 0.0f;
            }
        }
        float inv = 0.0f;
        AsymParams ap = {1.0f, 0.0f, 0.0f};
        if (ASYM) {
            block_max2(a, b, red);
            ap = asym_params(-b, a);   // lo = -max(0, -t) = min(0, t)
            if (tid == 0) {
                sx[m] = ap.sx;
                zx[m] = (int)ap.zf - 128;
            }
        } else {
            a = block_max(a, red);
            const bool zero_row = (a == 0.0f);
            inv = zero_row ? 0.0f : 127.0f / a;
            if (tid == 0) sx[m] = zero_row ? 1.0f : a / 127.0f;
        }
        int8_t *q = Xq + m * (int64_t)K;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int ch = tid + c * AQ_THREADS;
            if (ch < nchunks) {
                uint32_t w0 = 0, w1 = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int q0 = ASYM ? quant1_asym(t[c][j], ap.isx, ap.zf) : quant1(t[c][j], inv);
                    const int q1 = ASYM ? quant1_asym(t[c][j + 4], ap.isx, ap.zf) : quant1(t[c][j + 4], inv);
                    w0 |= (uint32_t)(q0 & 0xff) << (8 * j);
                    w1 |= (uint32_t)(q1 & 0xff) << (8 * j);
                }
                *reinterpret_cast<uint2 *>(q + (int64_t)ch * AQ_VEC) = make_uint2(w0, w1);
            }
        }
    }
}

// Any K, any alignment: one workgroup per row, scalar accesses, the row is read twice.
template <typename T, bool ASYM>
__global__ __launch_bounds__(AQ_THREADS) void act_quant_generic_kernel(
    const T *__restrict__ X, int64_t M, int64_t K, int64_t ldx, const float *__restrict__ s,
    int8_t *__restrict__ Xq, float *__restrict__ sx, int32_t *__restrict__ zx)
{
    __shared__ float red[8];
    const int64_t m = blockIdx.x;
    const T *x = X + m * ldx;
    float a = 0.0f, b = 0.0f;
    for (int64_t k = threadIdx.x; k < K; k += AQ_THREADS) {
        const float r = s ? 1.0f / s[k] : 1.0f;
        const float t = to_f32(x[k]) * r;
        if (ASYM) {
            a = fmaxf(a, t);
            b = fmaxf(b, -t);
        } else {
            a = fmaxf(a, fabsf(t));
        }
    }
    float inv = 0.0f;
    AsymParams ap = {1.0f, 0.0f, 0.0f};
    if (ASYM) {
        block_max2(a, b, red);
        ap = asym_params(-b, a);
        if (threadIdx.x == 0) {
            sx[m] = ap.sx;
            zx[m] = (int)ap.zf - 128;
        }
    } else {
        a = block_max(a, red);
        const bool zero_row = (a == 0.0f);
        inv = zero_row ? 0.0f : 127.0f / a;
        if (threadIdx.x == 0) sx[m] = zero_row ? 1.0f : a / 127.0f;
    }
    int8_t *q = Xq + m * K;
    for (int64_t k = threadIdx.x; k < K; k += AQ_THREADS) {
        const float r = s ? 1.0f / s[k] : 1.0f;
        const float t = to_f32(x[k]) * r;
        q[k] = (int8_t)(ASYM ? quant1_asym(t, ap.isx, ap.zf) : quant1(t, inv));
    }
}

template <typename T, bool ASYM>
static int launch_act_quant_t(const T *X, int64_t M, int64_t K, int64_t ldx, const float *s,
                              int8_t *Xq, float *sx, int32_t *zx, hipStream_t st)
{
    const bool aligned = (K % AQ_VEC == 0) && ((ldx * sizeof(T)) % 16 == 0) &&
                         ((uintptr_t)X % 16 == 0) && ((uintptr_t)Xq % 8 == 0) &&
                         (s == nullptr || (uintptr_t)s % 16 == 0) &&
                         K <= (int64_t)AQ_THREADS * AQ_VEC * 8;
    if (!aligned) {
        hipLaunchKernelGGL((act_quant_generic_kernel<T, ASYM>), dim3((unsigned)M), dim3(AQ_THREADS),
                           0, st, X, M, K, ldx, s, Xq, sx, zx);
        return hip_status(hipGetLastError());
    }
    // enough workgroups to fill 256 CUs twice; each amortizes its 1/s divisions over its rows
    int rows = (int)((M + 511) / 512);
    if (rows < 1) rows = 1;
    if (rows > 16) rows = 16;
    const unsigned grid = (unsigned)((M + rows - 1) / rows);
    const int nch = (int)((K / AQ_VEC + AQ_THREADS - 1) / AQ_THREADS);
#define W4A8_AQ_CASE(N_)                                                                       \
    case N_:                                                                                   \
        hipLaunchKernelGGL((act_quant_rows_kernel<T, N_, ASYM>), dim3(grid), dim3(AQ_THREADS), \
                           0, st, X, M, (int)K, ldx, s, Xq, sx, zx, rows);                     \
        break;
    switch (nch) {
        W4A8_AQ_CASE(1) W4A8_AQ_CASE(2) W4A8_AQ_CASE(3) W4A8_AQ_CASE(4)
        W4A8_AQ_CASE(5) W4A8_AQ_CASE(6) W4A8_AQ_CASE(7) W4A8_AQ_CASE(8)
        default: return W4A8_ERR_SHAPE;
    }
#undef W4A8_AQ_CASE
    return hip_status(hipGetLastError());
}

// zx == nullptr: symmetric absmax; else asymmetric min-max with the token zero-points in zx
int launch_act_quant(const void *X, int x_dtype, int64_t M, int64_t K, int64_t ldx, const float *s,
                     int8_t *Xq, float *sx, int32_t *zx, hipStream_t st)
{
#define W4A8_AQ_T(T_)                                                                       \
    (zx ? launch_act_quant_t<T_, true>((const T_ *)X, M, K, ldx, s, Xq, sx, zx, st)         \
        : launch_act_quant_t<T_, false>((const T_ *)X, M, K, ldx, s, Xq, sx, nullptr, st))
    switch (x_dtype) {
        case W4A8_F32: return W4A8_AQ_T(float);
        case W4A8_F16: return W4A8_AQ_T(__half);
        case W4A8_BF16: return W4A8_AQ_T(bf16_t);
        default: return W4A8_ERR_DTYPE;
    }
#undef W4A8_AQ_T
}

}  // namespace w4a8
