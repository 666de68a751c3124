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

constexpr float AQ_FLT_MAX = 3.402823466e+38f;   // a token whose 127 / max|t| is not finite counts as all-zero

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
    const float range = hi - lo;
    p.sx = range / 255.0f;
    p.isx = 1.0f / p.sx;
    if (!(p.isx <= AQ_FLT_MAX)) {   // all-zero token, or a range so small that the reciprocal scale overflows
        p.sx = 1.0f; p.isx = 0.0f; p.zf = 0.0f;
        return p;
    }
    p.zf = fminf(fmaxf(__builtin_rintf(-lo * p.isx), 0.0f), 255.0f);
    return p;
}

__device__ __forceinline__ int quant1(float t, float inv)
{
    float q = __builtin_rintf(t * inv);  // v_rndne_f32: round half to even
    q = fminf(fmaxf(q, -127.0f), 127.0f);
    return (int)q;
}

// Eight consecutive elements of a row as they come from memory (16 bytes of a 16-bit type, 32 of
// binary32), and their exact widening.
template <typename T> struct Raw8 { uint4 v; };
template <> struct Raw8<float> { float4 a, b; };

template <typename T>
__device__ __forceinline__ Raw8<T> load_raw8(const T *p)
{
    Raw8<T> r;
    // (streaming loads: the unquantized activations are read exactly once)
    const v4u t = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(p));
    r.v = make_uint4(t.x, t.y, t.z, t.w);
    return r;
}
template <>
__device__ __forceinline__ Raw8<float> load_raw8<float>(const float *p)
{
    Raw8<float> r;
    const v4f a = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(p));
    const v4f b = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(p + 4));
    r.a = make_float4(a.x, a.y, a.z, a.w);
    r.b = make_float4(b.x, b.y, b.z, b.w);
    return r;
}
__device__ __forceinline__ void widen8(const Raw8<float> &r, float (&v)[8])
{
    v[0] = r.a.x; v[1] = r.a.y; v[2] = r.a.z; v[3] = r.a.w;
    v[4] = r.b.x; v[5] = r.b.y; v[6] = r.b.z; v[7] = r.b.w;
}
__device__ __forceinline__ void widen8(const Raw8<__half> &r, float (&v)[8])
{
    const uint32_t w[4] = {r.v.x, r.v.y, r.v.z, r.v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = __half2float(__ushort_as_half((uint16_t)(w[i] & 0xffffu)));
        v[2 * i + 1] = __half2float(__ushort_as_half((uint16_t)(w[i] >> 16)));
    }
}
__device__ __forceinline__ void widen8(const Raw8<bf16_t> &r, float (&v)[8])
{
    const uint32_t w[4] = {r.v.x, r.v.y, r.v.z, r.v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}

// Four rounded codes (the low bytes of q0..q3) packed into one word.
__device__ __forceinline__ uint32_t pack4_low_bytes(uint32_t q0, uint32_t q1, uint32_t q2, uint32_t q3)
{
    const uint32_t lo = __builtin_amdgcn_perm(q1, q0, 0x0c0c0400u);   // [q0.b0, q1.b0, 0, 0]
    const uint32_t hi = __builtin_amdgcn_perm(q3, q2, 0x04000c0cu);   // [0, 0, q2.b0, q3.b0]
    return lo | hi;
}

// Symmetric form, rne and the conversion to an integer in one binary32 addition: y + 1.5 * 2^23 is
// 1.5 * 2^23 + rne(y) exactly for |y| <= 2^22 (the sum is rounded to nearest even at unit
// granularity), so the low byte of its bit pattern is rne(y) in two's complement.  The clamp to
// +-127 of the definition never changes a value: |t| <= a and inv = fl(127 / a) give
// |fl(t * inv)| <= 127 (1 + 2^-23), which rounds to 127.  (No contraction in this file: the product
// is rounded before the addition, as in the definition.)
__device__ __forceinline__ uint32_t quant1_bits(float t, float inv)
{
    return __float_as_uint(t * inv + 12582912.0f);
}

// Fast path: K % 8 == 0, 16-byte aligned rows, K <= 256 * 8 * NCH.  Rows r0 .. r0+rows_per_block.
// What bounds this kernel is memory latency, not bandwidth (a row is only 2 K bytes), so the loads
// of a workgroup's next row are issued before anything is done with the current one (the first row's
// before the reciprocal scales are computed; a second row of look-ahead measured the same), and the
// launch keeps about three workgroups on every CU.
template <typename T, int NCH, bool ASYM>
__global__ __launch_bounds__(AQ_THREADS) void act_quant_rows_kernel(
    const T *__restrict__ X, int64_t M, int K, int64_t ldx, const float *__restrict__ s,
    int8_t *__restrict__ Xq, float *__restrict__ sx, int32_t *__restrict__ zx, int rows_per_block)
{
    __shared__ float red[8];
    const int tid = threadIdx.x;
    const int nchunks = K / AQ_VEC;
    const int64_t row0 = (int64_t)blockIdx.x * rows_per_block;
    const int nrows = (int)min((int64_t)rows_per_block, M - row0);   // >= 1 by the grid size

    Raw8<T> cur[NCH], nxt[NCH];   // row m (being processed) and row m + 1 (on its way)
    auto load_row = [&](int64_t m, Raw8<T>(&dst)[NCH]) {
        const T *x = X + m * ldx;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int ch = tid + c * AQ_THREADS;
            if (ch < nchunks) dst[c] = load_raw8<T>(x + (int64_t)ch * AQ_VEC);
        }
    };
    load_row(row0, cur);

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

    for (int rr = 0; rr < nrows; ++rr) {
        const int64_t m = row0 + rr;
        if (rr + 1 < nrows) load_row(m + 1, nxt);   // (uniform over the workgroup)
        float t[NCH][AQ_VEC];
        float a = 0.0f, b = 0.0f;   // symmetric: a = max |t|;  asymmetric: a = max(0, t), b = max(0, -t)
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int ch = tid + c * AQ_THREADS;
            if (ch < nchunks) {
                float xv[8];
                widen8(cur[c], xv);
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
            const float inv0 = 127.0f / a;
            const bool zero_row = !(inv0 <= AQ_FLT_MAX);   // a == 0, or so small that 127 / a overflows
            inv = zero_row ? 0.0f : inv0;
            if (tid == 0) sx[m] = zero_row ? 1.0f : a / 127.0f;
        }
        int8_t *q = Xq + m * (int64_t)K;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int ch = tid + c * AQ_THREADS;
            if (ch < nchunks) {
                uint32_t w0 = 0, w1 = 0;
                if (ASYM) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int q0 = quant1_asym(t[c][j], ap.isx, ap.zf);
                        const int q1 = quant1_asym(t[c][j + 4], ap.isx, ap.zf);
                        w0 |= (uint32_t)(q0 & 0xff) << (8 * j);
                        w1 |= (uint32_t)(q1 & 0xff) << (8 * j);
                    }
                } else {   // rounding and conversion in one addition, four codes packed by two byte permutes
                    uint32_t b[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) b[j] = quant1_bits(t[c][j], inv);
                    w0 = pack4_low_bytes(b[0], b[1], b[2], b[3]);
                    w1 = pack4_low_bytes(b[4], b[5], b[6], b[7]);
                }
                *reinterpret_cast<uint2 *>(q + (int64_t)ch * AQ_VEC) = make_uint2(w0, w1);
            }
        }
#pragma unroll
        for (int c = 0; c < NCH; ++c) cur[c] = nxt[c];
    }
}

// One wavefront per token row (rows of up to 512 * NCW elements): no workgroup barrier in the row
// loop at all.  The lane keeps the scaled row t = x * r (binary32) in registers between the maximum and
// the rounding, and the raw chunks of the wave's next row, whose loads are issued as soon as the
// current row has been widened; the reciprocal scales 1 / s[k] are computed once per workgroup into
// LDS (true IEEE division) and read from there; the row maximum is a data-parallel-primitive
// reduction.  Rows are addressed through buffer descriptors of exactly one row: chunks beyond a
// ragged row's end load zeros and their stores are dropped by the bounds check (the whole offset
// is a vector offset: a scalar offset would not be checked), so the chunk code has no branches.
constexpr int AQW_WAVES = 4;
template <typename T, int NCW, bool ASYM>
__global__ __launch_bounds__(AQW_WAVES *WAVE, 2) void act_quant_wave_kernel(
    const T *__restrict__ X, int64_t M, int K, int64_t ldx, const float *__restrict__ s,
    int8_t *__restrict__ Xq, float *__restrict__ sx, int32_t *__restrict__ zx, int rows_per_wave)
{
    // [2][NCW * 64] float4: elements 0..3 and 4..7 of every chunk's reciprocals, each half contiguous
    // over the chunks so that a wave's 16-byte reads are conflict free; zero beyond the row's end
    extern __shared__ __attribute__((aligned(16))) float r_lds[];
    constexpr int CHUNKS = NCW * WAVE;
    constexpr int RAW = (int)sizeof(T) * AQ_VEC;   // bytes of a chunk in X
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nchunks = K / AQ_VEC;
    const int64_t row0 = ((int64_t)blockIdx.x * AQW_WAVES + wave) * rows_per_wave;
    const int nrows = (int)max((int64_t)0, min((int64_t)rows_per_wave, M - row0));

    Raw8<T> nxt[NCW];
    auto load_row = [&](int64_t m) {
        __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)(X + m * ldx), 0, K * (int)sizeof(T), 0x00020000);
#pragma unroll
        for (int c = 0; c < NCW; ++c) {
            if constexpr (sizeof(T) == 2) {
                const v4u v = __builtin_amdgcn_raw_buffer_load_b128(rx, (lane + c * WAVE) * RAW, 0, 2);   // (aux 2: non-temporal)
                nxt[c].v = make_uint4(v.x, v.y, v.z, v.w);
            } else {
                const v4u v0 = __builtin_amdgcn_raw_buffer_load_b128(rx, (lane + c * WAVE) * RAW, 0, 2);   // (aux 2: non-temporal)
                const v4u v1 = __builtin_amdgcn_raw_buffer_load_b128(rx, (lane + c * WAVE) * RAW + 16, 0, 2);
                nxt[c].a = make_float4(__uint_as_float(v0.x), __uint_as_float(v0.y), __uint_as_float(v0.z), __uint_as_float(v0.w));
                nxt[c].b = make_float4(__uint_as_float(v1.x), __uint_as_float(v1.y), __uint_as_float(v1.z), __uint_as_float(v1.w));
            }
        }
    };
    if (nrows > 0) load_row(row0);

    for (int ch = tid; ch < CHUNKS; ch += AQW_WAVES * WAVE) {
        float4 r0 = make_float4(0.0f, 0.0f, 0.0f, 0.0f), r1 = r0;
        if (ch < nchunks) {
            r0 = r1 = make_float4(1.0f, 1.0f, 1.0f, 1.0f);
            if (s != nullptr) {
                float sv[8];
                load8<float>(s + (int64_t)ch * AQ_VEC, sv);
                r0 = make_float4(1.0f / sv[0], 1.0f / sv[1], 1.0f / sv[2], 1.0f / sv[3]);
                r1 = make_float4(1.0f / sv[4], 1.0f / sv[5], 1.0f / sv[6], 1.0f / sv[7]);
            }
        }
        reinterpret_cast<float4 *>(r_lds)[ch] = r0;
        reinterpret_cast<float4 *>(r_lds)[CHUNKS + ch] = r1;
    }
    __syncthreads();
    const float4 *r_lane = reinterpret_cast<const float4 *>(r_lds) + lane;

    for (int rr = 0; rr < nrows; ++rr) {   // (uniform over the wave)
        const int64_t m = row0 + rr;
        float t[NCW][AQ_VEC];
        float a = 0.0f, b = 0.0f;   // symmetric: a = max |t|;  asymmetric: a = max(0, t), b = max(0, -t)
        // (the reciprocals are fetched one chunk ahead and no further: left to itself the compiler
        // reads all of them up front, 8 registers per chunk, and spills the row)
        float4 r0n = r_lane[0], r1n = r_lane[CHUNKS];
#pragma unroll
        for (int c = 0; c < NCW; ++c) {
            float xv[8];
            widen8(nxt[c], xv);
            const float4 r0 = r0n, r1 = r1n;
            if (c + 1 < NCW) {
                r0n = r_lane[(c + 1) * WAVE];
                r1n = r_lane[CHUNKS + (c + 1) * WAVE];
            }
            __builtin_amdgcn_sched_barrier(0);
            t[c][0] = xv[0] * r0.x; t[c][1] = xv[1] * r0.y; t[c][2] = xv[2] * r0.z; t[c][3] = xv[3] * r0.w;
            t[c][4] = xv[4] * r1.x; t[c][5] = xv[5] * r1.y; t[c][6] = xv[6] * r1.z; t[c][7] = xv[7] * r1.w;
#pragma unroll
            for (int j = 0; j < AQ_VEC; ++j) {
                if (ASYM) {
                    a = fmaxf(a, t[c][j]);
                    b = fmaxf(b, -t[c][j]);
                } else {
                    a = fmaxf(a, fabsf(t[c][j]));
                }
            }
        }
        // the raw registers are free again: the next row's loads go out before the reduction
        if (rr + 1 < nrows) load_row(m + 1);
        float inv = 0.0f;
        AsymParams ap = {1.0f, 0.0f, 0.0f};
        a = wave_max(a);
        if (ASYM) {
            b = wave_max(b);
            ap = asym_params(-b, a);   // lo = -max(0, -t) = min(0, t)
            if (lane == 0) {
                sx[m] = ap.sx;
                zx[m] = (int)ap.zf - 128;
            }
        } else {
            const float inv0 = 127.0f / a;
            const bool zero_row = !(inv0 <= AQ_FLT_MAX);   // a == 0, or so small that 127 / a overflows
            inv = zero_row ? 0.0f : inv0;
            if (lane == 0) sx[m] = zero_row ? 1.0f : a / 127.0f;
        }
        __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc((void *)(Xq + m * (int64_t)K), 0, K, 0x00020000);
#pragma unroll
        for (int c = 0; c < NCW; ++c) {
            uint32_t b8[8];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                b8[j] = ASYM ? (uint32_t)quant1_asym(t[c][j], ap.isx, ap.zf) : quant1_bits(t[c][j], inv);
            const v2u out = {pack4_low_bytes(b8[0], b8[1], b8[2], b8[3]), pack4_low_bytes(b8[4], b8[5], b8[6], b8[7])};
            __builtin_amdgcn_raw_buffer_store_b64(out, rq, (lane + c * WAVE) * AQ_VEC, 0, 0);
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
        const float inv0 = 127.0f / a;
        const bool zero_row = !(inv0 <= AQ_FLT_MAX);   // a == 0, or so small that 127 / a overflows
        inv = zero_row ? 0.0f : inv0;
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
    // Rows of up to 5120 16-bit (3072 binary32) elements: one wave per row, the scaled row and the next
    // row's raw chunks in its registers.
    const int ncw = (int)((K / AQ_VEC + WAVE - 1) / WAVE);
    if (ncw <= (sizeof(T) == 2 ? 10 : 6)) {
        // about eight waves per CU, all resident at once; a workgroup's four waves amortize its 1/s
        // divisions over their rows
        int rows = (int)((M + 2047) / 2048);
        if (rows > 8) rows = 8;
        const unsigned grid = (unsigned)((M + (int64_t)rows * AQW_WAVES - 1) / ((int64_t)rows * AQW_WAVES));
        size_t lds = 0;   // reciprocal scales of the instance's NCW * 64 chunks, <= 36 KB
#define W4A8_AQW_CASE(N_)                                                                          \
    if (ncw <= N_) {                                                                               \
        lds = (size_t)N_ * WAVE * AQ_VEC * sizeof(float);                                          \
        hipLaunchKernelGGL((act_quant_wave_kernel<T, N_, ASYM>), dim3(grid), dim3(AQW_WAVES *WAVE), \
                           lds, st, X, M, (int)K, ldx, s, Xq, sx, zx, rows);                       \
        return hip_status(hipGetLastError());                                                      \
    }
        W4A8_AQW_CASE(2) W4A8_AQW_CASE(4) W4A8_AQW_CASE(6)
        if constexpr (sizeof(T) == 2) {
            W4A8_AQW_CASE(8) W4A8_AQW_CASE(10)
        }
#undef W4A8_AQW_CASE
    }
    // longer rows: a workgroup of 256 lanes per row; about three workgroups per CU, all resident at once
    int rows = (int)((M + 767) / 768);
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
