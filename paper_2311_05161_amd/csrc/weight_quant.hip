// dINT4 weight quantization of W diag(s)  (Eq. 1 factor Q(W diag(s)); Sec. 4.2, Eq. 5 with b = 4,
// p = 13; min-max asymmetric ranges per output channel or per group of G input channels, App. A.1).
//
// Offline and HBM-bound.  One wavefront owns one (output row, group) segment: a first sweep takes
// the min / max of w' = W * s with the range extended to contain zero, the lane-0 value of
// step = (hi - lo) / 13, 1/step and the zero-point z is shared through the wave reduction, and a
// second sweep (served by the cache) applies Eq. 5 per element.  Every floating-point step is one
// binary32 operation in the order of the definition (no contraction), divisions are IEEE.
#include "w4a8_common.hpp"

namespace w4a8 {

constexpr int WQ_THREADS = 256;

template <typename T, int V>
__device__ __forceinline__ void loadv(const T *p, float (&v)[V])
{
    if constexpr (V == 1) {
        v[0] = to_f32(p[0]);
    } else if constexpr (sizeof(T) == 4) {
#pragma unroll
        for (int i = 0; i < V; i += 2) {
            const float2 a = *reinterpret_cast<const float2 *>(p + i);
            v[i] = a.x;
            v[i + 1] = a.y;
        }
    } else if constexpr (V == 2) {
        const uint32_t a = *reinterpret_cast<const uint32_t *>(p);
        T e[2];
        __builtin_memcpy(e, &a, 4);
        v[0] = to_f32(e[0]);
        v[1] = to_f32(e[1]);
    } else {
        static_assert(V == 8, "vector width");
        const uint4 a = *reinterpret_cast<const uint4 *>(p);
        T e[8];
        __builtin_memcpy(e, &a, 16);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = to_f32(e[i]);
    }
}

// Format of the code space (Sec. 4.2): p uniform steps, with or without the two special levels
// +-c, c = step / 2^shift.  dINT4: p = 13, special, shift 1 (Eq. 5); dINT3: p = 5, special; plain
// INT4: p = 15, none; shift 2 / 3: the other special values of the sweep in App. A.5 (Table 9).
struct CodeFormat {
    int p;
    int special;
    int shift = 1;
};
__host__ __device__ constexpr CodeFormat dint4_format() { return CodeFormat{DINT4_P, 1}; }

__device__ __forceinline__ uint32_t dint4_code(float w, float istep, int z, CodeFormat f = dint4_format())
{
    // (the vector ALU, not memory, is what bounds the quantizer kernels: about twenty operations per weight
    // hold them at 3.6 TB/s, so the rule is written for few operations)
    // u is clamped first (exactly: values beyond +-64 steps saturate at an end level whatever they are), so
    // that rne and the conversion are one addition: u + 1.5 * 2^23 holds rne(u) in its low bits for |u| < 2^22
    float u = w * istep;
    u = __builtin_amdgcn_fmed3f(u, -64.0f, 64.0f);
    const int r = (int)__float_as_uint(u + 12582912.0f) - 0x4B400000;
    int c = min(max(r + z, 0), f.p);   // (one v_med3_i32)
    if (f.special) {
        // nearest level: the band of +c runs from the midpoint between 0 and c to the midpoint
        // between c and one step (0.25 .. 0.75 for c = step/2), ends as in Eq. 5; both bounds exact.
        // The two bands mirror each other, (lo_t, hi_t] and [-hi_t, -lo_t), i.e. lo_t < |u| <= hi_t,
        // and the code is 14 + the sign bit (selects, not branches: the lanes of a wave disagree all the time)
        const float lo_t = f.shift == 1 ? 0.25f : (f.shift == 2 ? 0.125f : 0.0625f);
        const float hi_t = 0.5f + lo_t;
        const float au = __builtin_fabsf(u);
        const int sp = (int)(__float_as_uint(u) >> 31) | 14;
        c = (au > lo_t && au <= hi_t) ? sp : c;
    }
    return (uint32_t)c;
}

// Min-max asymmetric parameters of a range that contains zero: step = (hi - lo) / p,
// z = clamp(rne(-lo / step), 0, p); a degenerate range gives step 1, z 0.
__device__ __forceinline__ void range_params(float lo, float hi, float &st, float &istep, int &z,
                                             CodeFormat f = dint4_format())
{
    if (hi == lo) {
        st = 1.0f;
        istep = 1.0f;
        z = 0;
    } else {
        const float range = hi - lo;
        const float pf = (float)f.p;
        st = range / pf;
        istep = 1.0f / st;
        const float nlo = -lo;
        float zf = __builtin_rintf(nlo * istep);
        zf = fminf(fmaxf(zf, 0.0f), pf);
        z = (int)zf;
    }
}

// The V scales of a lane's V consecutive columns (1 where there is no scale vector).  Eight of
// them with two 16-byte loads where the vector is aligned: eight dword loads strided by 32 bytes
// over the lanes cost the memory pipeline several times as many cycles.
template <int V>
__device__ __forceinline__ void load_scales(const float *sg, int64_t k, int s_vec, float (&sv)[V])
{
    if (sg == nullptr) {
#pragma unroll
        for (int j = 0; j < V; ++j) sv[j] = 1.0f;
    } else if (V == 8 && s_vec) {
        const float4 s0 = *reinterpret_cast<const float4 *>(sg + k);
        const float4 s1 = *reinterpret_cast<const float4 *>(sg + k + 4);
        sv[0] = s0.x; sv[1] = s0.y; sv[2] = s0.z; sv[3] = s0.w;
        sv[4 % V] = s1.x; sv[5 % V] = s1.y; sv[6 % V] = s1.z; sv[7 % V] = s1.w;
    } else {
#pragma unroll
        for (int j = 0; j < V; ++j) sv[j] = sg[k + j];
    }
}

template <typename T, int V>
__global__ __launch_bounds__(WQ_THREADS) void weight_quant_kernel(
    const T *__restrict__ W, int64_t N, int64_t K, int64_t ldw, const float *__restrict__ s,
    int64_t G, int use_given, uint8_t *__restrict__ codes, float *__restrict__ step,
    uint8_t *__restrict__ zero, CodeFormat fmt, int s_vec)
{
    const int lane = threadIdx.x & 63;
    const int64_t ng = K / G;
    const int64_t seg = (int64_t)blockIdx.x * (WQ_THREADS / WAVE) + (threadIdx.x >> 6);
    if (seg >= N * ng) return;  // whole wave leaves together
    const int64_t n = seg / ng, g = seg % ng;
    const T *w = W + n * ldw + g * G;
    const float *sg = s ? s + g * G : nullptr;

    float st, istep;
    int z;
    if (use_given) {
        st = step[seg];
        z = zero[seg];
        istep = 1.0f / st;
    } else {
        float lo = 0.0f, hi = 0.0f;
        for (int64_t k = (int64_t)lane * V; k < G; k += (int64_t)WAVE * V) {
            float v[V], sv[V];
            loadv<T, V>(w + k, v);
            load_scales<V>(sg, k, s_vec, sv);
#pragma unroll
            for (int j = 0; j < V; ++j) {
                const float x = sg ? v[j] * sv[j] : v[j];
                lo = fminf(lo, x);
                hi = fmaxf(hi, x);
            }
        }
        lo = wave_min(lo);
        hi = wave_max(hi);
        range_params(lo, hi, st, istep, z, fmt);
        if (lane == 0) {
            step[seg] = st;
            zero[seg] = (uint8_t)z;
        }
    }

    uint8_t *c = codes + n * K + g * G;
    for (int64_t k = (int64_t)lane * V; k < G; k += (int64_t)WAVE * V) {
        float v[V], sv[V];
        loadv<T, V>(w + k, v);
        load_scales<V>(sg, k, s_vec, sv);
        uint32_t q[V];
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const float x = sg ? v[j] * sv[j] : v[j];
            q[j] = dint4_code(x, istep, z, fmt);
        }
        if constexpr (V == 8) {
            const uint32_t w0 = q[0] | q[1] << 8 | q[2] << 16 | q[3] << 24;
            const uint32_t w1 = q[4] | q[5] << 8 | q[6] << 16 | q[7] << 24;
            *reinterpret_cast<uint2 *>(c + k) = make_uint2(w0, w1);
        } else if constexpr (V == 2) {
            *reinterpret_cast<uint16_t *>(c + k) = (uint16_t)(q[0] | q[1] << 8);
        } else {
            c[k] = (uint8_t)q[0];
        }
    }
}

// Groups of 128 or 256 columns: a wave takes 512 consecutive columns of a row (8 per lane, one
// 16-byte load), i.e. 4 or 2 whole groups, each reduced over its own LANES = G / 8 lanes; the
// elements stay in registers between the range and the codes, so W is read once.
template <typename T, int LANES>
__global__ __launch_bounds__(WQ_THREADS) void weight_quant_small_groups_kernel(
    const T *__restrict__ W, int64_t N, int64_t K, int64_t ldw, const float *__restrict__ s,
    int use_given, uint8_t *__restrict__ codes, float *__restrict__ step, uint8_t *__restrict__ zero,
    CodeFormat fmt, int s_vec)
{
    constexpr int G = LANES * 8;
    const int lane = threadIdx.x & 63;
    const int64_t chunks = (K + 511) / 512;
    const int64_t seg = (int64_t)blockIdx.x * (WQ_THREADS / WAVE) + (threadIdx.x >> 6);   // (row, chunk)
    if (seg >= N * chunks) return;
    const int64_t n = seg / chunks, c = seg - n * chunks;
    const int64_t k = c * 512 + lane * 8;
    if (k >= K) return;   // whole groups of LANES lanes leave together (K % G == 0)
    float v[8], x[8];
    loadv<T, 8>(W + n * ldw + k, v);
    if (s == nullptr) {
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = v[j];
    } else if (s_vec) {
        // the lane's eight scales with two 16-byte loads (eight dword loads strided by 32 bytes
        // over the lanes cost the memory pipeline several times as many cycles)
        const float4 s0 = *reinterpret_cast<const float4 *>(s + k);
        const float4 s1 = *reinterpret_cast<const float4 *>(s + k + 4);
        const float sv[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = v[j] * sv[j];
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = v[j] * s[k + j];
    }
    const int64_t pidx = n * (K / G) + k / G;
    float st, istep;
    int z;
    if (use_given) {
        st = step[pidx];
        z = zero[pidx];
        istep = 1.0f / st;
    } else {
        float lo = 0.0f, hi = 0.0f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            lo = fminf(lo, x[j]);
            hi = fmaxf(hi, x[j]);
        }
#pragma unroll
        for (int off = LANES / 2; off >= 1; off >>= 1) {
            lo = fminf(lo, __shfl_xor(lo, off, WAVE));
            hi = fmaxf(hi, __shfl_xor(hi, off, WAVE));
        }
        range_params(lo, hi, st, istep, z, fmt);
        if ((lane & (LANES - 1)) == 0) {
            step[pidx] = st;
            zero[pidx] = (uint8_t)z;
        }
    }
    uint32_t q[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) q[j] = dint4_code(x[j], istep, z, fmt);
    *reinterpret_cast<uint2 *>(codes + n * K + k) =
        make_uint2(q[0] | q[1] << 8 | q[2] << 16 | q[3] << 24, q[4] | q[5] << 8 | q[6] << 16 | q[7] << 24);
}

template <typename T>
static int launch_weight_quant_t(const T *W, int64_t N, int64_t K, int64_t ldw, const float *s,
                                 int64_t G, int use_given, uint8_t *codes, float *step,
                                 uint8_t *zero, CodeFormat fmt, hipStream_t st)
{
    const int64_t segs = N * (K / G);
    if (segs == 0) return W4A8_OK;
    const int64_t blocks = (segs + (WQ_THREADS / WAVE) - 1) / (WQ_THREADS / WAVE);
    if (blocks > 0x7fffffffLL) return W4A8_ERR_SHAPE;
    const int s_vec = (uintptr_t)s % 16 == 0;   // (G % 8 == 0 wherever eight scales are loaded at once)
    const auto aligned = [&](int v) {
        return G % v == 0 && K % v == 0 && (ldw * sizeof(T)) % (v * sizeof(T)) == 0 &&
               (uintptr_t)W % (v * sizeof(T)) == 0 && (uintptr_t)codes % v == 0 && ldw % v == 0;
    };
#define W4A8_WQ_LAUNCH(V_)                                                                        \
    hipLaunchKernelGGL((weight_quant_kernel<T, V_>), dim3((unsigned)blocks), dim3(WQ_THREADS), 0, \
                       st, W, N, K, ldw, s, G, use_given, codes, step, zero, fmt, s_vec)
    if ((G == 128 || G == 256) && aligned(8)) {
        const int64_t wsegs = N * ((K + 511) / 512);
        const int64_t wblocks = (wsegs + (WQ_THREADS / WAVE) - 1) / (WQ_THREADS / WAVE);
        if (wblocks > 0x7fffffffLL) return W4A8_ERR_SHAPE;
        if (G == 128)
            hipLaunchKernelGGL((weight_quant_small_groups_kernel<T, 16>), dim3((unsigned)wblocks),
                               dim3(WQ_THREADS), 0, st, W, N, K, ldw, s, use_given, codes, step, zero, fmt,
                               s_vec);
        else
            hipLaunchKernelGGL((weight_quant_small_groups_kernel<T, 32>), dim3((unsigned)wblocks),
                               dim3(WQ_THREADS), 0, st, W, N, K, ldw, s, use_given, codes, step, zero, fmt,
                               s_vec);
    } else if (G >= 512 && aligned(8)) {
        W4A8_WQ_LAUNCH(8);
    } else if (aligned(2)) {
        W4A8_WQ_LAUNCH(2);
    } else {
        W4A8_WQ_LAUNCH(1);
    }
#undef W4A8_WQ_LAUNCH
    return hip_status(hipGetLastError());
}

int launch_weight_quant(const void *W, int w_dtype, int64_t N, int64_t K, int64_t ldw,
                        const float *s, int64_t G, int use_given, uint8_t *codes, float *step,
                        uint8_t *zero, int format, hipStream_t st)
{
    CodeFormat fmt;
    switch (format) {
        case W4A8_FMT_DINT4: fmt = CodeFormat{13, 1}; break;
        case W4A8_FMT_INT4: fmt = CodeFormat{15, 0}; break;
        case W4A8_FMT_DINT3: fmt = CodeFormat{5, 1}; break;
        case W4A8_FMT_DINT4_C4: fmt = CodeFormat{13, 1, 2}; break;
        case W4A8_FMT_DINT4_C8: fmt = CodeFormat{13, 1, 3}; break;
        default: return W4A8_ERR_DTYPE;
    }
    switch (w_dtype) {
        case W4A8_F32:
            return launch_weight_quant_t((const float *)W, N, K, ldw, s, G, use_given, codes, step,
                                         zero, fmt, st);
        case W4A8_F16:
            return launch_weight_quant_t((const __half *)W, N, K, ldw, s, G, use_given, codes, step,
                                         zero, fmt, st);
        case W4A8_BF16:
            return launch_weight_quant_t((const bf16_t *)W, N, K, ldw, s, G, use_given, codes, step,
                                         zero, fmt, st);
        default: return W4A8_ERR_DTYPE;
    }
}

// ---- clipped ranges (App. A.4: after the scale search the weights are additionally clipped) ------
// step / zero of the (zero-containing) min-max range of each (row, group) of W diag(s), shrunk by
// rho = 1 - 0.05 i: i = idx[n] per output row, or the same `uniform` index for all rows.  The codes
// then come from quantize_weight_dint4 with these parameters given (values beyond the shrunk range
// saturate at its end levels).  One wave per (row, group).
template <typename T>
__global__ __launch_bounds__(WQ_THREADS) void clip_params_kernel(
    const T *__restrict__ W, int64_t N, int64_t K, int64_t ldw, const float *__restrict__ s, int64_t G,
    const int32_t *__restrict__ idx, int uniform, float *__restrict__ step, uint8_t *__restrict__ zero)
{
    const int lane = threadIdx.x & 63;
    const int64_t ng = K / G;
    const int64_t seg = (int64_t)blockIdx.x * (WQ_THREADS / WAVE) + (threadIdx.x >> 6);
    if (seg >= N * ng) return;
    const int64_t n = seg / ng, g = seg % ng;
    const T *w = W + n * ldw + g * G;
    const float *sg = s ? s + g * G : nullptr;
    float lo = 0.0f, hi = 0.0f;
    for (int64_t k = lane; k < G; k += WAVE) {
        const float v = to_f32(w[k]);
        const float x = sg ? v * sg[k] : v;
        lo = fminf(lo, x);
        hi = fmaxf(hi, x);
    }
    lo = wave_min(lo);
    hi = wave_max(hi);
    const float rho = 1.0f - 0.05f * (float)(idx ? idx[n] : uniform);
    lo = lo * rho;
    hi = hi * rho;
    float st, istep;
    int z;
    range_params(lo, hi, st, istep, z);
    if (lane == 0) {
        step[seg] = st;
        zero[seg] = (uint8_t)z;
    }
}

int launch_clip_params(const void *W, int w_dtype, int64_t N, int64_t K, int64_t ldw, const float *s,
                       int64_t G, const int32_t *idx, int uniform, float *step, uint8_t *zero,
                       hipStream_t st)
{
    const int64_t segs = N * (K / G);
    if (segs == 0) return W4A8_OK;
    const dim3 grid((unsigned)((segs + (WQ_THREADS / WAVE) - 1) / (WQ_THREADS / WAVE)));
#define W4A8_CP_LAUNCH(T_)                                                                        \
    hipLaunchKernelGGL((clip_params_kernel<T_>), grid, dim3(WQ_THREADS), 0, st, (const T_ *)W, N, K, \
                       ldw, s, G, idx, uniform, step, zero)
    switch (w_dtype) {
        case W4A8_F32: W4A8_CP_LAUNCH(float); break;
        case W4A8_F16: W4A8_CP_LAUNCH(__half); break;
        case W4A8_BF16: W4A8_CP_LAUNCH(bf16_t); break;
        default: return W4A8_ERR_DTYPE;
    }
#undef W4A8_CP_LAUNCH
    return hip_status(hipGetLastError());
}

// ---- 4-bit Value cache (Sec. 5.1; App. A.1: channel-wise along the dimension the product with the
// attention map accumulates over, i.e. the tokens) -------------------------------------------------
// V [batch, T, D] is stored token-major, as a cache is appended to; the product wants V^T.  A
// workgroup owns 64 channels of one (head, token group): lane = channel, so every load is 64
// consecutive elements of one token; the four waves split the tokens, their ranges meet in LDS,
// and the codes go through an LDS transpose so that each channel row is written 16 bytes at a time.
template <typename T>
__global__ __launch_bounds__(256) void value_quant_kernel(const T *__restrict__ V, int64_t Tn,
                                                          int64_t D, int64_t ld_t, int64_t ld_b,
                                                          int64_t G, uint8_t *__restrict__ codes,
                                                          float *__restrict__ step,
                                                          uint8_t *__restrict__ zero, int vec_ok)
{
    __shared__ float s_lo[4][64], s_hi[4][64];
    __shared__ uint32_t s_codes[64][17];   // [channel][16 words of 4 tokens], odd stride
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t b = blockIdx.z, g = blockIdx.y;
    const int64_t d = (int64_t)blockIdx.x * 64 + lane;
    const bool live = d < D;
    const T *v = V + b * ld_b + g * G * ld_t + (live ? d : 0);

    float lo = 0.0f, hi = 0.0f;
    if (live) {
        // eight loads in flight per lane; tokens past the group re-read its first token
        for (int64_t t = wave; t < G; t += 32) {
            float x[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = to_f32(v[(t + 4 * i < G ? t + 4 * i : 0) * ld_t]);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                lo = fminf(lo, x[i]);
                hi = fmaxf(hi, x[i]);
            }
        }
    }
    s_lo[wave][lane] = lo;
    s_hi[wave][lane] = hi;
    __syncthreads();
    lo = fminf(fminf(s_lo[0][lane], s_lo[1][lane]), fminf(s_lo[2][lane], s_lo[3][lane]));
    hi = fmaxf(fmaxf(s_hi[0][lane], s_hi[1][lane]), fmaxf(s_hi[2][lane], s_hi[3][lane]));
    float st, istep;
    int z;
    range_params(lo, hi, st, istep, z);
    const int64_t ng = Tn / G;
    if (wave == 0 && live) {
        step[(b * D + d) * ng + g] = st;
        zero[(b * D + d) * ng + g] = (uint8_t)z;
    }

    const int r = threadIdx.x >> 2, q = threadIdx.x & 3;   // write side: channel row, 16-token quarter
    const int64_t dr = (int64_t)blockIdx.x * 64 + r;
    for (int64_t c0 = 0; c0 < G; c0 += 64) {
        float x[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int64_t t = c0 + wave * 16 + i;
            x[i] = to_f32(v[(t < G ? t : 0) * ld_t]);   // all sixteen loads issued before any is used
        }
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            uint32_t word = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t t = c0 + wave * 16 + i4 * 4 + i;
                if (live && t < G) word |= dint4_code(x[i4 * 4 + i], istep, z) << (8 * i);
            }
            s_codes[lane][wave * 4 + i4] = word;
        }
        __syncthreads();
        if (dr < D) {
            const int64_t t0 = c0 + q * 16;
            uint8_t *dst = codes + (b * D + dr) * Tn + g * G + t0;
            const uint32_t *w = &s_codes[r][q * 4];
            if (vec_ok && t0 + 16 <= G) {
                *reinterpret_cast<uint4 *>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
            } else {
                for (int i = 0; i < 16 && t0 + i < G; ++i) dst[i] = (uint8_t)(w[i >> 2] >> (8 * (i & 3)));
            }
        }
        __syncthreads();
    }
}

// The same for 16-bit elements with everything 16-byte aligned (D % 8 == 0, G % 128 == 0): a thread
// loads eight consecutive channels of a token at once, so a wave instruction moves eight 128-byte
// row segments instead of one (the channel-per-lane kernel above moves 128 bytes per instruction).
// Thread (c8, t4) = (tid % 8, tid / 8) owns channels 8 c8 .. + 7 and, per block of 128 tokens, the
// four tokens 4 t4 .. + 3: exactly one 32-bit word of codes per channel, which goes through LDS to
// the thread that stores the channel's row segment.
template <typename T>
__global__ __launch_bounds__(256) void value_quant_vec_kernel(const T *__restrict__ V, int64_t Tn,
                                                              int64_t D, int64_t ld_t, int64_t ld_b,
                                                              int64_t G, uint8_t *__restrict__ codes,
                                                              float *__restrict__ step,
                                                              uint8_t *__restrict__ zero)
{
    static_assert(sizeof(T) == 2, "16-bit elements");
    __shared__ float s_lo[4][64], s_hi[4][64];
    __shared__ float s_st[64], s_istep[64];
    __shared__ int s_z[64];
    __shared__ uint32_t s_codes[64][33];   // [channel][32 words of 4 tokens], odd stride
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c8 = tid & 7, t4 = tid >> 3;
    const int64_t b = blockIdx.z, g = blockIdx.y;
    const int64_t d0 = (int64_t)blockIdx.x * 64;
    const bool live = d0 + c8 * 8 < D;   // D % 8 == 0: the eight channels are valid together
    const T *v = V + b * ld_b + g * G * ld_t + (live ? d0 + c8 * 8 : 0);

    // ---- ranges: min / max of every channel over the group's tokens -------------------------------
    float lo[8], hi[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) lo[j] = hi[j] = 0.0f;
    for (int64_t t0 = 0; t0 < G; t0 += 128) {
        float x[4][8];
#pragma unroll
        for (int i = 0; i < 4; ++i) loadv<T, 8>(v + (t0 + 4 * t4 + i) * ld_t, x[i]);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                lo[j] = fminf(lo[j], x[i][j]);
                hi[j] = fmaxf(hi[j], x[i][j]);
            }
    }
    // over the eight lanes of the wave with the same channels (lane bits 3..5), then over the waves
#pragma unroll
    for (int j = 0; j < 8; ++j) {
#pragma unroll
        for (int off = 8; off <= 32; off <<= 1) {
            lo[j] = fminf(lo[j], __shfl_xor(lo[j], off, WAVE));
            hi[j] = fmaxf(hi[j], __shfl_xor(hi[j], off, WAVE));
        }
    }
    if (lane < 8) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            s_lo[wave][lane * 8 + j] = lo[j];
            s_hi[wave][lane * 8 + j] = hi[j];
        }
    }
    __syncthreads();
    const int64_t ng = Tn / G;
    if (tid < 64) {   // one thread per channel: step, zero-point
        const float l = fminf(fminf(s_lo[0][tid], s_lo[1][tid]), fminf(s_lo[2][tid], s_lo[3][tid]));
        const float h = fmaxf(fmaxf(s_hi[0][tid], s_hi[1][tid]), fmaxf(s_hi[2][tid], s_hi[3][tid]));
        float st, istep;
        int z;
        range_params(l, h, st, istep, z);
        s_st[tid] = st;
        s_istep[tid] = istep;
        s_z[tid] = z;
        if (d0 + tid < D) {
            step[(b * D + d0 + tid) * ng + g] = st;
            zero[(b * D + d0 + tid) * ng + g] = (uint8_t)z;
        }
    }
    __syncthreads();
    float istep[8];
    int z[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        istep[j] = s_istep[c8 * 8 + j];
        z[j] = s_z[c8 * 8 + j];
    }

    // ---- codes: 128 tokens per round, transposed through LDS to token-contiguous rows ------------
    const int r = tid >> 2, q = tid & 3;   // write side: channel row, 32-token quarter
    for (int64_t t0 = 0; t0 < G; t0 += 128) {
        float x[4][8];
#pragma unroll
        for (int i = 0; i < 4; ++i) loadv<T, 8>(v + (t0 + 4 * t4 + i) * ld_t, x[i]);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            uint32_t word = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) word |= dint4_code(x[i][j], istep[j], z[j]) << (8 * i);
            s_codes[c8 * 8 + j][t4] = word;
        }
        __syncthreads();
        if (d0 + r < D) {
            uint8_t *dst = codes + (b * D + d0 + r) * Tn + g * G + t0 + q * 32;
            const uint32_t *w = &s_codes[r][q * 8];
            *reinterpret_cast<uint4 *>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
            *reinterpret_cast<uint4 *>(dst + 16) = make_uint4(w[4], w[5], w[6], w[7]);
        }
        __syncthreads();
    }
}

int launch_value_quant(const void *V, int v_dtype, int64_t batch, int64_t T, int64_t D, int64_t ld_t,
                       int64_t ld_b, int64_t G, uint8_t *codes, float *step, uint8_t *zero,
                       hipStream_t st)
{
    const dim3 grid((unsigned)((D + 63) / 64), (unsigned)(T / G), (unsigned)batch);
    const int vec_ok = (uintptr_t)codes % 16 == 0 && T % 16 == 0 && G % 16 == 0;
    // 16-bit elements, every row and every store 16-byte aligned: eight channels per load
    if (v_dtype != W4A8_F32 && vec_ok && G % 128 == 0 && D % 8 == 0 && ld_t % 8 == 0 && ld_b % 8 == 0 &&
        (uintptr_t)V % 16 == 0) {
        if (v_dtype == W4A8_F16)
            hipLaunchKernelGGL((value_quant_vec_kernel<__half>), grid, dim3(256), 0, st, (const __half *)V, T,
                               D, ld_t, ld_b, G, codes, step, zero);
        else
            hipLaunchKernelGGL((value_quant_vec_kernel<bf16_t>), grid, dim3(256), 0, st, (const bf16_t *)V, T,
                               D, ld_t, ld_b, G, codes, step, zero);
        return hip_status(hipGetLastError());
    }
#define W4A8_VQ_LAUNCH(T_)                                                                     \
    hipLaunchKernelGGL((value_quant_kernel<T_>), grid, dim3(256), 0, st, (const T_ *)V, T, D, \
                       ld_t, ld_b, G, codes, step, zero, vec_ok)
    switch (v_dtype) {
        case W4A8_F32: W4A8_VQ_LAUNCH(float); break;
        case W4A8_F16: W4A8_VQ_LAUNCH(__half); break;
        case W4A8_BF16: W4A8_VQ_LAUNCH(bf16_t); break;
        default: return W4A8_ERR_DTYPE;
    }
#undef W4A8_VQ_LAUNCH
    return hip_status(hipGetLastError());
}

// ---- sums of the quantized weights (needed to take a token zero-point out of the product) ------
// wsum[n,b] = sum_{k in block b} d[n,k], d in half steps (Eq. 5, second half), over blocks of T
// consecutive input channels (T divides the group size G): one wave per (row, block).
__global__ __launch_bounds__(256) void weight_block_sums_kernel(const uint8_t *__restrict__ codes,
                                                                const uint8_t *__restrict__ zero,
                                                                int64_t N, int64_t K, int64_t G,
                                                                int64_t T, int32_t *__restrict__ wsum)
{
    const int lane = threadIdx.x & 63;
    const int64_t ng = K / G, nb = K / T;
    const int64_t seg = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);   // (row, block)
    if (seg >= N * nb) return;
    const int64_t n = seg / nb, b = seg - n * nb;
    const int z = zero[n * ng + (b * T) / G];
    const uint8_t *c = codes + n * K + b * T;
    int sum = 0;
    for (int64_t k = lane; k < T; k += WAVE) {
        const int code = c[k] & 15;
        sum += code <= DINT4_P ? 2 * (code - z) : (code == 14 ? 1 : -1);
    }
    sum = wave_sum_i32(sum);
    if (lane == 0) wsum[seg] = sum;
}

int launch_weight_sums(const uint8_t *codes, const uint8_t *zero, int64_t N, int64_t K, int64_t G,
                       int64_t T, int32_t *wsum, hipStream_t st)
{
    const int64_t segs = N * (K / T);
    hipLaunchKernelGGL(weight_block_sums_kernel, dim3((unsigned)((segs + 3) / 4)), dim3(256), 0, st,
                       codes, zero, N, K, G, T, wsum);
    return hip_status(hipGetLastError());
}

}  // namespace w4a8
