// Bit-packing of dINT4 codes, two per byte (the 4-bit storage of Sec. 4.2), in the canonical
// row-major layout and in the tiled layout the GEMM kernels stream (both defined in w4a8.h),
// plus the inverse maps and the canonical -> tiled conversion.  Pure integer byte shuffling.
#include "w4a8_common.hpp"

namespace w4a8 {

constexpr int PK_THREADS = 256;

// code -> stored nibble of the tiled layout and back (w4a8.h): integer code c = 2l + h becomes
// l | h << 3; the special pair (-step/2, +step/2) = codes (15, 14) becomes l = 7 with h = (0, 1).
__device__ __forceinline__ uint32_t recode(uint32_t c)
{
    c &= 15u;
    return c <= 13u ? ((c >> 1) | ((c & 1u) << 3)) : (c == 14u ? 15u : 7u);
}
__device__ __forceinline__ uint32_t uncode(uint32_t e)
{
    const uint32_t l = e & 7u, h = e >> 3;
    return l < 7u ? (2u * l + h) : (h ? 14u : 15u);
}

__global__ __launch_bounds__(PK_THREADS) void pack_canonical_kernel(
    const uint8_t *__restrict__ codes, int64_t total_bytes, uint8_t *__restrict__ packed)
{
    // rows are contiguous and K is even, so output byte i pairs codes 2i and 2i+1
    for (int64_t i = (int64_t)blockIdx.x * PK_THREADS + threadIdx.x; i < total_bytes;
         i += (int64_t)gridDim.x * PK_THREADS) {
        const uint32_t a = codes[2 * i] & 15u, b = codes[2 * i + 1] & 15u;
        packed[i] = (uint8_t)(a | (b << 4));
    }
}

__global__ __launch_bounds__(PK_THREADS) void unpack_canonical_kernel(
    const uint8_t *__restrict__ packed, int64_t total_bytes, uint8_t *__restrict__ codes)
{
    for (int64_t i = (int64_t)blockIdx.x * PK_THREADS + threadIdx.x; i < total_bytes;
         i += (int64_t)gridDim.x * PK_THREADS) {
        const uint32_t b = packed[i];
        codes[2 * i] = (uint8_t)(b & 15u);
        codes[2 * i + 1] = (uint8_t)(b >> 4);
    }
}

// Word index o of the tiled buffer -> (row n, first column k) of its 8 codes.
__device__ __forceinline__ void tiled_word_coords(int64_t o, int64_t KT, int64_t &n, int64_t &k)
{
    const int q = (int)(o & 3);
    const int lane = (int)((o >> 2) & 63);
    const int64_t tile = o >> 8;
    const int64_t nt = tile / KT, kt = tile % KT;
    n = nt * TILE_N + (lane & 15);
    k = kt * TILE_K + (lane >> 4) * 32 + q * 8;
}

// SRC = 0: one code per byte [N,K];  SRC = 1: canonical packed [N,K/2].
template <int SRC>
__global__ __launch_bounds__(PK_THREADS) void pack_tiled_kernel(
    const uint8_t *__restrict__ src, int64_t N, int64_t K, uint32_t *__restrict__ tiled, int plain)
{
    // plain (ordinary INT4): codes 14 and 15 are the integer pair of l = 7, lower member first, so they
    // trade places before the dINT re-encoding (which puts -step/2 = code 15 at the lower position)
    const uint32_t swap = plain ? 1u : 0u;
    const int64_t words = N * K / 8;
    const int64_t KT = K / TILE_K;
    for (int64_t o = (int64_t)blockIdx.x * PK_THREADS + threadIdx.x; o < words;
         o += (int64_t)gridDim.x * PK_THREADS) {
        int64_t n, k;
        tiled_word_coords(o, KT, n, k);
        uint32_t c[8];
        if (SRC == 0) {
            const uint8_t *p = src + n * K + k;
#pragma unroll
            for (int j = 0; j < 8; ++j) c[j] = p[j];
        } else {
            const uint8_t *p = src + (n * K + k) / 2;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t b = p[j];
                c[2 * j] = b & 15u;
                c[2 * j + 1] = b >> 4;
            }
        }
        uint32_t w = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {  // byte b: low nibble column +b, high nibble column +4+b
            w |= recode(c[b] >= 14u ? c[b] ^ swap : c[b]) << (8 * b);
            w |= recode(c[4 + b] >= 14u ? c[4 + b] ^ swap : c[4 + b]) << (8 * b + 4);
        }
        tiled[o] = w;
    }
}

__global__ __launch_bounds__(PK_THREADS) void unpack_tiled_kernel(
    const uint32_t *__restrict__ tiled, int64_t N, int64_t K, uint8_t *__restrict__ codes, int plain)
{
    const uint32_t swap = plain ? 1u : 0u;
    const int64_t words = N * K / 8;
    const int64_t KT = K / TILE_K;
    for (int64_t o = (int64_t)blockIdx.x * PK_THREADS + threadIdx.x; o < words;
         o += (int64_t)gridDim.x * PK_THREADS) {
        int64_t n, k;
        tiled_word_coords(o, KT, n, k);
        const uint32_t w = tiled[o];
        uint8_t *p = codes + n * K + k;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const uint32_t c0 = uncode((w >> (8 * b)) & 15u), c1 = uncode((w >> (8 * b + 4)) & 15u);
            p[b] = (uint8_t)(c0 >= 14u ? c0 ^ swap : c0);
            p[4 + b] = (uint8_t)(c1 >= 14u ? c1 ^ swap : c1);
        }
    }
}

__global__ __launch_bounds__(PK_THREADS) void fill_i32_kernel(int32_t *__restrict__ p, int64_t n,
                                                             int32_t v)
{
    for (int64_t i = (int64_t)blockIdx.x * PK_THREADS + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * PK_THREADS)
        p[i] = v;
}

// acc[m,n,g] -= zx[m] * wsum[n,g]: turns accumulators of the stored codes into those of
// (code - zero-point), exactly  (sum_k (q - zx) d = sum_k q d - zx sum_k d)
__global__ __launch_bounds__(PK_THREADS) void acc_zero_point_kernel(int32_t *__restrict__ acc,
                                                                   const int32_t *__restrict__ zx,
                                                                   const int32_t *__restrict__ wsum,
                                                                   int64_t M, int64_t per_token)
{
    const int64_t n = M * per_token;
    for (int64_t i = (int64_t)blockIdx.x * PK_THREADS + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * PK_THREADS) {
        const int64_t m = i / per_token;
        acc[i] -= zx[m] * wsum[i - m * per_token];
    }
}

static unsigned grid_for(int64_t items)
{
    int64_t b = (items + PK_THREADS - 1) / PK_THREADS;
    if (b < 1) b = 1;
    if (b > 256 * 64) b = 256 * 64;  // grid-stride beyond that
    return (unsigned)b;
}

int launch_pack(const uint8_t *codes, int64_t N, int64_t K, uint8_t *packed, int layout,
                hipStream_t st, int plain)
{
    if (N * K == 0) return W4A8_OK;
    if (layout == W4A8_LAYOUT_CANONICAL) {
        const int64_t bytes = N * K / 2;
        hipLaunchKernelGGL(pack_canonical_kernel, dim3(grid_for(bytes)), dim3(PK_THREADS), 0, st,
                           codes, bytes, packed);
    } else {
        hipLaunchKernelGGL(pack_tiled_kernel<0>, dim3(grid_for(N * K / 8)), dim3(PK_THREADS), 0, st,
                           codes, N, K, (uint32_t *)packed, plain);
    }
    return hip_status(hipGetLastError());
}

int launch_unpack(const uint8_t *packed, int64_t N, int64_t K, uint8_t *codes, int layout,
                  hipStream_t st, int plain)
{
    if (N * K == 0) return W4A8_OK;
    if (layout == W4A8_LAYOUT_CANONICAL) {
        const int64_t bytes = N * K / 2;
        hipLaunchKernelGGL(unpack_canonical_kernel, dim3(grid_for(bytes)), dim3(PK_THREADS), 0, st,
                           packed, bytes, codes);
    } else {
        hipLaunchKernelGGL(unpack_tiled_kernel, dim3(grid_for(N * K / 8)), dim3(PK_THREADS), 0, st,
                           (const uint32_t *)packed, N, K, codes, plain);
    }
    return hip_status(hipGetLastError());
}

int launch_repack_canonical_to_tiled(const uint8_t *canon, int64_t N, int64_t K, uint8_t *tiled,
                                     hipStream_t st, int plain)
{
    if (N * K == 0) return W4A8_OK;
    hipLaunchKernelGGL(pack_tiled_kernel<1>, dim3(grid_for(N * K / 8)), dim3(PK_THREADS), 0, st,
                       canon, N, K, (uint32_t *)tiled, plain);
    return hip_status(hipGetLastError());
}

int launch_fill_i32(int32_t *p, int64_t n, int32_t v, hipStream_t st)
{
    if (n == 0) return W4A8_OK;
    hipLaunchKernelGGL(fill_i32_kernel, dim3(grid_for(n)), dim3(PK_THREADS), 0, st, p, n, v);
    return hip_status(hipGetLastError());
}

int launch_acc_zero_point(int32_t *acc, const int32_t *zx, const int32_t *wsum, int64_t M,
                          int64_t per_token, hipStream_t st)
{
    if (M * per_token == 0) return W4A8_OK;
    hipLaunchKernelGGL(acc_zero_point_kernel, dim3(grid_for(M * per_token)), dim3(PK_THREADS), 0, st,
                       acc, zx, wsum, M, per_token);
    return hip_status(hipGetLastError());
}

// ---- 3-bit storage of dINT3 (Table 10): codes 0..5 and the special codes 14 / 15 of the 4-bit code
// space become 0..5, 6, 7; code i of a group of eight sits at bits 3i..3i+2 of a little-endian
// 24-bit word.  One thread per group of eight.
__global__ __launch_bounds__(PK_THREADS) void pack3_kernel(const uint8_t *__restrict__ codes, int64_t groups,
                                                           uint8_t *__restrict__ packed)
{
    for (int64_t i = (int64_t)blockIdx.x * PK_THREADS + threadIdx.x; i < groups;
         i += (int64_t)gridDim.x * PK_THREADS) {
        uint32_t word = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t c = codes[i * 8 + j] & 15u;
            word |= (c >= 14u ? c - 8u : (c & 7u)) << (3 * j);
        }
        packed[i * 3 + 0] = (uint8_t)word;
        packed[i * 3 + 1] = (uint8_t)(word >> 8);
        packed[i * 3 + 2] = (uint8_t)(word >> 16);
    }
}

__global__ __launch_bounds__(PK_THREADS) void unpack3_kernel(const uint8_t *__restrict__ packed, int64_t groups,
                                                             uint8_t *__restrict__ codes)
{
    for (int64_t i = (int64_t)blockIdx.x * PK_THREADS + threadIdx.x; i < groups;
         i += (int64_t)gridDim.x * PK_THREADS) {
        const uint32_t word = (uint32_t)packed[i * 3] | ((uint32_t)packed[i * 3 + 1] << 8) |
                              ((uint32_t)packed[i * 3 + 2] << 16);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t c = (word >> (3 * j)) & 7u;
            codes[i * 8 + j] = (uint8_t)(c >= 6u ? c + 8u : c);
        }
    }
}

int launch_pack3(const uint8_t *codes, int64_t N, int64_t K, uint8_t *packed, hipStream_t st)
{
    const int64_t groups = N * K / 8;
    hipLaunchKernelGGL(pack3_kernel, dim3(grid_for(groups)), dim3(PK_THREADS), 0, st, codes, groups, packed);
    return hip_status(hipGetLastError());
}

int launch_unpack3(const uint8_t *packed, int64_t N, int64_t K, uint8_t *codes, hipStream_t st)
{
    const int64_t groups = N * K / 8;
    hipLaunchKernelGGL(unpack3_kernel, dim3(grid_for(groups)), dim3(PK_THREADS), 0, st, packed, groups, codes);
    return hip_status(hipGetLastError());
}

// ---- dINT4 with the special value c = step / 2^t, t = 2, 3 (App. A.5, Table 9) as an ordinary dINT4
// matrix of twice the width:  +-c = +-step/2 -+ (1 - 2^(1-t)) step/2.  Columns K .. 2K-1 repeat the
// groups with step' = (1 - 2^(1-t)) step, the same zero-points, the special codes with their signs
// exchanged and every other code replaced by the zero level z.
__global__ __launch_bounds__(PK_THREADS) void expand_special_codes_kernel(
    const uint8_t *__restrict__ codes, const uint8_t *__restrict__ zero, int64_t N, int64_t K, int64_t G,
    uint8_t *__restrict__ out)
{
    const int64_t total = N * K;
    const int64_t ng = K / G;
    for (int64_t i = (int64_t)blockIdx.x * PK_THREADS + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * PK_THREADS) {
        const int64_t n = i / K, k = i - n * K;
        const uint8_t c = codes[i];
        const uint8_t z = zero[n * ng + k / G];
        out[n * 2 * K + k] = c;
        out[n * 2 * K + K + k] = c == 14 ? 15 : (c == 15 ? 14 : z);
    }
}

__global__ __launch_bounds__(PK_THREADS) void expand_special_params_kernel(
    const float *__restrict__ step, const uint8_t *__restrict__ zero, int64_t N, int64_t ng, float factor,
    float *__restrict__ step2, uint8_t *__restrict__ zero2)
{
    const int64_t total = N * ng;
    for (int64_t i = (int64_t)blockIdx.x * PK_THREADS + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * PK_THREADS) {
        const int64_t n = i / ng, g = i - n * ng;
        const float st = step[i];
        const uint8_t z = zero[i];
        step2[n * 2 * ng + g] = st;
        step2[n * 2 * ng + ng + g] = st * factor;
        zero2[n * 2 * ng + g] = z;
        zero2[n * 2 * ng + ng + g] = z;
    }
}

int launch_expand_special(const uint8_t *codes, const float *step, const uint8_t *zero, int64_t N,
                          int64_t K, int64_t G, int shift, uint8_t *codes2, float *step2, uint8_t *zero2,
                          hipStream_t st)
{
    const float factor = shift == 2 ? 0.5f : 0.75f;   // 1 - 2^(1-t)
    hipLaunchKernelGGL(expand_special_codes_kernel, dim3(grid_for(N * K)), dim3(PK_THREADS), 0, st, codes,
                       zero, N, K, G, codes2);
    hipLaunchKernelGGL(expand_special_params_kernel, dim3(grid_for(N * (K / G))), dim3(PK_THREADS), 0, st,
                       step, zero, N, K / G, factor, step2, zero2);
    return hip_status(hipGetLastError());
}

// out [M, 2K] = [Xq | Xq], 16 bytes per thread (K % 16 == 0, both pointers 16-byte aligned)
__global__ __launch_bounds__(PK_THREADS) void repeat_activations_kernel(const uint4 *__restrict__ Xq,
                                                                       int64_t M, int64_t K16,
                                                                       uint4 *__restrict__ out)
{
    const int64_t total = M * K16;
    for (int64_t i = (int64_t)blockIdx.x * PK_THREADS + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * PK_THREADS) {
        const int64_t m = i / K16, k = i - m * K16;
        const uint4 v = Xq[i];
        out[m * 2 * K16 + k] = v;
        out[m * 2 * K16 + K16 + k] = v;
    }
}

int launch_repeat_activations(const int8_t *Xq, int64_t M, int64_t K, int8_t *out, hipStream_t st)
{
    hipLaunchKernelGGL(repeat_activations_kernel, dim3(grid_for(M * (K / 16))), dim3(PK_THREADS), 0, st,
                       (const uint4 *)Xq, M, K / 16, (uint4 *)out);
    return hip_status(hipGetLastError());
}

}  // namespace w4a8
