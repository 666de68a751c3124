// AQAS scale search (Sec. 3.2, Eq. 1: the scale vector s minimizes the squared error of the quantized
// layer's output against the unquantized product on calibration activations; App. A.4: maximum
// magnitude per input channel as the representative of activations and weights, a grid search, then
// weight clipping).  Offline work whose inner loop is the layer itself: every candidate runs
// quantize_act_int8, quantize_weight_dint4, pack_dint4 and w4a8_gemm, the kernels below supply the
// representatives, the scale family, the unquantized product and the error sums.  Everything stays on
// the stream: the best grid point is picked on the device and the final scale is computed from it there.
//
// Scale family: s_k(j) = ax_k^(j/16) / aw_k^(1 - j/16), j = 0..16.  A sixteenth power is a chain of
// correctly rounded square roots, so the whole family is a fixed sequence of IEEE binary32 operations
// (this file is compiled without mul+add contraction).
#include "w4a8_common.hpp"

namespace w4a8 {

typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int AQ_GRID = 16;
constexpr int AQ_CLIP_STEPS = 11;

// ---- representatives: out[k] = max_r |A[r,k]| (out zeroed beforehand; non-negative floats order
// like their bit patterns, so an integer atomic max is exact and order-independent) ----------------
template <typename T>
__global__ __launch_bounds__(256) void channel_absmax_kernel(const T *__restrict__ A, int64_t R,
                                                             int64_t K, int64_t lda, int rows_per_block,
                                                             float *__restrict__ out)
{
    __shared__ float part[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t k = (int64_t)blockIdx.x * 64 + lane;
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_block;
    const int64_t r1 = min(R, r0 + rows_per_block);
    float m = 0.0f;
    if (k < K)
        for (int64_t r = r0 + wave; r < r1; r += 4) m = fmaxf(m, fabsf(to_f32(A[r * lda + k])));
    part[wave][lane] = m;
    __syncthreads();
    if (wave == 0 && k < K) {
        m = fmaxf(fmaxf(part[0][lane], part[1][lane]), fmaxf(part[2][lane], part[3][lane]));
        atomicMax(reinterpret_cast<unsigned int *>(out) + k, __float_as_uint(m));
    }
}

__global__ __launch_bounds__(256) void fill_f32_kernel(float *p, int64_t n, float v)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

int launch_channel_absmax(const void *A, int dtype, int64_t R, int64_t K, int64_t lda, float *out,
                          hipStream_t st)
{
    hipLaunchKernelGGL(fill_f32_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, out, K, 0.0f);
    if (R == 0) return hip_status(hipGetLastError());
    const int rpb = 256;
    const dim3 grid((unsigned)((K + 63) / 64), (unsigned)((R + rpb - 1) / rpb));
    switch (dtype) {
        case W4A8_F32:
            hipLaunchKernelGGL((channel_absmax_kernel<float>), grid, dim3(256), 0, st, (const float *)A, R, K, lda, rpb, out);
            break;
        case W4A8_F16:
            hipLaunchKernelGGL((channel_absmax_kernel<__half>), grid, dim3(256), 0, st, (const __half *)A, R, K, lda, rpb, out);
            break;
        case W4A8_BF16:
            hipLaunchKernelGGL((channel_absmax_kernel<bf16_t>), grid, dim3(256), 0, st, (const bf16_t *)A, R, K, lda, rpb, out);
            break;
        default: return W4A8_ERR_DTYPE;
    }
    return hip_status(hipGetLastError());
}

// ---- scale family -------------------------------------------------------------------------------
__device__ __forceinline__ float pow_sixteenths(float x, int j)
{
    if (j == AQ_GRID) return x;
    float out = 1.0f, r = x;
#pragma unroll
    for (int bit = 3; bit >= 0; --bit) {   // x^(1/2), x^(1/4), x^(1/8), x^(1/16)
        r = sqrtf(r);   // correctly rounded (hipcc default for binary32 sqrt and division)
        if ((j >> bit) & 1) out = out * r;
    }
    return out;
}

// j_dev != null: the grid point is read from device memory (the search's own result)
__global__ __launch_bounds__(256) void aqas_scale_kernel(const float *__restrict__ ax,
                                                         const float *__restrict__ aw, int64_t K, int j,
                                                         const int32_t *__restrict__ j_dev,
                                                         float *__restrict__ s)
{
    const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k >= K) return;
    if (j_dev != nullptr) j = *j_dev;
    const float x = ax[k], w = aw[k];
    float v = 1.0f;
    if (x != 0.0f && w != 0.0f) {
        v = pow_sixteenths(x, j) / pow_sixteenths(w, AQ_GRID - j);
        v = fminf(fmaxf(v, 1e-4f), 1e4f);
    }
    s[k] = v;
}

int launch_aqas_scale(const float *ax, const float *aw, int64_t K, int j, const int32_t *j_dev,
                      float *s, hipStream_t st)
{
    hipLaunchKernelGGL(aqas_scale_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, ax, aw, K,
                       j, j_dev, s);
    return hip_status(hipGetLastError());
}

// ---- the unquantized product Yref[m,n] = sum_k X[m,k] W[n,k] in fp32 on the matrix cores ----------
// One wave per 32 x 32 output tile, operands straight from global memory (offline work, small M).
// fp16 inputs: v_mfma_f32_32x32x8_f16, a lane fetches 8 consecutive k per 16-column step and feeds
// them as two MFMAs (any split of k over lanes and instructions is fine as long as both operands use
// the same one); other input types are widened exactly and go through v_mfma_f32_32x32x2_f32.
template <typename T>
__global__ __launch_bounds__(256) void ref_gemm_kernel(const T *__restrict__ X, int64_t M, int64_t K,
                                                       int64_t ldx, const T *__restrict__ W, int64_t N,
                                                       int64_t ldw, float *__restrict__ Y)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t m0 = ((int64_t)blockIdx.y * 2 + (wave >> 1)) * 32;
    const int64_t n0 = ((int64_t)blockIdx.x * 2 + (wave & 1)) * 32;
    if (m0 >= M || n0 >= N) return;   // whole wave
    const int r32 = lane & 31, kh = lane >> 5;
    const T *xr = X + min(m0 + r32, M - 1) * ldx;   // rows past the end recompute the last row (not stored)
    const T *wr = W + min(n0 + r32, N - 1) * ldw;
    v16f acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
    if constexpr (sizeof(T) == 2 && !__is_same(T, bf16_t)) {
        for (int64_t k = 0; k < K; k += 16) {
            const v8h a = *reinterpret_cast<const v8h *>(xr + k + 8 * kh);
            const v8h b = *reinterpret_cast<const v8h *>(wr + k + 8 * kh);
            acc = __builtin_amdgcn_mfma_f32_32x32x8f16(__builtin_shufflevector(a, a, 0, 1, 2, 3),
                                                       __builtin_shufflevector(b, b, 0, 1, 2, 3), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x8f16(__builtin_shufflevector(a, a, 4, 5, 6, 7),
                                                       __builtin_shufflevector(b, b, 4, 5, 6, 7), acc, 0, 0, 0);
        }
    } else {
        for (int64_t k = 0; k < K; k += 2)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(to_f32(xr[k + kh]), to_f32(wr[k + kh]), acc, 0, 0, 0);
    }
    // D[i][j] = sum_k A[i][k] B[k][j], A = tokens, B = channels: lane holds channel n0 + r32 and the
    // tokens m0 + 8 (r / 4) + 4 kh + r % 4
    const int64_t n = n0 + r32;
    if (n < N) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t m = m0 + 8 * (r >> 2) + 4 * kh + (r & 3);
            if (m < M) Y[m * N + n] = acc[r];
        }
    }
}

int launch_ref_gemm(const void *X, const void *W, int dtype, int64_t M, int64_t N, int64_t K,
                    int64_t ldx, int64_t ldw, float *Y, hipStream_t st)
{
    const dim3 grid((unsigned)((N + 63) / 64), (unsigned)((M + 63) / 64));
    switch (dtype) {
        case W4A8_F16:
            hipLaunchKernelGGL((ref_gemm_kernel<__half>), grid, dim3(256), 0, st, (const __half *)X, M, K, ldx,
                               (const __half *)W, N, ldw, Y);
            break;
        case W4A8_BF16:
            hipLaunchKernelGGL((ref_gemm_kernel<bf16_t>), grid, dim3(256), 0, st, (const bf16_t *)X, M, K, ldx,
                               (const bf16_t *)W, N, ldw, Y);
            break;
        case W4A8_F32:
            hipLaunchKernelGGL((ref_gemm_kernel<float>), grid, dim3(256), 0, st, (const float *)X, M, K, ldx,
                               (const float *)W, N, ldw, Y);
            break;
        default: return W4A8_ERR_DTYPE;
    }
    return hip_status(hipGetLastError());
}

// ---- error sums ---------------------------------------------------------------------------------
// err[n] = sum_m (Y[m,n] - Yref[m,n])^2, one lane per output channel, tokens in ascending order
// (deterministic); the difference in binary32, squares and sums in binary64.
__global__ __launch_bounds__(256) void output_sq_error_kernel(const uint16_t *__restrict__ Y, int y_dtype,
                                                              int64_t ldy, const float *__restrict__ Yref,
                                                              int64_t M, int64_t N, double *__restrict__ err)
{
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    double sum = 0.0;
    for (int64_t m = 0; m < M; ++m) {
        const uint16_t b = Y[m * ldy + n];
        const float y = (y_dtype == W4A8_F16) ? __half2float(__ushort_as_half(b)) : __uint_as_float((uint32_t)b << 16);
        const float d = y - Yref[m * N + n];
        sum += (double)d * (double)d;
    }
    err[n] = sum;
}

// loss[slot] = sum_n err[n]: one workgroup, fixed tree (deterministic)
__global__ __launch_bounds__(256) void loss_sum_kernel(const double *__restrict__ err, int64_t N,
                                                       double *__restrict__ losses, int slot)
{
    __shared__ double part[256];
    double s = 0.0;
    for (int64_t n = threadIdx.x; n < N; n += 256) s += err[n];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w >= 1; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) losses[slot] = part[0];
}

// first minimum of losses[0..count)
__global__ void argmin_kernel(const double *__restrict__ losses, int count, int32_t *__restrict__ best)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    int b = 0;
    for (int i = 1; i < count; ++i)
        if (losses[i] < losses[b]) b = i;
    *best = b;
}

// per-channel bookkeeping of the clipping search: candidate i replaces the incumbent only if strictly
// better (so ties keep the larger range); err_table (may be null) keeps every candidate's errors
__global__ __launch_bounds__(256) void clip_select_kernel(const double *__restrict__ err, int64_t N, int i,
                                                          double *__restrict__ best_err,
                                                          int32_t *__restrict__ best_idx,
                                                          double *__restrict__ err_table)
{
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    const double e = err[n];
    if (err_table != nullptr) err_table[(int64_t)i * N + n] = e;
    if (i == 0 || e < best_err[n]) {
        best_err[n] = e;
        best_idx[n] = i;
    }
}

int launch_output_sq_error(const void *Y, int y_dtype, int64_t ldy, const float *Yref, int64_t M,
                           int64_t N, double *err, hipStream_t st)
{
    hipLaunchKernelGGL(output_sq_error_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, st,
                       (const uint16_t *)Y, y_dtype, ldy, Yref, M, N, err);
    return hip_status(hipGetLastError());
}
int launch_loss_sum(const double *err, int64_t N, double *losses, int slot, hipStream_t st)
{
    hipLaunchKernelGGL(loss_sum_kernel, dim3(1), dim3(256), 0, st, err, N, losses, slot);
    return hip_status(hipGetLastError());
}
int launch_argmin(const double *losses, int count, int32_t *best, hipStream_t st)
{
    hipLaunchKernelGGL(argmin_kernel, dim3(1), dim3(64), 0, st, losses, count, best);
    return hip_status(hipGetLastError());
}
int launch_clip_select(const double *err, int64_t N, int i, double *best_err, int32_t *best_idx,
                       double *err_table, hipStream_t st)
{
    hipLaunchKernelGGL(clip_select_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, st, err, N, i,
                       best_err, best_idx, err_table);
    return hip_status(hipGetLastError());
}

// ---- the error split of Sec. 4.1 (Eq. 4) ---------------------------------------------------------
// delta = Wq - W diag(s) per weight, written to du where the quantized value is zero (underflow) and
// to dr otherwise (rounding); the other array gets 0.
template <typename T>
__global__ __launch_bounds__(256) void error_split_kernel(const T *__restrict__ W, int64_t N, int64_t K,
                                                          int64_t ldw, const float *__restrict__ s, int64_t G,
                                                          int special, const uint8_t *__restrict__ codes,
                                                          const float *__restrict__ step,
                                                          const uint8_t *__restrict__ zero,
                                                          float *__restrict__ du, float *__restrict__ dr)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= N * K) return;
    const int64_t n = i / K, k = i - n * K;
    const int64_t pi = n * (K / G) + k / G;
    const float w = to_f32(W[n * ldw + k]);
    const float wp = s ? w * s[k] : w;
    // special: 0 = no special levels, t = 1..3: codes 14 / 15 are +-step / 2^t
    const int code = codes[i] & 15, z = zero[pi];
    const int t = special ? special : 1;
    const int d = (special && code >= 14) ? (code == 14 ? 1 : -1) : (code - z) * (1 << t);   // units of step / 2^t
    const float unit = step[pi] * (t == 1 ? 0.5f : (t == 2 ? 0.25f : 0.125f));
    const float wq = (float)d * unit;
    const float delta = wq - wp;
    du[i] = d == 0 ? delta : 0.0f;
    dr[i] = d == 0 ? 0.0f : delta;
}

template <typename T>
__global__ __launch_bounds__(256) void scale_activations_kernel(const T *__restrict__ X, int64_t M, int64_t K,
                                                                int64_t ldx, const float *__restrict__ s,
                                                                float *__restrict__ xs)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= M * K) return;
    const int64_t m = i / K, k = i - m * K;
    const float x = to_f32(X[m * ldx + k]);
    xs[i] = s ? x * (1.0f / s[k]) : x;
}

// terms = {sum pu^2, sum pr^2, sum 2 pu pr, number of non-zero entries of du}; one workgroup, fixed order
__global__ __launch_bounds__(256) void error_terms_kernel(const float *__restrict__ pu,
                                                          const float *__restrict__ pr, int64_t n,
                                                          const float *__restrict__ du, int64_t nw,
                                                          double *__restrict__ terms)
{
    __shared__ double part[4][256];
    double a = 0.0, b = 0.0, c = 0.0, u = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += 256) {
        const double x = pu[i], y = pr[i];
        a += x * x;
        b += y * y;
        c += 2.0 * x * y;
    }
    for (int64_t i = threadIdx.x; i < nw; i += 256) u += du[i] != 0.0f ? 1.0 : 0.0;
    part[0][threadIdx.x] = a;
    part[1][threadIdx.x] = b;
    part[2][threadIdx.x] = c;
    part[3][threadIdx.x] = u;
    __syncthreads();
    for (int w = 128; w >= 1; w >>= 1) {
        if ((int)threadIdx.x < w)
            for (int t = 0; t < 4; ++t) part[t][threadIdx.x] += part[t][threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x < 4) terms[threadIdx.x] = part[threadIdx.x][0];
}

int launch_error_split(const void *W, int w_dtype, int64_t N, int64_t K, int64_t ldw, const float *s,
                       int64_t G, int special, const uint8_t *codes, const float *step,
                       const uint8_t *zero, float *du, float *dr, hipStream_t st)
{
    const dim3 grid((unsigned)((N * K + 255) / 256));
#define W4A8_ES_LAUNCH(T_)                                                                             \
    hipLaunchKernelGGL((error_split_kernel<T_>), grid, dim3(256), 0, st, (const T_ *)W, N, K, ldw, s, G, \
                       special, codes, step, zero, du, dr)
    switch (w_dtype) {
        case W4A8_F32: W4A8_ES_LAUNCH(float); break;
        case W4A8_F16: W4A8_ES_LAUNCH(__half); break;
        case W4A8_BF16: W4A8_ES_LAUNCH(bf16_t); break;
        default: return W4A8_ERR_DTYPE;
    }
#undef W4A8_ES_LAUNCH
    return hip_status(hipGetLastError());
}

int launch_scale_activations(const void *X, int x_dtype, int64_t M, int64_t K, int64_t ldx,
                             const float *s, float *xs, hipStream_t st)
{
    const dim3 grid((unsigned)((M * K + 255) / 256));
#define W4A8_SA_LAUNCH(T_) \
    hipLaunchKernelGGL((scale_activations_kernel<T_>), grid, dim3(256), 0, st, (const T_ *)X, M, K, ldx, s, xs)
    switch (x_dtype) {
        case W4A8_F32: W4A8_SA_LAUNCH(float); break;
        case W4A8_F16: W4A8_SA_LAUNCH(__half); break;
        case W4A8_BF16: W4A8_SA_LAUNCH(bf16_t); break;
        default: return W4A8_ERR_DTYPE;
    }
#undef W4A8_SA_LAUNCH
    return hip_status(hipGetLastError());
}

int launch_error_terms(const float *pu, const float *pr, int64_t n, const float *du, int64_t nw,
                       double *terms, hipStream_t st)
{
    hipLaunchKernelGGL(error_terms_kernel, dim3(1), dim3(256), 0, st, pu, pr, n, du, nw, terms);
    return hip_status(hipGetLastError());
}

}  // namespace w4a8
