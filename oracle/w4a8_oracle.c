/*
 * CPU oracle for the W4A8 (dINT4 x INT8) quantized linear layer of arXiv 2311.05161.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the plain, slow, obviously-correct
 * definition that the GPU library is checked against.  Only the test-suite, the
 * smoke check and the benchmark's "cpu_baseline" leg may call it.  It shares no
 * code, header, table or constant generator with the HIP path, and the HIP path
 * never calls it.
 *
 * Notation (paper -> here).  The paper writes the layer as
 *     Q(W diag(s)) Q(diag(s)^-1 X)                                   (Eq. 1)
 * with W [out, in], X [in, tokens], s [in].  Here tokens are rows:
 *     X [M, K]   M tokens, K input channels        (paper: T tokens, C channels)
 *     W [N, K]   N output channels                 (paper: M output features)
 *     s [K]      AQAS per-input-channel scale      (paper: s in Eq. 1)
 *     step[n,g]  dINT step size                    (paper: "s" in Eq. 5)
 *     zero[n,g]  integer zero-point z              (paper: z in Eq. 5)
 *     G          weights per quantization group along K (G = K: per output channel)
 *
 * dINT4 (Sec. 4.2, Eq. 5): b = 4 bits, p = 2^b - 3 = 13 uniform steps, so codes
 * 0..13 are ordinary asymmetric-integer levels (code - z) * step, and the two
 * reserved codes are the "denormal" levels: code 14 = c1 = +step/2,
 * code 15 = c2 = -step/2.
 *
 * Every floating-point step of the two quantizers is ONE IEEE-754 binary32
 * operation with round-to-nearest-even, in the order written below; compile
 * with -ffp-contract=off and without fast-math.  rne(.) is nearbyintf() in the
 * default rounding mode (round half to even).
 *
 * Parity status: every function in this file is pinned by tests that do not
 * call it to produce their expectation (closed-form level sets, hand-worked
 * examples of Eq. 5, brute-force nearest-level search in float64, a float64
 * matmul of dequantized operands, exhaustive product tables).
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define DINT4_P 13        /* p = 2^4 - 3 uniform steps (Sec. 4.2)            */
#define DINT4_C1 14       /* code of the positive special value  +step/2     */
#define DINT4_C2 15       /* code of the negative special value  -step/2     */

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------
 * Activation quantizer: per-token (row-wise) symmetric absmax INT8 of
 * diag(s)^-1 X  (Eq. 1, second factor; token-wise 8-bit, App. A.1).
 *
 *   r[k]   = 1 / s[k]                 (1 if s == NULL)
 *   t[m,k] = X[m,k] * r[k]
 *   a[m]   = max_k |t[m,k]|
 *   inv    = 127 / a
 *   inv not finite (a == 0, or a below 127 / FLT_MAX ~ 3.7e-37, where the reciprocal scale
 *   overflows binary32 and t * inv would be inf or nan): sx[m] = 1, Xq[m,:] = 0
 *   else   : sx[m] = a / 127
 *            Xq[m,k] = clamp(rne(t * inv), -127, 127)
 *
 * rbuf: caller-provided scratch of K floats.  Returns 0, or 1 on bad arguments.
 * ---------------------------------------------------------------------- */
int oracle_quantize_act_int8(const float *X, int64_t M, int64_t K, int64_t ldx,
                             const float *s, int8_t *Xq, float *sx, float *rbuf)
{
    if (!X || !Xq || !sx || !rbuf || M < 0 || K <= 0 || ldx < K) return 1;
    for (int64_t k = 0; k < K; ++k) rbuf[k] = s ? 1.0f / s[k] : 1.0f;

#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const float *x = X + m * ldx;
        float a = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            float t = x[k] * rbuf[k];
            float at = fabsf(t);
            if (at > a) a = at;
        }
        int8_t *q = Xq + m * K;
        float inv = 127.0f / a;
        if (!(inv <= FLT_MAX)) {   /* a == 0 or vanishingly small: no information at 8 bits */
            sx[m] = 1.0f;
            for (int64_t k = 0; k < K; ++k) q[k] = 0;
            continue;
        }
        sx[m] = a / 127.0f;
        for (int64_t k = 0; k < K; ++k) {
            float t = x[k] * rbuf[k];
            float v = nearbyintf(t * inv);
            if (v > 127.0f) v = 127.0f;
            if (v < -127.0f) v = -127.0f;
            q[k] = (int8_t)(int)v;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * One dINT4 code from one real value (Eq. 5, first half).
 *   u = w * istep                      (istep = 1/step, computed once per group)
 *    0.25 <  u <=  0.75  -> c1 (14)
 *   -0.75 <= u <  -0.25  -> c2 (15)
 *   else                 -> clamp(rne(u) + z, 0, 13)
 * ---------------------------------------------------------------------- */
static uint8_t dint4_code(float w, float istep, int z)
{
    float u = w * istep;
    if (u > 0.25f && u <= 0.75f) return DINT4_C1;
    if (u >= -0.75f && u < -0.25f) return DINT4_C2;
    int c = (int)nearbyintf(u) + z;
    if (c < 0) c = 0;
    if (c > DINT4_P) c = DINT4_P;
    return (uint8_t)c;
}

/* ------------------------------------------------------------------------
 * Weight quantizer: dINT4 of W diag(s) (Eq. 1, first factor), min-max
 * asymmetric per output channel or per group of G consecutive input
 * channels (App. A.1; Sec. 4.2: step = range / p, integer zero-point z).
 *
 *   w'[n,k] = W[n,k] * s[k]                       (s == NULL: w' = W)
 *   per (n,g): lo = min(0, min w'), hi = max(0, max w')
 *              hi == lo : step = 1, z = 0
 *              else     : step = (hi - lo) / 13 ; istep = 1 / step
 *                         z = clamp(rne(-lo * istep), 0, 13)
 *   per element: code = dint4_code(w', istep, z)
 *
 * use_given != 0: step[] and zero[] are inputs (externally chosen ranges, e.g.
 * after the weight clipping of App. A.4) and only the per-element rule runs.
 *
 * codes: [N,K] one code per byte.  step: [N,K/G] float.  zero: [N,K/G] u8.
 * Returns 0, or 1 on bad arguments.
 * ---------------------------------------------------------------------- */
int oracle_quantize_weight_dint4(const float *W, int64_t N, int64_t K, int64_t ldw,
                                 const float *s, int64_t G, int use_given,
                                 uint8_t *codes, float *step, uint8_t *zero)
{
    if (G == 0) G = K;
    if (!W || !codes || !step || !zero || N < 0 || K <= 0 || ldw < K || G <= 0 || K % G)
        return 1;
    const int64_t ng = K / G;

#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const float *w = W + n * ldw;
        for (int64_t g = 0; g < ng; ++g) {
            const int64_t k0 = g * G;
            float st, istep;
            int z;
            if (use_given) {
                st = step[n * ng + g];
                z = zero[n * ng + g];
                istep = 1.0f / st;
            } else {
                float lo = 0.0f, hi = 0.0f;
                for (int64_t k = k0; k < k0 + G; ++k) {
                    float v = s ? w[k] * s[k] : w[k];
                    if (v < lo) lo = v;
                    if (v > hi) hi = v;
                }
                if (hi == lo) {
                    st = 1.0f;
                    istep = 1.0f;
                    z = 0;
                } else {
                    float range = hi - lo;
                    st = range / 13.0f;
                    istep = 1.0f / st;
                    float nlo = -lo;
                    float zf = nearbyintf(nlo * istep);
                    if (zf < 0.0f) zf = 0.0f;
                    if (zf > 13.0f) zf = 13.0f;
                    z = (int)zf;
                }
                step[n * ng + g] = st;
                zero[n * ng + g] = (uint8_t)z;
            }
            for (int64_t k = k0; k < k0 + G; ++k) {
                float v = s ? w[k] * s[k] : w[k];
                codes[n * K + k] = dint4_code(v, istep, z);
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Canonical bit-packing: two codes per byte, even k in the low nibble.
 *   packed[n, j] = code[n, 2j] | code[n, 2j+1] << 4          (K even)
 * ---------------------------------------------------------------------- */
int oracle_pack_dint4(const uint8_t *codes, int64_t N, int64_t K, uint8_t *packed)
{
    if (!codes || !packed || N < 0 || K <= 0 || (K & 1)) return 1;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t j = 0; j < K / 2; ++j)
            packed[n * (K / 2) + j] =
                (uint8_t)((codes[n * K + 2 * j] & 0xF) | ((codes[n * K + 2 * j + 1] & 0xF) << 4));
    return 0;
}

int oracle_unpack_dint4(const uint8_t *packed, int64_t N, int64_t K, uint8_t *codes)
{
    if (!codes || !packed || N < 0 || K <= 0 || (K & 1)) return 1;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t j = 0; j < K / 2; ++j) {
            uint8_t b = packed[n * (K / 2) + j];
            codes[n * K + 2 * j] = b & 0xF;
            codes[n * K + 2 * j + 1] = b >> 4;
        }
    return 0;
}

/* ------------------------------------------------------------------------
 * Decode of one code to an integer in HALF-STEP units (Eq. 5, second half):
 *   code <= 13 : (code - z) * step      = 2 (code - z) * (step / 2)
 *   code == 14 : +step / 2              = +1           * (step / 2)
 *   code == 15 : -step / 2              = -1           * (step / 2)
 * The special magnitude is half a step, i.e. a power-of-two fraction of the
 * step, which is what lets a dINT4 x INT8 product stay an integer product.
 * ---------------------------------------------------------------------- */
int oracle_decode_dint4(int code, int z)
{
    if (code == DINT4_C1) return 1;
    if (code == DINT4_C2) return -1;
    return 2 * (code - z);
}

/* Dequantized weights as floats: Wdq[n,k] = decode(code, z) * (0.5f * step). */
int oracle_dequant_dint4(const uint8_t *codes, int64_t N, int64_t K, int64_t G,
                         const float *step, const uint8_t *zero, float *Wdq)
{
    if (G == 0) G = K;
    if (!codes || !step || !zero || !Wdq || K <= 0 || G <= 0 || K % G) return 1;
    const int64_t ng = K / G;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            int64_t g = k / G;
            float h = 0.5f * step[n * ng + g];
            Wdq[n * K + k] = (float)oracle_decode_dint4(codes[n * K + k], zero[n * ng + g]) * h;
        }
    return 0;
}

/* ------------------------------------------------------------------------
 * Integer GEMM (the product of Eq. 1 on the integer operands):
 *   acc[m,n,g] = sum_{k in group g} Xq[m,k] * decode(code[n,k], zero[n,g])
 * Plain triple loop, 64-bit running sum stored to int32
 * (|acc| <= 127 * 26 * K, far below 2^31 for any K < 650000).
 * packed: canonical layout [N, K/2].  acc: [M, N, K/G], g fastest.
 * ---------------------------------------------------------------------- */
int oracle_int_gemm(const int8_t *Xq, int64_t M, const uint8_t *packed, const uint8_t *zero,
                    int64_t N, int64_t K, int64_t G, int32_t *acc)
{
    if (G == 0) G = K;
    if (!Xq || !packed || !zero || !acc || K <= 0 || (K & 1) || G <= 0 || K % G) return 1;
    const int64_t ng = K / G;

#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n)
            for (int64_t g = 0; g < ng; ++g) {
                int z = zero[n * ng + g];
                int64_t sum = 0;
                for (int64_t k = g * G; k < (g + 1) * G; ++k) {
                    uint8_t b = packed[n * (K / 2) + k / 2];
                    int code = (k & 1) ? (b >> 4) : (b & 0xF);
                    sum += (int64_t)Xq[m * K + k] * (int64_t)oracle_decode_dint4(code, z);
                }
                acc[(m * N + n) * ng + g] = (int32_t)sum;
            }
    return 0;
}

/* Same sum for a list of nidx output coordinates (mi[i], ni[i]); acc: [nidx, K/G].
 * Used where the full triple loop would take hours. */
int oracle_int_gemm_sampled(const int8_t *Xq, int64_t M, const uint8_t *packed,
                            const uint8_t *zero, int64_t N, int64_t K, int64_t G,
                            const int64_t *mi, const int64_t *ni, int64_t nidx, int32_t *acc)
{
    if (G == 0) G = K;
    if (!Xq || !packed || !zero || !acc || !mi || !ni || K <= 0 || (K & 1) || G <= 0 || K % G)
        return 1;
    const int64_t ng = K / G;
    for (int64_t i = 0; i < nidx; ++i)
        if (mi[i] < 0 || mi[i] >= M || ni[i] < 0 || ni[i] >= N) return 1;

#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nidx; ++i) {
        const int64_t m = mi[i], n = ni[i];
        for (int64_t g = 0; g < ng; ++g) {
            int z = zero[n * ng + g];
            int64_t sum = 0;
            for (int64_t k = g * G; k < (g + 1) * G; ++k) {
                uint8_t b = packed[n * (K / 2) + k / 2];
                int code = (k & 1) ? (b >> 4) : (b & 0xF);
                sum += (int64_t)Xq[m * K + k] * (int64_t)oracle_decode_dint4(code, z);
            }
            acc[i * ng + g] = (int32_t)sum;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Dequantization of the accumulators (Eq. 5 second half applied to the
 * product; token scale sx from the activation quantizer):
 *   y = 0 ; for g ascending: y += (0.5 * step[n,g]) * acc[m,n,g]
 *   Y[m,n] = sx[m] * y
 * Y32 follows that sequence in binary32 (no contraction); Y64 evaluates the
 * same expression in binary64 and is the reference for the tolerance check.
 * Either output may be NULL.  acc: [M,N,ng]; rows may be a sample (then sx and
 * step are indexed through mi/ni, else pass mi = ni = NULL for the full grid).
 * ---------------------------------------------------------------------- */
int oracle_dequant_epilogue(const int32_t *acc, const float *sx, const float *step,
                            int64_t M, int64_t N, int64_t ng, float *Y32, double *Y64)
{
    if (!acc || !sx || !step || ng <= 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            const int32_t *a = acc + (m * N + n) * ng;
            float y = 0.0f;
            double yd = 0.0;
            for (int64_t g = 0; g < ng; ++g) {
                float h = 0.5f * step[n * ng + g];
                float prod = h * (float)a[g];
                y = y + prod;
                yd += (0.5 * (double)step[n * ng + g]) * (double)a[g];
            }
            if (Y32) Y32[m * N + n] = sx[m] * y;
            if (Y64) Y64[m * N + n] = (double)sx[m] * yd;
        }
    return 0;
}

/* ========================================================================
 * Asymmetric activations: the paper's own activation quantizer is min-max
 * asymmetric, token-wise, 8 bit (App. A.1, "Quantization Settings").  Same
 * convention as the weights: the range of a token is extended to contain 0, so
 * that the real value 0 is a level.
 *
 *   t[m,k] = X[m,k] * r[k]                           r[k] = 1 / s[k]
 *   lo = min(0, min_k t), hi = max(0, max_k t)
 *   sx = (hi - lo) / 255 ; isx = 1 / sx
 *   isx not finite (hi == lo, or a range so small that the reciprocal overflows binary32):
 *              sx = 1, zx = 0, Q[m,:] = 0
 *   else     :
 *              zx = clamp(rne(-lo * isx), 0, 255)
 *              Q[m,k] = clamp(rne(t * isx) + zx, 0, 255)      (codes 0..255)
 *   dequantized value: (Q - zx) * sx
 * ---------------------------------------------------------------------- */
int oracle_quantize_act_uint8_asym(const float *X, int64_t M, int64_t K, int64_t ldx,
                                   const float *s, uint8_t *Q, float *sx, int32_t *zx,
                                   float *rbuf)
{
    if (!X || !Q || !sx || !zx || !rbuf || M < 0 || K <= 0 || ldx < K) return 1;
    for (int64_t k = 0; k < K; ++k) rbuf[k] = s ? 1.0f / s[k] : 1.0f;

#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const float *x = X + m * ldx;
        float lo = 0.0f, hi = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            float t = x[k] * rbuf[k];
            if (t < lo) lo = t;
            if (t > hi) hi = t;
        }
        uint8_t *q = Q + m * K;
        float range = hi - lo;
        float st = range / 255.0f;
        float isx = 1.0f / st;
        if (!(isx <= FLT_MAX)) {   /* all-zero token, or a vanishing range */
            sx[m] = 1.0f;
            zx[m] = 0;
            for (int64_t k = 0; k < K; ++k) q[k] = 0;
            continue;
        }
        float zf = nearbyintf(-lo * isx);
        if (zf < 0.0f) zf = 0.0f;
        if (zf > 255.0f) zf = 255.0f;
        sx[m] = st;
        zx[m] = (int32_t)zf;
        for (int64_t k = 0; k < K; ++k) {
            float t = x[k] * rbuf[k];
            float v = nearbyintf(t * isx) + zf;
            if (v < 0.0f) v = 0.0f;
            if (v > 255.0f) v = 255.0f;
            q[k] = (uint8_t)(int)v;
        }
    }
    return 0;
}

/* Integer GEMM with a token zero-point:
 *   acc[m,n,g] = sum_{k in group g} (Q[m,k] - zx[m]) * decode(code[n,k], zero[n,g])
 * (|Q - zx| <= 255, |decode| <= 26: exact in the 64-bit running sum, and the
 * result fits int32 for any K < 300000.)  Layouts as in oracle_int_gemm. */
int oracle_int_gemm_asym(const uint8_t *Q, const int32_t *zx, int64_t M, const uint8_t *packed,
                         const uint8_t *zero, int64_t N, int64_t K, int64_t G, int32_t *acc)
{
    if (G == 0) G = K;
    if (!Q || !zx || !packed || !zero || !acc || K <= 0 || (K & 1) || G <= 0 || K % G) return 1;
    const int64_t ng = K / G;

#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n)
            for (int64_t g = 0; g < ng; ++g) {
                int z = zero[n * ng + g];
                int64_t sum = 0;
                for (int64_t k = g * G; k < (g + 1) * G; ++k) {
                    uint8_t b = packed[n * (K / 2) + k / 2];
                    int code = (k & 1) ? (b >> 4) : (b & 0xF);
                    int64_t xv = (int64_t)Q[m * K + k] - (int64_t)zx[m];
                    sum += xv * (int64_t)oracle_decode_dint4(code, z);
                }
                acc[(m * N + n) * ng + g] = (int32_t)sum;
            }
    return 0;
}

/* The same for a list of output coordinates (see oracle_int_gemm_sampled). */
int oracle_int_gemm_asym_sampled(const uint8_t *Q, const int32_t *zx, int64_t M,
                                 const uint8_t *packed, const uint8_t *zero, int64_t N, int64_t K,
                                 int64_t G, const int64_t *mi, const int64_t *ni, int64_t nidx,
                                 int32_t *acc)
{
    if (G == 0) G = K;
    if (!Q || !zx || !packed || !zero || !acc || !mi || !ni || K <= 0 || (K & 1) || G <= 0 ||
        K % G)
        return 1;
    const int64_t ng = K / G;
    for (int64_t i = 0; i < nidx; ++i)
        if (mi[i] < 0 || mi[i] >= M || ni[i] < 0 || ni[i] >= N) return 1;

#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nidx; ++i) {
        const int64_t m = mi[i], n = ni[i];
        for (int64_t g = 0; g < ng; ++g) {
            int z = zero[n * ng + g];
            int64_t sum = 0;
            for (int64_t k = g * G; k < (g + 1) * G; ++k) {
                uint8_t b = packed[n * (K / 2) + k / 2];
                int code = (k & 1) ? (b >> 4) : (b & 0xF);
                int64_t xv = (int64_t)Q[m * K + k] - (int64_t)zx[m];
                sum += xv * (int64_t)oracle_decode_dint4(code, z);
            }
            acc[i * ng + g] = (int32_t)sum;
        }
    }
    return 0;
}

/* Sums of the quantized weights in half steps over blocks of T consecutive input channels (T
 * divides the group size G): what an implementation needs to take the token zero-point out of
 * a product computed on the codes,  sum_k (Q - zx) d = sum_k Q d - zx * sum_k d.
 *   wsum[n,b] = sum_{k in block b} decode(code[n,k], zero[n, group of k])        (exact)
 * T = G gives the group sums.  wsum: [N, K/T]. */
int oracle_weight_sums(const uint8_t *packed, const uint8_t *zero, int64_t N, int64_t K, int64_t G,
                       int64_t T, int32_t *wsum)
{
    if (G == 0) G = K;
    if (T == 0) T = G;
    if (!packed || !zero || !wsum || K <= 0 || (K & 1) || G <= 0 || K % G || T <= 0 || G % T)
        return 1;
    const int64_t ng = K / G, nb = K / T;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t b = 0; b < nb; ++b) {
            int z = zero[n * ng + (b * T) / G];
            int64_t sum = 0;
            for (int64_t k = b * T; k < (b + 1) * T; ++k) {
                uint8_t by = packed[n * (K / 2) + k / 2];
                int code = (k & 1) ? (by >> 4) : (by & 0xF);
                sum += oracle_decode_dint4(code, z);
            }
            wsum[n * nb + b] = (int32_t)sum;
        }
    return 0;
}
