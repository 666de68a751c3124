/*
 * w4a8.h -- C ABI of the MI355X (gfx950) W4A8 linear layer of arXiv 2311.05161:
 *
 *     Y = dequant( Q8(X diag(s)^-1) . dINT4(W diag(s))^T )                 (Eq. 1)
 *
 *     X [M,K]  activations, one token per row          (paper: X in R^{C x T}, T tokens)
 *     W [N,K]  weights, one output channel per row     (paper: W in R^{M x C})
 *     s [K]    AQAS per-input-channel scale, an input  (paper: s in R^C)
 *
 * Conventions for EVERY entry point
 *   - All data pointers are DEVICE pointers (HIP global memory) owned by the caller; the
 *     library allocates nothing, frees nothing and keeps no state between calls.
 *     (The bench aids that time the machine's own ceilings are declared in w4a8_measure.h.)
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued on it and the call returns without synchronizing.
 *   - The return value is a w4a8_status.  Argument errors are detected on the host before
 *     anything is launched and leave the outputs untouched.  Nothing throws or aborts.
 *   - Rows are contiguous; `ld*` is the distance between rows in ELEMENTS.
 *   - Inputs must be finite and s[k] > 0; otherwise the result is undefined (no error).
 */
#ifndef W4A8_H
#define W4A8_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    W4A8_OK = 0,
    W4A8_ERR_NULL = 1,      /* a required pointer is NULL                                   */
    W4A8_ERR_SHAPE = 2,     /* a size, leading dimension, group size or alignment is invalid */
    W4A8_ERR_DTYPE = 3,     /* unknown / unsupported element type or layout id              */
    W4A8_ERR_WORKSPACE = 4, /* workspace missing or smaller than w4a8_gemm_workspace_bytes  */
    W4A8_ERR_HIP = 5        /* the HIP runtime reported a launch error                      */
} w4a8_status;

typedef enum { W4A8_F32 = 0, W4A8_F16 = 1, W4A8_BF16 = 2 } w4a8_dtype;

/* Packed-weight layouts (two 4-bit codes per byte).
 *
 * W4A8_LAYOUT_CANONICAL (0): row-major [N, K/2]; byte j of row n = code[n,2j] | code[n,2j+1]<<4.
 *
 * W4A8_LAYOUT_TILED (1): the same N*K/2 bytes rearranged for the GEMM kernels; requires
 *   N % 16 == 0 and K % 128 == 0.  The matrix is cut into tiles of 16 rows x 128 columns;
 *   tile (nt, kt) = (n/16, k/128) starts at byte (nt*(K/128) + kt) * 1024.  Inside a tile,
 *   "lane" l = (n%16) + 16*((k%128)/32) owns 16 consecutive bytes at offset 16*l, seen as four
 *   little-endian 32-bit words q = 0..3.  Word q holds the 8 codes of columns
 *   kk = 32*(l/16) + 8q + 0..7 of the tile: nibble i (bits 4i..4i+3, i = 0..7) holds column
 *   kk + (i>>1) + 4*(i&1), i.e. the low nibbles of the four bytes are columns +0..+3 and the
 *   high nibbles are columns +4..+7.  Each nibble stores the code re-encoded as e:
 *       code c <= 13 : e = (c >> 1) | ((c & 1) << 3)
 *       code 14 (+step/2) : e = 15          code 15 (-step/2) : e = 7
 *   so that e & 7 selects one of 8 base levels and bit 3 adds one whole step (= two half
 *   steps): the pairs (2l, 2l+1) of integer codes and the pair (-step/2, +step/2) all differ
 *   by exactly one step.
 */
enum { W4A8_LAYOUT_CANONICAL = 0, W4A8_LAYOUT_TILED = 1 };

/* Weight formats sharing the 4-bit code space (see quantize_weight_format). */
enum {
    W4A8_FMT_DINT4 = 0,
    W4A8_FMT_INT4 = 1,
    W4A8_FMT_DINT3 = 2,
    W4A8_FMT_DINT4_C4 = 3, /* dINT4 with the special value step/4 (quantizer and expand_special_value only) */
    W4A8_FMT_DINT4_C8 = 4  /* ... step/8 */
};

/* Per-token INT8 activation quantization with the AQAS scale folded in
 * (Eq. 1, factor Q(diag(s)^-1 X); token-wise 8-bit, App. A.1):
 *     t[m,k] = X[m,k] * (1 / s[k]);  a[m] = max_k |t[m,k]|;
 *     sx[m] = a[m] / 127;  Xq[m,k] = clamp(rne(t[m,k] * (127 / a[m])), -127, 127);
 *     an all-zero row gives sx = 1, Xq = 0.
 * Every step is one IEEE binary32 operation; divisions are correctly rounded.
 *   X   in   [M, ldx] elements of x_dtype (F32, F16 or BF16), ldx >= K
 *   s   in   [K] float, or NULL for s = 1
 *   Xq  out  [M, K] int8, contiguous
 *   sx  out  [M] float
 * M == 0 is a no-op.  K >= 1. */
int quantize_act_int8(const void *X, int x_dtype, int64_t M, int64_t K, int64_t ldx,
                      const float *s, int8_t *Xq, float *sx, void *stream);

/* dINT4 weight quantization of W diag(s) (Eq. 1 factor Q(W diag(s)); Sec. 4.2, Eq. 5 with
 * b = 4, p = 13; min-max asymmetric per output channel or per group, App. A.1):
 *     w' = W[n,k] * s[k];  per (n, group): lo = min(0, min w'), hi = max(0, max w'),
 *     step = (hi - lo) / 13, z = clamp(rne(-lo * (1/step)), 0, 13)   (hi == lo: step 1, z 0);
 *     u = w' * (1/step):  0.25 < u <= 0.75 -> code 14 (+step/2);
 *                        -0.75 <= u < -0.25 -> code 15 (-step/2);
 *                         else code = clamp(rne(u) + z, 0, 13).
 *   W      in   [N, ldw] elements of w_dtype, ldw >= K
 *   s      in   [K] float or NULL
 *   group_size  0 or K: one (step, z) per output channel; else K % group_size == 0
 *   use_given_params != 0: step/zero are INPUTS (externally chosen ranges, e.g. after the
 *               weight clipping of App. A.4) and only the per-element rule runs
 *   codes  out  [N, K] one code (0..15) per byte
 *   step   i/o  [N, K/G] float        zero  i/o  [N, K/G] uint8 (0..13)                    */
int quantize_weight_dint4(const void *W, int w_dtype, int64_t N, int64_t K, int64_t ldw,
                          const float *s, int64_t group_size, int use_given_params,
                          uint8_t *codes, float *step, uint8_t *zero, void *stream);

/* Bit-packing of dINT4 codes, two per byte (the storage format the 4-bit weights of
 * Sec. 4.2 are kept in), and its inverse.  `layout` is one of the ids above.
 *   codes  [N, K] bytes, values 0..15 (upper bits ignored)     packed  N*K/2 bytes
 * K must be even (layout 0) or N % 16 == 0 and K % 128 == 0 (layout 1). */
int pack_dint4(const uint8_t *codes, int64_t N, int64_t K, uint8_t *packed, int layout,
               void *stream);
int unpack_dint4(const uint8_t *packed, int64_t N, int64_t K, uint8_t *codes, int layout,
                 void *stream);

/* dINT4 x INT8 GEMM with int32 accumulation and fused dequantization (Eq. 1 product on the
 * integer operands; Eq. 5 second half; the dINT4 x INT8 MAC of Sec. 4.3):
 *     d[n,k]     = 2 (code - zero[n,g])  for code <= 13,  +1 for code 14,  -1 for code 15
 *                  (the weight in units of step/2)
 *     acc[m,n,g] = sum_{k in group g} Xq[m,k] * d[n,k]                      (int32, exact)
 *     Y[m,n]     = cast( sx[m] * sum_g (step[n,g] / 2) * acc[m,n,g] )
 *   Xq   in  [M, K] int8 contiguous        sx    in  [M] float
 *   Wp   in  packed weights in `layout`    step  in  [N, K/G] float   zero in [N, K/G] uint8
 *   group_size: 0 or K = per output channel, else a multiple of 128 dividing K
 *   Y    out [M, ldy] elements of y_dtype (F16 or BF16), ldy >= N
 *   acc_out  NULL, or int32 [M, N, K/G] (g fastest) that receives the exact accumulators
 *   workspace / workspace_bytes: device scratch of at least w4a8_gemm_workspace_bytes(...)
 *               bytes, 256-byte aligned, owned by the caller and free for reuse once the call's
 *               work on `stream` has finished; may be NULL when that function returns 0.  It
 *               holds, as needed: the tiled copy of canonical weights (N*K/2 bytes), the int32
 *               per-token row-sums of the per-channel prefill path, and the fp32 partial sums
 *               [splits, M, N] of launches that cut K across workgroups.
 * Requires N % 16 == 0, K % 128 == 0, K <= 65536, N*K/2 < 2^31 and, for M > 16, M*K < 2^31
 * (W4A8_ERR_SHAPE otherwise).  M == 0 or N == 0 is a no-op.
 * The M <= 16 path streams the packed weights once (memory-bound "decode" GEMV); larger M
 * uses the MFMA tile kernel ("prefill"), except that 17 .. 64 tokens (.. 128 on layers of at most
 * 48 Mi weights) run as 16-token blocks of the streaming kernel in one launch where that is
 * faster (w4a8_gemm_workspace_bytes knows which path a shape takes).  Results are deterministic (fixed reduction order). */
size_t w4a8_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t group_size,
                                 int layout);
int w4a8_gemm(const int8_t *Xq, const float *sx, int64_t M,
              const uint8_t *Wp, int layout, const float *step, const uint8_t *zero,
              int64_t N, int64_t K, int64_t group_size,
              void *Y, int y_dtype, int64_t ldy,
              int32_t *acc_out, void *workspace, size_t workspace_bytes, void *stream);

/* The whole quantized layer of Eq. 1 in one call, from unquantized activations:
 *     Y = dequant( Q8(X diag(s)^-1) . dINT4(W diag(s))^T )
 * i.e. quantize_act_int8 followed by w4a8_gemm, with the same results bit for bit (Xq, sx, the
 * accumulators, Y).  At most 16 tokens of F16 activations (rows 16-byte aligned: X % 16 == 0,
 * ldx % 8 == 0) on tiled weights whose K the streaming kernel takes in one range (K <= 5120 with
 * groups, <= 7168 per channel) run as ONE launch: every workgroup of the streaming kernel
 * quantizes the activations itself while its first weights are on their way, and the int8
 * activations never touch memory -- the decode step of the method without a second launch.  Every
 * other case runs the two steps one after the other on `stream`.
 *   X, x_dtype, M, K, ldx, s      as in quantize_act_int8
 *   Wp, layout, step, zero, N, group_size, Y, y_dtype, ldy, acc_out      as in w4a8_gemm
 *   Xq_out  NULL, or int8 [M, K] (16-byte aligned) that receives the quantized activations
 *   sx_out  NULL, or float [M] that receives the token scales        (both: checks, not needed for Y)
 *   workspace / workspace_bytes: at least w4a8_linear_workspace_bytes(...) bytes, 256-byte aligned: the int8
 *               activations, the token scales and w4a8_gemm's own workspace (untouched by the one-launch
 *               path, which needs none and accepts NULL).
 * Shape limits and errors as for quantize_act_int8 and w4a8_gemm; M == 0 or N == 0 is a no-op. */
size_t w4a8_linear_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t group_size, int layout);
int w4a8_linear(const void *X, int x_dtype, int64_t M, int64_t K, int64_t ldx, const float *s,
                const uint8_t *Wp, int layout, const float *step, const uint8_t *zero,
                int64_t N, int64_t group_size, void *Y, int y_dtype, int64_t ldy,
                int8_t *Xq_out, float *sx_out, int32_t *acc_out,
                void *workspace, size_t workspace_bytes, void *stream);

/* w4a8_gemm for callers that cannot allocate device memory or carry a workspace around: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, same
 * kernels, same results and same argument errors as w4a8_gemm; the workspace is a static device
 * array inside the library of W4A8_STATIC_SCRATCH_BYTES bytes (64 MiB; every GPU the library runs
 * on holds it until the process ends).  The call allocates and frees nothing.
 *   - A shape whose w4a8_gemm_workspace_bytes exceeds W4A8_STATIC_SCRATCH_BYTES is rejected with
 *     W4A8_ERR_WORKSPACE before anything is launched.  (What a shape needs: nothing for tiled
 *     weights whose K fits one range of the streaming kernel; splits * M * N * 4 bytes of partial
 *     sums where K is cut into ranges; 4 bytes per token for per-channel weights on the tile
 *     kernel; N * K / 2 bytes for canonical-layout weights.  64 MiB holds all of that for the
 *     LLaMA-7B/13B and OPT-66B layer shapes with tiled weights at any token count.)
 *   - All calls on one GPU share that GPU's array: calls whose work may overlap in time on one GPU
 *     (different streams, different threads) race on it and must be serialized by the caller.  A
 *     call needs nothing from what an earlier call left in the array.
 *   - The first call on a device that needs scratch asks the runtime for the array's address there
 *     (hipGetSymbolAddress, no allocation); make that call outside graph capture.
 *   w4a8_gemm_static_scratch_bytes returns W4A8_STATIC_SCRATCH_BYTES. */
#define W4A8_STATIC_SCRATCH_BYTES (64u << 20)
size_t w4a8_gemm_static_scratch_bytes(void);
int w4a8_gemm_static(const int8_t *Xq, const float *sx, int64_t M,
                     const uint8_t *Wp, int layout, const float *step, const uint8_t *zero,
                     int64_t N, int64_t K, int64_t group_size,
                     void *Y, int y_dtype, int64_t ldy, int32_t *acc_out, void *stream);

/* ---- Asymmetric activations: the min-max, token-wise 8-bit quantizer with a zero-point that the
 * paper itself uses for activations (App. A.1, "Quantization Settings"), and the GEMM for it. ----
 *
 * Per token m, with t = X[m,:] * (1 / s):  lo = min(0, min t), hi = max(0, max t),
 *     sx = (hi - lo) / 255,  zx = clamp(rne(-lo / sx), 0, 255),
 *     code[m,k] = clamp(rne(t[k] / sx) + zx, 0, 255)          (value = (code - zx) * sx)
 * (1/s and 1/sx are correctly rounded reciprocals, one binary32 operation per step; an all-zero
 * token gives sx = 1, zx = 0, codes 0).  Storage: the signed int8 matrix cores take
 *     Xq[m,k] = code - 128      and      zx[m] = zero-point - 128        (both in -128..127),
 * which leaves code - zero-point unchanged.
 *   X, s, ldx, Xq, sx as in quantize_act_int8;   zx  out  [M] int32                          */
int quantize_act_int8_asym(const void *X, int x_dtype, int64_t M, int64_t K, int64_t ldx,
                           const float *s, int8_t *Xq, float *sx, int32_t *zx, void *stream);

/* Sums of the quantized weights, computed once per weight matrix (offline, after
 * quantize_weight_dint4).  They take the token zero-point out of a product computed on the stored
 * codes, exactly, in int32:  sum_k (q - zx) d = sum_k q d - zx * sum_k d.
 *   codes  in  [N, K] one dINT4 code per byte      zero  in  [N, K/G]
 *   wsum   out [N, K/G] int32:    sum over the group of d[n,k] (weights in units of step/2)
 *   tsum   out [N, K/128] int32:  the same over each block of 128 input channels (the GEMM's
 *               k-tiles); NULL to skip it.  Needs K % 128 == 0 and G % 128 == 0.
 * With G = 128 the two arrays hold the same numbers. */
int dint4_weight_sums(const uint8_t *codes, const uint8_t *zero, int64_t N, int64_t K,
                      int64_t group_size, int32_t *wsum, int32_t *tsum, void *stream);

/* w4a8_gemm for activations quantized by quantize_act_int8_asym:
 *     acc[m,n,g] = sum_{k in g} (Xq[m,k] - zx[m]) * d[n,k]                    (int32, exact)
 *     Y[m,n]     = cast( sx[m] * sum_g (step[n,g] / 2) * acc[m,n,g] )
 * The kernels multiply the stored codes and subtract zx[m] * (sum of the weights) from the int32
 * accumulators before anything is converted to floating point.
 *   zx    in  [M] int32 (as written by quantize_act_int8_asym)
 *   wsum  in  [N, K/G] int32, tsum in [N, K/128] int32 (from dint4_weight_sums)
 * Everything else (shapes, limits, workspace, errors) as for w4a8_gemm, whose
 * w4a8_gemm_workspace_bytes also sizes this call's workspace. */
int w4a8_gemm_asym(const int8_t *Xq, const float *sx, const int32_t *zx, int64_t M,
                   const uint8_t *Wp, int layout, const float *step, const uint8_t *zero,
                   const int32_t *wsum, const int32_t *tsum,
                   int64_t N, int64_t K, int64_t group_size,
                   void *Y, int y_dtype, int64_t ldy,
                   int32_t *acc_out, void *workspace, size_t workspace_bytes, void *stream);

/* ---- 4-bit Value cache ("W4A8V4", Sec. 5.1).  Value is quantized channel-wise along the dimension
 * over which the product with the attention map accumulates (App. A.1), i.e. along the tokens:
 * for every head b and channel d, the T cached values V[b, :, d] (or each group of `group_size`
 * consecutive tokens of them) share one (step, zero), and are coded by the rule of
 * quantize_weight_dint4 (with s = 1).  The output is V^T per head -- exactly the operand layout of
 * a weight matrix with N = D output channels and K = T input channels -- so pack_dint4(codes,
 * batch*D, T, ...), dint4_weight_sums and w4a8_gemm_batched apply to it unchanged.
 *   V      in   element (b, t, d) at V[b*ld_b + t*ld_t + d], v_dtype F32 / F16 / BF16;
 *               ld_t >= D, ld_b >= 0 (token-major, as a cache is appended to; heads may be
 *               interleaved, e.g. a [T, heads, D] cache has ld_t = heads*D, ld_b = D)
 *   group_size  0 or T: per channel; else tokens per group, T % group_size == 0
 *   codes  out  [batch*D, T] one code per byte (row b*D + d, token fastest)
 *   step   out  [batch*D, T/G] float          zero  out  [batch*D, T/G] uint8
 * batch <= 65535, T/G <= 65535.  batch == 0 or D == 0 is a no-op. */
int quantize_value_dint4(const void *V, int v_dtype, int64_t batch, int64_t T, int64_t D,
                         int64_t ld_t, int64_t ld_b, int64_t group_size, uint8_t *codes,
                         float *step, uint8_t *zero, void *stream);

/* `batch` independent decode products of one shape in one launch -- e.g. the attention-times-Value
 * product with a 4-bit Value cache (Value is quantized channel-wise along the accumulation
 * dimension, App. A.1: each head's V^T [head_dim, tokens] is a per-channel dINT4 "weight" matrix
 * and the INT8 attention probabilities are the activations).  Problem b uses
 *     Xq + b*M*K, sx + b*M, zx + b*M, Wp + b*N*K/2, step/zero/wsum + b*N*(K/G), tsum + b*N*(K/128),
 *     Y + b*M*ldy
 * with the meaning of w4a8_gemm_asym (zx == NULL: of w4a8_gemm; wsum, tsum then unused).
 * Wp in the tiled layout only.  Requires M <= 16 (M*K a multiple of 16), K <= 9216 (5120 with groups), N % 16 == 0,
 * K % 128 == 0, batch <= 65535; needs no workspace and has no accumulator hook. */
int w4a8_gemm_batched(const int8_t *Xq, const float *sx, const int32_t *zx, int64_t M,
                      const uint8_t *Wp, const float *step, const uint8_t *zero,
                      const int32_t *wsum, const int32_t *tsum,
                      int64_t N, int64_t K, int64_t group_size,
                      void *Y, int y_dtype, int64_t ldy, int64_t batch, void *stream);

/* ---- AQAS scale search (Sec. 3.2, Eq. 1; App. A.4).  Offline calibration: on calibration activations
 * X [M, K] and the layer's weights W [N, K] it looks for the per-input-channel scale s that minimizes
 *     loss(s) = sum_{m,n} ( Yq[m,n] - sum_k X[m,k] W[n,k] )^2,    Yq = the fp16 output of the quantized
 * layer computed by this library's own kernels (quantize_act_int8, quantize_weight_dint4, pack_dint4,
 * w4a8_gemm) with that s.  Representatives are the maximum magnitudes per input channel (App. A.4):
 *     ax[k] = max_m |X[m,k]|,   aw[k] = max_n |W[n,k]|,
 * and the candidates are the 17 grid points j = 0..16 of
 *     s_k(j) = ax[k]^(j/16) / aw[k]^(1 - j/16)        (1 where ax[k] or aw[k] is 0; clamped to [1e-4, 1e4]),
 * a sixteenth power being the product, in the order 1/2, 1/4, 1/8, 1/16, of the correctly rounded
 * binary32 square-root chain of x selected by the bits of j (x for j = 16, 1 for j = 0): a fixed
 * sequence of IEEE operations.  The first grid point with the smallest loss wins; it is chosen on the
 * device, nothing synchronizes.
 *   X, W     in   one element type `dtype` for both (F32, F16, BF16); rows ldx / ldw elements apart;
 *                 F16: 16-byte aligned rows (pointer % 16 == 0, ld % 8 == 0)
 *   s_out    out  [K] float: s at the chosen grid point      best_j  out  int32 (device)
 *   losses   out  [17] double (device): loss of every grid point
 *   workspace     device scratch of aqas_search_workspace_bytes(M, N, K, group_size) bytes, 256-byte aligned
 * Shape limits as for w4a8_gemm (N % 16 == 0, K % 128 == 0, groups multiples of 128). */
size_t aqas_search_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t group_size);
int aqas_channel_absmax(const void *A, int dtype, int64_t R, int64_t K, int64_t lda, float *out,
                        void *stream);                         /* out[k] = max_r |A[r,k]|, exact */
int aqas_scale(const float *ax, const float *aw, int64_t K, int j, float *s, void *stream);
int aqas_search(const void *X, const void *W, int dtype, int64_t M, int64_t N, int64_t K, int64_t ldx,
                int64_t ldw, int64_t group_size, float *s_out, int32_t *best_j, double *losses,
                void *workspace, size_t workspace_bytes, void *stream);

/* Weight clipping after the scale search (App. A.4).  The (zero-containing) min / max of every group of
 * W diag(s) is shrunk by rho_i = 1 - 0.05 i, i = 0..10 (one binary32 multiply per end), step and
 * zero-point follow from the shrunk range by the rule of quantize_weight_dint4, and the codes come from
 * that function with use_given_params (values beyond the range saturate).
 *   dint4_clipped_params: index [N] int32 (device) gives i per output channel, or NULL: uniform_index for all.
 *   aqas_clip_search: tries every i for all channels, measures each output channel's own error
 *     sum_m (Yq[m,n] - Y[m,n])^2 with the layer's kernels as in aqas_search, and keeps per channel the
 *     first i with the smallest error.  index_out [N] int32, step_out / zero_out [N, K/G] the chosen
 *     parameters, err_table NULL or [11, N] double (every candidate's errors).  Workspace as aqas_search. */
int dint4_clipped_params(const void *W, int w_dtype, int64_t N, int64_t K, int64_t ldw, const float *s,
                         int64_t group_size, const int32_t *index, int uniform_index, float *step,
                         uint8_t *zero, void *stream);
int aqas_clip_search(const void *X, const void *W, int dtype, int64_t M, int64_t N, int64_t K,
                     int64_t ldx, int64_t ldw, const float *s, int64_t group_size, int32_t *index_out,
                     float *step_out, uint8_t *zero_out, double *err_table, void *workspace,
                     size_t workspace_bytes, void *stream);

/* ---- Weight-format variants that the paper compares dINT4 with (3-bit dINT, Table 10; ordinary INT4,
 * Tables 11-14), in one 4-bit code space so that pack_dint4 and the GEMM serve all of them:
 *     W4A8_FMT_DINT4  p = 13 integer steps (codes 0..13) + special levels +step/2 (14), -step/2 (15)  (Eq. 5)
 *     W4A8_FMT_DINT3  p = 2^3 - 3 = 5 (codes 0..5) + the same special codes 14, 15
 *     W4A8_FMT_INT4   p = 15 (codes 0..15 all integer levels, zero-point 0..15), no special levels
 * Rule as quantize_weight_dint4 with 13 replaced by p (and the two special cases dropped for INT4).
 * w4a8_gemm_format is w4a8_gemm with the meaning of codes 14 / 15 chosen by `format`. */
int quantize_weight_format(const void *W, int w_dtype, int64_t N, int64_t K, int64_t ldw, const float *s,
                           int64_t group_size, int format, int use_given_params, uint8_t *codes,
                           float *step, uint8_t *zero, void *stream);
/* pack_dint4 / unpack_dint4 for a format.  The canonical layout stores the codes as they are; in the
 * tiled layout INT4's codes 14 and 15 are the integer pair of the eighth base level, lower member first
 * (nibble e = (c >> 1) | ((c & 1) << 3) for all sixteen codes), whereas the dINT formats keep the
 * special pair as described at W4A8_LAYOUT_TILED. */
int pack_format(const uint8_t *codes, int64_t N, int64_t K, uint8_t *packed, int layout, int format,
                void *stream);
int unpack_format(const uint8_t *packed, int64_t N, int64_t K, uint8_t *codes, int layout, int format,
                  void *stream);
int w4a8_gemm_format(const int8_t *Xq, const float *sx, int64_t M, const uint8_t *Wp, int layout,
                     const float *step, const uint8_t *zero, int64_t N, int64_t K, int64_t group_size,
                     int format, void *Y, int y_dtype, int64_t ldy, int32_t *acc_out, void *workspace,
                     size_t workspace_bytes, void *stream);

/* ---- The special value of dINT4 (App. A.5, Table 9: c = step/4 and step/8 in place of step/2).
 * quantize_weight_format with W4A8_FMT_DINT4_C4 / _C8 keeps dINT4's code space (14 = +c, 15 = -c) and
 * rounds to the nearest level: +c for c/2 < w' <= (step + c)/2, i.e. 2^-(t+1) < w'/step <= 1/2 + 2^-(t+1)
 * with c = step / 2^t, ends open / closed as in Eq. 5, -c mirrored (for t = 1 this is Eq. 5 itself).
 * The GEMMs only know c = step/2.  Since  +-c = +-step/2 -+ (1 - 2^(1-t)) step/2,  such a matrix is the
 * ordinary dINT4 matrix of twice the width that expand_special_value writes:
 *     codes2 [N, 2K]:  columns 0..K-1 the codes; columns K..2K-1 the special codes with their signs
 *                      exchanged (14 <-> 15) and every other code replaced by the group's zero level z
 *     step2  [N, 2K/G]: the steps, then (1 - 2^(1-t)) * step (one binary32 multiply);  zero2: zero twice
 * Pack codes2 with pack_dint4 (N x 2K) and call w4a8_gemm_special, which multiplies it with [Xq | Xq]:
 * Y as w4a8_gemm would give for the variant format (same fp32 order over the 2K/G groups), and
 * acc_out [M, N, 2K/G] with the two sums A1 (groups 0..K/G-1) and A2 of every group, from which the sum
 * in units of step / 2^t is  2^(t-1) A1 + (2^(t-1) - 1) A2.  Twice the work of w4a8_gemm: a tool for the
 * format sweep, not a serving path.
 *   group_size: 0 (per channel) or a multiple of 128 that divides K; 2K <= 65536; other limits, workspace
 *   rules and errors as for w4a8_gemm with K replaced by 2K (the workspace also holds [Xq | Xq]). */
int expand_special_value(const uint8_t *codes, const float *step, const uint8_t *zero, int64_t N, int64_t K,
                         int64_t group_size, int format, uint8_t *codes2, float *step2, uint8_t *zero2,
                         void *stream);
size_t w4a8_gemm_special_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t group_size, int layout);
int w4a8_gemm_special(const int8_t *Xq, const float *sx, int64_t M, const uint8_t *Wp2, int layout,
                      const float *step2, const uint8_t *zero2, int64_t N, int64_t K, int64_t group_size,
                      void *Y, int y_dtype, int64_t ldy, int32_t *acc_out, void *workspace,
                      size_t workspace_bytes, void *stream);

/* 3-bit storage of dINT3 codes: 0..5 stay, special codes 14 / 15 become 6 / 7; code i of each group of
 * eight consecutive codes of a row sits at bits 3i..3i+2 of a little-endian 24-bit word (three bytes).
 *   codes [N, K] in the 4-bit code space, K % 8 == 0      packed [N, 3K/8] bytes
 * unpack_dint3 restores the 4-bit code space (ready for pack_dint4 and the GEMM). */
int pack_dint3(const uint8_t *codes, int64_t N, int64_t K, uint8_t *packed, void *stream);
int unpack_dint3(const uint8_t *packed, int64_t N, int64_t K, uint8_t *codes, void *stream);

/* The error split of Sec. 4.1 (Eq. 4) for weight quantization in `format`: with W' = W diag(s), Wq its
 * dequantized codes and X' = X diag(s)^-1 (unquantized), Delta_u = Wq - W' on the weights whose
 * quantized value is zero ("underflow"), Delta_r on the others ("rounding"):
 *     terms[0] = sum (X' Delta_u^T)^2    terms[1] = sum (X' Delta_r^T)^2
 *     terms[2] = sum 2 (X' Delta_u^T)(X' Delta_r^T)        terms[3] = number of underflowing weights
 * (their first three add up to the squared output error of weight quantization alone).
 *   format: any W4A8_FMT_* (the special-value variants included);
 *   X [M, ldx], W [N, ldw] of their dtypes; terms out [4] double (device);
 *   workspace of dint_error_terms_workspace_bytes(M, N, K, group_size) bytes, 256-byte aligned. */
size_t dint_error_terms_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t group_size);
int dint_error_terms(const void *X, int x_dtype, int64_t M, int64_t K, int64_t ldx, const void *W,
                     int w_dtype, int64_t N, int64_t ldw, const float *s, int64_t group_size, int format,
                     double *terms, void *workspace, size_t workspace_bytes, void *stream);

/* Human-readable name of a status code (static storage, never NULL). */
const char *w4a8_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* W4A8_H */
