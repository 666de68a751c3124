// Shared device helpers of the gfx950 W4A8 kernels (wave64, CDNA4).
#pragma once
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "../../include/w4a8.h"
#include "../../include/w4a8_measure.h"

namespace w4a8 {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));

constexpr int WAVE = 64;
constexpr int DINT4_P = 13;       // uniform steps of dINT4, 2^4 - 3 (Sec. 4.2)
constexpr int TILE_N = 16;        // rows of one packed-weight tile (layout 1)
constexpr int TILE_K = 128;       // columns of one packed-weight tile
constexpr int TILE_BYTES = 1024;  // 16 * 128 / 2

// ---- element loads, widened exactly to binary32 -------------------------------------------
struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(__half v) { return __half2float(v); }
__device__ __forceinline__ float to_f32(bf16_t v) { return __uint_as_float((uint32_t)v.bits << 16); }

// round-to-nearest-even narrowing of a finite binary32 value
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    const uint32_t u = __float_as_uint(f);
    const uint32_t rounded = u + 0x7fffu + ((u >> 16) & 1u);
    const uint32_t quiet = u | 0x400000u;                        // NaN stays NaN
    // (a select, not a branch: callers convert in the middle of long straight-line epilogues)
    return (uint16_t)(((u & 0x7fffffffu) > 0x7f800000u ? quiet : rounded) >> 16);
}
__device__ __forceinline__ uint16_t f32_to_f16_bits(float f)
{
    return __half_as_ushort(__float2half_rn(f));
}

// ---- wave-level reductions ------------------------------------------------------------------
// All 64 lanes must be active at the call (every caller reduces in wave-uniform control flow).
// Data-parallel-primitive operands instead of LDS permutes: the other lane's value comes in as a
// modifier of the max / min / add itself.  Two quad permutes, then the mirror of each half row and
// of each row of 16 lanes leave every row's result in all of its lanes; the four rows meet
// through scalar registers.
constexpr int DPP_QUAD_XOR1 = 0xB1;        // quad_perm [1, 0, 3, 2]
constexpr int DPP_QUAD_XOR2 = 0x4E;        // quad_perm [2, 3, 0, 1]
constexpr int DPP_ROW_HALF_MIRROR = 0x141; // lane i <-> 7 - i within 8 lanes
constexpr int DPP_ROW_MIRROR = 0x140;      // lane i <-> 15 - i within 16 lanes

template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v)
{
    return __int_as_float(dpp_i32<CTRL>(__float_as_int(v)));
}
__device__ __forceinline__ float lane_f32(float v, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, dpp_f32<DPP_QUAD_XOR1>(v));
    v = fmaxf(v, dpp_f32<DPP_QUAD_XOR2>(v));
    v = fmaxf(v, dpp_f32<DPP_ROW_HALF_MIRROR>(v));
    v = fmaxf(v, dpp_f32<DPP_ROW_MIRROR>(v));
    return fmaxf(fmaxf(lane_f32(v, 0), lane_f32(v, 16)), fmaxf(lane_f32(v, 32), lane_f32(v, 48)));
}
__device__ __forceinline__ float wave_min(float v)
{
    v = fminf(v, dpp_f32<DPP_QUAD_XOR1>(v));
    v = fminf(v, dpp_f32<DPP_QUAD_XOR2>(v));
    v = fminf(v, dpp_f32<DPP_ROW_HALF_MIRROR>(v));
    v = fminf(v, dpp_f32<DPP_ROW_MIRROR>(v));
    return fminf(fminf(lane_f32(v, 0), lane_f32(v, 16)), fminf(lane_f32(v, 32), lane_f32(v, 48)));
}
__device__ __forceinline__ int wave_sum_i32(int v)
{
    v += dpp_i32<DPP_QUAD_XOR1>(v);
    v += dpp_i32<DPP_QUAD_XOR2>(v);
    v += dpp_i32<DPP_ROW_HALF_MIRROR>(v);
    v += dpp_i32<DPP_ROW_MIRROR>(v);
    return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) +
           __builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48);
}

// ---- dINT4 nibble decode for the int8 matrix cores -----------------------------------------
//
// A stored nibble is e = l | h << 3 (see the tiled layout in w4a8.h): l in 0..6 names the pair
// of integer codes (2l, 2l+1), l = 7 the pair (-step/2, +step/2); h picks the upper member,
// which in every pair lies exactly one step = two half steps above the lower one.
//
// With z the zero-point of the (row, group), the weight in half steps is
//     d = 4 l + 2 h - 2 z   (l < 7)        d = 2 h - 1   (l = 7)          (Eq. 5, second half)
// The kernels feed the matrix cores  D = 4 (d + beta),  beta = 2 z + b0,  b0 = 1 - (z & 1):
//     D = (16 l + 4 b0) | (h << 3)          (l < 7)
//     D = (8 z + 4 b0 - 4) | (h << 3)       (l = 7)
// Both base terms always have bit 3 clear (that is what the parity-dependent b0 buys), so the
// per-byte "+8h" is a plain OR with the nibble's own bit 3 -- no carries between the four bytes
// of a register.  0 <= D <= 108 fits int8.  The GEMM accumulates sum_k Xq * D and removes the
// bias afterwards with the token's group row-sum:  sum_k Xq d = (acc - 4 beta * rowsum) / 4,
// which is exact in int32 (4 beta * |rowsum| and |acc| stay below 2^31 for K <= 65536).
struct DecodeLut {
    uint32_t lo;     // base levels of l = 0..3, one per byte
    uint32_t hi;     // base levels of l = 4..7
    int beta_q;      // 4 * beta = 8 z + 4 b0
};

// plain: the code space of ordinary INT4 (16 integer levels, zero-point up to 15): the pair l = 7 is
// the integer pair (14, 15) like the others, D = (112 + 4 b0) | (h << 3) <= 124.
__device__ __forceinline__ DecodeLut make_decode_lut(int z, bool plain = false)
{
    DecodeLut t;
    const uint32_t c4 = ((uint32_t)(~z) & 1u) << 2;  // 4 * b0
    const uint32_t c4x4 = c4 * 0x01010101u;
    t.lo = 0x30201000u | c4x4;
    t.hi = plain ? (0x70605040u | c4x4)
                 : ((0x00605040u | (c4x4 & 0x00ffffffu)) | ((uint32_t)(8 * z + (int)c4 - 4) << 24));
    t.beta_q = 8 * z + (int)c4;
    return t;
}

// Eight nibbles of one packed word -> eight int8 values D, columns +0..3 in `a`, +4..7 in `b`.
__device__ __forceinline__ void decode_word(uint32_t p, const DecodeLut &t, int &a, int &b)
{
    const uint32_t q = p >> 4;
    const uint32_t ra = __builtin_amdgcn_perm(t.hi, t.lo, p & 0x07070707u);
    const uint32_t rb = __builtin_amdgcn_perm(t.hi, t.lo, q & 0x07070707u);
    a = (int)(ra | (p & 0x08080808u));
    b = (int)(rb | (q & 0x08080808u));
}

// One lane's 16 packed bytes (32 weights) -> the two 16-byte matrix-core operands.
__device__ __forceinline__ void decode_lane(const v4u &p, const DecodeLut &t, v4i &w0, v4i &w1)
{
    int a, b;
    decode_word(p.x, t, a, b); w0.x = a; w0.y = b;
    decode_word(p.y, t, a, b); w0.z = a; w0.w = b;
    decode_word(p.z, t, a, b); w1.x = a; w1.y = b;
    decode_word(p.w, t, a, b); w1.z = a; w1.w = b;
}

// Signed variant for kernels that cannot afford the bias removal per accumulator: the table holds
// the levels in excess-128 form, T[l] = 128 + 16 l - 8 z (l < 7), T[7] = 124; adding 8 h never
// carries between bytes (T + 8 <= 232) and flipping bit 7 of every byte turns excess-128 into two's
// complement, giving 4 d directly.  Costs 11 instead of 7 operations per 8 weights.
struct SignedLut {
    uint32_t lo, hi;
};
__device__ __forceinline__ SignedLut make_signed_lut(int z, bool plain = false)
{
    SignedLut t;
    const uint32_t b = (uint32_t)(128 - 8 * z);           // 24 .. 128 (8 .. 128 for plain INT4)
    const uint32_t b4 = __builtin_amdgcn_perm(b, b, 0u);  // replicated to the four bytes
    t.lo = b4 + 0x30201000u;                              // no carries: b + 48 <= 176
    t.hi = plain ? b4 + 0x70605040u                       // b + 112 + 8 h <= 248
                 : (b4 & 0x00ffffffu) + 0x00605040u + (124u << 24);
    return t;
}
__device__ __forceinline__ void decode_word_signed(uint32_t p, const SignedLut &t, int &a, int &b)
{
    const uint32_t q = p >> 4;
    const uint32_t ra = __builtin_amdgcn_perm(t.hi, t.lo, p & 0x07070707u);
    const uint32_t rb = __builtin_amdgcn_perm(t.hi, t.lo, q & 0x07070707u);
    a = (int)((ra + (p & 0x08080808u)) ^ 0x80808080u);
    b = (int)((rb + (q & 0x08080808u)) ^ 0x80808080u);
}

// Host-side launchers (defined in the .hip files, called from the C ABI in api.hip).
// zx == nullptr: symmetric absmax; else asymmetric min-max, token zero-points (minus 128) to zx
int launch_act_quant(const void *X, int x_dtype, int64_t M, int64_t K, int64_t ldx, const float *s,
                     int8_t *Xq, float *sx, int32_t *zx, hipStream_t st);
// wsum[N, K/T]: sums of the weights in half steps over blocks of T columns (T divides G)
int launch_weight_sums(const uint8_t *codes, const uint8_t *zero, int64_t N, int64_t K, int64_t G,
                       int64_t T, int32_t *wsum, hipStream_t st);
int launch_acc_zero_point(int32_t *acc, const int32_t *zx, const int32_t *wsum, int64_t M,
                          int64_t per_token, hipStream_t st);
int launch_weight_quant(const void *W, int w_dtype, int64_t N, int64_t K, int64_t ldw,
                        const float *s, int64_t G, int use_given, uint8_t *codes, float *step,
                        uint8_t *zero, int format, hipStream_t st);
// step / zero of the ranges shrunk by rho = 1 - 0.05 i, i = idx[n] (or `uniform` when idx is null)
int launch_clip_params(const void *W, int w_dtype, int64_t N, int64_t K, int64_t ldw, const float *s,
                       int64_t G, const int32_t *idx, int uniform, float *step, uint8_t *zero,
                       hipStream_t st);
// AQAS scale search helpers (aqas_search.hip)
int launch_channel_absmax(const void *A, int dtype, int64_t R, int64_t K, int64_t lda, float *out,
                          hipStream_t st);
int launch_aqas_scale(const float *ax, const float *aw, int64_t K, int j, const int32_t *j_dev,
                      float *s, hipStream_t st);
int launch_ref_gemm(const void *X, const void *W, int dtype, int64_t M, int64_t N, int64_t K,
                    int64_t ldx, int64_t ldw, float *Y, hipStream_t st);
int launch_output_sq_error(const void *Y, int y_dtype, int64_t ldy, const float *Yref, int64_t M,
                           int64_t N, double *err, hipStream_t st);
int launch_loss_sum(const double *err, int64_t N, double *losses, int slot, hipStream_t st);
int launch_argmin(const double *losses, int count, int32_t *best, hipStream_t st);
int launch_clip_select(const double *err, int64_t N, int i, double *best_err, int32_t *best_idx,
                       double *err_table, hipStream_t st);
// 3-bit storage of dINT3 codes (0..5, 14 -> 6, 15 -> 7): eight codes in three bytes
int launch_pack3(const uint8_t *codes, int64_t N, int64_t K, uint8_t *packed, hipStream_t st);
int launch_unpack3(const uint8_t *packed, int64_t N, int64_t K, uint8_t *codes, hipStream_t st);
// error split of Sec. 4.1: du / dr [N,K] = quantization error of W diag(s) on the weights that
// quantize to zero / on the others; xs = X diag(s)^-1 in fp32; terms = {sum pu^2, sum pr^2,
// sum 2 pu pr, number of underflowing weights}; special: 0 = no special levels, t = 1..3: +-step / 2^t
int launch_error_split(const void *W, int w_dtype, int64_t N, int64_t K, int64_t ldw, const float *s,
                       int64_t G, int special, const uint8_t *codes, const float *step,
                       const uint8_t *zero, float *du, float *dr, hipStream_t st);
int launch_scale_activations(const void *X, int x_dtype, int64_t M, int64_t K, int64_t ldx,
                             const float *s, float *xs, hipStream_t st);
int launch_error_terms(const float *pu, const float *pr, int64_t n, const float *du, int64_t nw,
                       double *terms, hipStream_t st);
// Value cache: V [batch, T, D] (token stride ld_t, head stride ld_b) -> codes [batch * D, T]
int launch_value_quant(const void *V, int v_dtype, int64_t batch, int64_t T, int64_t D, int64_t ld_t,
                       int64_t ld_b, int64_t G, uint8_t *codes, float *step, uint8_t *zero,
                       hipStream_t st);
// plain != 0: code space of ordinary INT4 (codes 14 / 15 are the integer pair of l = 7)
int launch_pack(const uint8_t *codes, int64_t N, int64_t K, uint8_t *packed, int layout,
                hipStream_t st, int plain = 0);
int launch_unpack(const uint8_t *packed, int64_t N, int64_t K, uint8_t *codes, int layout,
                  hipStream_t st, int plain = 0);
int launch_repack_canonical_to_tiled(const uint8_t *canon, int64_t N, int64_t K, uint8_t *tiled,
                                     hipStream_t st, int plain = 0);
int launch_fill_i32(int32_t *p, int64_t n, int32_t v, hipStream_t st);
// dINT4 with special value step / 2^shift (shift 2, 3) -> ordinary dINT4 matrix [N, 2K]; [Xq | Xq]
int launch_expand_special(const uint8_t *codes, const float *step, const uint8_t *zero, int64_t N,
                          int64_t K, int64_t G, int shift, uint8_t *codes2, float *step2, uint8_t *zero2,
                          hipStream_t st);
int launch_repeat_activations(const int8_t *Xq, int64_t M, int64_t K, int8_t *out, hipStream_t st);
// measured ceilings (ceilings.hip): a streaming read of `bytes` bytes; `iters` rounds of the int8 MFMA loop
int launch_stream_read(const void *buf, int64_t bytes, uint32_t *sink, hipStream_t st);
int launch_mfma_i8_loop(int64_t iters, uint32_t *sink, int64_t *ops, hipStream_t st);
int launch_ktile_mix(int64_t iters, int fragment_reads, uint32_t *sink, hipStream_t st);
// Launch shape of the decode GEMV for a problem size (also sizes its K-split workspace).
struct GemvPlan {
    int splits;            // K is cut into this many ranges, each handled by its own workgroups
    int kt_per_split;      // 128-column k-tiles per range
    int at;                // k-tiles per compute wave (template instance)
    int q;                 // most 16-channel n-tiles any workgroup gets
    int blocks_per_split;
    int nt_lo, nt_rem;     // workgroup b of a split owns nt_lo (+1 if b < nt_rem) n-tiles: b, b + blocks_per_split, ...
    int lds_bytes;
    size_t partial_bytes;  // fp32 partial sums [splits][M][N] when splits > 1, else 0
};
GemvPlan plan_gemv(int64_t M, int64_t N, int64_t K, int64_t G, int64_t batch = 1);
// Asymmetric activations: zx = token zero-points, wsum = weight sums per group [N, K/G],
// tsum = weight sums per 128 columns [N, K/128]; all three null for the symmetric form.
struct ZeroPoint {
    const int32_t *zx, *wsum, *tsum;
};
// batch > 1: `batch` problems of one shape, every operand densely stacked (Y: M * ldy apart);
// needs a single K-range and no accumulator hook.
// 16 < M <= 128: the number of 16-token blocks that launch_gemv runs as one launch over shared weights
// where that is faster than the tile kernel (K within one K-range, few blocks or a small layer); else 0
int gemv_token_blocks(int64_t M, int64_t N, int64_t K, int64_t G);
// Unquantized activations for the streaming kernel's instances that quantize them in the launch
// (M <= 16, one K range of at most 7168 columns, symmetric form): X fp16 rows ldx elements apart
// (16-byte aligned), s the AQAS scale or null; Xq_out / sx_out: null, or where workgroup 0 leaves what
// it made (test hooks).
struct FusedAct {
    const void *X;
    int64_t ldx;
    const float *s;
    int8_t *Xq_out;
    float *sx_out;
};
// whether a shape can take those instances (they need K in one range and room in LDS for 1 / s)
bool gemv_can_fuse(int64_t M, int64_t N, int64_t K, int64_t G);
// fused != null: Xq and sx are ignored
int launch_gemv(const int8_t *Xq, const float *sx, ZeroPoint zp, int64_t M, const uint8_t *Wt,
                const float *step, const uint8_t *zero, int64_t N, int64_t K, int64_t G, void *Y,
                int y_dtype, int64_t ldy, int32_t *acc_out, float *partial, int64_t batch,
                hipStream_t st, int plain = 0, const FusedAct *fused = nullptr);
// Y = cast(sx * sum over splits of partial).  int_step != null: the partials are int32
// accumulators of a per-channel launch, scaled by int_step[n] / 8 after the exact zero-point term.
int launch_gemv_combine(const float *partial, const float *sx, const float *int_step, ZeroPoint zp,
                        int64_t M, int64_t N, int splits, void *Y, int y_dtype, int64_t ldy,
                        hipStream_t st);
// Launch shape of the prefill GEMM (also sizes its workspace).
struct GemmPlan {
    int bm;                // token rows per workgroup tile
    int splits;            // K ranges handled by separate workgroups (1 unless the output has few tiles)
    int kt_per_split;
    size_t rs_bytes;       // int32 row-sums [splits][M] (per-channel weights only)
    size_t partial_bytes;  // fp32 partial sums [splits][M][N] when splits > 1
    // Last round of tiles at most half full (group-wise 128 x 128 tiles, more than one round): the
    // channels of that round run as a launch of their own with K cut into rem_splits ranges
    // (0: no such remainder).  partial_bytes is then [rem_splits][M][rem_n].
    int rem_n;             // output channels of the remainder launch (the last ones)
    int rem_splits;
    int rem_kt_per_split;
};
GemmPlan plan_gemm(int64_t M, int64_t N, int64_t K, int64_t G);
int launch_gemm(const int8_t *Xq, const float *sx, ZeroPoint zp, int32_t *rs, int64_t M,
                const uint8_t *Wt, const float *step, const uint8_t *zero, int64_t N, int64_t K,
                int64_t G, void *Y, int y_dtype, int64_t ldy, int32_t *acc_out, float *partial,
                hipStream_t st, int plain = 0);

inline int hip_status(hipError_t e) { return e == hipSuccess ? W4A8_OK : W4A8_ERR_HIP; }

// More than 64 KB of dynamic LDS has to be opted into per kernel and per device.  `done` is that
// kernel's record of the devices it has been set on (bit = device ordinal modulo 64; setting it
// twice is harmless, so concurrent callers need no lock).
inline int opt_in_dynamic_lds(const void *kernel, int bytes, std::atomic<uint64_t> &done)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return W4A8_ERR_HIP;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_relaxed) & bit) return W4A8_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
        return W4A8_ERR_HIP;
    done.fetch_or(bit, std::memory_order_relaxed);
    return W4A8_OK;
}

}  // namespace w4a8
