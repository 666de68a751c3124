// dINT4 x INT8 GEMM, decode shape (M <= 16): a memory-bound GEMV that streams the packed
// weights exactly once  (Eq. 1 product on the integer operands; Eq. 5 second half fused as the
// epilogue; the dINT4 x INT8 multiply-accumulate of Sec. 4.3 mapped onto the int8 matrix cores).
//
// Work decomposition.  The tiled weight layout cuts W into 1 KB tiles of 16 output channels x
// 128 input channels.  A persistent workgroup owns a set of 16-channel "n-tiles" (all of K, or one
// K-split of it; n-tiles b, b + grid width, ...: sets differ by at most one tile, and the chip as
// a whole reads a contiguous window of the weights at a time) and has 8 compute wavefronts plus
// 1 helper wavefront:
//   * compute wave w owns the k-tiles kt = w, w+8, ... (at most AT of them).  Its int8 activation
//     fragments for those k-tiles are loaded once and stay in registers for the workgroup's
//     lifetime, so in steady state the only memory instructions it issues are 16-byte-per-lane
//     buffer loads of weight tiles (the wave reads one contiguous 1 KB tile per instruction).
//     The weight registers form a ring D n-tiles deep: right after slot (j % D, u) has been
//     consumed it is refilled with k-tile u of n-tile j + D, so D * AT KB per wave are in flight
//     towards HBM at any time.  Every load is issued unconditionally (tiles that do not exist are
//     addressed out of range, which a buffer load answers with zeros and no traffic), so the
//     s_waitcnt counts are static and a wave only ever waits for the one tile it is about to use.
//   * start-up is bound by the CU's memory pipeline, which takes one 1 KB request per 16 clocks
//     and serves requests in issue order: the compute waves first issue the (small, coalesced)
//     loads of the quantization parameters, meet at a barrier, and only then issue the bulk
//     loads, so that no wave's parameters queue behind another wave's weights.
//   * per tile: one ds_read_b128 fetches the precomputed decode record of (channel, k-tile), the
//     nibbles become int8 through the register LUT (w4a8_common.hpp), two MFMAs
//     (v_mfma_i32_16x16x64_i8, the <= 16 token rows are the other operand) accumulate the biased
//     product and two more against a constant "-4 beta" operand remove the decode bias exactly; the
//     int32 group sum is scaled into an fp32 running sum.
//   * the helper wave never touches the weight stream: after each n-tile's barrier it adds the 8
//     waves' partial sums in a fixed order (deterministic), applies the token scale and stores Y
//     (or an fp32 partial for a later combine when K is split across workgroups).
// Per-CU L2->L1 bandwidth (~30 B/clk) is what makes re-reading activations per tile unaffordable:
// at M = 16 they are twice the bytes of the 4-bit weights.
#include "w4a8_common.hpp"

namespace w4a8 {

constexpr int GV_CW = 8;                          // compute waves per workgroup
constexpr int GV_THREADS = (GV_CW + 1) * WAVE;    // + 1 helper wave
constexpr int GV_MAX_AT = 9;                      // k-tiles per compute wave -> K per split <= 9216 (5120 group-wise)
constexpr int GV_REC_THREADS = GV_CW * WAVE;      // the compute waves prepare the decode records
constexpr int GV_STAGE = 16;                      // decode records such a thread prepares at most
constexpr int GV_LDS_BUDGET = 128 * 1024;         // bytes of decode records per workgroup
constexpr int GV_OOB = 0x7fff0000;                // buffer offset beyond any buffer: loads return 0
constexpr int GV_RED_BYTES = 2 * GV_CW * 256 * 4; // partial sums of the compute waves, double buffered
constexpr int GV_MAX_LDS = GV_RED_BYTES + GV_LDS_BUDGET;
constexpr int GV_LDS_LIMIT = 160 * 1024;          // LDS of a CU: what a kernel may opt into
constexpr int GV_FUSED_STAGE = 8;                 // decode records such an instance's thread prepares at most
constexpr int GV_FUSED_MAX_AT = 7;                // k-tiles per wave of the instances that quantize the activations themselves

__device__ __forceinline__ void lds_barrier()
{
    // LDS-only barrier: outstanding global loads (the prefetched weight ring) stay in flight
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Pins the program order of memory instructions and of everything scheduled around them, at
// every level of the compiler (emits no instruction).
__device__ __forceinline__ void order_fence()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// Decode record of one (channel, k-tile): LUT halves, step / 8, and in the last word -4 beta as an
// int8 in byte 0 with 4 * tsum in the upper 24 bits (tsum: sum of the tile's weights in half steps,
// |4 tsum| <= 4 * 26 * 128; zero without a token zero-point).
__device__ __forceinline__ v4u decode_record(int z, float st, int tsum, bool plain)
{
    const DecodeLut t = make_decode_lut(z, plain);
    const uint32_t nb8 = (uint32_t)(-t.beta_q) & 0xffu;
    return v4u{t.lo, t.hi, __float_as_uint(st * 0.125f), ((uint32_t)(4 * tsum) << 8) | nb8};
}

__device__ __forceinline__ v4i as_v4i(const v4u &v) { return v4i{(int)v.x, (int)v.y, (int)v.z, (int)v.w}; }

// Kernel arguments (one block, so the prologue issues few scalar loads).
struct GemvArgs {
    const int8_t *Xq;      // [M, K]
    const float *sx;       // [M]
    const int32_t *zx;     // [M] token zero-points (asymmetric activations) or null
    const int32_t *wsum;   // [N, ng] sums of the weights per group, in half steps (with zx)
    const int32_t *tsum;   // [N, K / 128] the same per k-tile (with zx)
    const uint8_t *Wt;     // tiled packed weights
    const float *step;     // [N, ng]
    const uint8_t *zero;   // [N, ng]
    uint16_t *Y;           // [M, ldy]
    float *partial;        // [splits, M, N] or null
    int32_t *acc_out;      // test hook or null
    int64_t ldy;
    int M, N, K;
    int tiles_per_group, ng, y_dtype;
    int kt_per_split;      // k-tiles per K-split (blockIdx.y)
    int nt_lo, nt_rem;     // workgroup b owns nt_lo (+1 if b < nt_rem) n-tiles: b, b + width, ...
    int nt_stride;         // width: the number of workgroups per K-range
    int plain;             // code space of ordinary INT4 (16 integer levels) instead of dINT4
    int vec_store;         // Y and ldy allow 8-byte stores of four outputs
    int token_blocks;      // blockIdx.z: 16-token blocks of one problem (shared weights) instead of problems
    int part_rows;         // token rows of one K-range's slab of `partial` (all blocks' rows)
    // FUSED instances: the activations come unquantized and every workgroup quantizes them itself
    const void *X;         // [M, ldx] fp16
    const float *s;        // [K] AQAS scale or null
    int64_t ldx;
    int fused_lds_off;     // byte offset of the reciprocal scales [K] (then the row maxima [8][16]) in LDS
    int8_t *Xq_out;        // test hooks (workgroup 0 writes them) or null
    float *sx_out;
};

// GROUPED: one (step, zero) per k-tile or coarser group, rescaled per tile.  !GROUPED: per channel.
// AT k-tile slots per compute wave, weight ring D n-tiles deep; D = 0: the workgroups own a
// single n-tile each, so there is no ring and nothing is ever refilled.
// ASYM: the activations carry a token zero-point zx (stored codes and zx both offset by -128);
// the exact term zx * (sum of the weights) is taken out in int32, per tile (GROUPED) or once per
// output after the waves' int32 sums have been added (!GROUPED) -- never in floating point, where
// the two large terms would cancel badly.
// FUSED: the step before the product runs inside the launch (Eq. 1, factor Q(diag(s)^-1 X), per-token
// absmax INT8): Xq and sx are not read but made here from X and s, by every workgroup for itself --
// at <= 16 tokens that costs each workgroup about as much as waiting for another launch's result
// would, and saves the launch.  The weight ring is issued first (it does not depend on X); then the
// 512 compute lanes put the reciprocals 1 / s[k] into LDS (true divisions), load their own k-tiles'
// rows of X in the pattern of the int8 fragments (a quad of lanes reads 2 x 128 contiguous bytes of a
// row), take the row maxima of t = x * r (quad reduction, then the 8 waves' partial maxima meet in
// LDS) and round t * (127 / a) into the very registers the int8 fragments would have been loaded
// into.  Every floating-point step is the single binary32 operation of the definition, so Xq and sx
// have the bits quantize_act_int8 gives.  One K range only (every workgroup sees whole rows).
template <bool GROUPED, int AT, int D, bool ACC_OUT, bool ASYM, bool FUSED = false>
__global__ __launch_bounds__(GV_THREADS) void gemv_kernel(const GemvArgs args)
{
    // blockIdx.z: independent problems of one shape, densely stacked (batched launch), or the
    // 16-token blocks of one problem with more than 16 tokens: the same weights, and the last block
    // may be shorter
    GemvArgs a = args;
    if (gridDim.z > 1) {
        const int64_t b = blockIdx.z;
        const int64_t rows_w = a.token_blocks ? 0 : b * a.N;
        const int64_t rows_x = a.token_blocks ? b * 16 : b * a.M;
        if (a.token_blocks) {
            if (a.acc_out != nullptr) a.acc_out += rows_x * a.N * a.ng;
            if (a.partial != nullptr) a.partial += rows_x * a.N;
            a.M = min(16, a.M - (int)rows_x);
        }
        a.Xq += rows_x * a.K;
        a.sx += rows_x;
        a.Wt += rows_w * a.K / 2;
        a.step += rows_w * a.ng;
        a.zero += rows_w * a.ng;
        a.Y += rows_x * a.ldy;
        if (a.zx != nullptr) {
            a.zx += rows_x;
            a.wsum += rows_w * a.ng;
            a.tsum += rows_w * (a.K >> 7);
        }
    }
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    float *red = reinterpret_cast<float *>(smem);                        // [2][GV_CW][256]
    v4u *rec = reinterpret_cast<v4u *>(smem + GV_RED_BYTES);             // [n-tile][channel][RS]

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int M = a.M, N = a.N, K = a.K;
    const int KT = K >> 7;
    const int split = blockIdx.y;
    const int blk = blockIdx.x;
    // n-tiles are dealt out as evenly as possible, interleaved over the workgroups: the chip then
    // reads one contiguous window of the weights at a time (consecutive runs per workgroup, i.e.
    // 256 streams far apart, measured 5-10 % slower on weights of 85-340 MB)
    const int nt_stride = a.nt_stride;
    const int nt0 = blk;
    auto nt_of = [&](int j) { return nt0 + j * nt_stride; };
    const int my_nt = a.nt_lo + (blk < a.nt_rem ? 1 : 0);
    const int kt_begin = split * a.kt_per_split;
    const int KTs = min(a.kt_per_split, KT - kt_begin);     // k-tiles of this split
    const int recs_per_nt = GROUPED ? KTs : 1;
    // records of one channel are consecutive; an odd stride spreads the 16 channels that one
    // ds_read_b128 touches over all LDS banks
    const int RS = GROUPED ? (KTs | 1) : 1;

    // ---- quantization parameters of this workgroup -> decode records in LDS -------------------
    // Element e = (n-tile j, channel row, k-tile ktl), ktl fastest: consecutive lanes read
    // consecutive groups of one channel, i.e. consecutive addresses of step[] and zero[].
    // Loads first (only the stages that exist, uniform over the workgroup), LUT arithmetic
    // later.  Quotients by multiplication with an approximate reciprocal: exact here, since
    // (e + 0.5) / d is at least 1 / (2 d) away from any integer and e < 2^13, d <= 64, against
    // a relative error below 2^-21.
    constexpr int STAGES = FUSED ? GV_FUSED_STAGE : GV_STAGE;
    int st_z[STAGES], st_t[STAGES];
    float st_s[STAGES];
    const int n_rec = my_nt * 16 * recs_per_nt;
    const float inv_recs = __builtin_amdgcn_rcpf((float)recs_per_nt);
    auto issue_params = [&]() {
        __amdgpu_buffer_rsrc_t rstep =
            __builtin_amdgcn_make_buffer_rsrc((void *)a.step, 0, N * a.ng * 4, 0x00020000);
        __amdgpu_buffer_rsrc_t rzero =
            __builtin_amdgcn_make_buffer_rsrc((void *)a.zero, 0, N * a.ng, 0x00020000);
        const float inv_tpg = __builtin_amdgcn_rcpf((float)a.tiles_per_group);
#pragma unroll
        for (int i = 0; i < STAGES; ++i) {
            // (a stage that is skipped leaves its registers unset: write_records skips it too)
            if (i * GV_REC_THREADS >= n_rec) break;   // (uniform; one taken branch ends the stages)
            {
                const int e = min((int)threadIdx.x + i * GV_REC_THREADS, n_rec - 1);
                const int t = GROUPED ? (int)(((float)e + 0.5f) * inv_recs) : e;   // 16 j + row
                const int ktl = e - t * recs_per_nt;
                const int g = GROUPED ? (int)(((float)(kt_begin + ktl) + 0.5f) * inv_tpg) : 0;
                const int ch = nt_of(t >> 4) * TILE_N + (t & 15);
                const int idx = ch * a.ng + g;   // < N * ng <= N * K / 128 < 2^29
                st_z[i] = __builtin_amdgcn_raw_buffer_load_b8(rzero, idx, 0, 0);
                st_s[i] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rstep, idx * 4, 0, 0));
                st_t[i] = (ASYM && GROUPED) ? a.tsum[ch * KT + kt_begin + ktl] : 0;
            }
        }
    };
    auto write_records = [&]() {
#pragma unroll
        for (int i = 0; i < STAGES; ++i) {
            if (i * GV_REC_THREADS >= n_rec) break;   // (uniform; one taken branch ends the stages)
            {
                const int e = (int)threadIdx.x + i * GV_REC_THREADS;
                const int t = GROUPED ? (int)(((float)e + 0.5f) * inv_recs) : e;
                // (opaque copies: arithmetic on the loaded values must not be moved up to the
                // loads, where it would wait for each stage in turn)
                float sv = st_s[i];
                int zv = st_z[i];
                asm volatile("" : "+v"(sv), "+v"(zv));
                if (e < n_rec)
                    rec[t * RS + (e - t * recs_per_nt)] =
                        decode_record(zv & 0xff, sv, st_t[i], a.plain != 0);
            }
        }
    };

    // ---- FUSED: the unquantized activations of this wave's k-tiles and the AQAS scales, requested
    // before anything else: they are needed first (the row maxima), the parameters next, the weights last.
    // Raw rows: lane (row = lane / 4, q = lane % 4) holds columns 16 q .. + 15 and 64 + 16 q .. + 15 of
    // each of its k-tiles as four 16-byte pieces -- the columns its int8 fragments a0 / a1 cover.
    constexpr int NS = GV_FUSED_MAX_AT * 2;   // scales per thread: K <= 8 * 128 * GV_FUSED_MAX_AT, 512 threads
    v4u xr[FUSED ? AT : 1][4];
    float sv[FUSED ? NS : 1];
    float *r_lds = reinterpret_cast<float *>(smem + (FUSED ? a.fused_lds_off : 0));   // [K], then maxima [8][16]
    const int xcol = (lane & 3) * 16;   // first column of the lane's first half within a k-tile
    if (FUSED && wave < GV_CW) {
        const int tpw_x = (KTs - wave + GV_CW - 1) / GV_CW;
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            const int k = (int)threadIdx.x + i * GV_REC_THREADS;
            sv[i] = (a.s != nullptr && k < K) ? a.s[k] : 1.0f;
        }
        __amdgpu_buffer_rsrc_t rxx = __builtin_amdgcn_make_buffer_rsrc(
            (void *)a.X, 0, (int)((((int64_t)M - 1) * a.ldx + K) * 2), 0x00020000);
        const int voff_raw = ((lane >> 2) * (int)a.ldx + xcol) * 2;
#pragma unroll
        for (int u = 0; u < AT; ++u) {
            const int vo = u < tpw_x ? voff_raw + (wave + u * GV_CW) * (TILE_K * 2) : GV_OOB;
            xr[u][0] = __builtin_amdgcn_raw_buffer_load_b128(rxx, vo, 0, 0);
            xr[u][1] = __builtin_amdgcn_raw_buffer_load_b128(rxx, vo + 16, 0, 0);
            xr[u][2] = __builtin_amdgcn_raw_buffer_load_b128(rxx, vo + 128, 0, 0);
            xr[u][3] = __builtin_amdgcn_raw_buffer_load_b128(rxx, vo + 144, 0, 0);
        }
        order_fence();
    }
    if (wave < GV_CW) issue_params();
    if (FUSED && wave < GV_CW) {
        // the reciprocals (true divisions) go to LDS as soon as the scales are there (the first loads issued)
        order_fence();
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            const int k = (int)threadIdx.x + i * GV_REC_THREADS;
            if (k < K) r_lds[k] = 1.0f / sv[i];
        }
        order_fence();
    }

    if (wave == GV_CW) {
        // ================= helper wave: reduction across the compute waves + output ============
        // lane owns token m = lane / 4 and the four channels 4 (lane % 4) .. + 3: one 16-byte LDS
        // read per compute wave, one 8-byte store.
        // GROUPED: the waves publish fp32 sums (already scaled per group).  !GROUPED: they publish
        // their int32 accumulators; the sum is exact, then zero-point term, step / 8, token scale.
        const int hm = lane >> 2, hc = (lane & 3) * 4;
        const bool final_out = a.partial == nullptr;
        float sxm = (!FUSED && final_out && hm < M) ? a.sx[hm] : 0.f;
        const bool zp = ASYM && !GROUPED && final_out;
        const int zxm = (zp && hm < M) ? a.zx[hm] : 0;
        const v4i zero4i = {0, 0, 0, 0};
        // per-channel sums of the weights, fetched one n-tile ahead
        auto load_wn = [&](int j) {
            const int32_t *wp = a.wsum + nt_of(j) * TILE_N + hc;
            return v4i{wp[0], wp[1], wp[2], wp[3]};
        };
        v4i wn = zp ? load_wn(0) : zero4i;
        lds_barrier();   // every wave's parameter loads are under way
        lds_barrier();   // the records are complete
        if (FUSED) {
            lds_barrier();   // the compute waves have published their row maxima
            const float *mx = reinterpret_cast<const float *>(smem + a.fused_lds_off) + K;
            float am = 0.f;
#pragma unroll
            for (int w = 0; w < GV_CW; ++w) am = fmaxf(am, mx[w * 16 + hm]);
            sxm = !(127.0f / am <= 3.402823466e+38f) ? 1.0f : am / 127.0f;   // (all-zero or vanishing token: as in the quantizer kernels)
            if (a.sx_out != nullptr && blk == 0 && (lane & 3) == 0 && hm < M) a.sx_out[hm] = sxm;
        }
        for (int j = 0; j < my_nt; ++j) {
            lds_barrier();  // the compute waves have published their partial sums of n-tile j
            const v4i wn_next = (zp && j + 1 < my_nt) ? load_wn(j + 1) : zero4i;
            const float *rb = red + (j & 1) * GV_CW * 256 + 4 * lane;
            v4f sum = {0.f, 0.f, 0.f, 0.f};
            v4i isum = zero4i;
#pragma unroll
            for (int w = 0; w < GV_CW; ++w) {   // fixed order: deterministic
                const v4f part = *reinterpret_cast<const v4f *>(rb + w * 256);
                if (GROUPED) sum += part;
                else isum += v4i{__float_as_int(part.x), __float_as_int(part.y), __float_as_int(part.z),
                                 __float_as_int(part.w)};
            }
            if (hm < M) {
                const int n = nt_of(j) * TILE_N + hc;
                if (!final_out) {
                    float *pp = a.partial + ((int64_t)split * a.part_rows + hm) * N + n;
                    *reinterpret_cast<v4f *>(pp) =
                        GROUPED ? sum
                                : v4f{__int_as_float(isum.x), __int_as_float(isum.y),
                                      __int_as_float(isum.z), __int_as_float(isum.w)};
                } else {
                    uint16_t hh[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        float v = sum[i];
                        if (!GROUPED) {
                            const float es = __uint_as_float(rec[j * 16 + hc + i].z);
                            v = es * (float)(isum[i] - 4 * zxm * wn[i]);
                        }
                        float out = sxm * v;   // binary32 product, then the cast (never one fused
                        asm volatile("" : "+v"(out));   // mixed-precision operation: that rounds once)
                        hh[i] = (a.y_dtype == W4A8_F16) ? f32_to_f16_bits(out) : f32_to_bf16_bits(out);
                    }
                    uint16_t *yp = a.Y + (int64_t)hm * a.ldy + n;
                    if (a.vec_store) {
                        *reinterpret_cast<uint2 *>(yp) =
                            uint2{(uint32_t)hh[0] | ((uint32_t)hh[1] << 16), (uint32_t)hh[2] | ((uint32_t)hh[3] << 16)};
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i) yp[i] = hh[i];
                    }
                }
            }
            wn = wn_next;
        }
        return;
    }

    // ================= compute waves ==========================================================
    const int ln = lane & 15;   // weight operand: output channel;  accumulator: output channel
    const int kb = lane >> 4;   // which 32 of the tile's 128 input channels this lane holds
    const int tpw = (KTs - wave + GV_CW - 1) / GV_CW;   // k-tiles of this wave: kt = wave + 8 u
    __amdgpu_buffer_rsrc_t rw =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.Wt, 0, (int)((int64_t)N * K / 2), 0x00020000);
    __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)a.Xq, 0, M * K, 0x00020000);
    // Activation operand of the matrix cores: lane (ln, kb) holds token row ln, bytes kb*32 .. +32
    // of the k-tile.  Loading it in that pattern (16 rows per instruction, 16 bytes per lane and
    // row) moves a third of the bytes per clock that a row-coalesced load does (measured on L2-
    // resident data: 37 against 104 GB/s per CU), and at 16 tokens the activations are twice the
    // bytes of a tile's weights.  So a quad of lanes reads 64 contiguous bytes of one row (lane l:
    // row l / 4, bytes (l % 4) * 16 [+ 64]) and the fragments are transposed once through this
    // wave's own rows of the reduction buffer.  Rows >= M lie beyond the buffer and read as zero.
    const int voff_x = (lane >> 2) * K + (lane & 3) * 16 + kt_begin * TILE_K;
    const int wt_lane = lane * 16;
    const int tile0 = nt0 * KT + kt_begin + wave;       // first weight tile of this wave
    const int tile_step = nt_stride * KT;               // from one of its n-tiles to the next

    lds_barrier();   // every wave's parameter loads are under way: now the bulk loads
    // slot [d][u]: k-tile u of an n-tile j with j % D == d; out of range when there is none
    constexpr int DR = D > 0 ? D : 1;   // ring rows
    v4u p[DR][AT], a0[AT], a1[AT];
    // Streaming (non-temporal) loads where a workgroup walks several n-tiles, i.e. on matrices of tens of
    // megabytes that are read exactly once (36864 x 9216 at 16 tokens: 33.5 -> 30.7 us); the single-n-tile
    // instances serve small matrices, which measured 6 % slower with the hint.
    constexpr int W_AUX = D == 0 ? 0 : 2;
    auto load_w = [&](int j, int u) {
        const bool ok = j < my_nt && u < tpw;
        return __builtin_amdgcn_raw_buffer_load_b128(
            rw, ok ? wt_lane : GV_OOB, ok ? (tile0 + j * tile_step + u * GV_CW) * TILE_BYTES : 0, W_AUX);
    };
    // decode record of (n-tile j, this lane's channel, slot u), clamped into the staged range
    auto load_rec = [&](int j, int u) {
        const int jr = min(j, my_nt - 1);
        const int ktl = GROUPED ? min(wave + u * GV_CW, KTs - 1) : 0;
        return rec[(jr * 16 + ln) * RS + ktl];
    };
    // Issue order = arrival order (a wave's loads return in order): after the parameters, per
    // slot the activations and the first n-tile's weights, then ring rows 1 .. D-1.
#pragma unroll
    for (int u = 0; u < AT; ++u) {
        // slots without a k-tile hold zero activations, so whatever is computed there adds nothing
        if (!FUSED) {
            const int vo = u < tpw ? voff_x + (wave + u * GV_CW) * TILE_K : GV_OOB;
            a0[u] = __builtin_amdgcn_raw_buffer_load_b128(rx, vo, 0, 0);
            a1[u] = __builtin_amdgcn_raw_buffer_load_b128(rx, vo + 64, 0, 0);
        }
        p[0][u] = load_w(0, u);
    }
    if (!FUSED) {
#pragma unroll
        for (int d = 1; d < DR; ++d)
#pragma unroll
            for (int u = 0; u < AT; ++u) p[d][u] = load_w(d, u);
    }
    order_fence();
    write_records();

    // FUSED: the deeper ring rows are requested only now, into the registers the parameter staging held
    if (FUSED) {
        order_fence();
#pragma unroll
        for (int d = 1; d < DR; ++d)
#pragma unroll
            for (int u = 0; u < AT; ++u) p[d][u] = load_w(d, u);
        order_fence();
    }
    lds_barrier();   // the records (and the reciprocal scales) are complete

    // eight elements of one 16-byte piece, widened exactly and scaled: t = x * (1 / s)
    auto scaled8 = [&](const v4u &raw, const float *rk, float (&t)[8]) __attribute__((always_inline)) {
        const v4f r0 = *reinterpret_cast<const v4f *>(rk);
        const v4f r1 = *reinterpret_cast<const v4f *>(rk + 4);
        const uint32_t wd[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float lo, hi;
            // (fp16 only: with a run-time choice between two widenings inside this loop the compiler
            // keeps both variants' operands alive and every instance beyond one k-tile per wave spills)
            lo = __half2float(__ushort_as_half((uint16_t)(wd[i] & 0xffffu)));
            hi = __half2float(__ushort_as_half((uint16_t)(wd[i] >> 16)));
            const float ra = i < 2 ? r0[2 * i] : r1[2 * i - 4];
            const float rb = i < 2 ? r0[2 * i + 1] : r1[2 * i - 3];
            // (x * r + 0: the same single rounding of the exact product as x * r -- only the sign of a zero
            // can differ, which neither the maximum nor the code sees --, but the widening folds into it:
            // one mixed-precision multiply-add instead of a conversion and a multiply)
            t[2 * i] = __builtin_fmaf(lo, ra, 0.0f);
            t[2 * i + 1] = __builtin_fmaf(hi, rb, 0.0f);
        }
    };
    float q_inv = 0.f;   // 127 / (row maximum), 0 for an all-zero row
    // slot u: raw pieces -> int8 fragments.  rne and the conversion are one addition: y + 1.5 * 2^23
    // holds rne(y) in its low bits (|y| <= 127 (1 + 2^-23): the clamp of the definition never acts).
    // The product y = t * (127 / a) is rounded to binary32 BEFORE that addition, as in the definition:
    // fused into one multiply-add, a product just below a tie (x = a / 2 gives 63.5 - eps for about half
    // of all a) would round down where the definition's rounded product, the tie itself, goes to even.
    auto quantize_slot = [&](int u) __attribute__((always_inline)) {
#pragma clang fp contract(off)
        const float *rk = r_lds + (wave + u * GV_CW) * TILE_K + xcol;
        uint32_t o[8];
#pragma unroll
        for (int pc = 0; pc < 4; ++pc) {
            float t[8];
            // (slots without a k-tile hold zeros; their reciprocals are read from the last k-tile's place)
            scaled8(xr[u][pc], (u < tpw ? rk : r_lds) + (pc >> 1) * 64 + (pc & 1) * 8, t);
            uint32_t b[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float yq = t[i] * q_inv;
                asm volatile("" : "+v"(yq));   // (belt and braces: the rounded product is a value of its own)
                b[i] = __float_as_uint(yq + 12582912.0f);
            }
            o[2 * pc] = __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u) | __builtin_amdgcn_perm(b[3], b[2], 0x04000c0cu);
            o[2 * pc + 1] = __builtin_amdgcn_perm(b[5], b[4], 0x0c0c0400u) | __builtin_amdgcn_perm(b[7], b[6], 0x04000c0cu);
            __builtin_amdgcn_sched_barrier(0);   // (piece by piece, as above)
        }
        a0[u] = v4u{o[0], o[1], o[2], o[3]};
        a1[u] = v4u{o[4], o[5], o[6], o[7]};
        if (a.Xq_out != nullptr && blk == 0 && u < tpw && (lane >> 2) < M) {   // test hook
            int8_t *qo = a.Xq_out + (int64_t)(lane >> 2) * K + (wave + u * GV_CW) * TILE_K + xcol;
            *reinterpret_cast<v4u *>(qo) = a0[u];
            *reinterpret_cast<v4u *>(qo + 64) = a1[u];
        }
    };
    if (FUSED) {
        float am = 0.f;
#pragma unroll
        for (int u = 0; u < AT; ++u) {
            const float *rk = r_lds + (wave + u * GV_CW) * TILE_K + xcol;
#pragma unroll
            for (int pc = 0; pc < 4; ++pc) {
                float t[8];
                scaled8(xr[u][pc], (u < tpw ? rk : r_lds) + (pc >> 1) * 64 + (pc & 1) * 8, t);
#pragma unroll
                for (int i = 0; i < 8; i += 2) am = fmaxf(fmaxf(am, fabsf(t[i])), fabsf(t[i + 1]));
                // (piece by piece: scheduled freely, all reciprocals are read and all pieces widened
                // up front -- some 80 registers per slot -- and the wave spills)
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // (the rounding pass widens the raw pieces again: kept widened from here they would be 32
        // registers per slot)
#pragma unroll
        for (int u = 0; u < AT; ++u)
            asm volatile("" : "+v"(xr[u][0]), "+v"(xr[u][1]), "+v"(xr[u][2]), "+v"(xr[u][3]));
        // the row's four lanes, then the eight waves through LDS
        am = fmaxf(am, dpp_f32<DPP_QUAD_XOR1>(am));
        am = fmaxf(am, dpp_f32<DPP_QUAD_XOR2>(am));
        float *mx = r_lds + K;
        if ((lane & 3) == 0) mx[wave * 16 + (lane >> 2)] = am;
        lds_barrier();   // the row maxima are complete
        float arow = 0.f;
#pragma unroll
        for (int w = 0; w < GV_CW; ++w) arow = fmaxf(arow, mx[w * 16 + (lane >> 2)]);
        q_inv = 127.0f / arow;
        if (!(q_inv <= 3.402823466e+38f)) q_inv = 0.f;   // all-zero token, or one so small that 127 / a overflows
    }

    // fragments -> operand layout: lane (ln, kb) takes bytes kb*32 .. +32 of row ln, i.e. the
    // 16-byte pieces 2 (kb % 2) and 2 (kb % 2) + 1 that lanes 4 ln + .. loaded, from the first
    // (kb < 2) or second half-row load.  LDS executes a wave's accesses in order, so the two 1 KB
    // staging rows are reused from slot to slot without further synchronization.  A workgroup
    // with a single n-tile does this slot by slot, so that its first tiles are computed while
    // the later fragments are still on their way (inside the ring loop the extra branch costs
    // more than it hides).
    uint8_t *stg0 = reinterpret_cast<uint8_t *>(red + wave * 256);
    uint8_t *stg1 = reinterpret_cast<uint8_t *>(red + (GV_CW + wave) * 256);
    const uint8_t *stg_src = ((kb & 2) ? stg1 : stg0) + (4 * ln + 2 * (kb & 1)) * 16;
    auto to_operand_layout = [&](int u) __attribute__((always_inline)) {
        *reinterpret_cast<v4u *>(stg0 + lane * 16) = a0[u];
        *reinterpret_cast<v4u *>(stg1 + lane * 16) = a1[u];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        a0[u] = *reinterpret_cast<const v4u *>(stg_src);
        a1[u] = *reinterpret_cast<const v4u *>(stg_src + 16);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    if (D != 0) {
#pragma unroll
        for (int u = 0; u < AT; ++u) {
            if (FUSED) quantize_slot(u);
            to_operand_layout(u);
        }
    }

    const v4i zero4 = {0, 0, 0, 0};
    v4i acc = zero4;
    v4f y = {0.f, 0.f, 0.f, 0.f};
    v4u r = load_rec(0, 0);
    int nzx[4] = {0, 0, 0, 0};   // minus the zero-points of this lane's tokens m = 4 kb + rr
    if (ASYM && GROUPED) {
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) nzx[rr] = 4 * kb + rr < M ? -a.zx[4 * kb + rr] : 0;
    }
    // one n-tile: consume ring row d, optionally refilling it for n-tile j + D
    auto step_ntile = [&](int j, int d, bool refill) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < AT; ++u) {
            if (D == 0) {
                if (FUSED) quantize_slot(u);
                to_operand_layout(u);
            }
            // the record of the next slot is fetched one slot ahead
            v4u rn = r;
            if (u + 1 < AT) {
                if (GROUPED) rn = load_rec(j, u + 1);
            } else {
                rn = load_rec(j + 1, 0);
            }
            const DecodeLut lut = {r.x, r.y, 0};
            const int nb = (int)__builtin_amdgcn_perm(r.w, r.w, 0u);   // byte 0 replicated
            const v4i negb = {nb, nb, nb, nb};
            const v4i c0 = as_v4i(a0[u]), c1 = as_v4i(a1[u]);
            const bool live = u < tpw;   // uniform over the wave
            // D[i][j] = sum_k A[i][k] B[k][j]: rows i = tokens, columns j = output channels.
            // sum Xq 4(d + beta) - 4 beta sum Xq = 4 sum Xq d, exact in int32: the bias goes
            // first (it needs no weights), then each half of the tile as soon as it is decoded.
            v4i w1 = zero4;
            if (live) {
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(c0, negb, GROUPED ? zero4 : acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(c1, negb, acc, 0, 0, 0);
                v4i w0;
                int x0, x1;
                decode_word(p[d][u].x, lut, x0, x1); w0.x = x0; w0.y = x1;
                decode_word(p[d][u].y, lut, x0, x1); w0.z = x0; w0.w = x1;
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(c0, w0, acc, 0, 0, 0);
                decode_word(p[d][u].z, lut, x0, x1); w1.x = x0; w1.y = x1;
                decode_word(p[d][u].w, lut, x0, x1); w1.z = x0; w1.w = x1;
            }
            // Refill the slot with the same k-tile of the n-tile D further on.  The load comes
            // after the last read of the old contents, so it can land in the same registers and
            // the ring needs no copies (which would have to wait for the data to arrive).
            order_fence();
            if (refill) p[d][u] = load_w(j + DR, u);
            order_fence();
            if (live) acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(c1, w1, acc, 0, 0, 0);
            if (GROUPED && live) {
                const float es = __uint_as_float(r.z);
                if (ASYM) {
                    const int t4 = (int)r.w >> 8;   // 4 * (sum of the tile's weights)
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr)
                        y[rr] = __builtin_fmaf(es, (float)(acc[rr] + __mul24(nzx[rr], t4)), y[rr]);
                } else {
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) y[rr] = __builtin_fmaf(es, (float)acc[rr], y[rr]);
                }
                if (ACC_OUT) {
                    const int g = (kt_begin + wave + u * GV_CW) / a.tiles_per_group;
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        const int m = 4 * kb + rr;
                        if (m < M)
                            atomicAdd(&a.acc_out[((int64_t)m * N + nt_of(j) * TILE_N + ln) * a.ng + g],
                                      acc[rr] >> 2);
                    }
                }
            }
            if (!GROUPED && u == AT - 1) {
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) y[rr] = __int_as_float(acc[rr]);   // summed exactly by the helper
                if (ACC_OUT && tpw > 0) {
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        const int m = 4 * kb + rr;
                        if (m < M)
                            atomicAdd(&a.acc_out[(int64_t)m * N + nt_of(j) * TILE_N + ln], acc[rr] >> 2);
                    }
                }
                acc = zero4;
            }
            r = rn;
            order_fence();   // keeps the unrolled slots from being interleaved
        }
        // accumulator layout: lane holds tokens m = 4 kb + rr of output channel ln
        float *rb = red + ((j & 1) * GV_CW + wave) * 256;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            rb[(4 * kb + rr) * 16 + ln] = y[rr];
            y[rr] = 0.f;
        }
        lds_barrier();
    };

    // whole rounds of D n-tiles with refill (loads past the last n-tile go out of range), then
    // the last my_nt % D n-tiles, which only consume
    if (D == 0) {
        step_ntile(0, 0, false);
        return;
    }
    int j0 = 0;
    for (; j0 + DR <= my_nt; j0 += DR) {
#pragma unroll
        for (int d = 0; d < DR; ++d) step_ntile(j0 + d, d, true);
    }
#pragma unroll
    for (int d = 0; d < DR - 1; ++d)
        if (j0 + d < my_nt) step_ntile(j0 + d, d, false);
}

// Y[m,n] = cast(sx[m] * sum_s partial[s,m,n]), fixed order over the K-splits.  int_step != null:
// the partials are the int32 accumulators (times 4) of a per-channel launch; their exact sum,
// minus the zero-point term when zx is given, is scaled by int_step[n] / 8.
__global__ __launch_bounds__(256) void gemv_combine_kernel(const float *__restrict__ partial,
                                                           const float *__restrict__ sx,
                                                           const float *__restrict__ int_step,
                                                           const int32_t *__restrict__ zx,
                                                           const int32_t *__restrict__ wsum, int M,
                                                           int N, int splits, uint16_t *__restrict__ Y,
                                                           int y_dtype, int64_t ldy)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)M * N) return;
    const int m = (int)(i / N), n = (int)(i - (int64_t)m * N);
    float sum = 0.f;
    if (int_step != nullptr) {
        int isum = 0;
        for (int s = 0; s < splits; ++s) isum += __float_as_int(partial[(int64_t)s * M * N + i]);
        if (zx != nullptr) isum -= 4 * zx[m] * wsum[n];
        sum = (int_step[n] * 0.125f) * (float)isum;
    } else {
        for (int s = 0; s < splits; ++s) sum += partial[(int64_t)s * M * N + i];
    }
    float out = sx[m] * sum;   // binary32 product, then the cast (see gemv_kernel)
    asm volatile("" : "+v"(out));
    Y[(int64_t)m * ldy + n] = (y_dtype == W4A8_F16) ? f32_to_f16_bits(out) : f32_to_bf16_bits(out);
}

GemvPlan plan_gemv(int64_t M, int64_t N, int64_t K, int64_t G, int64_t batch)
{
    GemvPlan pl{};
    const int KT = (int)(K / TILE_K), NT = (int)(N / TILE_N);
    if (KT < 1 || NT < 1 || batch < 1) return pl;   // nothing to launch (callers check shapes first)
    // group-wise weights keep at most 5 k-tiles per wave: their decode records (one per channel and
    // k-tile) would otherwise leave room for too few n-tiles per workgroup in LDS
    const int max_at = (G != K) ? 5 : GV_MAX_AT;
    pl.splits = (KT + GV_CW * max_at - 1) / (GV_CW * max_at);
    pl.kt_per_split = (KT + pl.splits - 1) / pl.splits;
    pl.splits = (KT + pl.kt_per_split - 1) / pl.kt_per_split;
    const int tpw = (pl.kt_per_split + GV_CW - 1) / GV_CW;
    pl.at = tpw;   // 1 .. GV_MAX_AT
    const bool grouped = G != K;
    // about one workgroup per CU, n-tiles dealt out evenly (more, shorter-lived workgroups
    // measured slower: each one reloads its activation fragments)
    int bps = (int)(256 / (pl.splits * batch));   // batched: the 256 CUs are shared by all problems
    if (bps < 1) bps = 1;
    if (bps > NT) bps = NT;
    int q = (NT + bps - 1) / bps;   // most n-tiles any workgroup gets
    const int recs = grouped ? pl.kt_per_split : 1;
    const int rs = grouped ? (pl.kt_per_split | 1) : 1;
    const int q_lds = GV_LDS_BUDGET / (rs * 16 * 16);
    const int q_stage = GV_STAGE * GV_REC_THREADS / (recs * 16);
    const int q_cap = q_lds < q_stage ? q_lds : q_stage;
    if (q > q_cap) {
        // more than 256 workgroups: whole generations of them, all equally long (a short last
        // generation still costs a workgroup's whole lifetime)
        const int per = (int)(pl.splits * batch);
        const int at_cap = (NT + q_cap - 1) / q_cap * per;
        const int gens = (at_cap + 255) / 256;
        bps = 256 * gens / per;
        if (bps < (NT + q_cap - 1) / q_cap) bps = (NT + q_cap - 1) / q_cap;
        if (bps > NT) bps = NT;
        q = (NT + bps - 1) / bps;
    }
    pl.q = q;
    pl.blocks_per_split = bps;
    pl.nt_lo = NT / bps;
    pl.nt_rem = NT % bps;
    pl.lds_bytes = GV_RED_BYTES + q * rs * 16 * 16;
    pl.partial_bytes = pl.splits > 1 ? (size_t)pl.splits * M * N * sizeof(float) : 0;
    return pl;
}

template <bool GROUPED, bool ACC_OUT, bool ASYM, bool FUSED = false>
static int launch_gemv_at(const GemvPlan &pl, const GemvArgs &ga, int batch, hipStream_t st)
{
    const dim3 grid((unsigned)pl.blocks_per_split, (unsigned)pl.splits, (unsigned)batch);
    // FUSED: the reciprocal scales [K] and the waves' row maxima [8][16] follow the decode records
    const int lds_bytes = pl.lds_bytes + (FUSED ? ga.K * 4 + GV_CW * 16 * 4 : 0);
    // more than 64 KB of dynamic LDS has to be opted into, once per instance and device
#define W4A8_GV_LAUNCH(AT_, D_)                                                                  \
    do {                                                                                         \
        static std::atomic<uint64_t> lds_opted{0};                                               \
        if (lds_bytes > 64 * 1024 &&                                                             \
            opt_in_dynamic_lds((const void *)gemv_kernel<GROUPED, AT_, D_, ACC_OUT, ASYM, FUSED>, \
                               GV_LDS_LIMIT, lds_opted) != W4A8_OK)                              \
            return W4A8_ERR_HIP;                                                                 \
        hipLaunchKernelGGL((gemv_kernel<GROUPED, AT_, D_, ACC_OUT, ASYM, FUSED>), grid,          \
                           dim3(GV_THREADS), lds_bytes, st, ga);                                 \
    } while (0)
    // ring depth: 8 - 10 KB per wave in flight, within the register budget of 9 waves per CU;
    // no ring when every workgroup has a single n-tile (the accumulator hook keeps the ring form)
#define W4A8_GV_CASE(AT_, D_)                                 \
    case AT_:                                                 \
        if (pl.q == 1 && !ACC_OUT) W4A8_GV_LAUNCH(AT_, 0);    \
        else W4A8_GV_LAUNCH(AT_, D_);                         \
        break
    switch (pl.at) {
        W4A8_GV_CASE(1, 4);
        W4A8_GV_CASE(2, 4);
        W4A8_GV_CASE(3, 3);
        W4A8_GV_CASE(4, 2);
        W4A8_GV_CASE(5, 2);
        default:
            // 6 .. 9 k-tiles per wave: per-channel weights only (see plan_gemv)
            if constexpr (!GROUPED) {
                switch (pl.at) {
                    W4A8_GV_CASE(6, 1);
                    W4A8_GV_CASE(7, 1);
                    default:
                        if constexpr (!FUSED) {
                            switch (pl.at) {
                                W4A8_GV_CASE(8, 1);
                                W4A8_GV_CASE(9, 1);
                                default: return W4A8_ERR_SHAPE;
                            }
                        } else {
                            return W4A8_ERR_SHAPE;
                        }
                        break;
                }
            } else {
                return W4A8_ERR_SHAPE;
            }
            break;
    }
#undef W4A8_GV_CASE
#undef W4A8_GV_LAUNCH
    return hip_status(hipGetLastError());
}

int gemv_token_blocks(int64_t M, int64_t N, int64_t K, int64_t G)
{
    // Measured against the tile kernel: up to four blocks win on every layer shape tried (C2 at 32
    // tokens 16 -> 7 us, 13824 x 5120 group-128 at 64 tokens 46 -> 31 us), five to eight blocks only
    // on smaller layers (5120 x 5120 at 128 tokens: 27 -> 20 us); each block streams the weights again.
    if (M <= 16 || M > 128 || N <= 0) return 0;
    if (M > 64 && N * K > 48LL * (1 << 20)) return 0;
    // (weights beyond the last-level cache's reach are re-streamed from memory by every block:
    // 36864 x 9216 at 64 tokens 87 us in four blocks against 58 us on the tile kernel)
    if (M > 32 && N * K > 128LL * (1 << 20)) return 0;
    const int nb = (int)((M + 15) / 16);
    // the decode records cap the n-tiles per workgroup: not more than two generations of workgroups
    // (one for more than four blocks)
    const GemvPlan pl = plan_gemv(16, N, K, G, nb);
    if ((int64_t)pl.blocks_per_split * pl.splits * nb > (nb > 4 ? 256 : 512)) return 0;
    return nb;
}

bool gemv_can_fuse(int64_t M, int64_t N, int64_t K, int64_t G)
{
    if (M < 1 || M > 16 || N < TILE_N || K < TILE_K) return false;
    const GemvPlan pl = plan_gemv(M, N, K, G, 1);
    // (8 and 9 k-tiles per wave would spill: 16 registers of raw activations per k-tile)
    const int recs = (G != K) ? pl.kt_per_split : 1;   // decode records per channel
    return pl.splits == 1 && pl.at <= GV_FUSED_MAX_AT && pl.q * 16 * recs <= GV_FUSED_STAGE * GV_REC_THREADS &&
           pl.lds_bytes + (int)K * 4 + GV_CW * 16 * 4 <= GV_LDS_LIMIT;
}

int launch_gemv(const int8_t *Xq, const float *sx, ZeroPoint zp, int64_t M, const uint8_t *Wt,
                const float *step, const uint8_t *zero, int64_t N, int64_t K, int64_t G, void *Y,
                int y_dtype, int64_t ldy, int32_t *acc_out, float *partial, int64_t batch,
                hipStream_t st, int plain, const FusedAct *fused)
{
    if (fused != nullptr && (batch != 1 || zp.zx != nullptr || !gemv_can_fuse(M, N, K, G))) return W4A8_ERR_SHAPE;
    // 16 < M <= 128 where gemv_token_blocks says so: one launch over the 16-token blocks (batch must be 1)
    const int token_blocks = M > 16 ? gemv_token_blocks(M, N, K, G) : 0;
    if (M > 16 && (token_blocks == 0 || batch != 1)) return W4A8_ERR_SHAPE;
    if (token_blocks) batch = token_blocks;
    const GemvPlan pl = plan_gemv(token_blocks ? 16 : M, N, K, G, batch);
    if (batch > 1 && !token_blocks && (pl.splits > 1 || acc_out != nullptr)) return W4A8_ERR_SHAPE;
    const bool grouped = G != K;
    float *part = pl.splits > 1 ? partial : nullptr;
    GemvArgs ga;
    ga.Xq = Xq; ga.sx = sx; ga.zx = zp.zx; ga.wsum = zp.wsum; ga.tsum = zp.tsum; ga.Wt = Wt;
    ga.step = step; ga.zero = zero;
    ga.Y = (uint16_t *)Y; ga.partial = part; ga.acc_out = acc_out; ga.ldy = ldy;
    ga.M = (int)M; ga.N = (int)N; ga.K = (int)K;
    ga.tiles_per_group = (int)(G / TILE_K); ga.ng = (int)(K / G); ga.y_dtype = y_dtype;
    ga.kt_per_split = pl.kt_per_split; ga.nt_lo = pl.nt_lo; ga.nt_rem = pl.nt_rem;
    ga.nt_stride = pl.blocks_per_split;
    ga.token_blocks = token_blocks;
    ga.part_rows = (int)M;
    ga.plain = plain;
    ga.vec_store = ((uintptr_t)Y % 8 == 0) && (ldy % 4 == 0);
    ga.X = nullptr; ga.s = nullptr; ga.ldx = 0; ga.Xq_out = nullptr; ga.sx_out = nullptr;
    ga.fused_lds_off = pl.lds_bytes;
    const bool asym = zp.zx != nullptr;
    int rc;
    if (fused != nullptr) {
        ga.X = fused->X; ga.s = fused->s; ga.ldx = fused->ldx;
        ga.Xq_out = fused->Xq_out; ga.sx_out = fused->sx_out;
        if (grouped) {
            if (acc_out) rc = launch_gemv_at<true, true, false, true>(pl, ga, 1, st);
            else rc = launch_gemv_at<true, false, false, true>(pl, ga, 1, st);
        } else {
            if (acc_out) rc = launch_gemv_at<false, true, false, true>(pl, ga, 1, st);
            else rc = launch_gemv_at<false, false, false, true>(pl, ga, 1, st);
        }
        return rc;
    }
    if (grouped) {
        // the per-tile zero-point term only exists in its own instances (asymmetric, grouped)
        if (asym) {
            if (acc_out) rc = launch_gemv_at<true, true, true>(pl, ga, (int)batch, st);
            else rc = launch_gemv_at<true, false, true>(pl, ga, (int)batch, st);
        } else {
            if (acc_out) rc = launch_gemv_at<true, true, false>(pl, ga, (int)batch, st);
            else rc = launch_gemv_at<true, false, false>(pl, ga, (int)batch, st);
        }
    } else {
        if (asym) {
            if (acc_out) rc = launch_gemv_at<false, true, true>(pl, ga, (int)batch, st);
            else rc = launch_gemv_at<false, false, true>(pl, ga, (int)batch, st);
        } else {
            if (acc_out) rc = launch_gemv_at<false, true, false>(pl, ga, (int)batch, st);
            else rc = launch_gemv_at<false, false, false>(pl, ga, (int)batch, st);
        }
    }
    if (rc != W4A8_OK || pl.splits == 1) return rc;
    return launch_gemv_combine(part, sx, grouped ? nullptr : step, zp, M, N, pl.splits, Y, y_dtype,
                               ldy, st);
}

int launch_gemv_combine(const float *partial, const float *sx, const float *int_step, ZeroPoint zp,
                        int64_t M, int64_t N, int splits, void *Y, int y_dtype, int64_t ldy,
                        hipStream_t st)
{
    const int64_t outs = M * N;
    hipLaunchKernelGGL(gemv_combine_kernel, dim3((unsigned)((outs + 255) / 256)), dim3(256), 0, st,
                       partial, sx, int_step, int_step ? zp.zx : nullptr, zp.wsum, (int)M, (int)N,
                       splits, (uint16_t *)Y, y_dtype, ldy);
    return hip_status(hipGetLastError());
}

}  // namespace w4a8
