// dINT4 x INT8 GEMM, prefill shape (M > 16): a compute-bound tile kernel on the int8 matrix cores
// (Eq. 1 product on the integer operands with int32 accumulation; Eq. 5 second half fused as the
// dequantizing epilogue; the dINT4 x INT8 multiply-accumulate of Sec. 4.3).
//
// v_mfma_i32_32x32x32_i8 is the instruction to build on: measured on MI355X it sustains ~4.5 POPS,
// twice what v_mfma_i32_16x16x64_i8 reaches.  A workgroup of WM x 4 wavefronts (WM = 1 or 2)
// computes a BM x 256 output tile; a wave owns BM / WM token rows of 64 output channels (two
// 32-channel sub-tiles).  Packed weights never touch LDS: per 128 columns of K a wave reads the
// 4 KB of its 64 channels straight from global memory (16-byte buffer loads, issued two k-tiles
// ahead), turns the nibbles into int8 through the per-channel register LUT and reuses each
// decoded operand for all its 32-token sub-tiles.  The int8 activations are shared by the waves
// through a ring of four LDS tiles that are filled global -> LDS directly (buffer_load ... lds, no
// staging registers, no ds_write), three k-tiles ahead of the MFMAs; their 16-byte chunks are
// XOR-swizzled by row pair -- on the global side, since a wave's copy lands in lane order -- so that
// the ds_read_b128 operand reads are conflict free on the 64-bank LDS.  One barrier per k-tile; the
// operands of the first k-step of the next tile are fetched before it.
//
// Per-channel weights use the biased decode (7 operations per 8 weights); the bias is removed once,
// in the epilogue, with per-token row-sums from a small pre-pass.  Group-wise weights must rescale
// every accumulator once per group, so they use the signed decode (no bias term) and keep fp32
// running sums next to the int32 group accumulators (BM <= 128); the group's (step, zero) pairs
// reach the waves through LDS, fetched three groups ahead.
//
// When the output has too few tiles to occupy 256 CUs (mid-size M) K is cut into ranges as well:
// each workgroup writes an fp32 partial of its range and a small kernel adds the ranges in a fixed
// order, applies the token scale and casts (deterministic; the int32 hook uses exact atomic adds).
#include <algorithm>
#include <type_traits>

#include "w4a8_common.hpp"

namespace w4a8 {

typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int GM_BN = 256;  // output channels per workgroup
constexpr int GM_OOB = 0x7fff0000;
constexpr int GM_RING = 4;  // activation tiles in LDS
constexpr int GM_PANEL = 4; // token tiles per panel of the tile numbering

// Pins the program order of memory instructions and of everything scheduled around them, at every
// level of the compiler (emits no instruction).
__device__ __forceinline__ void gm_order_fence()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// Global -> LDS copy that bypasses the registers: lane l of the wave writes its 16 bytes to
// lds_addr + 16 l (lds_addr: byte address in LDS, wave-uniform); addresses beyond the buffer
// write zeros.  Completion is counted by vmcnt like any buffer load, but the compiler does not
// know that this one writes LDS: whoever reads the bytes waits for vmcnt and a barrier first.
__device__ __forceinline__ void dma_b128(v4i rsrc, int voff, int soff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, %2 offen lds"
                 :: "v"(voff), "s"(rsrc), "s"(soff), "s"(lds_addr) : "memory");
}

// Copies issued by dma_b128 are invisible to the compiler's own wait insertion: wait_copies<Y>()
// returns once at most Y accesses issued after the copies in question are outstanding (vmcnt
// retires in issue order), and must be followed by a barrier before other waves read the tile.
template <int YOUNGER>
__device__ __forceinline__ void wait_copies()
{
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(YOUNGER) : "memory");
}
// A use of every register of p (emits nothing): the compiler completes all the loads into p here,
// with one wait, instead of piecemeal in front of later uses -- a later wait of its own could only
// allow fewer accesses in flight, and it does not know of the LDS copies issued in between.
// (In / out operands: what is computed from p afterwards depends on this statement and stays behind it.)
__device__ __forceinline__ void use_all(v4u (&p)[2][2])
{
    asm volatile("" : "+v"(p[0][0]), "+v"(p[0][1]), "+v"(p[1][0]), "+v"(p[1][1]));
}
__device__ __forceinline__ void use_all(v4u (&p)[1][2])
{
    asm volatile("" : "+v"(p[0][0]), "+v"(p[0][1]));
}
// keeps the computation of v in front of this point (emits nothing)
__device__ __forceinline__ void pin_value(v4i &v) { asm volatile("" : "+v"(v)); }

// ---- per-token row-sums of Xq over each K-range (bias removal of the per-channel path) ----------
__global__ __launch_bounds__(256) void rowsum_kernel(const int8_t *__restrict__ Xq, int64_t M, int K,
                                                     int splits, int k_per_split,
                                                     int32_t *__restrict__ rs)
{
    const int lane = threadIdx.x & 63;
    const int64_t seg = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);   // (split, token)
    if (seg >= M * splits) return;
    const int sp = (int)(seg / M);
    const int64_t m = seg - (int64_t)sp * M;
    const int k0 = sp * k_per_split;
    const int kn = min(k_per_split, K - k0);
    const v4i *x = reinterpret_cast<const v4i *>(Xq + m * K + k0);
    int sum = 0;
    for (int i = lane; i < kn / 16; i += WAVE) {
        const v4i v = x[i];
        sum = __builtin_amdgcn_sdot4(v.x, 0x01010101, sum, false);
        sum = __builtin_amdgcn_sdot4(v.y, 0x01010101, sum, false);
        sum = __builtin_amdgcn_sdot4(v.z, 0x01010101, sum, false);
        sum = __builtin_amdgcn_sdot4(v.w, 0x01010101, sum, false);
    }
    sum = wave_sum_i32(sum);
    if (lane == 0) rs[seg] = sum;
}

// ---- the tile kernel ------------------------------------------------------------------------
// WM wave rows x WN wave columns (8 waves for BM >= 128: every SIMD hosts two, so one wave's
// MFMAs cover the other's LDS and decode latency); a wave owns BM / WM token rows of 256 / WN output
// channels.  WN = 4 (64 channels per wave) suits the per-channel kernel; group-wise weights take
// 128 tokens x 32 channels per wave: every decoded weight then feeds twice as many MFMAs, and
// instruction issue -- decode plus the per-group rescale -- is what bounds them.  BN is the tile's
// width in channels: 256, or 128 for the group-wise 128-token tile (WM = 1, WN = 4, two workgroups
// per CU that share no barrier).
// Token zero-points zx (asymmetric activations; codes and zx stored offset by -128): the exact
// term zx * (sum of the weights) leaves the int32 accumulators before any floating-point step --
// per group in the flush (GROUPED; its own instances, ASYM) or once in the epilogue (!GROUPED,
// decided at run time by zx != null).
template <int BM, int WM, int WN, bool GROUPED, bool ACC_OUT, bool ASYM, bool TWO, int BN>
__global__ __launch_bounds__(WM * WN * 64, TWO ? 4 : (BN < GM_BN ? 2 : 1)) void gemm_kernel(
    const int8_t *__restrict__ Xq, const float *__restrict__ sx, const int32_t *__restrict__ zx,
    const int32_t *__restrict__ wsum, const int32_t *__restrict__ tsum,
    const int32_t *__restrict__ rs, int M,
    const uint8_t *__restrict__ Wt, const float *__restrict__ step,
    const uint8_t *__restrict__ zero, int N, int K, int tiles_per_group, int ng,
    uint16_t *__restrict__ Y, int y_dtype, int64_t ldy, int vec_store,
    int32_t *__restrict__ acc_out, int grid_m, int grid_n, int kt_per_split,
    float *__restrict__ partial, int plain, int acc_ld)
{
    // (acc_ld: channels per token row of acc_out -- N, or the whole layer's when this launch covers a
    // range of its channels)
    constexpr int GM_THREADS = WM * WN * 64;
    constexpr int GM_NS = BN / (WN * 32);       // 32-channel sub-tiles per wave
    constexpr int WROWS = BM / WM;                 // token rows per wave
    constexpr int MS = WROWS / 32;                 // 32-token sub-tiles per wave
    constexpr int NW = WM * WN;                    // waves
    constexpr int LD_ITERS = BM * 8 / GM_THREADS;  // 16-byte chunks of the A tile per thread
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
    uint8_t(*lds)[BM * TILE_K] = reinterpret_cast<uint8_t(*)[BM * TILE_K]>(lds_raw);   // [GM_RING][BM * 128]
    // group-wise weights: step / 8 and zero-point of the workgroup's 256 channels, a ring of four groups
    __shared__ __attribute__((aligned(16))) float s_ges[GROUPED ? 4 : 1][GROUPED ? BN : 4];
    __shared__ int s_gz[GROUPED ? 4 : 1][GROUPED ? BN : 4];
    __shared__ __attribute__((aligned(16))) int s_gw[GROUPED && ASYM ? 4 : 1][GROUPED && ASYM ? BN : 4];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r32 = lane & 31;   // operand row: output channel (weights) / token (activations)
    const int kh = lane >> 5;    // which 16 of a k-step's 32 input channels this lane holds
    const int KT = K / TILE_K;

    // Workgroups are handed to the 8 XCDs round-robin; renumber so that each XCD works on a
    // contiguous range of tiles and its private L2 sees the reuse.
    // With few output tiles K is also split over workgroups (each writes an fp32 partial).
    const int tiles = grid_m * grid_n;
    const int split = blockIdx.x / tiles;
    const int kt0 = split * kt_per_split;              // first k-tile of this workgroup
    const int KTl = min(kt_per_split, KT - kt0);       // its number of k-tiles
    int bid = blockIdx.x - split * tiles;
    {
        const int per = tiles / 8;
        if (bid < per * 8) bid = (bid & 7) * per + (bid >> 3);
    }
    // tiles are numbered down panels of GM_PANEL token tiles, channel tiles next: the 32 tiles an
    // XCD works on at a time then share their activations 8 ways and their weights 4 ways
    const int panel = bid / (GM_PANEL * grid_n);
    const int pr = bid - panel * (GM_PANEL * grid_n);
    const int ph = min(GM_PANEL, grid_m - panel * GM_PANEL);   // rows of this (possibly last, lower) panel
    const int bn = pr / ph;
    const int bm = panel * GM_PANEL + pr - bn * ph;
    const int m0 = bm * BM;
    const int nb0 = bn * BN;                        // first output channel of the workgroup
    const int wn = wave % WN;                          // wave column
    const int wr0 = (wave / WN) * WROWS;               // first token row of this wave within the tile
    const int n0 = nb0 + wn * (GM_NS * 32);            // first output channel of this wave

    __amdgpu_buffer_rsrc_t rw =
        __builtin_amdgcn_make_buffer_rsrc((void *)Wt, 0, (int)((int64_t)N * K / 2), 0x00020000);
    // the LDS copies take the descriptor of Xq as plain words (base, high bits with stride 0, bytes, flags)
    const uint64_t xq_addr = (uint64_t)Xq;
    const v4i rx = {(int)(uint32_t)xq_addr, (int)((xq_addr >> 32) & 0xffffu), (int)((int64_t)M * K),
                    0x00020000};

    // Weight operand of k-step s = 2 sp + h of a k-tile: MFMA lane (r32, kh) takes half h of the 16
    // bytes that lane (r32 % 16) + 16 (2 sp + kh) of tile (n / 16, kt) holds (w4a8.h), i.e. input
    // channels (2 sp + kh) * 32 + h * 16 + 0..15 of the tile.  One 16-byte load covers two k-steps.
    int wvoff[GM_NS];   // per-lane byte offset inside the wave's tile row (out of range if n >= N)
    int wsoff[GM_NS];   // byte offset of tile (n-subtile, kt = 0)
    bool ns_valid[GM_NS];
#pragma unroll
    for (int ns = 0; ns < GM_NS; ++ns) {
        const int nn = n0 + ns * 32;
        ns_valid[ns] = nn < N;
        const bool lane_ok = nn + r32 < N;
        wvoff[ns] = lane_ok ? (r32 >> 4) * KT * TILE_BYTES + ((r32 & 15) + 16 * kh) * 16 : GM_OOB;
        wsoff[ns] = ns_valid[ns] ? (nn / TILE_N) * KT * TILE_BYTES : 0;
    }

    v16i acc[MS][GM_NS];
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int ns = 0; ns < GM_NS; ++ns)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[ms][ns][r] = 0;

    constexpr int YS = GROUPED ? MS : 1;
    float y[YS][GM_NS][16];
#pragma unroll
    for (int ms = 0; ms < YS; ++ms)
#pragma unroll
        for (int ns = 0; ns < GM_NS; ++ns)
#pragma unroll
            for (int r = 0; r < 16; ++r) y[ms][ns][r] = 0.f;

    // A-tile staging: chunk c (16 bytes) of row r lives at r*128 + ((c ^ ((r >> 1) & 7)) * 16): with 64
    // LDS banks (256 B per clock) 16 consecutive rows x one chunk index cover all banks exactly once.
    // The tile goes global -> LDS directly: copy i of wave w fills the 1 KB block q = i * NW + w
    // (rows 8q .. 8q+7) in lane order, so lane l fetches, for row 8q + l/8 and physical chunk l%8,
    // the logical chunk that the swizzle puts there.  Rows >= M lie beyond the buffer: zeros.
    int avoff[LD_ITERS];
#pragma unroll
    for (int i = 0; i < LD_ITERS; ++i) {
        const int row = (i * NW + wave) * 8 + (lane >> 3);
        avoff[i] = (m0 + row) * K + (((lane & 7) ^ ((row >> 1) & 7)) << 4);
    }
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lds_raw;
    auto dma_a = [&](int kt, int buf) {
#pragma unroll
        for (int i = 0; i < LD_ITERS; ++i)
            dma_b128(rx, avoff[i], (kt0 + kt) * TILE_K,
                     lds_base + (uint32_t)(buf * (BM * TILE_K) + (i * NW + wave) * 1024));
    };

    v4u pa[GM_NS][2], pb[GM_NS][2];   // packed weights of two consecutive k-tiles (ping-pong)
    auto load_b = [&](int kt, v4u(&dst)[GM_NS][2]) {
#pragma unroll
        for (int ns = 0; ns < GM_NS; ++ns)
#pragma unroll
            for (int sp = 0; sp < 2; ++sp)
                dst[ns][sp] = __builtin_amdgcn_raw_buffer_load_b128(
                    rw, wvoff[ns] + sp * 512, wsoff[ns] + (kt0 + kt) * TILE_BYTES, 0);
    };

    // per-lane decode tables of its two output channels
    DecodeLut lut[GM_NS];
    SignedLut slut[GM_NS];
    auto load_luts = [&](int g) {
#pragma unroll
        for (int ns = 0; ns < GM_NS; ++ns) {
            if (GROUPED) {
                slut[ns] = make_signed_lut(s_gz[g & 3][wn * (GM_NS * 32) + ns * 32 + r32], plain != 0);
            } else {
                const int nn = (n0 + ns * 32 + r32 < N) ? n0 + ns * 32 + r32 : 0;
                lut[ns] = make_decode_lut(zero[(int64_t)nn * ng], plain != 0);
            }
        }
    };
    // group parameters of channel nb0 + tid (threads 0..255), fetched one group ahead
    float gp_es = 0.f;
    int gp_z = 0, gp_w = 0;
    auto fetch_group = [&](int g) {
        if (tid < BN) {
            const int nn = nb0 + tid < N ? nb0 + tid : 0;
            gp_es = step[(int64_t)nn * ng + g] * 0.125f;
            gp_z = zero[(int64_t)nn * ng + g];
            if (ASYM) gp_w = 4 * wsum[(int64_t)nn * ng + g];
        }
    };
    auto publish_group = [&](int g) {
        if (tid < BN) {
            s_ges[g & 3][tid] = gp_es;
            s_gz[g & 3][tid] = gp_z;
            if (ASYM) s_gw[g & 3][tid] = gp_w;
        }
    };
    int nzx[MS];   // minus the zero-point of this lane's token in each sub-tile (GROUPED && ASYM)
#pragma unroll
    for (int ms = 0; ms < MS; ++ms) {
        const int m = m0 + wr0 + ms * 32 + r32;
        nzx[ms] = (GROUPED && ASYM && m < M) ? -zx[m] : 0;
    }

    // Accumulator layout (32x32): lane holds token m = 32 ms + r32 and the 16 output channels
    // n = n0 + 32 ns + 8 (r / 4) + 4 kh + (r % 4), r = 0..15.
    auto flush_group = [&](int g) {   // GROUPED only: y += (step / 8) * acc, acc = 0
#pragma unroll
        for (int ns = 0; ns < GM_NS; ++ns) {
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int nl = wn * (GM_NS * 32) + ns * 32 + 8 * b + 4 * kh;
                const v4f es = *reinterpret_cast<const v4f *>(&s_ges[g & 3][nl]);
                v4i gw = {0, 0, 0, 0};   // 4 * (sum of the group's weights), |.| < 2^23
                if (ASYM) gw = *reinterpret_cast<const v4i *>(&s_gw[g & 3][nl]);
#pragma unroll
                for (int ms = 0; ms < MS; ++ms) {
                    const int m = m0 + wr0 + ms * 32 + r32;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int v = acc[ms][ns][4 * b + r];
                        const int vz = ASYM ? v + __mul24(nzx[ms], gw[r]) : v;
                        // (an explicit fused multiply-add: left to contraction, instances of this
                        // kernel could round the running sum differently)
                        float &yr = y[GROUPED ? ms : 0][ns][4 * b + r];
                        yr = __builtin_fmaf(es[r], (float)vz, yr);
                        if (ACC_OUT && m < M) {
                            const int nn = nb0 + nl + r;
                            if (nn < N) acc_out[((int64_t)m * acc_ld + nn) * ng + g] = v >> 2;
                        }
                    }
                }
            }
        }
    };

    // activation fragments of k-step s = 2 sp + h: 16-byte chunk 2 (2 sp + kh) + h of the token's row
    // (the swizzle term of a row does not depend on its 32-token block -- wr0 and 32 ms are multiples
    // of 16 rows --, so block and ring slot are plain offsets on four per-lane addresses instead of
    // sixteen)
    int frag_off[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int chunk = 2 * (2 * (s >> 1) + kh) + (s & 1);
        frag_off[s] = (wr0 + r32) * TILE_K + ((chunk ^ ((r32 >> 1) & 7)) << 4);
    }
    auto read_a = [&](int buf, int s, v4i(&dst)[MS]) {
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
            dst[ms] = *reinterpret_cast<const v4i *>(&lds_raw[buf * (BM * TILE_K) + ms * (32 * TILE_K) + frag_off[s]]);
    };
    auto decode_step = [&](const v4u(&pk)[GM_NS][2], int s, v4i(&dst)[GM_NS]) {
        const int sp = s >> 1, h = s & 1;
#pragma unroll
        for (int ns = 0; ns < GM_NS; ++ns) {
            const uint32_t q0 = h ? pk[ns][sp].z : pk[ns][sp].x;
            const uint32_t q1 = h ? pk[ns][sp].w : pk[ns][sp].y;
            int a, b, c, d;
            if (GROUPED) {
                decode_word_signed(q0, slut[ns], a, b);
                decode_word_signed(q1, slut[ns], c, d);
            } else {
                decode_word(q0, lut[ns], a, b);
                decode_word(q1, lut[ns], c, d);
            }
            dst[ns] = v4i{a, b, c, d};
        }
    };

    // ---- pipeline ------------------------------------------------------------------------------
    // LDS holds four activation tiles: kt (being consumed), kt + 1 (its first fragments are fetched
    // before this iteration's barrier), kt + 2 (landing, published by this iteration's barrier) and
    // kt + 3 (copy issued right before that barrier).  The packed weights of tile kt + 2 are loaded
    // at the start of iteration kt's last k-step into the registers that tile kt has just been
    // decoded from (ordinary loads: the compiler places their waits), one whole iteration before
    // their first decode.  The LDS copies are waited for explicitly at the end of the next
    // iteration, one barrier before anyone reads the tile: the only accesses issued after them by
    // then are that iteration's NB weight loads (vmcnt retires in issue order), and every access
    // of the loop is unconditional (tiles past the end are clamped), which keeps that count exact.
    // The k-tile loop is unrolled by two so that the two weight register sets swap roles without
    // copies.
    constexpr int NB = GM_NS * 2;   // weight loads per k-tile and lane
    const int ktl = KTl - 1;
    const int g0 = GROUPED ? kt0 / tiles_per_group : 0;            // groups [g0, g_end) of this split
    const int g_end = GROUPED ? g0 + KTl / tiles_per_group : 1;
    dma_a(0, 0);
    dma_a(min(1, ktl), 1);
    dma_a(min(2, ktl), 2);
    load_b(0, pa);
    load_b(min(1, ktl), pb);
    if (GROUPED) {
        fetch_group(g0);
        publish_group(g0);
        if (g0 + 1 < g_end) {
            fetch_group(g0 + 1);
            publish_group(g0 + 1);
        }
        if (g0 + 2 < g_end) fetch_group(g0 + 2);
    } else {
        load_luts(0);
    }
    use_all(pa);
    use_all(pb);
    wait_copies<0>();
    __syncthreads();
    if (GROUPED) load_luts(g0);

    // TWO: per-channel 128-token tiles of a launch with more workgroups than CUs keep one set of
    // activation fragments and refill each right behind the MFMA that consumed it (the same block's
    // fragment of the next k-step: three MFMAs of lead); with 128 registers two workgroups share a
    // CU, and one's barrier waits and epilogue run under the other's main loop.  (With at most one
    // workgroup per CU the two fragment sets are 1-2 % faster.)
    constexpr bool ROLL = TWO;
    static_assert(!TWO || (!GROUPED && BM == 128 && GM_NS == 1), "two workgroups per CU: per-channel 128-token tiles");
    v4i af[ROLL ? 1 : 2][MS], w[2][GM_NS];
    read_a(0, 0, af[0]);
    decode_step(pa, 0, w[0]);

    // One k-tile: P holds its packed weights, PN those of the next tile.  For group-wise weights
    // the group is rescaled into the fp32 sums behind its last k-tile.  Ring of group parameters:
    // group g + 2 is published before the barrier of group g's first tile (its slot was last read
    // for group g - 2, at least one barrier ago) and read from the end of group g + 1 on (at least
    // one barrier later).
    const int tiles_in_group = GROUPED ? tiles_per_group : KTl;
    auto k_tile = [&](v4u(&P)[GM_NS][2], v4u(&PN)[GM_NS][2], int kt, int t, int g)
                      __attribute__((always_inline)) {
        const int cur = kt & (GM_RING - 1), nxt = (kt + 1) & (GM_RING - 1);
        // Software pipeline over the four 32-column k-steps: fragments and decoded weights of
        // the next step (for the last step: of the next tile's first step) are produced while
        // the MFMAs of the current step run.
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (s < 3) {
                if (!ROLL) read_a(cur, s + 1, af[ROLL ? 0 : ((s + 1) & 1)]);
                decode_step(P, s + 1, w[(s + 1) & 1]);
            } else {
                gm_order_fence();
                load_b(min(kt + 2, ktl), P);   // P: last read by the decode during the previous k-step
                gm_order_fence();
                if (GROUPED && t == tiles_in_group - 1 && g + 1 < g_end) load_luts(g + 1);
                if (!ROLL) read_a(nxt, 0, af[0]);
                use_all(PN);
                decode_step(PN, 0, w[0]);
            }
            // D[i][j]: rows i = output channels (weights operand), columns j = tokens.  The
            // first k-step of a group starts from a zero operand instead of cleared accumulators.
            if (ROLL) {
#pragma unroll
                for (int ms = 0; ms < MS; ++ms) {
                    acc[ms][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w[s & 1][0], af[0][ms], acc[ms][0], 0, 0, 0);
                    af[0][ms] = *reinterpret_cast<const v4i *>(
                        &lds_raw[(s < 3 ? cur : nxt) * (BM * TILE_K) + ms * (32 * TILE_K) + frag_off[(s + 1) & 3]]);
                }
#pragma unroll
                for (int i = 0; i < MS; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
                }
                continue;
            }
            if (GROUPED && s == 0 && t == 0) {
                const v16i z16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                    for (int ns = 0; ns < GM_NS; ++ns)
                        acc[ms][ns] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w[s & 1][ns], af[ROLL ? 0 : (s & 1)][ms],
                                                                            z16, 0, 0, 0);
            } else {
#pragma unroll
                for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                    for (int ns = 0; ns < GM_NS; ++ns)
                        acc[ms][ns] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w[s & 1][ns], af[ROLL ? 0 : (s & 1)][ms],
                                                                            acc[ms][ns], 0, 0, 0);
            }
            // issue order for this step: the LDS reads of the next step first, then the decode
            // arithmetic spread evenly between the MFMAs
            __builtin_amdgcn_sched_group_barrier(0x100, MS, 0);
#pragma unroll
            for (int i = 0; i < MS * GM_NS; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, GROUPED ? 6 : 4, 0);
            }
        }
#pragma unroll
        for (int ns = 0; ns < GM_NS; ++ns) pin_value(w[0][ns]);
        gm_order_fence();
        // group parameters: the values fetched an iteration (or more) ago go to LDS, the next
        // fetch joins this iteration's loads as the youngest
        // tile kt + 2 has landed, and so have the group parameters fetched a group ago (younger:
        // the loads into P)
        if (GROUPED && t == 0 && g + 2 < g_end) publish_group(g + 2);
        wait_copies<NB>();
        dma_a(min(kt + 3, ktl), (kt + 3) & (GM_RING - 1));
        if (GROUPED && t == 0 && g + 3 < g_end) fetch_group(g + 3);
        gm_order_fence();
        __syncthreads();
        if (GROUPED && t == tiles_in_group - 1) flush_group(g);
    };

    {
        int kt = 0, t = 0, g = g0;
        auto advance = [&]() {
            ++kt;
            if (GROUPED && ++t == tiles_in_group) {
                t = 0;
                ++g;
            }
        };
        while (kt + 2 <= KTl) {
            k_tile(pa, pb, kt, t, g);
            advance();
            k_tile(pb, pa, kt, t, g);
            advance();
        }
        if (kt < KTl) k_tile(pa, pb, kt, t, g);
    }
    // the staging buffers are reused below: no copy may still be on its way
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // Per-token values of the epilogue, fetched for all of the wave's rows at once and together
    // with the per-channel parameters below.
    const bool asym = !GROUPED && zx != nullptr;
    float sxm_a[MS];
    int nzx4_a[MS], rs_a[MS];
#pragma unroll
    for (int ms = 0; ms < MS; ++ms) {
        const int m = min(m0 + wr0 + ms * 32 + r32, M - 1);
        sxm_a[ms] = sx[m];
        nzx4_a[ms] = asym ? -4 * zx[m] : 0;
        rs_a[ms] = GROUPED ? 0 : rs[(int64_t)split * M + m];
    }

    // epilogue parameters of the workgroup's 256 channels
    __shared__ __attribute__((aligned(16))) int s_epi[3 * BN];
    float *s_es = reinterpret_cast<float *>(&s_epi[0]);           // step / 8
    int *s_bq = &s_epi[BN];                                    // 4 beta
    if (!GROUPED) {
        if (tid < BN) {
            const int nn = nb0 + tid < N ? nb0 + tid : 0;
            const int z = zero[(int64_t)nn * ng];
            s_es[tid] = step[(int64_t)nn * ng] * 0.125f;
            s_bq[tid] = 8 * z + ((~z & 1) << 2);
        }
        __syncthreads();
    }
    // per-channel weights with token zero-points: sums of each channel's weights over this
    // workgroup's K-range (all of K: the group sum; a K-split: its k-tiles added up)
    int *s_w = &s_epi[2 * BN];
    if (asym) {
        if (tid < BN) {
            const int nn = nb0 + tid < N ? nb0 + tid : 0;
            int w = 0;
            if (partial == nullptr) {
                w = wsum[nn];
            } else {
                for (int kt = 0; kt < KTl; ++kt) w += tsum[(int64_t)nn * KT + kt0 + kt];
            }
            s_w[tid] = w;
        }
        __syncthreads();
    }

    // epilogue: Y[m, n..n+3] = cast(sx[m] * y).  In the accumulator layout a lane holds four
    // consecutive channels of one token, so direct stores are 8-byte pieces scattered over 32 rows
    // of Y per instruction.  Where Y allows 16-byte stores the tile is staged in the (now free)
    // activation ring as [token][256 channels] fp16 -- 16-byte columns XOR-swizzled with the row
    // so that the 8-byte writes of 32 different rows spread over the banks -- and written out row
    // by row, 32 lanes x 16 bytes = one whole 512-byte row segment per half wave.
    // Everything uniform (output type, destination, token zero-points or none) is decided once, outside the loops, and the
    // channel parameters of four outputs come with one 16-byte LDS read, reused over the wave's
    // token blocks: as a single loop with those decisions per element the compiler produced one
    // LDS read, one wait and several branches per output (17 us per 256 x 256 tile).
    uint8_t *ytile = lds_raw;                                         // [BM][2 BN]
    enum { TO_PARTIAL = 0, TO_TILE = 1, TO_Y = 2 };
    auto epilogue = [&](auto f16_tag, auto dest_tag, auto full_tag, auto zp_tag) __attribute__((always_inline)) {
        constexpr bool F16 = decltype(f16_tag)::value;
        constexpr int DEST = decltype(dest_tag)::value;
        constexpr bool FULL = decltype(full_tag)::value;   // the tile lies inside Y: no range checks
        constexpr bool ZP = decltype(zp_tag)::value;       // per-channel weights with token zero-points
#pragma unroll
        for (int ns = 0; ns < GM_NS; ++ns) {
            if (!FULL && !ns_valid[ns]) continue;   // uniform over the wave
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int nl = wn * (GM_NS * 32) + ns * 32 + 8 * b + 4 * kh;   // channel within the workgroup
                const int nn = nb0 + nl;
                // N % 16 == 0: the eight channels of (ns, b) are valid together, uniformly over the wave
                if (!FULL && nb0 + wn * (GM_NS * 32) + ns * 32 + 8 * b >= N) continue;
                v4f es4 = {0.f, 0.f, 0.f, 0.f};
                v4i bq4 = {0, 0, 0, 0}, sw4 = {0, 0, 0, 0};
                if (!GROUPED) {
                    es4 = *reinterpret_cast<const v4f *>(&s_es[nl]);
                    bq4 = *reinterpret_cast<const v4i *>(&s_bq[nl]);
                    if (asym) sw4 = *reinterpret_cast<const v4i *>(&s_w[nl]);
                }
                const v4i nbq4 = -bq4;
#pragma unroll
                for (int ms = 0; ms < MS; ++ms) {
                    const int m = m0 + wr0 + ms * 32 + r32;
                    const bool row_ok = FULL || m < M;
                    const float sxm = sxm_a[ms];
                    uint16_t hh[4];
                    v4f part;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float yv;
                        if (GROUPED) {
                            yv = y[GROUPED ? ms : 0][ns][4 * b + r];
                        } else {
                            // remove the decode bias: 4 sum Xq d = acc - 4 beta * rowsum (exact)
                            // (24-bit multiplies: 4 beta <= 124, |row-sum| <= 2^23, |weight sum| < 2^23)
                            int v = __mul24(nbq4[r], rs_a[ms]) + acc[ms][ns][4 * b + r];
                            if (ACC_OUT && row_ok) {
                                if (partial != nullptr) atomicAdd(&acc_out[(int64_t)m * acc_ld + nn + r], v >> 2);
                                else acc_out[(int64_t)m * acc_ld + nn + r] = v >> 2;
                            }
                            // (the accumulator hook keeps the raw sum)
                            if (ZP) v = __mul24(nzx4_a[ms], sw4[r]) + v;
                            yv = es4[r] * (float)v;
                        }
                        part[r] = yv;
                        // binary32 product first, then the cast: the opaque copy keeps the compiler
                        // from fusing the two into one mixed-precision operation, which rounds once
                        // (it did so for some outputs and not for others, differently per instance)
                        float out = sxm * yv;
                        asm volatile("" : "+v"(out));
                        hh[r] = F16 ? f32_to_f16_bits(out) : f32_to_bf16_bits(out);
                    }
                    if (DEST == TO_PARTIAL) {   // K-split: the combine kernel applies sx and the cast
                        if (row_ok) *reinterpret_cast<v4f *>(&partial[((int64_t)split * M + m) * N + nn]) = part;
                        continue;
                    }
                    const uint2 h4 = make_uint2((uint32_t)hh[0] | ((uint32_t)hh[1] << 16),
                                                (uint32_t)hh[2] | ((uint32_t)hh[3] << 16));
                    if (DEST == TO_TILE) {
                        const int rl = wr0 + ms * 32 + r32;   // row within the tile
                        const int c8 = nl >> 2;               // 8-byte column within the row
                        *reinterpret_cast<uint2 *>(ytile + rl * (2 * BN) +
                                                   ((((c8 >> 1) ^ (rl & 15)) << 4) | ((c8 & 1) << 3))) = h4;
                    } else if (row_ok) {
                        uint16_t *yp = Y + (int64_t)m * ldy + nn;
                        if (vec_store & 1) {
                            *reinterpret_cast<uint2 *>(yp) = h4;
                        } else {
#pragma unroll
                            for (int r = 0; r < 4; ++r) yp[r] = hh[r];
                        }
                    }
                }
            }
        }
    };
    using std::integral_constant;
    const bool staged = partial == nullptr && (vec_store & 2) != 0;   // uniform
    const bool full = m0 + BM <= M && nb0 + BN <= N;                // uniform
    auto epilogue_zp = [&](auto f16_tag, auto dest_tag, auto full_tag) __attribute__((always_inline)) {
        if (asym) epilogue(f16_tag, dest_tag, full_tag, integral_constant<bool, true>{});
        else epilogue(f16_tag, dest_tag, full_tag, integral_constant<bool, false>{});
    };
    auto epilogue_for = [&](auto f16_tag, auto dest_tag) __attribute__((always_inline)) {
        if (full) epilogue_zp(f16_tag, dest_tag, integral_constant<bool, true>{});
        else epilogue_zp(f16_tag, dest_tag, integral_constant<bool, false>{});
    };
    if (partial != nullptr) {
        epilogue_zp(integral_constant<bool, true>{}, integral_constant<int, TO_PARTIAL>{}, integral_constant<bool, false>{});
    } else if (y_dtype == W4A8_F16) {
        if (staged) epilogue_for(integral_constant<bool, true>{}, integral_constant<int, TO_TILE>{});
        else epilogue_for(integral_constant<bool, true>{}, integral_constant<int, TO_Y>{});
    } else {
        if (staged) epilogue_for(integral_constant<bool, false>{}, integral_constant<int, TO_TILE>{});
        else epilogue_for(integral_constant<bool, false>{}, integral_constant<int, TO_Y>{});
    }
    if (staged) {
        __syncthreads();
        constexpr int NWV = WM * WN;
        constexpr int LPR = BN / 8;       // lanes per row of the tile (16 bytes each)
        constexpr int RPW = 64 / LPR;     // rows per wave and store instruction
        for (int r = wave * RPW + lane / LPR; r < BM; r += NWV * RPW) {
            const int c16 = lane % LPR;
            const int m = m0 + r, nn = nb0 + c16 * 8;
            if (m < M && nn < N) {
                const v4u v = *reinterpret_cast<const v4u *>(ytile + r * (2 * BN) + ((c16 ^ (r & 15)) << 4));
                // (streaming stores: nobody in this launch reads Y, and the caches are what serves the
                // re-reads of the activations and weights by the other tiles)
                __builtin_nontemporal_store(v, reinterpret_cast<v4u *>(Y + (int64_t)m * ldy + nn));
            }
        }
    }
}

template <int BM, int WM, int WN, bool GROUPED, bool ACC_OUT, bool ASYM, bool TWO, int BN>
static int launch_gemm_t2(const GemmPlan &pl, const int8_t *Xq, const float *sx, ZeroPoint zp,
                          const int32_t *rs, int64_t M, const uint8_t *Wt, const float *step,
                          const uint8_t *zero, int64_t N, int64_t K, int64_t G, void *Y, int y_dtype,
                          int64_t ldy, int32_t *acc_out, float *partial, hipStream_t st, int plain, int64_t acc_ld)
{
    const int grid_m = (int)((M + BM - 1) / BM);
    const int grid_n = (int)((N + BN - 1) / BN);
    // bit 0: 8-byte stores of four outputs are aligned; bit 1: 16-byte stores of eight are
    const int vec_store = ((((uintptr_t)Y % 8 == 0) && (ldy % 4 == 0)) ? 1 : 0) |
                          ((((uintptr_t)Y % 16 == 0) && (ldy % 8 == 0)) ? 2 : 0);
    constexpr int lds_bytes = GM_RING * BM * TILE_K;
    static std::atomic<uint64_t> lds_opted{0};
    if (lds_bytes > 48 * 1024 &&
        opt_in_dynamic_lds((const void *)gemm_kernel<BM, WM, WN, GROUPED, ACC_OUT, ASYM, TWO, BN>, lds_bytes,
                           lds_opted) != W4A8_OK)
        return W4A8_ERR_HIP;
    hipLaunchKernelGGL((gemm_kernel<BM, WM, WN, GROUPED, ACC_OUT, ASYM, TWO, BN>),
                       dim3((unsigned)(grid_m * grid_n * pl.splits)), dim3(WM * WN * 64), lds_bytes, st,
                       Xq, sx, zp.zx, zp.wsum, zp.tsum, rs, (int)M, Wt, step, zero, (int)N, (int)K,
                       (int)(G / TILE_K), (int)(K / G), (uint16_t *)Y, y_dtype, ldy, vec_store,
                       acc_out, grid_m, grid_n, pl.kt_per_split, pl.splits > 1 ? partial : nullptr, plain,
                       (int)(acc_ld > 0 ? acc_ld : N));
    return hip_status(hipGetLastError());
}

template <int BM, int WM, int WN, bool GROUPED, bool TWO = false, int BN = GM_BN>
static int launch_gemm_t(const GemmPlan &pl, const int8_t *Xq, const float *sx, ZeroPoint zp,
                         const int32_t *rs, int64_t M, const uint8_t *Wt, const float *step,
                         const uint8_t *zero, int64_t N, int64_t K, int64_t G, void *Y, int y_dtype,
                         int64_t ldy, int32_t *acc_out, float *partial, hipStream_t st, int plain,
                         int64_t acc_ld = 0)
{
    // The accumulator test hook is a separate instance so that the fast path carries none of it;
    // so is the per-group zero-point term of group-wise weights.
#define W4A8_GM2(AO_, AS_)                                                                       \
    return launch_gemm_t2<BM, WM, WN, GROUPED, AO_, AS_, TWO, BN>(pl, Xq, sx, zp, rs, M, Wt, step, zero, N, K, \
                                                     G, Y, y_dtype, ldy, acc_out, partial, st, plain, acc_ld)
    if (GROUPED && zp.zx != nullptr) {
        if (acc_out) W4A8_GM2(true, GROUPED);
        W4A8_GM2(false, GROUPED);
    }
    if (acc_out) W4A8_GM2(true, false);
    W4A8_GM2(false, false);
#undef W4A8_GM2
}

// ---- group-128 weights at a few hundred tokens ---------------------------------------------------
// Between the streaming kernel (<= 16 tokens per pass over the weights) and the tile kernel at full
// occupancy lies the ridge of the roofline (M ~ 156): a 128-token tile kernel has only N / 256 tiles for
// 256 CUs there, and cutting K into ranges over more workgroups moves more fp32 partial sums through
// memory than the layer has weights.  This kernel cuts K inside the workgroup instead.  A workgroup
// owns 128 tokens x 64 channels; its 8 waves are 2 (channel halves of 32) x 4 (K phases): phase q takes
// the k-tiles kt = 4 i + q -- with 128-wide groups each k-tile is one whole group, so a wave decodes,
// multiplies and rescales complete groups exactly like the tile kernel does, and no group is shared.
// The four k-tiles of a super-step are consumed concurrently from four LDS slots while the next four
// land in the other four (global -> LDS copies, issued right behind the barrier that frees the slots):
// one barrier per FOUR k-tiles.  At the end the phases' fp32 sums meet through LDS in a fixed order
// ((q0 + q1) + (q2 + q3)), and the two phase-0 waves apply the token scale and store.  N / 64 workgroups
// per 128 tokens, no workspace, no second launch.
constexpr int MD_BM = 128, MD_BN = 64, MD_KQ = 4, MD_THREADS = 512;
constexpr int MD_TILE = MD_BM * TILE_K;   // bytes of one activation k-tile in LDS

template <bool ACC_OUT>
__global__ __launch_bounds__(MD_THREADS, 2) void gemm_mid_kernel(
    const int8_t *__restrict__ Xq, const float *__restrict__ sx, int M, const uint8_t *__restrict__ Wt,
    const float *__restrict__ step, const uint8_t *__restrict__ zero, int N, int K,
    uint16_t *__restrict__ Y, int y_dtype, int64_t ldy, int vec_store, int32_t *__restrict__ acc_out,
    int grid_m, int plain)
{
    constexpr int MS = MD_BM / 32;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];   // [2 * MD_KQ][MD_TILE]
    __shared__ __attribute__((aligned(16))) float s_ges[4 * MD_KQ][MD_BN];   // step / 8 per k-tile (= group) of four super-steps, and channel
    __shared__ int s_gz[4 * MD_KQ][MD_BN];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave & 1;      // channel half
    const int kq = wave >> 1;     // K phase
    const int r32 = lane & 31;
    const int kh = lane >> 5;
    const int KT = K / TILE_K;    // = number of groups
    const int SS = (KT + MD_KQ - 1) / MD_KQ;
    const int bm = blockIdx.x % grid_m, bn = blockIdx.x / grid_m;
    const int m0 = bm * MD_BM;
    const int nb0 = bn * MD_BN;
    const int n0 = nb0 + wn * 32;

    __amdgpu_buffer_rsrc_t rw =
        __builtin_amdgcn_make_buffer_rsrc((void *)Wt, 0, (int)((int64_t)N * K / 2), 0x00020000);
    const uint64_t xq_addr = (uint64_t)Xq;
    const v4i rx = {(int)(uint32_t)xq_addr, (int)((xq_addr >> 32) & 0xffffu), (int)((int64_t)M * K), 0x00020000};

    // weights of this wave's 32 channels (see gemm_kernel): one 16-byte load covers two k-steps
    const bool lane_ok = n0 + r32 < N;
    const int wvoff = lane_ok ? (r32 >> 4) * KT * TILE_BYTES + ((r32 & 15) + 16 * kh) * 16 : GM_OOB;
    const int wsoff = n0 < N ? (n0 / TILE_N) * KT * TILE_BYTES : 0;
    auto load_b = [&](int kt, v4u(&dst)[2]) {
        const int ktc = min(kt, KT - 1);
        dst[0] = __builtin_amdgcn_raw_buffer_load_b128(rw, wvoff, wsoff + ktc * TILE_BYTES, 0);
        dst[1] = __builtin_amdgcn_raw_buffer_load_b128(rw, wvoff + 512, wsoff + ktc * TILE_BYTES, 0);
    };

    // activation k-tile -> LDS slot: 16 blocks of 8 rows, two per wave (swizzle as in gemm_kernel)
    int avoff[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = (i * 8 + wave) * 8 + (lane >> 3);
        avoff[i] = (m0 + row) * K + (((lane & 7) ^ ((row >> 1) & 7)) << 4);
    }
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lds_raw;
    // this wave's share of the four k-tiles of super-step ss (into the slots of its parity): eight copies
    // of 1 KB, c = 2 j + i for block i of k-tile j
    auto dma_one = [&](int ss, int c) {
        const int j = c >> 1, i = c & 1;
        const int kt = min(ss * MD_KQ + j, KT - 1);
        const int slot = (ss & 1) * MD_KQ + j;
        dma_b128(rx, avoff[i], kt * TILE_K, lds_base + (uint32_t)(slot * MD_TILE + (i * 8 + wave) * 1024));
    };
    auto dma_super_step = [&](int ss) {
#pragma unroll
        for (int c = 0; c < 2 * MD_KQ; ++c) dma_one(ss, c);
    };
    // group parameters of a super-step: thread (j = tid / 64, ch = tid % 64), tid < 256
    float gp_es = 0.f;
    int gp_z = 0;
    auto fetch_params = [&](int ss) {
        if (tid < MD_KQ * MD_BN) {
            const int kt = min(ss * MD_KQ + (tid >> 6), KT - 1);
            const int nn = nb0 + (tid & 63) < N ? nb0 + (tid & 63) : 0;
            gp_es = step[(int64_t)nn * KT + kt];   // (used only in publish_params: nothing here waits for the load)
            gp_z = zero[(int64_t)nn * KT + kt];
        }
    };
    auto publish_params = [&](int ss) {
        if (tid < MD_KQ * MD_BN) {
            s_ges[(ss & 3) * MD_KQ + (tid >> 6)][tid & 63] = gp_es * 0.125f;
            s_gz[(ss & 3) * MD_KQ + (tid >> 6)][tid & 63] = gp_z;
        }
    };

    v16i acc[MS];
    float y[MS][16];
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int r = 0; r < 16; ++r) y[ms][r] = 0.f;

    int frag_off[4];
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
        const int chunk = 2 * (2 * (s4 >> 1) + kh) + (s4 & 1);
        frag_off[s4] = r32 * TILE_K + ((chunk ^ ((r32 >> 1) & 7)) << 4);
    }
    auto read_a = [&](int slot, int ms, int s4) {   // fragment of token block ms, k-step s4
        return *reinterpret_cast<const v4i *>(&lds_raw[slot * MD_TILE + ms * (32 * TILE_K) + frag_off[s4]]);
    };
    SignedLut slut;
    auto decode_step = [&](const v4u(&pk)[2], int s4, v4i &dst) {
        const int sp = s4 >> 1, h = s4 & 1;
        const uint32_t q0 = h ? pk[sp].z : pk[sp].x;
        const uint32_t q1 = h ? pk[sp].w : pk[sp].y;
        int a, b, c, d;
        decode_word_signed(q0, slut, a, b);
        decode_word_signed(q1, slut, c, d);
        dst = v4i{a, b, c, d};
    };
    // y += (step / 8) * acc for accumulator registers 4 b .. 4 b + 3 of token block ms (group kt)
    v4f es4[4];   // step / 8 of this lane's 16 channels for the group in the accumulators
    auto flush_quarter = [&](int ms, int b, int kt) {
        const int m = m0 + ms * 32 + r32;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int v = acc[ms][4 * b + r];
            y[ms][4 * b + r] = __builtin_fmaf(es4[b][r], (float)v, y[ms][4 * b + r]);
            if (ACC_OUT && m < M) {
                const int nn = nb0 + wn * 32 + 8 * b + 4 * kh + r;
                if (nn < N) acc_out[((int64_t)m * N + nn) * KT + kt] = v >> 2;
            }
        }
    };

    // ---- prologue: super-steps 0 and 1 on their way, this wave's first four k-tiles of weights, the
    // group parameters of super-steps 0 and 1 published and those of 2 requested
    v4u pw[4][2];   // packed weights of this wave's next four k-tiles (the weights come from HBM, read once)
    dma_super_step(0);
#pragma unroll
    for (int i = 0; i < 4; ++i) load_b(i * MD_KQ + kq, pw[i]);
    fetch_params(0);
    publish_params(0);
    fetch_params(min(1, SS - 1));
    publish_params(1);
    fetch_params(min(2, SS - 1));
    asm volatile("" : "+v"(pw[0][0]), "+v"(pw[0][1]), "+v"(pw[1][0]), "+v"(pw[1][1]));
    wait_copies<0>();
    __syncthreads();

    v4i w[4], af[4];   // decoded weights of the four k-steps of the current k-tile; activation fragments
    slut = make_signed_lut(s_gz[kq][wn * 32 + r32], plain != 0);
#pragma unroll
    for (int k = 0; k < 4; ++k) decode_step(pw[0], k, w[k]);
    bool pending = false;   // (uniform) accumulators of token block 3 of the previous k-tile wait for their rescale

    // One super-step of this wave: k-tile kt = 4 ss + q (= one group) from LDS slot (ss parity, q).
    // The MFMAs run token block by token block (four k-steps each), so that the rescale of block ms - 1
    // -- whose group sum is complete -- and, under the last block, the decode of the NEXT k-tile (each
    // w[k] is free once the last MFMA that reads it has issued) sit between the MFMAs of block ms:
    // a wave overlaps its own vector and matrix work instead of relying on its SIMD neighbour.
    // The last block's rescale is deferred to the start of the next super-step, where it covers the
    // latency of the first fragment reads.
    // P: packed weights of this k-tile, refilled for the wave's k-tile four super-steps on; PN: those of
    // the next super-step (decoded here); PNN: those of the one after (completed here, see below).
    // Order of the memory accesses of a wave (vmcnt retires in this order):
    //   behind barrier(ss - 1): [2 parameter loads of ss + 2]
    //   in super-step ss:       8 copies of super-step ss + 1 (their slots were freed by barrier(ss - 1))
    //   at the end of ss:       2 weight loads for ss + 4
    // so "at most 2 outstanding" at the end of super-step ss means the copies of ss + 1 have landed and
    // every older weight load is complete; the barrier then publishes the copies and frees the slots
    // of ss for ss + 2.  Group parameters: ring of four super-steps, published two ahead (the decode of
    // the next k-tile needs its zero-points before the next barrier).
    auto super_step = [&](v4u(&P)[2], v4u(&PN)[2], v4u(&PNN)[2], int ss) __attribute__((always_inline)) {
        const int kt = ss * MD_KQ + kq;
        const int slot = (ss & 1) * MD_KQ + kq;
        const int pslot = (ss & 3) * MD_KQ + kq;
        const int pslot_next = ((ss + 1) & 3) * MD_KQ + kq;
        const bool live = kt < KT;   // (uniform over the wave; live k-tiles come first)
        if (live) {
#pragma unroll
            for (int k = 0; k < 4; ++k) af[k] = read_a(slot, 0, k);
        }
        if (pending) {
#pragma unroll
            for (int b = 0; b < 4; ++b) flush_quarter(3, b, kt - MD_KQ);
            pending = false;
        }
        if (live) {
#pragma unroll
            for (int b = 0; b < 4; ++b)
                es4[b] = *reinterpret_cast<const v4f *>(&s_ges[pslot][wn * 32 + 8 * b + 4 * kh]);
            int z_next = s_gz[pslot_next][wn * 32 + r32];
            const v16i z16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int ms = 0; ms < MS; ++ms) {
                if (ms == 1) {
                    // the scales and the next zero-point are in registers from here on (their reads were
                    // issued before the first block's MFMAs; without this the reads sink to their uses)
                    asm volatile("" : "+v"(es4[0]), "+v"(es4[1]), "+v"(es4[2]), "+v"(es4[3]), "+v"(z_next));
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    if (k == 0) acc[ms] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w[0], af[0], z16, 0, 0, 0);
                    else acc[ms] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w[k], af[k], acc[ms], 0, 0, 0);
                    if (ms + 1 < MS) af[k] = read_a(slot, ms + 1, k);
                    // the copies of the next super-step, two per MFMA of the first block: issued in one burst
                    // by all eight waves they fill the address queue of the CU and hold every wave up
                    if (ms == 0) {
                        dma_one(ss + 1, 2 * k);
                        dma_one(ss + 1, 2 * k + 1);
                    }
                    if (ms > 0) flush_quarter(ms - 1, k, kt);
                    if (ms + 1 == MS) {
                        if (k == 0) slut = make_signed_lut(z_next, plain != 0);
                        decode_step(PN, k, w[k]);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    if (ms + 1 < MS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    if (ms + 1 == MS) __builtin_amdgcn_sched_group_barrier(0x002, 32, 0);
                    else if (ms > 0) __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
                }
            }
            pending = true;
        } else {
            dma_super_step(ss + 1);
        }
        gm_order_fence();
        load_b((ss + 4) * MD_KQ + kq, P);
        gm_order_fence();
        wait_copies<2>();
        // (a use in every lane, outside any branch: all waits for the parameter loads and for PNN happen
        // here, none behind the copies issued below)
        asm volatile("" : "+v"(PNN[0]), "+v"(PNN[1]), "+v"(gp_es), "+v"(gp_z));
        publish_params(ss + 2);   // (fetched behind the last barrier)
        __syncthreads();
        fetch_params(min(ss + 3, SS - 1));
        gm_order_fence();
    };

    {
        int ss = 0;
        for (; ss + 4 <= SS; ss += 4) {
            super_step(pw[0], pw[1], pw[2], ss);
            super_step(pw[1], pw[2], pw[3], ss + 1);
            super_step(pw[2], pw[3], pw[0], ss + 2);
            super_step(pw[3], pw[0], pw[1], ss + 3);
        }
        if (ss < SS) super_step(pw[0], pw[1], pw[2], ss);
        if (ss + 1 < SS) super_step(pw[1], pw[2], pw[3], ss + 1);
        if (ss + 2 < SS) super_step(pw[2], pw[3], pw[0], ss + 2);
        if (pending) {   // the last live k-tile of this wave: 4 (SS - 1) + q, or the one before
            const int kt_last = (SS - 1) * MD_KQ + kq;
#pragma unroll
            for (int b = 0; b < 4; ++b) flush_quarter(3, b, kt_last < KT ? kt_last : kt_last - MD_KQ);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // ---- the four phases' sums meet in LDS: (q0 + q1) + (q2 + q3)
    float *red = reinterpret_cast<float *>(lds_raw);   // [..][64 lanes][64 floats], 16 KB per wave
    auto red_ptr = [&](int slot) { return red + ((size_t)slot * 64 + lane) * 64; };
    auto put = [&](int slot) {
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
            for (int r = 0; r < 16; r += 4)
                *reinterpret_cast<v4f *>(red_ptr(slot) + ((ms * 16 + r) ^ ((lane & 15) << 2))) =
                    v4f{y[ms][r], y[ms][r + 1], y[ms][r + 2], y[ms][r + 3]};
    };
    auto add = [&](int slot) {
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
            for (int r = 0; r < 16; r += 4) {
                const v4f t = *reinterpret_cast<const v4f *>(red_ptr(slot) + ((ms * 16 + r) ^ ((lane & 15) << 2)));
                y[ms][r] += t.x; y[ms][r + 1] += t.y; y[ms][r + 2] += t.z; y[ms][r + 3] += t.w;
            }
    };
    if (kq & 1) put((kq >> 1) * 2 + wn);          // q1 -> slots 0, 1; q3 -> slots 2, 3
    __syncthreads();
    if (!(kq & 1)) add((kq >> 1) * 2 + wn);       // q0 += q1, q2 += q3
    __syncthreads();
    if (kq == 2) put(wn);
    __syncthreads();
    if (kq != 0) return;
    add(wn);

    // ---- epilogue (phase-0 waves): Y[m, n .. n+3] = cast(sx[m] * y)
#pragma unroll
    for (int ms = 0; ms < MS; ++ms) {
        const int m = m0 + ms * 32 + r32;
        if (m >= M) continue;
        const float sxm = sx[m];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int nn = nb0 + wn * 32 + 8 * b + 4 * kh;
            if (nn >= N) continue;   // (N % 16 == 0: four channels are valid together)
            uint16_t hh[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float out = sxm * y[ms][4 * b + r];   // binary32 product, then the cast (see gemm_kernel)
                asm volatile("" : "+v"(out));
                hh[r] = (y_dtype == W4A8_F16) ? f32_to_f16_bits(out) : f32_to_bf16_bits(out);
            }
            uint16_t *yp = Y + (int64_t)m * ldy + nn;
            if (vec_store & 1) {
                *reinterpret_cast<uint2 *>(yp) = make_uint2((uint32_t)hh[0] | ((uint32_t)hh[1] << 16),
                                                            (uint32_t)hh[2] | ((uint32_t)hh[3] << 16));
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) yp[r] = hh[r];
            }
        }
    }
}

// The same decomposition for per-channel weights: no group parameters and no rescale per group -- the
// int32 accumulators run over all of a phase's k-tiles (biased decode, 7 instead of 11 operations per
// eight weights), the four phases' int32 sums are added exactly through LDS, and the phase-0 waves remove
// the decode bias with the token's row-sum (rs[m], from rowsum_kernel), scale and store.
// A super-step of this kernel is short (8 MFMAs per wave), far shorter than the time a copy of
// activations needs to arrive when every workgroup asks for the same k-tiles at the same moment, so the
// tile is 64 tokens (8 KB per k-tile) and LDS holds FOUR super-steps: the copies of super-step ss + 3 are
// issued during ss.  Every memory access of the loop is issued by hand (the copies, and the weight
// loads as plain buffer loads into registers), in a fixed order, so that one explicit wait per
// super-step is exact: at its end everything up to the copies of ss + 1 must have landed, and the
// accesses issued after those are 2 + 4 + 2 + 4 + 2 = 14 (weights of ss + 2, copies of ss + 2, weights of
// ss + 3, copies of ss + 3, weights of ss + 4).
constexpr int MP_BM = 64, MP_RING = 4;
constexpr int MP_TILE = MP_BM * TILE_K;   // 8 KB

__device__ __forceinline__ void load_b128_by_hand(v4u &dst, v4i rsrc, int voff, int soff)
{
    asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen" : "=v"(dst) : "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}

template <bool ACC_OUT>
__global__ __launch_bounds__(MD_THREADS, 2) void gemm_mid_pc_kernel(
    const int8_t *__restrict__ Xq, const float *__restrict__ sx, const int32_t *__restrict__ rs, int M,
    const uint8_t *__restrict__ Wt, const float *__restrict__ step, const uint8_t *__restrict__ zero, int N,
    int K, uint16_t *__restrict__ Y, int y_dtype, int64_t ldy, int vec_store, int32_t *__restrict__ acc_out,
    int grid_m, int plain)
{
    constexpr int MS = MP_BM / 32;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];   // [MP_RING * MD_KQ][MP_TILE]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave & 1;      // channel half
    const int kq = wave >> 1;     // K phase
    const int r32 = lane & 31;
    const int kh = lane >> 5;
    const int KT = K / TILE_K;
    const int SS = (KT + MD_KQ - 1) / MD_KQ;
    const int bm = blockIdx.x % grid_m, bn = blockIdx.x / grid_m;
    const int m0 = bm * MP_BM;
    const int nb0 = bn * MD_BN;
    const int n0 = nb0 + wn * 32;

    const uint64_t wt_addr = (uint64_t)Wt;
    const v4i rwv = {(int)(uint32_t)wt_addr, (int)((wt_addr >> 32) & 0xffffu), (int)((int64_t)N * K / 2), 0x00020000};
    const uint64_t xq_addr = (uint64_t)Xq;
    const v4i rx = {(int)(uint32_t)xq_addr, (int)((xq_addr >> 32) & 0xffffu), (int)((int64_t)M * K), 0x00020000};

    // the decode table of this lane's channel (one zero-point for all of K); loaded before anything is
    // issued by hand, so that the compiler's wait for it covers nothing else
    const bool lane_ok = n0 + r32 < N;
    const DecodeLut lut = make_decode_lut(zero[lane_ok ? n0 + r32 : 0], plain != 0);

    const int wvoff = lane_ok ? (r32 >> 4) * KT * TILE_BYTES + ((r32 & 15) + 16 * kh) * 16 : GM_OOB;
    const int wsoff = n0 < N ? (n0 / TILE_N) * KT * TILE_BYTES : 0;
    auto load_b = [&](int kt, v4u(&dst)[2]) {
        const int ktc = min(kt, KT - 1);
        load_b128_by_hand(dst[0], rwv, wvoff, wsoff + ktc * TILE_BYTES);
        load_b128_by_hand(dst[1], rwv, wvoff + 512, wsoff + ktc * TILE_BYTES);
    };
    // activation k-tile (64 rows) -> LDS slot: 8 blocks of 8 rows, one per wave (swizzle as in gemm_kernel)
    const int arow = wave * 8 + (lane >> 3);
    const int avoff = (m0 + arow) * K + (((lane & 7) ^ ((arow >> 1) & 7)) << 4);
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lds_raw;
    auto dma_one = [&](int ss, int j) {   // this wave's block of k-tile j of super-step ss
        const int kt = min(ss * MD_KQ + j, KT - 1);
        const int slot = (ss & (MP_RING - 1)) * MD_KQ + j;
        dma_b128(rx, avoff, kt * TILE_K, lds_base + (uint32_t)(slot * MP_TILE + wave * 1024));
    };

    v16i acc[MS];
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[ms][r] = 0;

    int frag_off[4];
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
        const int chunk = 2 * (2 * (s4 >> 1) + kh) + (s4 & 1);
        frag_off[s4] = r32 * TILE_K + ((chunk ^ ((r32 >> 1) & 7)) << 4);
    }
    auto read_a = [&](int slot, int s4, v4i(&dst)[MS]) {
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
            dst[ms] = *reinterpret_cast<const v4i *>(&lds_raw[slot * MP_TILE + ms * (32 * TILE_K) + frag_off[s4]]);
    };
    auto decode_step = [&](const v4u(&pk)[2], int s4, v4i &dst) {
        const int sp = s4 >> 1, h = s4 & 1;
        const uint32_t q0 = h ? pk[sp].z : pk[sp].x;
        const uint32_t q1 = h ? pk[sp].w : pk[sp].y;
        int a, b, c, d;
        decode_word(q0, lut, a, b);
        decode_word(q1, lut, c, d);
        dst = v4i{a, b, c, d};
    };

    // ---- prologue, in the order the loop continues: copies of super-steps 0, 1, 2 and the weights of this
    // wave's first four k-tiles (every access unconditional: k-tiles past the end are clamped)
    v4u pw[4][2];
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // (the zero-point above)
#pragma unroll
    for (int j = 0; j < MD_KQ; ++j) dma_one(0, j);
    load_b(kq, pw[0]);
    load_b(MD_KQ + kq, pw[1]);
#pragma unroll
    for (int j = 0; j < MD_KQ; ++j) dma_one(1, j);
    load_b(2 * MD_KQ + kq, pw[2]);
#pragma unroll
    for (int j = 0; j < MD_KQ; ++j) dma_one(2, j);
    load_b(3 * MD_KQ + kq, pw[3]);
    // super-step 0's copies and weights: everything but the 4 + 2 + 4 + 2 + 2 accesses issued behind them
    // (weights of 1 were issued together with those of 0: waited for as well)
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(pw[0][0]), "+v"(pw[0][1]), "+v"(pw[1][0]), "+v"(pw[1][1]) :: "memory");
    __syncthreads();

    // One super-step: k-tile kt = 4 ss + q from slot (ss mod 4, q); P: its packed weights (complete since
    // the previous super-step's wait), refilled at the end for ss + 4; PN: the next super-step's.
    auto super_step = [&](v4u(&P)[2], v4u(&PN)[2], int ss, bool drain) __attribute__((always_inline)) {
        const int kt = ss * MD_KQ + kq;
        const int slot = (ss & (MP_RING - 1)) * MD_KQ + kq;
        if (kt < KT) {   // (uniform over the wave; live k-tiles come first)
            v4i af[2][MS], w[2];
            read_a(slot, 0, af[0]);
            decode_step(P, 0, w[0]);
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
                if (s4 < 3) {
                    read_a(slot, s4 + 1, af[(s4 + 1) & 1]);
                    decode_step(P, s4 + 1, w[(s4 + 1) & 1]);
                }
#pragma unroll
                for (int ms = 0; ms < MS; ++ms)
                    acc[ms] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w[s4 & 1], af[s4 & 1][ms], acc[ms], 0, 0, 0);
                dma_one(ss + 3, s4);   // (the slots of ss + 3 = those of ss - 1: freed by the last barrier)
            }
        } else {
#pragma unroll
            for (int j = 0; j < MD_KQ; ++j) dma_one(ss + 3, j);
        }
        // (P's last read, by the decode above, comes before its refill: both are pinned in program order)
        asm volatile("" : "+v"(P[0]), "+v"(P[1]) :: "memory");
        load_b((ss + 4) * MD_KQ + kq, P);
        // (the waits name no register: a choice between two statements that do would make the compiler
        // merge register sets behind them, with copies; the use of PN that follows is what keeps the
        // next super-step's decode behind the wait)
        if (drain) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the loop's last super-step
        else asm volatile("s_waitcnt vmcnt(14)" ::: "memory");
        asm volatile("" : "+v"(PN[0]), "+v"(PN[1]) :: "memory");
        __syncthreads();
    };
    // The loop body is four super-steps (the four weight register sets take turns without copies) and is
    // the ONLY code between the prologue and the reduction: super-steps past the last one have no live
    // k-tile and only keep the order of the accesses (clamped copies and loads).  A separate tail would
    // have the compiler move the weight registers between their homes of the loop and those of the tail
    // while loads that it cannot see are still writing them.  For the same reason the loop's last
    // super-step waits for everything: behind the loop no register or LDS slot has a load on its way.
    for (int ss = 0; ss < SS; ss += 4) {
        super_step(pw[0], pw[1], ss, false);
        super_step(pw[1], pw[2], ss + 1, false);
        super_step(pw[2], pw[3], ss + 2, false);
        super_step(pw[3], pw[0], ss + 3, ss + 4 >= SS);
    }

    // ---- the four phases' int32 sums meet in LDS (exact: the order does not matter)
    int *red = reinterpret_cast<int *>(lds_raw);   // [..][64 lanes][32 ints], 8 KB per wave
    auto red_ptr = [&](int slot) { return red + ((size_t)slot * 64 + lane) * (MS * 16); };
    auto put = [&](int slot) {
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
            for (int r = 0; r < 16; r += 4)
                *reinterpret_cast<v4i *>(red_ptr(slot) + ((ms * 16 + r) ^ ((lane & 7) << 2))) =
                    v4i{acc[ms][r], acc[ms][r + 1], acc[ms][r + 2], acc[ms][r + 3]};
    };
    auto add = [&](int slot) {
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
            for (int r = 0; r < 16; r += 4) {
                const v4i t = *reinterpret_cast<const v4i *>(red_ptr(slot) + ((ms * 16 + r) ^ ((lane & 7) << 2)));
                acc[ms][r] += t.x; acc[ms][r + 1] += t.y; acc[ms][r + 2] += t.z; acc[ms][r + 3] += t.w;
            }
    };
    if (kq & 1) put((kq >> 1) * 2 + wn);
    __syncthreads();
    if (!(kq & 1)) add((kq >> 1) * 2 + wn);
    __syncthreads();
    if (kq == 2) put(wn);
    __syncthreads();
    if (kq != 0) return;
    add(wn);

    // ---- epilogue (phase-0 waves): remove the decode bias, scale, store
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int nn = nb0 + wn * 32 + 8 * b + 4 * kh;
        if (nn >= N) continue;   // (N % 16 == 0: four channels are valid together)
        float es[4];
        int nbq[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int z = zero[nn + r];
            es[r] = step[nn + r] * 0.125f;
            nbq[r] = -(8 * z + ((~z & 1) << 2));   // - 4 beta
        }
#pragma unroll
        for (int ms = 0; ms < MS; ++ms) {
            const int m = m0 + ms * 32 + r32;
            if (m >= M) continue;
            const float sxm = sx[m];
            const int rsm = rs[m];
            uint16_t hh[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                // 4 sum Xq d = acc - 4 beta * rowsum (exact; 24-bit multiply: 4 beta <= 124, |row-sum| <= 2^23)
                const int v = __mul24(nbq[r], rsm) + acc[ms][4 * b + r];
                if (ACC_OUT) acc_out[(int64_t)m * N + nn + r] = v >> 2;
                float out = sxm * (es[r] * (float)v);   // binary32 products, then the cast (see gemm_kernel)
                asm volatile("" : "+v"(out));
                hh[r] = (y_dtype == W4A8_F16) ? f32_to_f16_bits(out) : f32_to_bf16_bits(out);
            }
            uint16_t *yp = Y + (int64_t)m * ldy + nn;
            if (vec_store & 1) {
                *reinterpret_cast<uint2 *>(yp) = make_uint2((uint32_t)hh[0] | ((uint32_t)hh[1] << 16),
                                                            (uint32_t)hh[2] | ((uint32_t)hh[3] << 16));
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) yp[r] = hh[r];
            }
        }
    }
}

// Whether a shape takes gemm_mid_kernel: 128-wide groups, symmetric activations, 65 .. 256 tokens, and a
// grid of at most one workgroup per CU.  Measured against the tile kernel with K cut into ranges (which
// is what these shapes would otherwise run): ahead wherever the grid covers at least half the CUs
// (LLaMA-13B up-projection at 128 tokens: 39 -> 26 us; 4096 x 4096 at 256: 29 -> 22 us), behind on long K
// with few workgroups (13824 -> 5120 at 128 tokens: 80 workgroups, 27 super-steps, 45 against 37 us) and
// with more than one workgroup per CU.
bool gemm_mid_applies(int64_t M, int64_t N, int64_t K, int64_t G, bool asym)
{
    if (asym || G != TILE_K || G == K || M <= 64 || M > 256) return false;
    const int64_t wgs = (M + MD_BM - 1) / MD_BM * ((N + MD_BN - 1) / MD_BN);
    const int64_t KT = K / TILE_K;
    return KT >= 8 && wgs <= 256 && (wgs >= 128 || KT <= 48);
}

static int launch_gemm_mid(const int8_t *Xq, const float *sx, int64_t M, const uint8_t *Wt, const float *step,
                           const uint8_t *zero, int64_t N, int64_t K, void *Y, int y_dtype, int64_t ldy,
                           int32_t *acc_out, hipStream_t st, int plain)
{
    const int grid_m = (int)((M + MD_BM - 1) / MD_BM);
    const int grid_n = (int)((N + MD_BN - 1) / MD_BN);
    const int vec_store = (((uintptr_t)Y % 8 == 0) && (ldy % 4 == 0)) ? 1 : 0;
    constexpr int lds_bytes = 2 * MD_KQ * MD_TILE;   // 128 KB
#define W4A8_MD(AO_)                                                                                      \
    do {                                                                                                  \
        static std::atomic<uint64_t> lds_opted{0};                                                        \
        if (opt_in_dynamic_lds((const void *)gemm_mid_kernel<AO_>, lds_bytes, lds_opted) != W4A8_OK)      \
            return W4A8_ERR_HIP;                                                                          \
        hipLaunchKernelGGL((gemm_mid_kernel<AO_>), dim3((unsigned)(grid_m * grid_n)), dim3(MD_THREADS),   \
                           lds_bytes, st, Xq, sx, (int)M, Wt, step, zero, (int)N, (int)K, (uint16_t *)Y,  \
                           y_dtype, ldy, vec_store, acc_out, grid_m, plain);                              \
    } while (0)
    if (acc_out) W4A8_MD(true);
    else W4A8_MD(false);
#undef W4A8_MD
    return hip_status(hipGetLastError());
}

// The per-channel variant (gemm_mid_pc_kernel), same token range and grid condition.
bool gemm_mid_pc_applies(int64_t M, int64_t N, int64_t K, int64_t G, bool asym)
{
    if (asym || G != K || M <= 64 || M > 256) return false;
    const int64_t wgs = (M + MP_BM - 1) / MP_BM * ((N + MD_BN - 1) / MD_BN);
    const int64_t KT = K / TILE_K;
    return KT >= 8 && wgs <= 256;
}

static int launch_gemm_mid_pc(const int8_t *Xq, const float *sx, int32_t *rs, int64_t M, const uint8_t *Wt,
                              const float *step, const uint8_t *zero, int64_t N, int64_t K, void *Y, int y_dtype,
                              int64_t ldy, int32_t *acc_out, hipStream_t st, int plain)
{
    // the tokens' row-sums over all of K (bias removal in the epilogue)
    hipLaunchKernelGGL(rowsum_kernel, dim3((unsigned)((M + 3) / 4)), dim3(256), 0, st, Xq, M, (int)K, 1, (int)K, rs);
    if (hipGetLastError() != hipSuccess) return W4A8_ERR_HIP;
    const int grid_m = (int)((M + MP_BM - 1) / MP_BM);
    const int grid_n = (int)((N + MD_BN - 1) / MD_BN);
    const int vec_store = (((uintptr_t)Y % 8 == 0) && (ldy % 4 == 0)) ? 1 : 0;
    constexpr int lds_bytes = MP_RING * MD_KQ * MP_TILE;   // 128 KB
#define W4A8_MDP(AO_)                                                                                     \
    do {                                                                                                  \
        static std::atomic<uint64_t> lds_opted{0};                                                        \
        if (opt_in_dynamic_lds((const void *)gemm_mid_pc_kernel<AO_>, lds_bytes, lds_opted) != W4A8_OK)   \
            return W4A8_ERR_HIP;                                                                          \
        hipLaunchKernelGGL((gemm_mid_pc_kernel<AO_>), dim3((unsigned)(grid_m * grid_n)), dim3(MD_THREADS), \
                           lds_bytes, st, Xq, sx, rs, (int)M, Wt, step, zero, (int)N, (int)K, (uint16_t *)Y, \
                           y_dtype, ldy, vec_store, acc_out, grid_m, plain);                              \
    } while (0)
    if (acc_out) W4A8_MDP(true);
    else W4A8_MDP(false);
#undef W4A8_MDP
    return hip_status(hipGetLastError());
}

GemmPlan plan_gemm(int64_t M, int64_t N, int64_t K, int64_t G)
{
    GemmPlan pl{};
    const bool grouped = G != K;
    const int64_t gn = (N + GM_BN - 1) / GM_BN;
    if (M < 1 || gn < 1 || K < TILE_K) return pl;   // nothing to launch (callers check shapes first)
    if (M <= 64 && grouped) {
        pl.bm = 64;    // (per-channel layers with so few tokens run as token blocks of the streaming kernel)
    } else if (grouped || M <= 128) {
        pl.bm = 128;   // group-wise: int32 group accumulators plus fp32 running sums
    } else {
        // 256-row tiles reuse each decoded weight twice as often, but whole rounds of 256 CUs are
        // what count.  128-row tiles run two to a CU: 512 of them cost about what a round of 256-row
        // tiles costs, a remainder of up to 256 (one per CU) about 0.6 of it.  Take them when
        // that is clearly less machine time.
        const int64_t t128 = (M + 127) / 128 * gn;
        const double rounds256 = (double)(((M + 255) / 256 * gn + 255) / 256);
        const int64_t rem = t128 % 512;
        const double rounds128 = (double)(t128 / 512) + (rem == 0 ? 0.0 : rem <= 256 ? 0.6 : 1.0);
        pl.bm = rounds128 < 0.95 * rounds256 ? 128 : 256;
    }
    // too few output tiles for 256 CUs: split K as well (whole groups, at least 4 k-tiles each)
    const bool half = grouped && pl.bm == 128;   // 128-channel tiles, two workgroups per CU
    const int64_t tiles = (M + pl.bm - 1) / pl.bm * (half ? (N + 127) / 128 : gn);
    const int KT = (int)(K / TILE_K), tpg = (int)(G / TILE_K);
    pl.splits = 1;
    pl.kt_per_split = KT;
    if (tiles < (half ? 256 : 128) && KT >= 8) {
        // (rounded down: a few workgroups beyond 256 make a second generation that costs as much as
        // the first)
        const int want = (int)((half ? 512 : 256) / tiles);
        int unit = grouped ? tpg : 1;           // k-tiles that must stay together
        while (unit < 4) unit += grouped ? tpg : 1;
        int kps = (KT + want - 1) / want;
        kps = (kps + unit - 1) / unit * unit;
        if (kps < KT) {
            pl.kt_per_split = kps;
            pl.splits = (KT + kps - 1) / kps;
        }
    }
    pl.rs_bytes = grouped ? 0 : (size_t)pl.splits * M * sizeof(int32_t);
    pl.partial_bytes = pl.splits > 1 ? (size_t)pl.splits * M * N * sizeof(float) : 0;
    // More than one round of 512 resident 128 x 128 tiles with the last round at most half full: a round
    // costs the same however full it is, so the channels of the last round become a launch of their own
    // with K cut into ranges over (about) 512 workgroups, and a combine pass over that slice of Y.
    // (Per-channel layers do not gain: their rounds are short against the partial sums' traffic.)
    if (half && pl.splits == 1 && tiles > 512) {
        const int64_t gm = (M + 127) / 128, gn128 = (N + 127) / 128;
        const int64_t gn_main = tiles / 512 * 512 / gm;   // whole channel tiles that fill whole rounds
        const int64_t rem_tiles = (gn128 - gn_main) * gm;
        int unit = tpg;
        while (unit < 4) unit += tpg;
        // (measured: it pays where a round is long against the two extra launches and the partial sums --
        // K >= 5120 with the last round under a third full, K >= 10240 with it up to half full;
        // at K = 2048 it costs 20 %)
        const bool pays = (KT >= 40 && rem_tiles <= 160) || (KT >= 80 && rem_tiles <= 256);
        if (gn_main > 0 && rem_tiles > 0 && pays && KT >= 2 * unit) {
            const int want = (int)std::min<int64_t>(512 / rem_tiles, 4);
            int kps = (KT + want - 1) / want;
            kps = (kps + unit - 1) / unit * unit;
            const int sp = (KT + kps - 1) / kps;
            if (sp >= 2) {
                pl.rem_n = (int)(N - gn_main * 128);
                pl.rem_splits = sp;
                pl.rem_kt_per_split = kps;
                pl.partial_bytes = (size_t)sp * M * pl.rem_n * sizeof(float);
            }
        }
    }
    return pl;
}

int launch_gemm(const int8_t *Xq, const float *sx, ZeroPoint zp, int32_t *rs, int64_t M,
                const uint8_t *Wt, const float *step, const uint8_t *zero, int64_t N, int64_t K,
                int64_t G, void *Y, int y_dtype, int64_t ldy, int32_t *acc_out, float *partial,
                hipStream_t st, int plain)
{
    const bool grouped = G != K;
    if ((M + 63) / 64 * ((N + 255) / 256) * 64 > 0x7fffffLL || M * K > 0x7fffffffLL)
        return W4A8_ERR_SHAPE;
    if (gemm_mid_applies(M, N, K, G, zp.zx != nullptr))
        return launch_gemm_mid(Xq, sx, M, Wt, step, zero, N, K, Y, y_dtype, ldy, acc_out, st, plain);
    if (gemm_mid_pc_applies(M, N, K, G, zp.zx != nullptr))
        return launch_gemm_mid_pc(Xq, sx, rs, M, Wt, step, zero, N, K, Y, y_dtype, ldy, acc_out, st, plain);
    const GemmPlan pl = plan_gemm(M, N, K, G);
    if (!grouped) {
        const int64_t segs = M * pl.splits;
        hipLaunchKernelGGL(rowsum_kernel, dim3((unsigned)((segs + 3) / 4)), dim3(256), 0, st, Xq, M,
                           (int)K, pl.splits, pl.kt_per_split * TILE_K, rs);
        if (hipGetLastError() != hipSuccess) return W4A8_ERR_HIP;
    }
    int rc;
#define W4A8_GM(BM_, WM_, WN_, GR_, TWO_)                                                                \
    rc = launch_gemm_t<BM_, WM_, WN_, GR_, TWO_>(pl, Xq, sx, zp, rs, M, Wt, step, zero, N, K, G, Y, y_dtype, ldy, \
                                            acc_out, partial, st, plain)
    // more workgroups than CUs: the 128-token per-channel tile in its two-per-CU form
    const int64_t wgs = (M + pl.bm - 1) / pl.bm * ((N + GM_BN - 1) / GM_BN) * pl.splits;
    if (grouped) {
        // 128-token group-wise tiles are 128 channels wide, four waves of 128 x 32, two workgroups per CU:
        // the same two waves per SIMD as one 256-channel workgroup, but from workgroups that do not share
        // a barrier, so that one's rescale (vector ALU only) drifts under the other's MFMAs
        if (pl.bm == 64) {
            W4A8_GM(64, 1, 4, true, false);
        } else if (pl.rem_n == 0) {
            rc = launch_gemm_t<128, 1, 4, true, false, 128>(pl, Xq, sx, zp, rs, M, Wt, step, zero, N, K, G, Y, y_dtype,
                                                            ldy, acc_out, partial, st, plain);
        } else {
            // whole rounds of tiles first, then the last channels with K in ranges (plan_gemm); every
            // parameter array is per output channel, the tiled weights are channel-tile major
            const int64_t n1 = N - pl.rem_n, ng = K / G, KT = K / TILE_K;
            GemmPlan p1 = pl;
            p1.splits = 1;
            p1.kt_per_split = (int)KT;
            rc = launch_gemm_t<128, 1, 4, true, false, 128>(p1, Xq, sx, zp, rs, M, Wt, step, zero, n1, K, G, Y, y_dtype,
                                                            ldy, acc_out, nullptr, st, plain, N);
            if (rc != W4A8_OK) return rc;
            GemmPlan p2 = pl;
            p2.splits = pl.rem_splits;
            p2.kt_per_split = pl.rem_kt_per_split;
            ZeroPoint zp2 = zp;
            if (zp.zx != nullptr) {
                zp2.wsum = zp.wsum + n1 * ng;
                zp2.tsum = zp.tsum + n1 * KT;
            }
            uint16_t *y2 = (uint16_t *)Y + n1;
            rc = launch_gemm_t<128, 1, 4, true, false, 128>(
                p2, Xq, sx, zp2, rs, M, Wt + n1 / TILE_N * KT * TILE_BYTES, step + n1 * ng, zero + n1 * ng, pl.rem_n, K, G,
                y2, y_dtype, ldy, acc_out ? acc_out + n1 * ng : nullptr, partial, st, plain, N);
            if (rc != W4A8_OK) return rc;
            return launch_gemv_combine(partial, sx, nullptr, ZeroPoint{nullptr, nullptr, nullptr}, M, pl.rem_n,
                                       pl.rem_splits, y2, y_dtype, ldy, st);
        }
    } else {
        if (pl.bm == 128 && wgs > 256) W4A8_GM(128, 1, 8, false, true);
        else if (pl.bm == 128) W4A8_GM(128, 1, 8, false, false);
        else W4A8_GM(256, 2, 4, false, false);
    }
#undef W4A8_GM
    if (rc != W4A8_OK || pl.splits == 1) return rc;
    return launch_gemv_combine(partial, sx, nullptr, ZeroPoint{nullptr, nullptr, nullptr}, M, N,
                               pl.splits, Y, y_dtype, ldy, st);
}

}  // namespace w4a8
