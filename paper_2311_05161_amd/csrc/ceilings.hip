// Measured ceilings of the machine, for the bench to print beside the nominal peaks: what a plain
// streaming read reaches on the box the kernels are timed on, what a register-resident loop of
// the int8 MFMA that the prefill kernel is built on reaches, and what the instruction mix of the
// group-wise tile kernel's k-tile costs with and without its LDS fragment reads.  None is a step of the
// W4A8 path (Eq. 1 / Eq. 5 are computed by the other files); they only put the roofline fractions in context.
#include "w4a8_common.hpp"

namespace w4a8 {

typedef int v16i_c __attribute__((ext_vector_type(16)));

constexpr int SR_THREADS = 512;
constexpr int SR_BLOCKS = 256 * 2;
constexpr int SR_UNROLL = 4;   // 16-byte loads in flight per lane

// Every lane streams 16-byte pieces, a wave 1 KB per instruction, the grid a contiguous window of
// SR_BLOCKS x SR_THREADS x SR_UNROLL x 16 bytes per round.  The loaded words are folded into one
// value per lane that is stored only if it equals a value it never takes in practice, so that the
// loads cannot be removed and nothing is written.
__global__ __launch_bounds__(SR_THREADS) void stream_read_kernel(const v4u *__restrict__ src, int64_t n16,
                                                                uint32_t *__restrict__ sink)
{
    const int64_t stride = (int64_t)gridDim.x * SR_THREADS;
    int64_t i = (int64_t)blockIdx.x * SR_THREADS + threadIdx.x;
    uint32_t fold = 0;
    for (; i + (SR_UNROLL - 1) * stride < n16; i += SR_UNROLL * stride) {
        v4u v[SR_UNROLL];
#pragma unroll
        for (int u = 0; u < SR_UNROLL; ++u) v[u] = __builtin_nontemporal_load(&src[i + u * stride]);   // (streaming, as the decode kernel's weight loads)
#pragma unroll
        for (int u = 0; u < SR_UNROLL; ++u) fold ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < n16; i += stride) {
        const v4u v = __builtin_nontemporal_load(&src[i]);
        fold ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (fold == 0x9e3779b9u && sink != nullptr) sink[0] = fold;
}

constexpr int MF_THREADS = 256;
constexpr int MF_BLOCKS = 256 * 2;   // two workgroups of four waves per CU: two waves per SIMD
constexpr int MF_CHAINS = 8;         // independent accumulators per wave

// `iters` rounds of MF_CHAINS independent v_mfma_i32_32x32x32_i8 per wave, operands in registers.
__global__ __launch_bounds__(MF_THREADS) void mfma_i8_loop_kernel(int64_t iters, uint32_t *__restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    v4i a = {lane, lane + 1, lane + 2, lane + 3};
    v4i b = {lane * 3, lane * 5, lane * 7, lane * 11};
    v16i_c acc[MF_CHAINS];
#pragma unroll
    for (int c = 0; c < MF_CHAINS; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[c][r] = c;
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < MF_CHAINS; ++c)
            acc[c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[c], 0, 0, 0);
    }
    int fold = 0;
#pragma unroll
    for (int c = 0; c < MF_CHAINS; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) fold ^= acc[c][r];
    if (fold == 0x5bd1e995 && sink != nullptr) sink[0] = (uint32_t)fold;
}

// The instruction mix of one k-tile (= one 128-wide group) of the group-wise tile kernel, per wave: 16
// v_mfma_i32_32x32x32_i8 (four k-steps x four token blocks, each block's four MFMAs chained on its
// accumulators) with six independent vector instructions behind each (the nibble decode's share), then the
// rescale: one convert and one multiply-add per accumulator register (128 vector instructions that read
// the MFMA results).  FRAGS: each MFMA's second operand comes from LDS (one conflict-free ds_read_b128
// per MFMA, the kernel's swizzled fragment addresses, a 64 KB ring) instead of a register.  Two workgroups
// of four waves per CU, as the kernel runs.  What the pair of timings shows: in registers the matrix
// cores hide under the vector instructions; the fragment reads add their time on top.
constexpr int KM_THREADS = 256;
constexpr int KM_BLOCKS = 256 * 2;
template <bool FRAGS>
__global__ __launch_bounds__(KM_THREADS, 2) void ktile_mix_kernel(int64_t iters, float es, uint32_t *__restrict__ sink)
{
    __shared__ __attribute__((aligned(16))) uint8_t ring[FRAGS ? 65536 : 16];
    if (FRAGS) {
        for (int i = threadIdx.x; i < 65536 / 4; i += KM_THREADS) reinterpret_cast<int *>(ring)[i] = i;
        __syncthreads();
    }
    const int lane = threadIdx.x & 63;
    const int r32 = lane & 31, kh = lane >> 5;
    int frag_off[4];
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
        const int chunk = 2 * (2 * (s4 >> 1) + kh) + (s4 & 1);
        frag_off[s4] = r32 * 128 + ((chunk ^ ((r32 >> 1) & 7)) << 4);
    }
    const v4i a = {lane, 1, 2, 3}, b = {4, 5, 6, (int)blockIdx.x};
    const v16i_c z16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    v16i_c acc[4] = {z16, z16, z16, z16};
    float y[4][16];
#pragma unroll
    for (int ms = 0; ms < 4; ++ms)
#pragma unroll
        for (int r = 0; r < 16; ++r) y[ms][r] = 0.f;
    float f[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) f[r] = lane * 0.5f + r;
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
#pragma unroll
            for (int ms = 0; ms < 4; ++ms) {
                v4i bb = b;
                if (FRAGS) bb = *reinterpret_cast<const v4i *>(&ring[((int)it & 3) * 16384 + ms * 4096 + frag_off[s]]);
                acc[ms] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, bb, s == 0 ? z16 : acc[ms], 0, 0, 0);
#pragma unroll
                for (int v = 0; v < 6; ++v) f[(ms * 6 + v) & 7] = __builtin_fmaf(f[(ms * 6 + v) & 7], 1.0001f, 0.5f);
            }
#pragma unroll
            for (int ms = 0; ms < 4; ++ms) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ms = 0; ms < 4; ++ms)
#pragma unroll
            for (int r = 0; r < 16; ++r) y[ms][r] = __builtin_fmaf(es, (float)acc[ms][r], y[ms][r]);
        __builtin_amdgcn_sched_barrier(0);
    }
    float fold = 0.f;
#pragma unroll
    for (int r = 0; r < 8; ++r) fold += f[r];
#pragma unroll
    for (int ms = 0; ms < 4; ++ms)
#pragma unroll
        for (int r = 0; r < 16; ++r) fold += y[ms][r];
    if (fold == 12345.678f && sink != nullptr) sink[0] = __float_as_uint(fold);
}

int launch_stream_read(const void *buf, int64_t bytes, uint32_t *sink, hipStream_t st)
{
    hipLaunchKernelGGL(stream_read_kernel, dim3(SR_BLOCKS), dim3(SR_THREADS), 0, st,
                       reinterpret_cast<const v4u *>(buf), bytes / 16, sink);
    return hip_status(hipGetLastError());
}

int launch_mfma_i8_loop(int64_t iters, uint32_t *sink, int64_t *ops, hipStream_t st)
{
    if (ops != nullptr)
        *ops = (int64_t)MF_BLOCKS * (MF_THREADS / WAVE) * MF_CHAINS * iters * (2LL * 32 * 32 * 32);
    hipLaunchKernelGGL(mfma_i8_loop_kernel, dim3(MF_BLOCKS), dim3(MF_THREADS), 0, st, iters, sink);
    return hip_status(hipGetLastError());
}

int launch_ktile_mix(int64_t iters, int fragment_reads, uint32_t *sink, hipStream_t st)
{
    if (fragment_reads)
        hipLaunchKernelGGL((ktile_mix_kernel<true>), dim3(KM_BLOCKS), dim3(KM_THREADS), 0, st, iters, 0.5f, sink);
    else
        hipLaunchKernelGGL((ktile_mix_kernel<false>), dim3(KM_BLOCKS), dim3(KM_THREADS), 0, st, iters, 0.5f, sink);
    return hip_status(hipGetLastError());
}

}  // namespace w4a8
