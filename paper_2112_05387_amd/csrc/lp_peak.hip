// What the matrix cores of THIS device sustain: two synthetic kernels with the wave tile of the convolution kernels
// (eight waves per workgroup, two per SIMD, 2 x 5 micro-tiles of v_mfma_f32_32x32x16_bf16 per wave), timed by the
// caller.  Mode 0 issues nothing but MFMAs on register operands; mode 1 reads, for every k-step, the seven 16-byte
// operand fragments from LDS that a k-step of the convolution kernels reads (conflict-free, swizzled rows), so that
// the LDS traffic per MFMA is the kernels' own.  Each workgroup also records the shader-clock and the constant
// 100 MHz counter at its start and end, from which the caller derives the clock the chip ran at under that load.
// The published peak (2.5 PFLOP/s dense bf16) assumes 2.4 GHz; these kernels say what power management leaves of it.
#include "lp_kernels.h"
#include "lp_mma.h"

namespace lp {

template <int MODE>
__global__ __launch_bounds__(512) void mfma_peak_kernel(int iters, unsigned long long* __restrict__ clk, float* __restrict__ sink) {
    constexpr int FM = 2, FN = 5;
    __shared__ __attribute__((aligned(16))) unsigned char tile[(FM + FN) * 32 * 128];      // 7 operand pieces of 32 rows x 128 B
    const int lane = threadIdx.x & 63;
    // operand values with random signs and mantissas in +-[1, 2): the power an MFMA draws depends on its operands, and
    // all-equal operands would flatter the result
    auto rnd2 = [](unsigned i) {
        unsigned h = i * 2654435761u; h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
        return (h & 0x807f807fu) | 0x3f803f80u;
    };
    for (int i = threadIdx.x; i < (int)sizeof(tile) / 4; i += blockDim.x) reinterpret_cast<unsigned*>(tile)[i] = rnd2((unsigned)i + 7919u * blockIdx.x);
    __syncthreads();
    unsigned long long t0 = 0, r0 = 0;
    if (threadIdx.x == 0) { t0 = __builtin_readcyclecounter(); r0 = wall_clock64(); }
    f32x16 acc[FN][FM];
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;
    u32x4 af[FM], bf[FN];
#pragma unroll
    for (int i = 0; i < FM; ++i) af[i] = u32x4{rnd2(threadIdx.x * 8 + i), rnd2(threadIdx.x * 8 + i + 100000), rnd2(threadIdx.x * 8 + i + 200000), rnd2(threadIdx.x * 8 + i + 300000)};
#pragma unroll
    for (int j = 0; j < FN; ++j) bf[j] = u32x4{rnd2(threadIdx.x * 8 + j + 400000), rnd2(threadIdx.x * 8 + j + 500000), rnd2(threadIdx.x * 8 + j + 600000), rnd2(threadIdx.x * 8 + j + 700000)};
    // fragment addressing of the convolution kernels: lane l reads row l % 32, chunk (2*ks + l/32) ^ ((row >> 1) & 7)
    const int lr = lane & 31, lkc = lane >> 5, sw = (lr >> 1) & 7;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if constexpr (MODE == 1) {
                asm volatile("" ::: "memory");          // the tile is read again in every k-step, as the kernels' tiles are
                const int ck = ((2 * ks + lkc) ^ sw) << 4;
#pragma unroll
                for (int i = 0; i < FM; ++i) af[i] = *reinterpret_cast<const u32x4*>(tile + (i * 32 + lr) * 128 + ck);
#pragma unroll
                for (int j = 0; j < FN; ++j) bf[j] = *reinterpret_cast<const u32x4*>(tile + ((FM + j) * 32 + lr) * 128 + ck);
            }
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int i = 0; i < FM; ++i) Mma<bf16_t, 32>::run(bf[j], af[i], acc[j][i]);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) s += acc[j][i][r];
    if (s == -1.f) sink[0] = s;                       // keeps the accumulators alive; never true
    if (threadIdx.x == 0 && clk) {
        clk[2 * blockIdx.x] = __builtin_readcyclecounter() - t0;
        clk[2 * blockIdx.x + 1] = wall_clock64() - r0;
    }
}

hipError_t launch_mfma_peak(int mode, int blocks, int iters, unsigned long long* clk, float* sink, hipStream_t s) {
    if (mode == 0) hipLaunchKernelGGL(mfma_peak_kernel<0>, dim3(blocks), dim3(512), 0, s, iters, clk, sink);
    else hipLaunchKernelGGL(mfma_peak_kernel<1>, dim3(blocks), dim3(512), 0, s, iters, clk, sink);
    return hipGetLastError();
}

}  // namespace lp
