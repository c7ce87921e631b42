// bf16 filter-gradient kernel for the wide 3x3 stride-1 layers on gfx950.
//
//   dW[co][r][s][ci] = sum over pixels m=(n,oh,ow) of dY[m][co] * X[n, oh+r-1, ow+s-1][ci]
//
// The reduction runs over pixels, and both operands are stored pixel-major ([pixel][channel]), so a k-tile of
// pixels of either operand is a run of whole channel rows: it is fetched with direct-to-LDS loads of 1 KiB per wave
// instruction (contiguous in memory, not the 64-byte gathers of the forward operand) and lands in LDS in its
// natural [pixel][channel] order.  The MFMA wants the reduction index contiguous inside a lane, i.e. the
// transpose; ds_read_tr16_b64 delivers exactly that: within 16 lanes it reads a 4-pixel x 16-channel block and
// hands lane c the 4 pixels of channel c.
//
// One block (768 threads, 12 waves, three per SIMD) owns a 160 (co) x 160 (ci) filter tile for the three taps of
// one filter row r and a chunk of the pixel range; partial sums are added to dW with fp32 atomics (split-K).
// Wave (wc, wj): co half wc, tap s = wj/2, ci half wj%2 -> an 80 x 80 tile of 5 x 5 v_mfma_f32_16x16x32_bf16
// micro-tiles (100 accumulators).
//
// A ring stage holds 64 pixels: the dY rows of pixels m0..m0+63 and ONE window of X shared by the three taps,
// the 66 pixels m0-1+(r-1)W .. m0+64+(r-1)W (flattened pixel index; tap s of pixel m reads window row m-m0+s).
// What the flattened window cannot express is patched in two places: window pixels whose image row is outside the
// image for this filter row are loaded as zeros (out-of-range offsets), and the column wrap of taps 0 and 2 (the
// left neighbour of column 0 is the last pixel of the previous row) is masked in the fragments.  One barrier per
// stage; inside a stage the two 32-pixel k-steps of a wave follow each other, so that after the first k-step the
// waves of a SIMD are out of phase and LDS reads overlap MFMAs.
// LDS rows are 320 B; the 32-byte channel pairs of a row swap places in rows with bit 3 set, which keeps the
// transposing reads of a half-wave (pixel rows p..p+3 and p+8..p+11) on distinct banks.
//
// Blocks are numbered XCD-major: the hardware deals consecutive block ids round-robin to the 8 XCDs, so logical
// neighbours (the filter-row and channel tiles that read the same pixel chunk) are given ids that are 8 apart and
// share one L2.
#include <algorithm>

#include "lp_kernels.h"
#include "lp_mma.h"

namespace lp {
namespace {

constexpr unsigned kOOB = 0x80000000u;      // byte offset beyond any buffer

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr_t;

template <int N> __device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// n / d for n < 2^31 with the (mul, shift) pair of fastdiv_make
__device__ __forceinline__ unsigned fastdiv(unsigned n, unsigned mul, unsigned shift) {
    return (__umulhi(n, mul) + n) >> shift;
}

constexpr int WF_NW = 12, WF_NT = 768, WF_BK = 64;   // pixels per ring stage (two MFMA k-steps of 32)
constexpr int WF_TILE = 160;                         // channels per operand tile
constexpr int WF_ROW = WF_TILE * 2;                  // bytes per LDS row
constexpr int WF_Y_BYTES = WF_BK * WF_ROW;           // dY rows of a stage: 20 KiB = 20 wave-loads
constexpr int WF_Y_SLABS = WF_Y_BYTES / 1024;
constexpr int WF_X_ROWS = WF_BK + 2;                 // window rows of a stage
constexpr int WF_X_SLABS = (WF_X_ROWS * WF_ROW + 1023) / 1024;     // 21 wave-loads
constexpr int WF_STAGE_BYTES = WF_Y_BYTES + WF_X_SLABS * 1024;
constexpr int WF_STAGES = 3;
constexpr int WF_SLABS = WF_Y_SLABS + WF_X_SLABS;    // 41 wave-loads per stage
constexpr int WF_LPW = (WF_SLABS + WF_NW - 1) / WF_NW;   // at most 4 per wave

}  // namespace

// (mul, shift) with n / d == (mulhi(n, mul) + n) >> shift for every n < 2^31 (d >= 1)
void fastdiv_make(unsigned d, unsigned* mul, unsigned* shift) {
    unsigned s = 0;
    while ((1ull << s) < d) ++s;
    *shift = s;
    *mul = (unsigned)((((1ull << s) - d) << 32) / d + 1);
}

// Parameter update of a finished 160 (co) x 3 taps x 160 (ci) gradient tile by the whole workgroup: 480 runs of up to 160
// consecutive channels.  Not inlined: the kernel's registers are allotted for its main loop, and this runs once per
// tile in one workgroup, after the accumulators are dead.
__device__ __attribute__((noinline)) void wgrad_fast_update_tile(void* w, float* vel, float* master, const float* dw, int co0,
                                                                 int ci0, int r, int Cin, int Cout, bool lowp, float lr,
                                                                 float momentum, float wd, int tid) {
    const SgdCoef c{lr, momentum, wd, lowp};
    const int nrows = 3 * min(WF_TILE, Cout - co0), ncols = min(WF_TILE, Cin - ci0);
    sgd_update_tile<WF_NT, 5>(w, vel, master, dw, nrows, ncols, true,
                              [=](int q) { const int co = co0 + q / 3, s = q - (q / 3) * 3; return ((size_t)co * 9 + r * 3 + s) * Cin + ci0; },
                              c, tid);
}

__global__ __launch_bounds__(WF_NT) void conv_wgrad_fast_kernel(const WgradGroup g) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int pi = 0;
    for (int i = 1; i < g.nprob; ++i)
        if ((int)blockIdx.x >= g.p[i].tile_start) pi = i;
    const WgradProb& P = g.p[pi];
    // XCD-major numbering (tile_start is a multiple of 8)
    const int T = P.tiles_m * P.tiles_n;
    const int nb = T * P.ksplit;
    const int local = blockIdx.x - P.tile_start;
    const int L = (local & 7) * ((nb + 7) >> 3) + (local >> 3);
    if (L >= nb) return;
    // (block-uniform quotients: the division runs on the vector ALU; readfirstlane puts the results into scalar registers)
    const int split = __builtin_amdgcn_readfirstlane(L / T), tile = L - split * T;
    const int tile_m = __builtin_amdgcn_readfirstlane(tile / P.tiles_n), tile_n = tile - tile_m * P.tiles_n;
    const int r = tile_n % 3, ci0 = (tile_n / 3) * WF_TILE, co0 = tile_m * WF_TILE;
    const int Cin = P.Cin, Cout = P.Cout, H = P.IH, W = P.IW;
    const int k_begin = split * P.kchunk;
    const int k_end = min(P.M, k_begin + P.kchunk);
    const int nk = (k_end - k_begin + WF_BK - 1) / WF_BK;

    const __amdgpu_buffer_rsrc_t rsrc_y = make_rsrc(P.dy, (unsigned)((size_t)P.M * Cout * 2));
    const __amdgpu_buffer_rsrc_t rsrc_x = make_rsrc(P.x, (unsigned)((size_t)P.M * Cin * 2));

    // ---- loads: wave-load q = wave + 12*i; q < 20: bytes [1024*q, +1024) of the dY rows, else of the X window.
    // Lane l supplies the 16 bytes that land at +16*l, i.e. row b/320 and the (swizzled) channel chunk of that row.
    // (Everything is recomputed per stage rather than kept in registers: the accumulators need them.)
    const int nld = wave + WF_NW * (WF_LPW - 1) < WF_SLABS ? WF_LPW : WF_LPW - 1;
    const int Mtot = P.M;
    // the division constants in scalar registers for good (left alone, the compiler re-reads them from the kernel
    // arguments inside the loops and every re-read is a wait on the scalar cache)
    unsigned mulW = P.mulW, shW = P.shW, mulH = P.mulH, shH = P.shH;
    asm volatile("" : "+s"(mulW), "+s"(shW), "+s"(mulH), "+s"(shH));
    auto issue_loads = [&](int st, int kt) {
        const int mt = k_begin + kt * WF_BK;                 // first pixel of the stage (beyond k_end: all zeros)
        const bool live = mt < k_end;
#pragma unroll
        for (int i = 0; i < WF_LPW; ++i) {
            const int q = wave + WF_NW * i;
            if (q < WF_SLABS) {
                const bool isx = q >= WF_Y_SLABS;
                const int b = (isx ? q - WF_Y_SLABS : q) * 1024 + lane * 16;
                const int row = b / WF_ROW, cb = b - row * WF_ROW;
                const int ce = ((((cb >> 5) ^ ((row >> 3) & 1)) << 5) | (cb & 31)) >> 1;   // first channel fetched
                bool ok = live;
                unsigned off;
                if (!isx) {
                    ok = ok && (co0 + ce < Cout) && (mt + row < k_end);
                    off = (unsigned)(((mt + row) * Cout + co0 + ce) * 2);
                } else {
                    // window pixel p; zero unless it exists and its image row hp has hp-(r-1) inside the image
                    const int p = mt + row - 1 + (r - 1) * W;
                    const unsigned t = fastdiv((unsigned)p, mulW, shW);
                    const int hp = (int)t - (int)fastdiv(t, mulH, shH) * H;
                    ok = ok && row < WF_X_ROWS && (ci0 + ce < Cin) && p >= 0 && p < Mtot && (unsigned)(hp - (r - 1)) < (unsigned)H;
                    off = (unsigned)((p * Cin + ci0 + ce) * 2);
                }
                if (!ok) off = kOOB;
                unsigned char* dst = smem + st * WF_STAGE_BYTES + q * 1024;
                if (!isx) __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_y, (lds_ptr_t)dst, 16, (int)off, 0, 0, 0);
                else __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_x, (lds_ptr_t)dst, 16, (int)off, 0, 0, 0);
            }
        }
    };

    // ---- fragment addressing (transposing reads): lane l, l' = l%16, g = l/16 supplies pixel row 8g + 4h + l'/4
    // (h = which half of the 8 reduction elements) and channels cbase + 4*(l'%4)..+3, and receives channel cbase + l'.
    // The 32-byte channel pair P of a row sits at pair slot P ^ s, s = bit 3 of the LDS row: P + s for even P, P - s
    // for odd P.  So a fragment address is one of two lane registers (even / odd pair) plus a compile-time offset.
    const int wc = wave & 1, wj = wave >> 1;
    const int tap_s = wj >> 1, half = wj & 1;
    const int lq = lane & 15, lg = lane >> 4;
    const int lrow = 8 * lg + (lq >> 2);                 // this lane's row inside a 32-pixel k-step (h = 0)
    // dY: pairs 5*wc + i, row bit 3 = g & 1 in both halves
    const int a_row_off = lrow * WF_ROW + 8 * (lq & 3) + 160 * wc;
    const int a_sw = (lg & 1) * 32;
    const int a_even = a_row_off + ((wc & 1) ? -a_sw : a_sw);      // pair parity of i = 0 is wc & 1
    const int a_odd = a_row_off + ((wc & 1) ? a_sw : -a_sw);
    const int b_row_off = WF_Y_BYTES + (lrow + tap_s) * WF_ROW + 8 * (lq & 3) + 160 * half;
    // The transposing LDS read as inline assembly with explicit lgkmcnt waits below.  Through the compiler's builtin
    // the read carries no memory operand, so the waitcnt pass cannot tell it from the in-flight direct-to-LDS loads
    // and puts s_waitcnt vmcnt(0) in front of it: every k-step then waited for the loads of the stage two ahead.
    auto tr_read = [&](const unsigned char* p) -> u32x2 {
        u32x2 r;
        const unsigned a = (unsigned)(uintptr_t)(lds_ptr_t)const_cast<unsigned char*>(p);
        asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(r) : "v"(a));
        return r;
    };

    f32x4 acc[5][5];
#pragma unroll
    for (int i = 0; i < 5; ++i)
#pragma unroll
        for (int j = 0; j < 5; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    if (nk > 0) {
        issue_loads(0, 0);
        issue_loads(1, 1);
        // this wave's share of stage 0 landed once at most one stage of its loads (nld of them) is outstanding
        if (nld == 4) wait_vmcnt<4>(); else wait_vmcnt<3>();
        __builtin_amdgcn_s_barrier();
        int st = 0;
        for (int kt = 0; kt < nk; ++kt) {
            int st_free = st + WF_STAGES - 1;
            if (st_free >= WF_STAGES) st_free -= WF_STAGES;
            issue_loads(st_free, kt + WF_STAGES - 1);          // into the stage that stage kt-1 used
            const unsigned char* S = smem + st * WF_STAGE_BYTES;
#pragma unroll 1
            for (int sub = 0; sub < 2; ++sub) {     // not unrolled: the second k-step's addresses would be kept in registers
                const unsigned char* Ss = S + sub * (32 * WF_ROW);
                // column wrap: pixel k of this lane's 8 reduction elements is invalid for tap 0 at column 0 and for
                // tap 2 at column W-1 (tap 1 never)
                unsigned km0 = 0xffffffffu, km1 = 0xffffffffu, km2 = 0xffffffffu, km3 = 0xffffffffu;
                if (tap_s != 1) {
                    const int k0 = k_begin + kt * WF_BK + sub * 32 + 8 * lg;
                    const int ow0 = k0 - (int)fastdiv((unsigned)k0, mulW, shW) * W;
                    const int bad = tap_s == 0 ? 0 : W - 1;
                    int e = bad - ow0;                        // first of this lane's 8 elements in the bad column
                    if (e < 0) e += W;
                    if (W >= 8) {
                        // at most one of the 8 is bad: one half of one mask register
                        const unsigned half = (e & 1) ? 0x0000ffffu : 0xffff0000u;
                        const int d = e >> 1;
                        km0 = d == 0 ? half : 0xffffffffu; km1 = d == 1 ? half : 0xffffffffu;
                        km2 = d == 2 ? half : 0xffffffffu; km3 = d == 3 ? half : 0xffffffffu;
                    } else {
                        unsigned bits = 0xffu;
                        for (; e < 8; e += W) bits &= ~(1u << e);
                        km0 = ((bits & 1u) ? 0xffffu : 0u) | ((bits & 2u) ? 0xffff0000u : 0u);
                        km1 = ((bits & 4u) ? 0xffffu : 0u) | ((bits & 8u) ? 0xffff0000u : 0u);
                        km2 = ((bits & 16u) ? 0xffffu : 0u) | ((bits & 32u) ? 0xffff0000u : 0u);
                        km3 = ((bits & 64u) ? 0xffffu : 0u) | ((bits & 128u) ? 0xffff0000u : 0u);
                    }
                }
                // The compiler does not know that the results of these reads are pending: nothing may touch them before
                // the s_waitcnt that covers them, and the empty asm behind that wait is where their values become
                // usable (it orders every use after the wait).  LDS reads return in order.
                u32x2 alo[5], ahi[5];
#pragma unroll
                for (int i = 0; i < 5; ++i) {
                    const unsigned char* pa = Ss + ((i & 1) ? a_odd : a_even) + 32 * i;
                    alo[i] = tr_read(pa);
                    ahi[i] = tr_read(pa + 4 * WF_ROW);
                }
                // window rows of this lane for h = 0 and h = 1; the pair swizzle follows the actual LDS row
                const int wr0 = 32 * sub + lrow + tap_s, wr1 = wr0 + 4;
                const int s0 = ((wr0 >> 3) & 1) * 32, s1 = ((wr1 >> 3) & 1) * 32;
                const unsigned char* B0 = Ss + b_row_off;
                const unsigned char* B1 = B0 + 4 * WF_ROW;
                // pair 5*half + j: its parity for j = 0 is half & 1
                const unsigned char* B0e = B0 + ((half & 1) ? -s0 : s0);
                const unsigned char* B0o = B0 + ((half & 1) ? s0 : -s0);
                const unsigned char* B1e = B1 + ((half & 1) ? -s1 : s1);
                const unsigned char* B1o = B1 + ((half & 1) ? s1 : -s1);
                // the X fragments one ahead of the MFMAs that use them (and no further: registers)
                u32x2 blo[5], bhi[5];
                blo[0] = tr_read(B0e); bhi[0] = tr_read(B1e);
                u32x4 af[5];
#pragma unroll
                for (int j = 0; j < 5; ++j) {
                    if (j + 1 < 5) {
                        blo[j + 1] = tr_read((((j + 1) & 1) ? B0o : B0e) + 32 * (j + 1));
                        bhi[j + 1] = tr_read((((j + 1) & 1) ? B1o : B1e) + 32 * (j + 1));
                        __builtin_amdgcn_s_waitcnt(0xc07f | (2 << 8));                 // lgkmcnt(2): all but the pair just issued
                    } else {
                        __builtin_amdgcn_s_waitcnt(0xc07f);                            // lgkmcnt(0)
                    }
                    if (j == 0) {
#pragma unroll
                        for (int i = 0; i < 5; ++i) {
                            asm volatile("" : "+v"(alo[i]), "+v"(ahi[i]));
                            af[i] = u32x4{alo[i][0], alo[i][1], ahi[i][0], ahi[i][1]};
                        }
                    }
                    asm volatile("" : "+v"(blo[j]), "+v"(bhi[j]));
                    const u32x4 bfj = {blo[j][0] & km0, blo[j][1] & km1, bhi[j][0] & km2, bhi[j][1] & km3};
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int i = 0; i < 5; ++i) Mma<bf16_t, 16>::run(af[i], bfj, acc[i][j]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (nld == 4) wait_vmcnt<4>(); else wait_vmcnt<3>();    // stage kt+1 landed (this wave's share)
            __builtin_amdgcn_s_barrier();                         // ... everyone's; and stage st is free again
            if (++st == WF_STAGES) st = 0;
        }
    }
    wait_vmcnt<0>();                     // trailing out-of-range loads still write zeros into LDS

    // ---- epilogue: partial sums -> dW[co][r][s][ci]
    float* __restrict__ dw = P.dw;
    const int tap = r * 3 + tap_s;
#pragma unroll
    for (int i = 0; i < 5; ++i)
#pragma unroll
        for (int j = 0; j < 5; ++j) {
            const int ci = ci0 + 80 * half + 16 * j + lq;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int co = co0 + 80 * wc + 16 * i + 4 * lg + e;
                if (co < Cout && ci < Cin) {
                    float* dst = dw + ((size_t)co * 9 + tap) * Cin + ci;
                    if (P.ksplit == 1) *dst = acc[i][j][e];
                    else atomicAdd(dst, acc[i][j][e]);
                }
            }
        }
    // ---- parameter update by the workgroup that completed this tile (Cin and Cout are multiples of 8: whole vectors)
    if (P.w) {
        __shared__ unsigned s_last;
        // the thread index afresh (not the one of the kernel's head: that would stay live through the main loop)
        const int t2 = wave * 64 + (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
        // This workgroup's partial sums must have been added before its ticket is taken: they are device-scope atomics
        // (performed at the memory side, not held in this XCD's L2), so waiting for their acknowledgement is all a release
        // needs here -- a device-scope fence would also write back and invalidate the whole L2 under the other workgroups
        // (measured: the step took 2.4 ms longer).
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
        if (P.ksplit > 1) {
            if (t2 == 0) s_last = __hip_atomic_fetch_add(P.cnt + tile, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (unsigned)(P.ksplit - 1);
            __syncthreads();
            if (!s_last) return;
        }
        wgrad_fast_update_tile(P.w, P.vel, P.master, dw, co0, ci0, r, Cin, Cout, g.lowp != 0, g.lr, g.momentum, g.wd, t2);
    }
}

// number of blocks the kernel is launched with for one problem (a multiple of 8: XCD-major numbering)
int wgrad_fast_blocks(const WgradProb& p) {
    const int nb = p.tiles_m * p.tiles_n * p.ksplit;
    return (nb + 7) / 8 * 8;
}

hipError_t launch_wgrad_fast(const WgradGroup& g, hipStream_t s) {
    if (g.total_tiles <= 0) return hipSuccess;
    const size_t lds = (size_t)WF_STAGES * WF_STAGE_BYTES;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void*)conv_wgrad_fast_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured = true;
    }
    hipLaunchKernelGGL(conv_wgrad_fast_kernel, dim3(g.total_tiles), dim3(WF_NT), lds, s, g);
    return hipGetLastError();
}

}  // namespace lp
