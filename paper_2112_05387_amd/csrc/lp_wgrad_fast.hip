// bf16 filter-gradient kernel for the wide 3x3 stride-1 layers on gfx950.
//
//   dW[co][r][s][ci] = sum over pixels m=(n,oh,ow) of dY[m][co] * X[n, oh+r-1, ow+s-1][ci]
//
// The reduction runs over pixels, and both operands are stored pixel-major ([pixel][channel]), so a k-tile of 32
// pixels of either operand is a run of whole channel rows: it is fetched with direct-to-LDS loads of 1 KiB per wave
// instruction (contiguous in memory, not the 64-byte gathers of the forward operand) and lands in LDS in its
// natural [pixel][channel] order.  The MFMA wants the reduction index contiguous inside a lane, i.e. the
// transpose; ds_read_tr16_b64 delivers exactly that: within 16 lanes it reads a 4-pixel x 16-channel block and
// hands lane c the 4 pixels of channel c.
//
// One block (768 threads, 12 waves, three per SIMD) owns a 160 (co) x 160 (ci) filter tile for the three taps of
// one filter row r and a chunk of the pixel range; partial sums are added to dW with fp32 atomics (split-K).
// Wave (wc, wj): co half wc, tap s = wj/2, ci half wj%2 -> an 80 x 80 tile of 5 x 5 v_mfma_f32_16x16x32_bf16
// micro-tiles (100 accumulators).  Per k-tile a block stages the dY tile and one X tile per tap (the same pixels
// shifted by one column; the zero padding is written by the loads themselves as out-of-range offsets).
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

constexpr int WF_NW = 12, WF_NT = 768, WF_BK = 32;
constexpr int WF_TILE = 160;                         // channels per operand tile
constexpr int WF_ROW = WF_TILE * 2;                  // bytes per LDS row
constexpr int WF_TILE_BYTES = WF_BK * WF_ROW;        // 10 KiB
constexpr int WF_STAGE_BYTES = 4 * WF_TILE_BYTES;    // dY + three taps of X
constexpr int WF_STAGES = 3;
constexpr int WF_SLABS = 4 * WF_TILE_BYTES / 1024;   // 40 wave-loads per stage
constexpr int WF_LPW = (WF_SLABS + WF_NW - 1) / WF_NW;   // at most 4 per wave

}  // namespace

// (mul, shift) with n / d == (mulhi(n, mul) + n) >> shift for every n < 2^31 (d >= 1)
void fastdiv_make(unsigned d, unsigned* mul, unsigned* shift) {
    unsigned s = 0;
    while ((1ull << s) < d) ++s;
    *shift = s;
    *mul = (unsigned)((((1ull << s) - d) << 32) / d + 1);
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
    const int split = L / T, tile = L - split * T;
    const int tile_m = tile / P.tiles_n, tile_n = tile - tile_m * P.tiles_n;
    const int r = tile_n % 3, ci0 = (tile_n / 3) * WF_TILE, co0 = tile_m * WF_TILE;
    const int Cin = P.Cin, Cout = P.Cout, H = P.IH, W = P.IW;
    const int k_begin = split * P.kchunk;
    const int k_end = min(P.M, k_begin + P.kchunk);
    const int nk = (k_end - k_begin + WF_BK - 1) / WF_BK;

    const __amdgpu_buffer_rsrc_t rsrc_y = make_rsrc(P.dy, (unsigned)((size_t)P.M * Cout * 2));
    const __amdgpu_buffer_rsrc_t rsrc_x = make_rsrc(P.x, (unsigned)((size_t)P.M * Cin * 2));

    // ---- load plan: wave-load q = wave + 12*i covers bytes [1024*(q%10), +1024) of operand tile q/10 of the stage;
    // lane l supplies the 16 bytes that land at +16*l, i.e. pixel row krow and (swizzled) channel chunk of that row.
    int ld_base[WF_LPW];      // byte offset of the lane's chunk for pixel 0 of the chunk's tap-shifted position
    int ld_krow[WF_LPW];      // pixel row inside the k-tile, or -1 if the lane's channels lie beyond the tensor
    int nld = 0;
#pragma unroll
    for (int i = 0; i < WF_LPW; ++i) {
        const int q = wave + WF_NW * i;
        ld_base[i] = 0; ld_krow[i] = -1;
        if (q < WF_SLABS) {
            ++nld;
            const int op = q / 10, slab = q - op * 10;
            const int b = slab * 1024 + lane * 16;
            const int krow = b / WF_ROW, cb = b - krow * WF_ROW;
            const int gb = ((((cb >> 5) ^ ((krow >> 3) & 1)) << 5) | (cb & 31));     // byte of the channel row fetched
            const int ce = gb >> 1;
            if (op == 0) {
                if (co0 + ce < Cout) { ld_krow[i] = krow; ld_base[i] = (krow * Cout + co0 + ce) * 2; }
            } else {
                if (ci0 + ce < Cin) { ld_krow[i] = krow; ld_base[i] = ((krow + (r - 1) * W + (op - 2)) * Cin + ci0 + ce) * 2; }
            }
        }
    }
    auto issue_loads = [&](int st, int kt) {
        const int mt = k_begin + kt * WF_BK;                 // first pixel of the k-tile (beyond k_end: all zeros)
#pragma unroll
        for (int i = 0; i < WF_LPW; ++i) {
            const int q = wave + WF_NW * i;
            if (q < WF_SLABS) {
                const int op = q / 10, slab = q - op * 10;
                const int m = mt + ld_krow[i];
                bool ok = ld_krow[i] >= 0 && m < k_end;
                unsigned off;
                if (op == 0) {
                    off = (unsigned)(ld_base[i] + mt * Cout * 2);
                } else {
                    const unsigned t = fastdiv((unsigned)m, P.mulW, P.shW);
                    const int ow = m - (int)t * W;
                    const int oh = (int)t - (int)fastdiv(t, P.mulH, P.shH) * H;
                    ok = ok && (unsigned)(oh + r - 1) < (unsigned)H && (unsigned)(ow + op - 2) < (unsigned)W;
                    off = (unsigned)(ld_base[i] + mt * Cin * 2);
                }
                if (!ok) off = kOOB;
                unsigned char* dst = smem + st * WF_STAGE_BYTES + op * WF_TILE_BYTES + slab * 1024;
                if (op == 0) __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_y, (lds_ptr_t)dst, 16, (int)off, 0, 0, 0);
                else __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_x, (lds_ptr_t)dst, 16, (int)off, 0, 0, 0);
            }
        }
    };

    // ---- fragment addressing (transposing reads): lane l, l' = l%16, g = l/16 supplies pixel row 8g + 4h + l'/4
    // (h = which half of the 8 reduction elements) and channels cbase + 4*(l'%4)..+3, and receives channel cbase + l'.
    const int wc = wave & 1, wj = wave >> 1;
    const int tap_s = wj >> 1, half = wj & 1;
    const int lq = lane & 15, lg = lane >> 4;
    const int row_off = (8 * lg + (lq >> 2)) * WF_ROW + 8 * (lq & 3);
    const int sw = lg & 1;
    int a_off[5], b_off[5];
#pragma unroll
    for (int i = 0; i < 5; ++i) {
        a_off[i] = row_off + (((5 * wc + i) ^ sw) << 5);
        b_off[i] = (1 + tap_s) * WF_TILE_BYTES + row_off + (((5 * half + i) ^ sw) << 5);
    }
    auto read_frag = [&](const unsigned char* base) -> u32x4 {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr_t)(lds_ptr_t)const_cast<unsigned char*>(base));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr_t)(lds_ptr_t)const_cast<unsigned char*>(base + 4 * WF_ROW));
        const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
        u32x4 f = {l2.x, l2.y, h2.x, h2.y};
        return f;
    };

    f32x4 acc[5][5];
#pragma unroll
    for (int i = 0; i < 5; ++i)
#pragma unroll
        for (int j = 0; j < 5; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    if (nk > 0) {
        issue_loads(0, 0);
        issue_loads(1, 1);
        // this wave's share of tile 0 landed once at most one tile of its loads (nld of them) is outstanding
        if (nld == 4) wait_vmcnt<4>(); else wait_vmcnt<3>();
        __builtin_amdgcn_s_barrier();
        int st = 0;
        for (int kt = 0; kt < nk; ++kt) {
            int st_free = st + WF_STAGES - 1;
            if (st_free >= WF_STAGES) st_free -= WF_STAGES;
            issue_loads(st_free, kt + WF_STAGES - 1);          // into the stage tile kt-1 used
            const unsigned char* S = smem + st * WF_STAGE_BYTES;
            u32x4 af[5];
#pragma unroll
            for (int i = 0; i < 5; ++i) af[i] = read_frag(S + a_off[i]);
#pragma unroll
            for (int j = 0; j < 5; ++j) {
                const u32x4 bfj = read_frag(S + b_off[j]);
#pragma unroll
                for (int i = 0; i < 5; ++i) Mma<bf16_t, 16>::run(af[i], bfj, acc[i][j]);
            }
            if (nld == 4) wait_vmcnt<4>(); else wait_vmcnt<3>();    // tile kt+1 landed (this wave's share)
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
