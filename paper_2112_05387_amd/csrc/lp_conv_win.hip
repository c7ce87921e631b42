// bf16 3x3 stride-1 convolution (forward / data-gradient of the same-size layers) for the wide layers on gfx950, with
// the input held in LDS as a window instead of being gathered once per filter tap.
//
// Why: a compute unit's L1 accepts about one cache-line request per four clocks, whatever part of the line is used.
// The implicit-GEMM kernel (lp_conv_fast.hip) gathers an A tile per (tap, channel slab): for a 512 x 160 tile and 32
// channels that is 672 line requests per 1280 matrix-core clocks, so the requests, not the MFMAs, set the pace.
// Here the tile is a band of whole image rows (or whole images); the band plus a one-pixel halo is loaded ONCE per
// channel slab ("window", rows of BK channels) and all nine taps read their A fragments from it at shifted pixel
// positions.  Per channel slab the requests drop from 9 x (BM + BN) to NP + 9 x BN (NP = window pixels, about
// 1.2 - 1.6 x BM), which leaves the matrix core as the bound.
//
// Layout of LDS: [window: NP rows of BK channels, rounded up to 1 KiB slabs][ring of STAGES filter tiles (BN rows of
// BK channels)][output row offsets]; the epilogue staging reuses the front.  Rows are unpadded with the XOR swizzle
// of the 16-byte chunk that makes sixteen consecutive rows conflict-free at any alignment (64-byte rows: (row>>2)&3,
// 128-byte rows: (row>>1)&7); the direct-to-LDS loads apply it by choosing which global chunk a lane fetches.
// Halo pixels outside the image are out-of-range buffer offsets (the hardware writes zeros).
//
// Pipeline: the window of a channel slab is single-buffered: after the last tap of a slab every wave has its last
// fragments in registers (barrier), the next window is requested, the last MFMAs run, and one more barrier makes the
// window visible.  Filter tiles run through their ring exactly as in the implicit-GEMM kernel.
//
// Restrictions (checked on the host, conv_win_ok): bf16, 3x3 taps at offsets -1..1, stride 1, input and output of the
// same H x W, BM a multiple of W and a tile either a band inside one image or a whole number of images,
// Cin % 32 == 0 (channel slabs of 64, the last one may be half).
#include <algorithm>

#include "lp_addr.h"
#include "lp_kernels.h"
#include "lp_mma.h"

namespace lp {

namespace {

using addr::kOOB;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
typedef __attribute__((address_space(3))) void* lds_ptr_t;

// s_waitcnt vmcnt(n) only (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] at [15:14])
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// s_waitcnt vmcnt(n) for a wave-uniform run-time n
__device__ __forceinline__ void wait_vmcnt_rt(int n) {
    switch (n) {
        case 0: wait_vmcnt<0>(); break;   case 1: wait_vmcnt<1>(); break;   case 2: wait_vmcnt<2>(); break;
        case 3: wait_vmcnt<3>(); break;   case 4: wait_vmcnt<4>(); break;   case 5: wait_vmcnt<5>(); break;
        case 6: wait_vmcnt<6>(); break;   case 7: wait_vmcnt<7>(); break;   case 8: wait_vmcnt<8>(); break;
        case 9: wait_vmcnt<9>(); break;   case 10: wait_vmcnt<10>(); break; case 11: wait_vmcnt<11>(); break;
        case 12: wait_vmcnt<12>(); break; case 13: wait_vmcnt<13>(); break; case 14: wait_vmcnt<14>(); break;
        case 15: wait_vmcnt<15>(); break; case 16: wait_vmcnt<16>(); break; case 17: wait_vmcnt<17>(); break;
        case 18: wait_vmcnt<18>(); break; case 19: wait_vmcnt<19>(); break; case 20: wait_vmcnt<20>(); break;
        default: wait_vmcnt<0>(); break;
    }
}

}  // namespace

template <int WGM, int WGN, int STAGES, int BK>
__global__ __launch_bounds__(WGM * WGN * 64) void conv_win_kernel(const ConvGroup g) {
    constexpr int MT = 32, FM = 2, FN = 5, NW = WGM * WGN, NT = NW * 64;
    static_assert(NW == 8, "eight waves: with one wave per SIMD the same tiles ran at half the rate per compute unit");
    static_assert(BK == 64, "channel slabs of 64 channels (a last half slab is allowed)");
    constexpr int TM = FM * MT, TN = FN * MT, BM = WGM * TM, BN = WGN * TN;
    constexpr int ROWB = BK * 2;                      // bytes of an LDS row
    constexpr int RPS = 1024 / ROWB;                  // rows per 1 KiB slab (one wave-load)
    constexpr int CPR = ROWB / 16;                    // 16-byte chunks per row
    constexpr int KS = BK / 16;                       // MFMA k-steps per tap
    constexpr int B_BYTES = BN * ROWB;
    constexpr int NSBT = BN / RPS;                    // slabs of a filter tile
    constexpr int NSB = (NSBT + NW - 1) / NW;         // per wave (the last one may be absent)
    constexpr int BPER = (NSB + FN - 1) / FN;         // filter loads issued behind each of the FN MFMA pairs of a k-step
    constexpr int NSWMAX = conv_win_max_slabs(BM, NW);   // window slabs per wave
    constexpr int EP_PITCH = 336, EP_WAVE = 32 * EP_PITCH;
    constexpr int EP_BYTES = NW * EP_WAVE;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int pi = 0;
    for (int i = 1; i < g.nprob; ++i)
        if ((int)blockIdx.x >= g.p[i].tile_start) pi = i;
    const ConvProb& P = g.p[pi];
    const int t = blockIdx.x - P.tile_start;
    const int tile_n = t % P.tiles_n, tile_m = t / P.tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int M = P.M, Cin = P.Cin;
    // tile = TH image rows: nseg segments of SH rows, each inside one image; window of a segment: (SH+2) x (W+2) pixels
    const addr::WinGeom wg = addr::win_geom(P, BM);
    const int per = wg.per, WW = wg.WW, NP = wg.NP;
    const int nslab = (NP + RPS - 1) / RPS;
    const int win_bytes = nslab * 1024;
    unsigned char* s_b = smem + win_bytes;
    const int ring_end = win_bytes + STAGES * B_BYTES;
    int* s_rowoff = reinterpret_cast<int*>(smem + (ring_end > EP_BYTES ? ring_end : EP_BYTES));
    unsigned* s_abase = reinterpret_cast<unsigned*>(s_rowoff + BM) + tid;     // [NSWMAX][NT]: window addresses of this lane

    for (int r = tid; r < BM; r += NT) {
        const int m = m0 + r;
        s_rowoff[r] = m < M ? addr::out_row_offset(P, m) : -1;
    }

    const int nimg = M / per;
    const __amdgpu_buffer_rsrc_t rsrc_a = make_rsrc(P.in, (unsigned)((size_t)nimg * per * Cin * 2));
    const __amdgpu_buffer_rsrc_t rsrc_b = make_rsrc(P.wt, (unsigned)((size_t)P.Ncol * P.ldw * 2));

    // ---- window loads: slab sl = wave + NW*i holds window pixels RPS*sl .. RPS*sl + RPS-1; lane l writes LDS slot
    // (pixel RPS*sl + l/CPR, chunk l%CPR) and fetches global chunk (l%CPR) ^ swizzle(pixel)
    // (kept in LDS: they are needed once per channel slab, and the registers are needed for the accumulators)
#pragma unroll 1
    for (int i = 0; i < NSWMAX; ++i) {
        const int wp = (wave + NW * i) * RPS + lane / CPR;
        const int f = BK == 64 ? ((wp >> 1) & 7) : ((wp >> 2) & 3);
        const int lc = (lane % CPR) ^ f;                 // logical 8-channel chunk of the slab this lane fetches
        s_abase[i * NT] = addr::win_slot_offset(P, wg, m0, wp, lc, CPR);     // 0xffffffff: no pixel behind this slot
    }
    // channel slabs: Cin / BK full ones and, when Cin is an odd multiple of BK/2, a last half slab whose upper
    // chunks are out of range (zeros) and whose upper k-steps are skipped
    const int nslabc = (Cin + BK - 1) / BK;
    const bool half_last = (Cin % BK) != 0;
    auto load_window = [&](int ci0) {
        const bool half = half_last && ci0 + BK > Cin;
#pragma unroll
        for (int i = 0; i < NSWMAX; ++i) {
            const int sl = wave + NW * i;
            if (sl < nslab) {
                const unsigned ab = s_abase[i * NT];
                const unsigned off = (ab == 0xffffffffu || (half && (ab >> 31))) ? kOOB : (ab & 0x7fffffffu) + (unsigned)(ci0 * 2);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (lds_ptr_t)(smem + sl * 1024), 16, (int)off, 0, 0, 0);
            }
        }
    };

    // ---- filter tiles (as in the implicit-GEMM kernel) ----
    const int lrow = lane / CPR;
    const int kvg = addr::filter_kvg(BK, lane, wave);
    const addr::FilterRows frows = addr::filter_rows(n0, RPS, NW, wave, lrow, kvg, P.ldw, P.Ncol);
    const bool last_b = (wave + NW * (NSB - 1)) < NSBT;
    const int nk = 9 * nslabc;
    const bool b_hi = kvg >= CPR / 2;
    // Order of the channel slabs: the sum over channels may run in any order.  With a half last slab, odd workgroups
    // start with it, so that the two halves of the chip reach their slab boundaries (where every workgroup requests a
    // whole window at once and waits for it) at different times.
    const int ci_first = (half_last && (blockIdx.x & 1)) ? (nslabc - 1) * BK : 0;
    const int ci_wrap = nslabc * BK;
    int tr = 0, ts = 0, ci0 = ci_first, issued = 0;
    bool t_live = false;
    unsigned t_offb = 0;
    unsigned char* t_dst = s_b;
    auto tile_begin = [&](int st) {
        t_live = issued < nk && !(b_hi && half_last && ci0 + BK > Cin);
        t_offb = addr::filter_tap_offset(P, tr, ts, ci0);
        t_dst = s_b + st * B_BYTES + wave * 1024;
        ++issued;
        if (++ts == 3) {
            ts = 0;
            if (++tr == 3) { tr = 0; ci0 += BK; if (ci0 >= ci_wrap) ci0 = 0; }
        }
    };
    auto issue_b = [&](int j) {
        if (j < NSB && (j + 1 < NSB || last_b)) {
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_b, (lds_ptr_t)(t_dst + j * (NW * 1024)), 16,
                                                     (int)addr::filter_voffset(frows, j, t_live),
                                                     (int)addr::filter_soffset(frows, t_offb, j), 0, 0);
        }
    };

    // ---- fragment addressing ----
    const int wm = wave / WGN, wn = wave % WGN;
    const int lr = lane & 31, lkc = lane >> 5;
    // a_row[i]: LDS byte offset of the window row this lane reads for micro-tile i at the current tap; it moves by a
    // wave-uniform number of rows from tap to tap (taps of a slab run ts-fastest, then tr, then wrap)
    int a_row[FM];
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        a_row[i] = addr::win_frag_row(P, wg, wm * TM + i * MT + lr, 0, 0) * ROWB;             // tap (0, 0)
    }
    const int swb4 = (BK == 32 ? ((lr >> 2) & 3) : ((lr >> 1) & 7)) << 4;
    const int b_rd = (wn * TN + lr) * ROWB;
    const int step_s = P.dws * ROWB;                                  // next tap in the same filter row
    const int step_r = (P.dhs * WW - 2 * P.dws) * ROWB;               // first tap of the next filter row
    const int step_w = (-2 * P.dhs * WW - 2 * P.dws) * ROWB;          // back to tap (0, 0)
    int rtr = 0, rts = 0;                             // tap of the tile being read
    auto next_tap = [&]() {
        int d = step_s;
        if (++rts == 3) {
            rts = 0; d = step_r;
            if (++rtr == 3) { rtr = 0; d = step_w; }
        }
#pragma unroll
        for (int i = 0; i < FM; ++i) a_row[i] += d;
    };
    // Fragments: the pixel operand (two micro-tiles) is double-buffered over k-steps; each of the five filter
    // fragments is refilled in place for the next k-step right after its two MFMAs, so the other four fragments'
    // MFMAs cover the LDS latency and only one set of filter fragments occupies registers.
    u32x4 af[2][FM], bf[FN];
    auto load_a = [&](int ks, int slot) {
        const int q = (2 * ks + lkc) << 4;
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            // swizzle of the row: (row >> 2) & 3 for 64-byte rows, (row >> 1) & 7 for 128-byte rows, times 16
            const int asw = BK == 64 ? ((a_row[i] >> 4) & 0x70) : ((a_row[i] >> 4) & 0x30);
            af[slot][i] = *reinterpret_cast<const u32x4*>(smem + a_row[i] + (q ^ asw));
        }
    };
    auto load_b = [&](int st, int ks, int j) {
        const int q = (2 * ks + lkc) << 4;
        bf[j] = *reinterpret_cast<const u32x4*>(s_b + st * B_BYTES + (q ^ swb4) + b_rd + j * (MT * ROWB));
    };

    f32x16 acc[FN][FM];
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

    __syncthreads();                     // row offsets and window addresses visible; nothing in flight yet
    if (nk > 0) {
        const int LT = last_b ? NSB : NSB - 1;                 // filter loads per tile of this wave
        load_window(ci_first);
#pragma unroll
        for (int s = 0; s < STAGES; ++s) {
            tile_begin(s);
#pragma unroll
            for (int j = 0; j < NSB; ++j) issue_b(j);
        }
        wait_vmcnt_rt((STAGES - 1) * LT);                      // the window and tile 0 landed (they are the oldest)
        __builtin_amdgcn_s_barrier();
        load_a(0, 0);
#pragma unroll
        for (int j = 0; j < FN; ++j) load_b(0, 0, j);
        int st = 0, tap = 0, rci = ci_first;                   // ring stage, tap and channel slab of tile kt
        t_live = false;
        for (int kt = 0; kt < nk; ++kt) {
            // a tile of the half slab has KS/2 k-steps: the first ones and, in the code of the last one below, k-step
            // KS/2-1, whose fragments sit in the slot the last k-step reads ((KS/2-1) & 1 == (KS-1) & 1 for KS = 4)
            const bool short_tile = half_last && rci + BK > Cin;
#pragma unroll
            for (int ks = 0; ks + 1 < KS; ++ks) {
                if (short_tile && ks + 1 >= KS / 2) continue;
                load_a(ks + 1, (ks + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < FN; ++j) {
#pragma unroll
                    for (int i = 0; i < FM; ++i) Mma<bf16_t, 32>::run(bf[j], af[ks & 1][i], acc[j][i]);
                    load_b(st, ks + 1, j);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            const bool slab_end = tap == 8;
            const bool more = kt + 1 < nk;
            __builtin_amdgcn_s_waitcnt(0xc07f);                // lgkmcnt(0): the last fragments of this tile are in registers
            wait_vmcnt_rt((STAGES - 2) * LT);                  // filter tile kt+1 landed (this wave's share)
            __builtin_amdgcn_s_barrier();                      // every wave is done with stage st (and, at slab_end, with the window)
            int nst = st + 1;
            if (nst == STAGES) nst = 0;
            if (!slab_end) {
                next_tap();
                load_a(0, 0);
            } else if (more) {
                rci += BK;
                if (rci >= ci_wrap) rci = 0;
                load_window(rci);                              // ahead of the filter tile: the window is the older request
            }
            tile_begin(st);                                    // filter tile kt+STAGES into the stage just freed
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < FN; ++j) {
#pragma unroll
                for (int i = 0; i < FM; ++i) Mma<bf16_t, 32>::run(bf[j], af[(KS - 1) & 1][i], acc[j][i]);
                if (more) load_b(nst, 0, j);
#pragma unroll
                for (int q = j * BPER; q < (j + 1) * BPER; ++q) issue_b(q);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (slab_end && more) {
                wait_vmcnt<0>();                               // the new window (and whatever else was in flight) landed
                __builtin_amdgcn_s_barrier();
                next_tap();
                load_a(0, 0);
            }
            tap = slab_end ? 0 : tap + 1;
            st = nst;
        }
    }
    wait_vmcnt<0>();                     // trailing (all out-of-range) filter loads still write zeros into the ring
    __syncthreads();
    // ---- epilogue: registers -> (addends) -> bf16 -> LDS [pixel][channel] -> 16-byte coalesced stores + statistics ----
    bf16_t* __restrict__ out = reinterpret_cast<bf16_t*>(P.out);
    const bf16_t* __restrict__ add0 = reinterpret_cast<const bf16_t*>(P.add0);
    const bf16_t* __restrict__ add1 = reinterpret_cast<const bf16_t*>(P.add1);
    unsigned char* E = smem + wave * EP_WAVE;            // staging over the (dead) operand area; the host sizes LDS for it
    const int cg = lane % 20, pl = lane / 20;           // read-back: 16-byte channel group, pixel lane (pl == 3: idle)
    const int colg = n0 + wn * TN + cg * 8;
    float s1[8], s2[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { s1[e] = 0.f; s2[e] = 0.f; }
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int prow = wm * TM + i * MT;              // first tile row of this pixel group
        // Addends (skip connections of the data-gradient) come in the way the result goes out: the 32 x 160 piece of the
        // addend tensor is copied into the staging area with 16-byte accesses along the channels, and every lane then
        // picks the elements of its accumulators from LDS.  Read straight from memory in the accumulator layout, a
        // wave-load touched 32 rows for 16 bytes each, and the cache-line requests of the epilogue cost 10-15 us per launch.
#pragma unroll
        for (int which = 0; which < 2; ++which) {
            const bf16_t* __restrict__ ap = which == 0 ? add0 : add1;
            if (!ap) continue;
            constexpr int NLD = (MT + 2) / 3;           // rows per pixel lane
            u32x4 araw[NLD];
#pragma unroll
            for (int t = 0; t < NLD; ++t) {             // all loads first, unconditional (a row that is not there reads element 0)
                const int p = pl + 3 * t;
                const int ro = s_rowoff[prow + (p < MT ? p : MT - 1)];
                const bool ok = pl < 3 && p < MT && ro >= 0 && colg < P.Ncol;
                araw[t] = *reinterpret_cast<const u32x4*>(ap + (ok ? (size_t)ro + colg : (size_t)0));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < NLD; ++t) {
                const int p = pl + 3 * t;
                const int ro = s_rowoff[prow + (p < MT ? p : MT - 1)];
                const bool ok = ro >= 0 && colg < P.Ncol;
                u32x4 q = araw[t];
#pragma unroll
                for (int e = 0; e < 4; ++e) q[e] = ok ? q[e] : 0u;
                if (pl < 3 && p < MT) *reinterpret_cast<u32x4*>(E + p * EP_PITCH + cg * 16) = q;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_s_waitcnt(0xc07f);         // lgkmcnt(0): the piece is in LDS
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    const int c0 = j * MT + 8 * rg + 4 * lkc;
                    const uint2 a = *reinterpret_cast<const uint2*>(E + lr * EP_PITCH + c0 * 2);
                    acc[j][i][rg * 4 + 0] += __uint_as_float(a.x << 16); acc[j][i][rg * 4 + 1] += __uint_as_float(a.x & 0xffff0000u);
                    acc[j][i][rg * 4 + 2] += __uint_as_float(a.y << 16); acc[j][i][rg * 4 + 3] += __uint_as_float(a.y & 0xffff0000u);
                }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            __builtin_amdgcn_s_waitcnt(0xc07f);         // read before the staging area is written again
        }
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int c0 = j * MT + 8 * rg + 4 * lkc;          // channel inside the wave tile
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[j][i][rg * 4 + e];
                uint2 pk;
                pk.x = pack_bf16x2(v[0], v[1]);
                pk.y = pack_bf16x2(v[2], v[3]);
                *reinterpret_cast<uint2*>(E + lr * EP_PITCH + c0 * 2) = pk;
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_s_waitcnt(0xc07f);             // lgkmcnt(0): this wave's LDS writes are done
        if (pl < 3) {
            for (int p = pl; p < MT; p += 3) {
                const u32x4 q = *reinterpret_cast<const u32x4*>(E + p * EP_PITCH + cg * 16);
                const int ro = s_rowoff[prow + p];
                if (ro >= 0) {
                    if (colg < P.Ncol) *reinterpret_cast<u32x4*>(out + (size_t)ro + colg) = q;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float lo = __uint_as_float(q[e] << 16), hi = __uint_as_float(q[e] & 0xffff0000u);
                        s1[2 * e] += lo; s2[2 * e] += lo * lo;
                        s1[2 * e + 1] += hi; s2[2 * e + 1] += hi * hi;
                    }
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_s_waitcnt(0xc07f);             // reads done before the next group overwrites the staging area
    }
    if (P.stats) {
        __syncthreads();                                // every wave is done with its staging area
        float* red = reinterpret_cast<float*>(smem);    // [wave][pl][160][2]
        if (pl < 3) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                red[(((wave * 3 + pl) * TN) + cg * 8 + e) * 2 + 0] = s1[e];
                red[(((wave * 3 + pl) * TN) + cg * 8 + e) * 2 + 1] = s2[e];
            }
        }
        __syncthreads();
        for (int c = tid; c < BN; c += NT) {
            const int col = n0 + c;
            if (col < P.Ncol) {
                const int wn_c = c / TN, cc = c % TN;
                float a1 = 0.f, a2 = 0.f;
#pragma unroll
                for (int w = 0; w < WGM; ++w)
#pragma unroll
                    for (int q = 0; q < 3; ++q) {
                        const int idx = ((((w * WGN + wn_c) * 3 + q) * TN) + cc) * 2;
                        a1 += red[idx]; a2 += red[idx + 1];
                    }
                double* st = P.stats + (size_t)(blockIdx.x % stat_stripes(P.Ncol)) * 2 * P.Ncol;      // this workgroup's stripe
                atomicAdd(&st[col], (double)a1);
                atomicAdd(&st[P.Ncol + col], (double)a2);
            }
        }
    }
}


namespace {

template <int WGM, int WGN, int STAGES, int BK>
hipError_t win_launch(const ConvGroup& g, hipStream_t s) {
    constexpr int BM = WGM * 64, BN = WGN * 160, RPS = 1024 / (BK * 2);
    size_t lds = 0;
    for (int i = 0; i < g.nprob; ++i) {
        const ConvProb& c = g.p[i];
        const int TH = BM / c.OB, SH = std::min(TH, c.OA), nseg = TH / SH;
        const int NP = nseg * (SH + 2) * (c.OB + 2);
        const size_t ring_end = (size_t)((NP + RPS - 1) / RPS) * 1024 + (size_t)STAGES * BN * BK * 2;
        lds = std::max(lds, std::max(ring_end, (size_t)WGM * WGN * 32 * 336) + BM * sizeof(int) +
                                (size_t)conv_win_max_slabs(BM, WGM * WGN) * WGM * WGN * 64 * sizeof(unsigned));
    }
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    static bool configured = false;
    auto kern = conv_win_kernel<WGM, WGN, STAGES, BK>;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3(g.total_tiles), dim3(WGM * WGN * 64), lds, s, g);
    return hipGetLastError();
}

}  // namespace

CfgInfo conv_win_cfg_info(int cfg) {
    switch (cfg) {
        case WIN64_512x160: return {512, 160, 64};
        default: return {256, 320, 64};
    }
}

hipError_t launch_conv_win(const ConvGroup& g, int cfg, hipStream_t s) {
    if (g.total_tiles <= 0) return hipSuccess;
    switch (cfg) {
        case WIN64_512x160: return win_launch<8, 1, 2, 64>(g, s);
        case WIN64_256x320: return win_launch<4, 2, 2, 64>(g, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace lp
