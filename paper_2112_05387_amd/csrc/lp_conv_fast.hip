// bf16 implicit-GEMM convolution (forward / data-gradient) for the wide layers on gfx950.
//
// Each wave owns a 64-pixel x 160-channel output tile (2 x 5 micro-tiles of v_mfma_f32_32x32x16_bf16, 160 fp32
// accumulators); a block is WGM x WGN waves: eight (512x160 or 256x320 tiles), or four (128x320) or two (128x160)
// for launches that would otherwise have fewer tiles than the chip has CUs.  What was measured on the
// machine and shaped this kernel:
//  * an MFMA loop fed from LDS is bound by LDS bandwidth (about 128 B/clk/CU), so the wave tile is as large
//    as the register file allows at two waves per SIMD;
//  * one k-tile of register-staged prefetch does not cover a miss to HBM, and every k-tile waits for its
//    slowest load, so operands go global -> LDS directly (buffer_load ... lds, no staging registers) into a
//    ring of STAGES k-tiles, with STAGES-1 tiles of loads in flight;
//  * LDS rows are unpadded (64 B = 32 bf16) with an XOR swizzle of the 16-byte chunk, conflict-free for the
//    fragment reads; the direct loads write lane l at slab + 16*l, so the swizzle is applied by choosing which
//    global chunk each lane fetches;
//  * the output tile goes back through LDS so that global stores are 16 bytes per lane and coalesced, and the
//    per-channel batch statistics are taken from the staged values on the way out.
// The zero padding of the convolution and the ragged edges of the GEMM are out-of-range buffer offsets, which
// the hardware returns (and writes to LDS) as zeros.
//
// k-tiles of 64 channels (128-byte rows, two ring stages) are used where Cin allows: a CU's L1 accepts about one
// cache line per four clocks whatever part of the line is used, so the 64-byte gathers of the 32-channel k-tile
// reach half the bytes per clock of 128-byte ones.
//
// Restrictions (the caller falls back to the general kernel otherwise): bf16, Cin % BK == 0 (a k-tile lies
// inside one filter tap, so the tap geometry is wave-uniform), at most 32 taps, tensors < 2 GiB.
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
__global__ __launch_bounds__(WGM * WGN * 64) void conv_igemm_fast_kernel(const ConvGroup g) {
    constexpr int MT = 32, FM = 2, FN = 5, NW = WGM * WGN, NT = NW * 64;
    static_assert(NW == 8 || NW == 4 || NW == 2, "eight waves (two per SIMD), four or two");
    static_assert(BK == 32 || BK == 64, "k-tile of 32 or 64 channels");
    constexpr int TM = FM * MT, TN = FN * MT, BM = WGM * TM, BN = WGN * TN;
    constexpr int ROWB = BK * 2;                      // bytes of an LDS row (one tile row, BK channels)
    constexpr int RPS = 1024 / ROWB;                  // rows per 1 KiB slab (one wave-load): 16 or 8
    constexpr int CPR = ROWB / 16;                    // 16-byte chunks per row: 4 or 8
    constexpr int KS = BK / 16;                       // MFMA k-steps per k-tile
    constexpr int A_BYTES = BM * ROWB, STAGE_BYTES = (BM + BN) * ROWB;
    constexpr int NSA = BM / RPS / NW;                // slabs of A per wave
    constexpr int NSBT = BN / RPS;                    // slabs of B in total
    constexpr int NSB = (NSBT + NW - 1) / NW;         // per wave (the last one may be absent)
    constexpr int EP_PITCH = 336, EP_WAVE = 32 * EP_PITCH;
    constexpr int EP_BYTES = NW * EP_WAVE;            // epilogue staging, over the dead operand area
    constexpr int OP_BYTES = STAGES * STAGE_BYTES > EP_BYTES ? STAGES * STAGE_BYTES : EP_BYTES;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform by construction: keep it in an SGPR
    int pi = 0;
    for (int i = 1; i < g.nprob; ++i)
        if ((int)blockIdx.x >= g.p[i].tile_start) pi = i;
    const ConvProb& P = g.p[pi];
    const int t = blockIdx.x - P.tile_start;
    const int tile_n = t % P.tiles_n, tile_m = t / P.tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int M = P.M, Cin = P.Cin, IH = P.IH, IW = P.IW, ntr = P.ntr, nts = P.nts;
    const int per = P.OA * P.OB;
    // LDS map: [ring of STAGES x (A tile, B tile)] [output row offsets]
    int* s_rowoff = reinterpret_cast<int*>(smem + OP_BYTES);

    for (int r = tid; r < BM; r += NT) {
        const int m = m0 + r;
        s_rowoff[r] = m < M ? addr::out_row_offset(P, m) : -1;
    }

    const __amdgpu_buffer_rsrc_t rsrc_a = make_rsrc(P.in, (unsigned)((size_t)(M / per) * IH * IW * Cin * 2));
    const __amdgpu_buffer_rsrc_t rsrc_b = make_rsrc(P.wt, (unsigned)((size_t)P.Ncol * P.ldw * 2));

    // ---- gather state.  Slab s covers tile rows RPS*s .. RPS*s+RPS-1; lane l writes LDS slot (row RPS*s + l/CPR,
    // chunk l%CPR) and therefore fetches global chunk (l%CPR) ^ swizzle(row).  64-byte rows: swizzle(row) = (row>>2)&3;
    // 128-byte rows: (row>>1)&7, which inside a slab is 4*(s&1) + (l>>4), and s&1 = wave&1 for every slab of a wave.
    const int lrow = lane / CPR;
    const int kvg = addr::filter_kvg(BK, lane, wave);
    int a_base[NSA];
    unsigned a_mask[NSA];
#pragma unroll
    for (int i = 0; i < NSA; ++i) {
        const int m = m0 + RPS * (wave + NW * i) + lrow;
        a_base[i] = 0; a_mask[i] = 0u;
        if (m < M) {
            const addr::RowGeom rg = addr::row_geom(P, m);
            a_base[i] = addr::fast_row_base(P, rg, kvg);
            a_mask[i] = addr::fast_row_mask(P, rg);
        }
    }
    // filter rows at or beyond Ncol (ragged last column tile) are marked out of range per lane, in every round
    const addr::FilterRows frows = addr::filter_rows(n0, RPS, NW, wave, lrow, kvg, P.ldw, P.Ncol);
    const bool last_b = (wave + NW * (NSB - 1)) < NSBT;          // does this wave own a slab in the last round?

    const int nk = ntr * nts * (Cin / BK);
    int tr = 0, ts = 0, ci0 = 0, issued = 0;
    // One k-tile of direct-to-LDS loads, one wave-load at a time: a wave that issues a load stalls until the address
    // unit takes it (about 30 clocks per wave-load with every wave of the CU loading), so the loads are spread
    // between the MFMAs of the k-tile and the matrix core keeps running on what this and the other wave of the SIMD
    // issued before.  tile_begin fixes the tap geometry of the tile, issue_one(i) issues wave-load i of it.
    // Past the end every offset is out of range (zeros).
    bool t_live = false;
    unsigned t_offb = 0;
    int t_offa = 0, t_bit = 0;
    unsigned char* t_dst = smem;
    auto tile_begin = [&](int st) {
        t_live = issued < nk;
        t_offb = addr::filter_tap_offset(P, tr, ts, ci0);
        t_offa = addr::fast_tap_offset(P, tr, ts, ci0);
        t_bit = tr * nts + ts;
        t_dst = smem + st * STAGE_BYTES + wave * 1024;
        ++issued;
        // taps innermost: the shifted reads of one channel slab follow each other and hit the same cache lines
        if (++ts == nts) {
            ts = 0;
            if (++tr == ntr) { tr = 0; ci0 += BK; }
        }
    };
    auto issue_one = [&](int i) {
        if (i < NSA) {
            const unsigned off = (t_live && ((a_mask[i] >> t_bit) & 1u)) ? (unsigned)(a_base[i] + t_offa) : kOOB;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (lds_ptr_t)(t_dst + i * (NW * 1024)), 16, (int)off, 0, 0, 0);
        } else if (i < NSA + NSB) {
            const int j = i - NSA;
            if (j + 1 < NSB || last_b) {
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_b, (lds_ptr_t)(t_dst + A_BYTES + j * (NW * 1024)), 16,
                                                         (int)addr::filter_voffset(frows, j, t_live),
                                                         (int)addr::filter_soffset(frows, t_offb, j), 0, 0);
            }
        }
    };
    auto issue_loads = [&](int st) {
        tile_begin(st);
#pragma unroll
        for (int i = 0; i < NSA + NSB; ++i) issue_one(i);
    };

    // ---- fragment addressing: lane l reads tile row (l % 32) and chunk (2*ks + l/32) ^ swizzle(row) ----
    const int wm = wave / WGN, wn = wave % WGN;
    const int lr = lane & 31, lkc = lane >> 5;
    const int sw = BK == 32 ? ((lr >> 2) & 3) : ((lr >> 1) & 7);
    const int a_rd = (wm * TM + lr) * ROWB, b_rd = A_BYTES + (wn * TN + lr) * ROWB;
    int ck[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) ck[ks] = ((2 * ks + lkc) ^ sw) << 4;
    u32x4 af[2][FM], bf[2][FN];
    auto load_frags = [&](int st, int ks, int slot) {
        const unsigned char* T = smem + st * STAGE_BYTES + ck[ks];
#pragma unroll
        for (int i = 0; i < FM; ++i) af[slot][i] = *reinterpret_cast<const u32x4*>(T + a_rd + i * (MT * ROWB));
#pragma unroll
        for (int j = 0; j < FN; ++j) bf[slot][j] = *reinterpret_cast<const u32x4*>(T + b_rd + j * (MT * ROWB));
    };

    // acc[j][i]: rows = channels of micro-tile j, columns = pixels of micro-tile i (filters are the row operand, so
    // that a lane ends up with 4 consecutive channels of one pixel)
    f32x16 acc[FN][FM];
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

    __syncthreads();                     // row offsets visible; nothing in flight yet
    if (nk > 0) {
        const int LT = NSA + (last_b ? NSB : NSB - 1);         // loads per k-tile of this wave
        // Ring of STAGES k-tiles, all of them filled before the loop.  The barrier of an iteration sits BEFORE the
        // MFMAs of its last k-step (whose fragments are in registers by then): it says that every wave has read all
        // of stage st and that tile kt+1 is visible.  Behind it come the first fragments of tile kt+1 and the loads
        // of tile kt+STAGES into stage st, spread evenly over the MFMA pairs of one k-tile (the address unit takes
        // about as long for a tile's loads as the matrix core for its MFMAs): they start under the last k-step of this
        // iteration and end under the first k-steps of the next one.
#pragma unroll
        for (int s = 0; s < STAGES; ++s) issue_loads(s);
        wait_vmcnt_rt((STAGES - 1) * LT);                      // tile 0 landed: all but the STAGES-1 younger tiles
        __builtin_amdgcn_s_barrier();
        load_frags(0, 0, 0);
        int st = 0;                      // ring stage of tile kt
        constexpr int NL = NSA + NSB;    // wave-loads per k-tile
        constexpr int NSLOT = KS * FN;   // MFMA pairs of a k-tile = places to issue a load
        constexpr int PER = (NL + 2 * FN - 1) / (2 * FN);      // loads per place: the tile is issued within 2*FN places
        static_assert(NL <= PER * NSLOT, "more loads than places");
        t_live = false;                  // nothing pending before the first barrier of the loop
        for (int kt = 0; kt < nk; ++kt) {
#pragma unroll
            for (int ks = 0; ks + 1 < KS; ++ks) {
                load_frags(st, ks + 1, (ks + 1) & 1);          // next k-step's fragments behind these MFMAs
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < FN; ++j) {
#pragma unroll
                    for (int i = 0; i < FM; ++i) Mma<bf16_t, 32>::run(bf[ks & 1][j], af[ks & 1][i], acc[j][i]);
                    // slots FN.. of the tile whose issue began under the last k-step of the previous iteration
                    if (kt > 0) {
                        const int slot = FN + ks * FN + j;      // a constant after unrolling
#pragma unroll
                        for (int i = slot * PER; i < (slot + 1) * PER; ++i) issue_one(i);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            __builtin_amdgcn_s_waitcnt(0xc07f);                // lgkmcnt(0): the last fragments of stage st are in registers
            wait_vmcnt_rt((STAGES - 2) * LT);                  // tile kt+1 landed (this wave's share)
            __builtin_amdgcn_s_barrier();
            int nst = st + 1;
            if (nst == STAGES) nst = 0;
            if (kt + 1 < nk) load_frags(nst, 0, 0);
            tile_begin(st);                                    // tile kt+STAGES into the stage just freed
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < FN; ++j) {
#pragma unroll
                for (int i = 0; i < FM; ++i) Mma<bf16_t, 32>::run(bf[(KS - 1) & 1][j], af[(KS - 1) & 1][i], acc[j][i]);
#pragma unroll
                for (int i = j * PER; i < (j + 1) * PER; ++i) issue_one(i);
                __builtin_amdgcn_sched_barrier(0);
            }
            st = nst;
        }
        // the last tile_begin's loads that were due under the next iteration: issue what is left (all out of range)
#pragma unroll
        for (int i = FN * PER; i < NL; ++i) issue_one(i);
    }
    wait_vmcnt<0>();                     // the trailing (all out-of-range) loads still write zeros into the ring
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
hipError_t fast_launch(const ConvGroup& g, hipStream_t s) {
    constexpr int BM = WGM * 64, BN = WGN * 160;
    const size_t operands = std::max((size_t)STAGES * (BM + BN) * BK * 2, (size_t)WGM * WGN * 32 * 336);   // ring / epilogue staging
    const size_t lds = operands + BM * sizeof(int);
    static_assert((size_t)STAGES * (BM + BN) * BK * 2 + BM * sizeof(int) <= 160 * 1024, "LDS budget");
    static bool configured = false;
    auto kern = conv_igemm_fast_kernel<WGM, WGN, STAGES, BK>;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3(g.total_tiles), dim3(WGM * WGN * 64), lds, s, g);
    return hipGetLastError();
}

}  // namespace

CfgInfo conv_fast_cfg_info(int cfg) {
    switch (cfg) {
        case FAST_512x160: return {512, 160, 32};
        case FAST_128x320: return {128, 320, 32};
        case FAST_128x160: return {128, 160, 32};
        case FAST64_256x320: return {256, 320, 64};
        case FAST64_128x320: return {128, 320, 64};
        case FAST64_128x160: return {128, 160, 64};
        case FAST_256x160: return {256, 160, 32};
        case FAST64_256x160: return {256, 160, 64};
        default: return {256, 320, 32};
    }
}

hipError_t launch_conv_fast(const ConvGroup& g, int cfg, hipStream_t s) {
    if (g.total_tiles <= 0) return hipSuccess;
    switch (cfg) {
        case FAST_512x160: return fast_launch<8, 1, 3, 32>(g, s);
        case FAST_256x320: return fast_launch<4, 2, 4, 32>(g, s);
        case FAST_128x320: return fast_launch<2, 2, 4, 32>(g, s);
        case FAST_128x160: return fast_launch<2, 1, 4, 32>(g, s);
        case FAST64_256x320: return fast_launch<4, 2, 2, 64>(g, s);
        case FAST64_128x320: return fast_launch<2, 2, 2, 64>(g, s);
        case FAST64_128x160: return fast_launch<2, 1, 2, 64>(g, s);
        case FAST_256x160: return fast_launch<4, 1, 4, 32>(g, s);
        case FAST64_256x160: return fast_launch<4, 1, 2, 64>(g, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace lp
