// Grouped implicit-GEMM convolution kernels for gfx950: forward / data-gradient (one kernel, the
// problem descriptor carries the tap geometry), weight-gradient (split over the reduction), the filter
// re-layout that the data-gradient needs, and a debug kernel that exposes the im2col address function.
//
// These are the products P dX_{m+1}/dX_m and P dF/dW of the discrete adjoint recursion and of the weight
// update (Sec. 4.1) and the convolutions inside F of the feature-flow equation; a dense contraction, so
// they run on the matrix cores: operands are staged through LDS as [row][k] tiles (k contiguous, padded
// pitch), read as 16-byte MFMA fragments, accumulated in fp32.
#include "lp_addr.h"
#include "lp_kernels.h"
#include "lp_mma.h"

namespace lp {

// -------------------------------------------------------------------------------------------------
// forward / data-gradient
// -------------------------------------------------------------------------------------------------
template <typename T, int BM, int BN, int BK, int WGM, int WGN, int MT, bool VEC>
__global__ __launch_bounds__(WGM* WGN * 64) void conv_igemm_kernel(const ConvGroup g) {
    constexpr int NT = WGM * WGN * 64;
    constexpr int EPV = 16 / (int)sizeof(T);
    constexpr int VPR = BK / EPV;
    constexpr int PITCH = BK + EPV;
    constexpr int A_VECS = BM * VPR, B_VECS = BN * VPR;
    constexpr int A_PER_T = (A_VECS + NT - 1) / NT, B_PER_T = (B_VECS + NT - 1) / NT;
    constexpr int TM = BM / WGM, TN = BN / WGN, FM = TM / MT, FN = TN / MT;
    static_assert(NT % VPR == 0, "k-chunk of a thread must not depend on the pass");
    static_assert(TM % MT == 0 && TN % MT == 0, "wave tile must be whole micro-tiles");
    typedef typename AccT<MT>::type acc_t;

    // both operands' buffers in one array: the epilogue stages the result tile over it
    // Narrow tiles (16 / 32 output channels) keep ONE operand buffer: their 256 rows of pixels are what fills the LDS, a
    // layer has 512 of them per 32 x 32 x 128 tensor, and with one buffer five workgroups fit a CU instead of three, so
    // that a launch is one generation of workgroups (measured: -15 % on the 16-channel layers; the second barrier per
    // k-tile costs nothing there, the kernel being bound by its chain of latencies, not by the k-loop).
    constexpr int NBUF = (BN <= 32) ? 1 : 2;
    __shared__ __attribute__((aligned(16))) T s_ab[NBUF * (BM + BN) * PITCH];
    T* const As0 = s_ab;
    T* const Bs0 = s_ab + NBUF * BM * PITCH;
    __shared__ int s_rowoff[BM];

    // ---- which problem, which tile ------------------------------------------------------------
    const int tid = threadIdx.x;
    int pi = 0;
    {
        const int bid = blockIdx.x;
        for (int i = 1; i < g.nprob; ++i)
            if (bid >= g.p[i].tile_start) pi = i;
    }
    const ConvProb& P = g.p[pi];
    const int t = blockIdx.x - P.tile_start;
    const int tile_n = t % P.tiles_n, tile_m = t / P.tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int M = P.M, Cin = P.Cin, IH = P.IH, IW = P.IW, ntr = P.ntr, nts = P.nts;
    const T* __restrict__ in = reinterpret_cast<const T*>(P.in);
    const T* __restrict__ wt = reinterpret_cast<const T*>(P.wt);

    // ---- per-row output offsets (also used by the epilogue) ---------------------------------------
    for (int r = tid; r < BM; r += NT) {
        const int m = m0 + r;
        s_rowoff[r] = m < M ? addr::out_row_offset(P, m) : -1;
    }

    // ---- per-thread gather state ---------------------------------------------------------------
    const int kv = tid % VPR;                // this thread's 16-byte k-chunk inside a k-tile
    addr::RowGeom a_g[A_PER_T];
#pragma unroll
    for (int i = 0; i < A_PER_T; ++i) {
        const int v = tid + i * NT;
        const int row = v / VPR;
        const int m = m0 + row;
        a_g[i].pix = 0; a_g[i].ih0 = -(1 << 28); a_g[i].iw0 = 0;       // a row that is not there: every tap outside
        if (v < A_VECS && m < M) a_g[i] = addr::row_geom(P, m);
    }
    int b_off[B_PER_T];
#pragma unroll
    for (int i = 0; i < B_PER_T; ++i) {
        const int v = tid + i * NT;
        const int col = n0 + v / VPR;
        b_off[i] = (v < B_VECS && col < P.Ncol) ? col * P.ldw : -1;
    }
    // (ci, tr, ts) of this thread's chunk, advanced by BK per k-tile (vector path only)
    int ci, tr, ts;
    {
        const int q0 = kv * EPV;
        const int tap = q0 / Cin;
        ci = q0 - tap * Cin;
        tr = tap / nts;
        ts = tap - tr * nts;
    }

    u32x4 a_reg[A_PER_T], b_reg[B_PER_T];
    auto load_tile = [&](int k0) {
        if constexpr (VEC) {
            const bool kok = tr < ntr;
            const int wk = ((P.r0 + P.rs * tr) * P.S + (P.s0 + P.ss * ts)) * Cin + ci;
#pragma unroll
            for (int i = 0; i < A_PER_T; ++i) {
                int ih, iw;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (addr::tap_inside(P, a_g[i], tr, ts, ih, iw) && kok)
                    v = *reinterpret_cast<const u32x4*>(in + addr::elem_offset(P, a_g[i], ih, iw, ci));
                a_reg[i] = v;
            }
#pragma unroll
            for (int i = 0; i < B_PER_T; ++i) {
                u32x4 v = {0u, 0u, 0u, 0u};
                if (kok && b_off[i] >= 0) v = *reinterpret_cast<const u32x4*>(wt + ((size_t)b_off[i] + wk));
                b_reg[i] = v;
            }
            // advance to the next k-tile
            ci += BK;
            while (ci >= Cin) {
                ci -= Cin;
                if (++ts == nts) { ts = 0; ++tr; }
            }
        } else {
            // element-wise gather: any Cin (used for the image-facing convolutions, Cin = 3)
            T av[A_PER_T][EPV], bv[B_PER_T][EPV];
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                const int q = k0 + kv * EPV + e;
                const int tap = q / Cin, c = q - tap * Cin;
                const int r = tap / nts, s = tap - r * nts;
                const bool kok = q < P.Kg;
                const int wk = ((P.r0 + P.rs * r) * P.S + (P.s0 + P.ss * s)) * Cin + c;
#pragma unroll
                for (int i = 0; i < A_PER_T; ++i) {
                    int ih, iw;
                    T v = from_float<T>(0.f);
                    if (addr::tap_inside(P, a_g[i], r, s, ih, iw) && kok)
                        v = in[addr::elem_offset(P, a_g[i], ih, iw, c)];
                    av[i][e] = v;
                }
#pragma unroll
                for (int i = 0; i < B_PER_T; ++i) {
                    T v = from_float<T>(0.f);
                    if (kok && b_off[i] >= 0) v = wt[(size_t)b_off[i] + wk];
                    bv[i][e] = v;
                }
            }
#pragma unroll
            for (int i = 0; i < A_PER_T; ++i) a_reg[i] = *reinterpret_cast<u32x4*>(&av[i][0]);
#pragma unroll
            for (int i = 0; i < B_PER_T; ++i) b_reg[i] = *reinterpret_cast<u32x4*>(&bv[i][0]);
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i) {
            const int v = tid + i * NT;
            if (A_VECS % NT == 0 || v < A_VECS)
                *reinterpret_cast<u32x4*>(As0 + buf * (BM * PITCH) + (v / VPR) * PITCH + kv * EPV) = a_reg[i];
        }
#pragma unroll
        for (int i = 0; i < B_PER_T; ++i) {
            const int v = tid + i * NT;
            if (B_VECS % NT == 0 || v < B_VECS)
                *reinterpret_cast<u32x4*>(Bs0 + buf * (BN * PITCH) + (v / VPR) * PITCH + kv * EPV) = b_reg[i];
        }
    };

    // ---- main loop: register-staged prefetch, double-buffered LDS ---------------------------------
    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WGN, wn = wave % WGN;
    acc_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < AccT<MT>::N; ++r) acc[i][j][r] = 0.f;

    const int nk = (P.Kg + BK - 1) / BK;
    load_tile(0);
    store_tile(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = NBUF == 2 ? (kt & 1) : 0;
        if (kt + 1 < nk) load_tile((kt + 1) * BK);
        mma_ktile<T, MT, FM, FN, BK, PITCH>(As0 + cur * (BM * PITCH), Bs0 + cur * (BN * PITCH), wm * TM, wn * TN, lane, acc);
        if (NBUF == 1) __syncthreads();
        if (kt + 1 < nk) store_tile(NBUF == 2 ? (cur ^ 1) : 0);
        __syncthreads();
    }

    // ---- epilogue: [+ addends] -> store; per-column sum / sum of squares -------------------------------
    // Every wave passes its result through a private LDS slice, one micro-tile row (MT pixels x TN channels) at a time:
    // the accumulators go in as they lie in the registers (a lane holds single elements of 4 or 16 pixels), and come out
    // as 16-byte vectors along the channels, so that addends are loaded and results stored with one 16-byte access per
    // lane instead of one 2- or 4-byte access per element (each of which the compiler followed by a full wait: the
    // addend loads of a data-gradient ran one after another).  The rounded values go back into the slice, where each lane
    // picks up its own elements again for the batch statistics, which describe the values as stored.
    T* __restrict__ out = reinterpret_cast<T*>(P.out);
    const T* __restrict__ add0 = reinterpret_cast<const T*>(P.add0);
    const T* __restrict__ add1 = reinterpret_cast<const T*>(P.add1);
    const int lc = lane % MT;
    float cs1[FN], cs2[FN];
#pragma unroll
    for (int j = 0; j < FN; ++j) { cs1[j] = 0.f; cs2[j] = 0.f; }
    constexpr int SP = TN + 4;                          // floats per slice row (16-byte aligned, staggers the banks)
    constexpr int G = TN / EPV;                         // output vectors per row
    constexpr int ITEMS = MT * G, IPL = (ITEMS + 63) / 64;
    static_assert(TN % EPV == 0, "wave tile columns must be whole vectors");
    static_assert((size_t)WGM * WGN * MT * SP * sizeof(float) <= sizeof(s_ab), "result slices must fit the operand buffers");
    float* const slice = reinterpret_cast<float*>(s_ab) + wave * (MT * SP);
    if (P.Ncol % EPV == 0) {
#pragma unroll
        for (int i = 0; i < FM; ++i) {
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int r = 0; r < AccT<MT>::N; ++r) slice[acc_row<MT>(r, lane) * SP + j * MT + lc] = acc[i][j][r];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            // all addend loads of this row first (a vector that does not exist reads element 0 and is dropped)
            u32x4 a0[IPL], a1[IPL];
            size_t off[IPL];
            bool ok[IPL];
#pragma unroll
            for (int t = 0; t < IPL; ++t) {
                const int item = lane + 64 * t;
                const int row = item / G, grp = item - row * G;
                const int ro = (ITEMS % 64 == 0 || item < ITEMS) ? s_rowoff[wm * TM + i * MT + row] : -1;
                const int col = n0 + wn * TN + grp * EPV;
                ok[t] = ro >= 0 && col < P.Ncol;
                off[t] = ok[t] ? (size_t)ro + col : (size_t)0;
                if (add0) a0[t] = *reinterpret_cast<const u32x4*>(add0 + off[t]);
                if (add1) a1[t] = *reinterpret_cast<const u32x4*>(add1 + off[t]);
            }
#pragma unroll
            for (int t = 0; t < IPL; ++t) {
                if (!ok[t]) continue;
                const int item = lane + 64 * t;
                const int row = item / G, grp = item - row * G;
                float* sp = slice + row * SP + grp * EPV;
                float v[EPV];
#pragma unroll
                for (int e = 0; e < EPV; e += 4) {
                    const f32x4 q = *reinterpret_cast<const f32x4*>(sp + e);
                    v[e] = q[0]; v[e + 1] = q[1]; v[e + 2] = q[2]; v[e + 3] = q[3];
                }
                u32x4 st;
                if constexpr (sizeof(T) == 4) {
                    if (add0) { const f32x4 a = __builtin_bit_cast(f32x4, a0[t]); v[0] += a[0]; v[1] += a[1]; v[2] += a[2]; v[3] += a[3]; }
                    if (add1) { const f32x4 a = __builtin_bit_cast(f32x4, a1[t]); v[0] += a[0]; v[1] += a[1]; v[2] += a[2]; v[3] += a[3]; }
                    st = u32x4{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (add0) { v[2 * e] += __uint_as_float(a0[t][e] << 16); v[2 * e + 1] += __uint_as_float(a0[t][e] & 0xffff0000u); }
                        if (add1) { v[2 * e] += __uint_as_float(a1[t][e] << 16); v[2 * e + 1] += __uint_as_float(a1[t][e] & 0xffff0000u); }
                        st[e] = pack_bf16x2(v[2 * e], v[2 * e + 1]);
                        v[2 * e] = __uint_as_float(st[e] << 16); v[2 * e + 1] = __uint_as_float(st[e] & 0xffff0000u);
                    }
                }
                *reinterpret_cast<u32x4*>(out + off[t]) = st;
#pragma unroll
                for (int e = 0; e < EPV; e += 4) *reinterpret_cast<f32x4*>(sp + e) = f32x4{v[e], v[e + 1], v[e + 2], v[e + 3]};
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if (P.stats) {
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    const int col = n0 + wn * TN + j * MT + lc;
#pragma unroll
                    for (int r = 0; r < AccT<MT>::N; ++r) {
                        const int prow = acc_row<MT>(r, lane);
                        if (s_rowoff[wm * TM + i * MT + prow] >= 0 && col < P.Ncol) {
                            const float vs = slice[prow * SP + j * MT + lc];
                            cs1[j] += vs;
                            cs2[j] += vs * vs;
                        }
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    } else {
        // output channel counts that are no multiple of a vector: element by element
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int col = n0 + wn * TN + j * MT + lc;
#pragma unroll
                for (int r = 0; r < AccT<MT>::N; ++r) {
                    const int row = wm * TM + i * MT + acc_row<MT>(r, lane);
                    const int ro = s_rowoff[row];
                    float v = acc[i][j][r];
                    if (ro >= 0 && col < P.Ncol) {
                        const size_t o = (size_t)ro + col;
                        if (add0) v += to_float(add0[o]);
                        if (add1) v += to_float(add1[o]);
                        const T st = from_float<T>(v);
                        out[o] = st;
                        const float vs = to_float(st);
                        cs1[j] += vs;
                        cs2[j] += vs * vs;
                    }
                }
            }
    }
    __syncthreads();                                    // the slices are done with before the statistics reuse the buffer
    if (P.stats) {
        float* red = reinterpret_cast<float*>(s_ab);           // [WGM][BN][2], operands and slices are dead by now
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            float s1 = cs1[j], s2 = cs2[j];
#pragma unroll
            for (int sh = MT; sh < 64; sh <<= 1) {
                s1 += __shfl_xor(s1, sh, 64);
                s2 += __shfl_xor(s2, sh, 64);
            }
            if (lane < MT) {
                const int c = wn * TN + j * MT + lane;
                red[(wm * BN + c) * 2 + 0] = s1;
                red[(wm * BN + c) * 2 + 1] = s2;
            }
        }
        __syncthreads();
        for (int c = tid; c < BN; c += NT) {
            const int col = n0 + c;
            if (col < P.Ncol) {
                float s1 = 0.f, s2 = 0.f;
#pragma unroll
                for (int w = 0; w < WGM; ++w) { s1 += red[(w * BN + c) * 2]; s2 += red[(w * BN + c) * 2 + 1]; }
                double* st = P.stats + (size_t)(blockIdx.x % stat_stripes(P.Ncol)) * 2 * P.Ncol;      // this workgroup's stripe
                atomicAdd(&st[col], (double)s1);
                atomicAdd(&st[P.Ncol + col], (double)s2);
            }
        }
    }
}

// -------------------------------------------------------------------------------------------------
// weight gradient
// -------------------------------------------------------------------------------------------------
// GEMM rows = output channels (operand dY, read as [m][co]), GEMM columns j = (r,s,ci) (operand X gathered
// as [m][ci] at the tap of j), reduction over m.  Both operands arrive with the reduction index slowest, so
// each thread loads 4 consecutive m rows of one 16-byte channel vector and writes the 4 x EPV block
// transposed, giving the same [row][k] LDS layout as the forward kernel.
template <typename T, int BM, int BN, int BK, int WGM, int WGN, int MT, bool VEC>
__global__ __launch_bounds__(WGM* WGN * 64) void conv_wgrad_kernel(const WgradGroup g) {
    constexpr int NT = WGM * WGN * 64;
    constexpr int EPV = 16 / (int)sizeof(T);
    constexpr int PITCH = BK + EPV;
    constexpr int RG = BK / 4;                         // row groups (4 reduction rows each) per k-tile
    constexpr int A_CV = BM / EPV, B_CV = BN / EPV;    // channel vectors per operand
    constexpr int A_GROUPS = A_CV * RG, B_GROUPS = B_CV * RG;
    constexpr int A_PER_T = (A_GROUPS + NT - 1) / NT, B_PER_T = (B_GROUPS + NT - 1) / NT;
    constexpr int TM = BM / WGM, TN = BN / WGN, FM = TM / MT, FN = TN / MT;
    static_assert(BM % EPV == 0 && BN % EPV == 0 && BK % 4 == 0, "tile shape");
    static_assert(TM % MT == 0 && TN % MT == 0, "wave tile must be whole micro-tiles");
    typedef typename AccT<MT>::type acc_t;

    constexpr int NBUF = (BM <= 64) ? 1 : 2;             // narrow filters: one operand buffer, twice the workgroups per CU (as in the forward kernel)
    __shared__ __attribute__((aligned(16))) T As[NBUF][BM * PITCH];
    __shared__ __attribute__((aligned(16))) T Bs[NBUF][BN * PITCH];

    const int tid = threadIdx.x;
    int pi = 0;
    for (int i = 1; i < g.nprob; ++i)
        if ((int)blockIdx.x >= g.p[i].tile_start) pi = i;
    const WgradProb& P = g.p[pi];
    int t = blockIdx.x - P.tile_start;
    const int tile_n = t % P.tiles_n; t /= P.tiles_n;
    const int tile_m = t % P.tiles_m;
    const int split = t / P.tiles_m;
    const int co0 = tile_m * BM, j0 = tile_n * BN;
    const int k_begin = split * P.kchunk;
    const int k_end = min(P.M, k_begin + P.kchunk);
    const int Cin = P.Cin, Cout = P.Cout, Kg = P.Kg, IH = P.IH, IW = P.IW, Ho = P.Ho, Wo = P.Wo;
    const T* __restrict__ x = reinterpret_cast<const T*>(P.x);
    const T* __restrict__ dy = reinterpret_cast<const T*>(P.dy);

    // thread -> (row group, channel vector); row group fastest so that the transposed LDS stores of a
    // wave spread over banks
    int a_rg[A_PER_T], a_cv[A_PER_T];
    bool a_ok[A_PER_T];
#pragma unroll
    for (int i = 0; i < A_PER_T; ++i) {
        const int gi = tid + i * NT;
        a_rg[i] = gi % RG; a_cv[i] = gi / RG;
        a_ok[i] = gi < A_GROUPS && (co0 + a_cv[i] * EPV) < Cout;
    }
    int b_rg[B_PER_T], b_cv[B_PER_T];
    int b_dh[B_PER_T][VEC ? 1 : EPV], b_dw[B_PER_T][VEC ? 1 : EPV], b_ci[B_PER_T][VEC ? 1 : EPV];
#pragma unroll
    for (int i = 0; i < B_PER_T; ++i) {
        const int gi = tid + i * NT;
        b_rg[i] = gi % RG; b_cv[i] = gi / RG;
#pragma unroll
        for (int e = 0; e < (VEC ? 1 : EPV); ++e) {
            const int j = j0 + b_cv[i] * EPV + e;
            if (gi < B_GROUPS && j < Kg) {
                const int tap = j / Cin;
                b_ci[i][e] = j - tap * Cin;
                const int r = tap / P.S;
                b_dh[i][e] = r - P.pad;
                b_dw[i][e] = (tap - r * P.S) - P.pad;
            } else {
                b_ci[i][e] = -1; b_dh[i][e] = 0; b_dw[i][e] = 0;
            }
        }
    }

    u32x4 a_reg[A_PER_T][4], b_reg[B_PER_T][4];
    auto load_tile = [&](int k0) {
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i) {
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int m = k0 + a_rg[i] * 4 + rr;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (a_ok[i] && m < k_end) v = *reinterpret_cast<const u32x4*>(dy + ((size_t)m * Cout + co0 + a_cv[i] * EPV));
                a_reg[i][rr] = v;
            }
        }
#pragma unroll
        for (int i = 0; i < B_PER_T; ++i) {
            const int mb = k0 + b_rg[i] * 4;
            // decode the first row of the group, then step
            const int per = Ho * Wo;
            int n = mb / per;
            int rem = mb - n * per;
            int ho = rem / Wo, wo = rem - ho * Wo;
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int m = mb + rr;
                if constexpr (VEC) {
                    u32x4 v = {0u, 0u, 0u, 0u};
                    const int ih = ho * P.stride + b_dh[i][0], iw = wo * P.stride + b_dw[i][0];
                    if (b_ci[i][0] >= 0 && m < k_end && (unsigned)ih < (unsigned)IH && (unsigned)iw < (unsigned)IW)
                        v = *reinterpret_cast<const u32x4*>(x + ((size_t)((n * IH + ih) * IW + iw) * Cin + b_ci[i][0]));
                    b_reg[i][rr] = v;
                } else {
                    T tmp[EPV];
#pragma unroll
                    for (int e = 0; e < EPV; ++e) {
                        const int ih = ho * P.stride + b_dh[i][e], iw = wo * P.stride + b_dw[i][e];
                        T v = from_float<T>(0.f);
                        if (b_ci[i][e] >= 0 && m < k_end && (unsigned)ih < (unsigned)IH && (unsigned)iw < (unsigned)IW)
                            v = x[(size_t)((n * IH + ih) * IW + iw) * Cin + b_ci[i][e]];
                        tmp[e] = v;
                    }
                    b_reg[i][rr] = *reinterpret_cast<u32x4*>(&tmp[0]);
                }
                if (++wo == Wo) { wo = 0; if (++ho == Ho) { ho = 0; ++n; } }
            }
        }
    };
    // transposed store of a 4 x EPV block: element e of the 4 rows -> LDS row (cv*EPV+e), k = rg*4..rg*4+3
    auto store_block = [&](T* dst, int cv, int rg, const u32x4 (&v)[4]) {
        if constexpr (sizeof(T) == 4) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                u32x4 o = {v[0][e], v[1][e], v[2][e], v[3][e]};
                *reinterpret_cast<u32x4*>(dst + (cv * EPV + e) * PITCH + rg * 4) = o;
            }
        } else {
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {       // dword e2 holds channels 2*e2 (low half) and 2*e2+1 (high half)
                const unsigned d0 = v[0][e2], d1 = v[1][e2], d2 = v[2][e2], d3 = v[3][e2];
                uint2 lo, hi;
                lo.x = (d0 & 0xffffu) | (d1 << 16);
                lo.y = (d2 & 0xffffu) | (d3 << 16);
                hi.x = (d0 >> 16) | (d1 & 0xffff0000u);
                hi.y = (d2 >> 16) | (d3 & 0xffff0000u);
                *reinterpret_cast<uint2*>(dst + (cv * EPV + 2 * e2) * PITCH + rg * 4) = lo;
                *reinterpret_cast<uint2*>(dst + (cv * EPV + 2 * e2 + 1) * PITCH + rg * 4) = hi;
            }
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i)
            if (A_GROUPS % NT == 0 || tid + i * NT < A_GROUPS) store_block(As[buf], a_cv[i], a_rg[i], a_reg[i]);
#pragma unroll
        for (int i = 0; i < B_PER_T; ++i)
            if (B_GROUPS % NT == 0 || tid + i * NT < B_GROUPS) store_block(Bs[buf], b_cv[i], b_rg[i], b_reg[i]);
    };

    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WGN, wn = wave % WGN;
    acc_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < AccT<MT>::N; ++r) acc[i][j][r] = 0.f;

    const int nk = (k_end - k_begin + BK - 1) / BK;
    if (nk > 0) {
        load_tile(k_begin);
        store_tile(0);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = NBUF == 2 ? (kt & 1) : 0;
        if (kt + 1 < nk) load_tile(k_begin + (kt + 1) * BK);
        mma_ktile<T, MT, FM, FN, BK, PITCH>(As[cur], Bs[cur], wm * TM, wn * TN, lane, acc);
        if (NBUF == 1) __syncthreads();
        if (kt + 1 < nk) store_tile(NBUF == 2 ? (cur ^ 1) : 0);
        __syncthreads();
    }

    if (nk > 0) {
        const int lc = lane % MT;
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int col = j0 + wn * TN + j * MT + lc;
#pragma unroll
                for (int r = 0; r < AccT<MT>::N; ++r) {
                    const int co = co0 + wm * TM + i * MT + acc_row<MT>(r, lane);
                    if (co < Cout && col < Kg) {
                        float* dst = P.dw + (size_t)co * Kg + col;
                        if (P.ksplit == 1) *dst = acc[i][j][r];
                        else atomicAdd(dst, acc[i][j][r]);
                    }
                }
            }
    }
    // ---- parameter update by the workgroup that completed this tile: BM runs of up to BN consecutive columns
    if (P.w) {
        __shared__ unsigned s_last;
        // This workgroup's partial sums must have been added before its ticket is taken: they are device-scope atomics
        // (performed at the memory side, not held in this XCD's L2), so waiting for their acknowledgement is all a release
        // needs here -- a device-scope fence would also write back and invalidate the whole L2 under the other workgroups
        // (measured: the step took 2.4 ms longer).
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
        if (P.ksplit > 1) {
            if (tid == 0) s_last = __hip_atomic_fetch_add(P.cnt + tile_m * P.tiles_n + tile_n, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (unsigned)(P.ksplit - 1);
            __syncthreads();
            if (!s_last) return;
        }
        const SgdCoef c{g.lr, g.momentum, g.wd, g.lowp != 0};
        const int nrows = min(BM, Cout - co0), ncols = min(BN, Kg - j0);
        sgd_update_tile<NT, 4>(P.w, P.vel, P.master, P.dw, nrows, ncols, (Kg & 3) == 0 && (ncols & 3) == 0,
                               [=](int q) { return (size_t)(co0 + q) * Kg + j0; }, c, tid);
    }
}

// -------------------------------------------------------------------------------------------------
// filter re-layout for the data-gradient: w[co][rs][ci] -> wt[ci][rs][co]
// -------------------------------------------------------------------------------------------------
template <typename T>
__global__ void wtrans_kernel(const WtransGroup g) {
    int pi = 0;
    for (int i = 1; i < g.nprob; ++i)
        if ((int)blockIdx.x >= g.p[i].block_start) pi = i;
    const WtransProb& P = g.p[pi];
    const T* __restrict__ w = reinterpret_cast<const T*>(P.w);
    T* __restrict__ wt = reinterpret_cast<T*>(P.wt);
    // 64 x 64 (co, ci) tile of one tap through LDS; both sides move 4 consecutive elements per thread (channel counts
    // are multiples of 4), so a wave reads and writes whole 128-byte (bf16) or 256-byte (fp32) rows
    constexpr int TS = 64;
    __shared__ T tile[TS][TS + 4];
    const int tiles_ci = (P.Cin + TS - 1) / TS, tiles_co = (P.Cout + TS - 1) / TS;
    int b = blockIdx.x - P.block_start;
    const int tci = b % tiles_ci; b /= tiles_ci;
    const int tco = b % tiles_co;
    const int rs = b / tiles_co;
    const int tx = (threadIdx.x % 16) * 4, ty = threadIdx.x / 16;   // 256 threads: 16 column groups x 16 rows
    struct alignas(4 * sizeof(T)) V4 { T v[4]; };
    for (int r = ty; r < TS; r += 16) {
        const int co = tco * TS + r, ci = tci * TS + tx;
        if (co < P.Cout && ci < P.Cin) {
            const V4 q = *reinterpret_cast<const V4*>(w + ((size_t)co * P.RS + rs) * P.Cin + ci);
#pragma unroll
            for (int e = 0; e < 4; ++e) tile[r][tx + e] = q.v[e];
        }
    }
    __syncthreads();
    for (int r = ty; r < TS; r += 16) {
        const int ci = tci * TS + r, co = tco * TS + tx;
        if (co < P.Cout && ci < P.Cin) {
            V4 q;
#pragma unroll
            for (int e = 0; e < 4; ++e) q.v[e] = tile[tx + e][r];
            *reinterpret_cast<V4*>(wt + ((size_t)ci * P.RS + rs) * P.Cout + co) = q;
        }
    }
}

// -------------------------------------------------------------------------------------------------
// debug kernels: the address functions the convolution kernels use (lp_addr.h), evaluated one sample per thread
// -------------------------------------------------------------------------------------------------
__global__ void im2col_offsets_kernel(const ConvProb P, const int64_t* __restrict__ ms, const int64_t* __restrict__ qs,
                                      int64_t* __restrict__ out, int count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    const int m = (int)ms[i], q = (int)qs[i];
    const int tap = q / P.Cin, ci = q - tap * P.Cin;
    const int tr = tap / P.nts, ts = tap - tr * P.nts;
    const addr::RowGeom rg = addr::row_geom(P, m);
    int ih, iw;
    int64_t o = -1;
    if (tr < P.ntr && addr::tap_inside(P, rg, tr, ts, ih, iw)) o = (int64_t)addr::elem_offset(P, rg, ih, iw, ci);
    out[i] = o;
}

// kernel: 0 conv_igemm_kernel, 1 conv_igemm_fast_kernel (tile height BM, k-tiles of bk channels, nw waves),
// 2 conv_win_kernel (tile height BM, 64-channel slabs).  For GEMM element (m, q = (tr*nts + ts)*Cin + ci) and
// filter row `col`: in_off = element offset of the activation the kernel's loads fetch for it (-1: zero padding),
// w_off = element offset of the filter element, out_off = element offset of output (m, column 0).
__global__ void conv_offsets_kernel(const ConvProb P, int kernel, int BM, int bk, int nw, const int64_t* __restrict__ ms,
                                    const int64_t* __restrict__ qs, const int64_t* __restrict__ cols,
                                    int64_t* __restrict__ in_off, int64_t* __restrict__ w_off, int64_t* __restrict__ out_off,
                                    int count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    const int m = (int)ms[i], q = (int)qs[i], col = (int)cols[i];
    const int tap = q / P.Cin, ci = q - tap * P.Cin;
    const int tr = tap / P.nts, ts = tap - tr * P.nts;
    const addr::RowGeom rg = addr::row_geom(P, m);
    int64_t o = -1;
    if (kernel == 0) {
        int ih, iw;
        if (addr::tap_inside(P, rg, tr, ts, ih, iw)) o = (int64_t)addr::elem_offset(P, rg, ih, iw, ci);
    } else if (kernel == 1) {
        // the lane of the row's wave-load that fetches the 16-byte chunk holding channel ci of the slab
        const int rps = 1024 / (bk * 2), cpr = bk * 2 / 16;
        const int r = m % BM, slab = r / rps, lrow = r % rps, wave = slab % nw;
        const int ci0 = ci - ci % bk, c8 = (ci % bk) / 8;
        int found = 0, kvg = -1;
        for (int x = 0; x < cpr; ++x) {
            const int k = addr::filter_kvg(bk, lrow * cpr + x, wave);
            if (k == c8) { ++found; kvg = k; }
        }
        if (found != 1) o = -2;                                  // the chunk permutation of a row is broken
        else if ((addr::fast_row_mask(P, rg) >> (tr * P.nts + ts)) & 1u)
            o = ((int64_t)addr::fast_row_base(P, rg, kvg) + addr::fast_tap_offset(P, tr, ts, ci0)) / 2 + ci % 8;
    } else {
        const addr::WinGeom wg = addr::win_geom(P, BM);
        const int m0 = m / BM * BM;
        const int wp = addr::win_frag_row(P, wg, m - m0, tr, ts);        // window pixel the fragment read addresses
        const int ci0 = ci / 64 * 64, c8 = (ci % 64) / 8;
        const unsigned ab = addr::win_slot_offset(P, wg, m0, wp, c8, 8);
        if (wp < 0 || wp >= wg.NP) o = -2;                               // a fragment read outside the window
        else if (ab != 0xffffffffu) o = ((int64_t)(ab & 0x7fffffffu) + ci0 * 2) / 2 + ci % 8;
    }
    in_off[i] = o;
    const int ci0w = ci - ci % bk;
    w_off[i] = (int64_t)col * P.ldw + addr::filter_tap_offset(P, tr, ts, ci0w) / 2 + (ci - ci0w);
    out_off[i] = addr::out_row_offset(P, m);
}

// -------------------------------------------------------------------------------------------------
// launchers
// -------------------------------------------------------------------------------------------------
namespace {
template <typename T> struct CfgK { static constexpr int BK = sizeof(T) == 2 ? 32 : 16; };

template <typename T, int BM, int BN, int BK, int WGM, int WGN, int MT, bool VEC>
hipError_t conv_launch_bk(const ConvGroup& g, hipStream_t s) {
    hipLaunchKernelGGL((conv_igemm_kernel<T, BM, BN, BK, WGM, WGN, MT, VEC>), dim3(g.total_tiles), dim3(WGM * WGN * 64), 0, s, g);
    return hipGetLastError();
}
template <typename T, int BM, int BN, int WGM, int WGN, int MT, bool VEC>
hipError_t conv_launch(const ConvGroup& g, hipStream_t s) {
    hipLaunchKernelGGL((conv_igemm_kernel<T, BM, BN, CfgK<T>::BK, WGM, WGN, MT, VEC>), dim3(g.total_tiles),
                       dim3(WGM * WGN * 64), 0, s, g);
    return hipGetLastError();
}
template <typename T, bool VEC>
hipError_t conv_dispatch(const ConvGroup& g, int cfg, hipStream_t s) {
    switch (cfg) {
        case CFG_N16: return conv_launch<T, 256, 16, 4, 1, 16, VEC>(g, s);
        case CFG_N32: return conv_launch<T, 256, 32, 4, 1, 16, VEC>(g, s);
        case CFG_N64: return conv_launch<T, 128, 64, 2, 2, 32, VEC>(g, s);
        case CFG_N64S: return conv_launch_bk<T, 64, 64, 2 * CfgK<T>::BK, 2, 2, 16, VEC>(g, s);
        case CFG_N128: if constexpr (VEC) return conv_launch<T, 128, 128, 2, 2, 32, true>(g, s); else break;
        case CFG_N160: if constexpr (VEC) return conv_launch<T, 128, 160, 2, 2, 16, true>(g, s); else break;
        default: break;
    }
    return hipErrorInvalidValue;
}
template <typename T, int BM, int BN, int BK, int WGM, int WGN, int MT, bool VEC>
hipError_t wgrad_launch_bk(const WgradGroup& g, hipStream_t s) {
    hipLaunchKernelGGL((conv_wgrad_kernel<T, BM, BN, BK, WGM, WGN, MT, VEC>), dim3(g.total_tiles), dim3(WGM * WGN * 64), 0, s, g);
    return hipGetLastError();
}
template <typename T, int BM, int BN, int WGM, int WGN, int MT, bool VEC>
hipError_t wgrad_launch(const WgradGroup& g, hipStream_t s) {
    hipLaunchKernelGGL((conv_wgrad_kernel<T, BM, BN, CfgK<T>::BK, WGM, WGN, MT, VEC>), dim3(g.total_tiles),
                       dim3(WGM * WGN * 64), 0, s, g);
    return hipGetLastError();
}
template <typename T, bool VEC>
hipError_t wgrad_dispatch(const WgradGroup& g, int cfg, hipStream_t s) {
    switch (cfg) {
        // narrow filters: k-tiles of twice the pixels (half as many load -> LDS -> barrier rounds per chunk; measured
        // -4 % on the ResNet-56 step, -3 % on ResNet-20)
        // ... and 144 columns: the 9 taps x 16 / 32 / 64 channels of a 3x3 filter are 1 / 2 / 4 whole tiles (128 columns left
        // a second or fifth tile that is one eighth full and reads the whole dY chunk again; measured: ResNet-56 step
        // 1.06 -> 1.02 ms, ResNet-20 0.925 -> 0.895; the 64-channel bf16 tile is the exception: 0.086 -> 0.094 ms)
        case CFG_N16: return wgrad_launch_bk<T, 16, 144, 2 * CfgK<T>::BK, 1, 3, 16, VEC>(g, s);
        case CFG_N32: return wgrad_launch_bk<T, 32, 144, 2 * CfgK<T>::BK, 1, 3, 16, VEC>(g, s);
        case CFG_N64:
            if constexpr (sizeof(T) == 4) return wgrad_launch_bk<T, 64, 144, 2 * CfgK<T>::BK, 2, 3, 16, VEC>(g, s);
            else return wgrad_launch_bk<T, 64, 128, 2 * CfgK<T>::BK, 2, 2, 32, VEC>(g, s);
        case CFG_N128: if constexpr (VEC) return wgrad_launch_bk<T, 128, 128, 2 * CfgK<T>::BK, 2, 2, 32, true>(g, s); else break;
        case CFG_N160: if constexpr (VEC) return wgrad_launch<T, 160, 160, 2, 2, 16, true>(g, s); else break;
        default: break;
    }
    return hipErrorInvalidValue;
}
}  // namespace

CfgInfo conv_cfg_info(int cfg, int dtype) {
    const int bk = dtype == 1 ? 32 : 16;
    switch (cfg) {
        case CFG_N16: return {256, 16, bk};
        case CFG_N32: return {256, 32, bk};
        case CFG_N64: return {128, 64, bk};
        case CFG_N64S: return {64, 64, 2 * bk};
        case CFG_N128: return {128, 128, bk};
        default: return {128, 160, bk};
    }
}
CfgInfo wgrad_cfg_info(int cfg, int dtype) {
    const int bk = dtype == 1 ? 32 : 16;
    switch (cfg) {
        case CFG_N16: return {16, 144, 2 * bk};
        case CFG_N32: return {32, 144, 2 * bk};
        case CFG_N64: return {64, dtype == 1 ? 128 : 144, 2 * bk};
        case CFG_N128: return {128, 128, 2 * bk};
        default: return {160, 160, bk};      // (doubled k-tiles cost this one its second workgroup per CU: slower)
    }
}

hipError_t launch_conv(const ConvGroup& g, int dtype, int cfg, bool vec, hipStream_t s) {
    if (g.total_tiles <= 0) return hipSuccess;
    if (dtype == 1) return vec ? conv_dispatch<bf16_t, true>(g, cfg, s) : conv_dispatch<bf16_t, false>(g, cfg, s);
    return vec ? conv_dispatch<float, true>(g, cfg, s) : conv_dispatch<float, false>(g, cfg, s);
}
hipError_t launch_wgrad(const WgradGroup& g, int dtype, int cfg, bool vec, hipStream_t s) {
    if (g.total_tiles <= 0) return hipSuccess;
    if (dtype == 1) return vec ? wgrad_dispatch<bf16_t, true>(g, cfg, s) : wgrad_dispatch<bf16_t, false>(g, cfg, s);
    return vec ? wgrad_dispatch<float, true>(g, cfg, s) : wgrad_dispatch<float, false>(g, cfg, s);
}
hipError_t launch_wtrans(const WtransGroup& g, int dtype, hipStream_t s) {
    if (g.total_blocks <= 0) return hipSuccess;
    if (dtype == 1) hipLaunchKernelGGL(wtrans_kernel<bf16_t>, dim3(g.total_blocks), dim3(256), 0, s, g);
    else hipLaunchKernelGGL(wtrans_kernel<float>, dim3(g.total_blocks), dim3(256), 0, s, g);
    return hipGetLastError();
}
hipError_t launch_im2col_offsets(const ConvProb& p, const int64_t* m, const int64_t* q, int64_t* out, int count, hipStream_t s) {
    if (count <= 0) return hipSuccess;
    hipLaunchKernelGGL(im2col_offsets_kernel, dim3((count + 255) / 256), dim3(256), 0, s, p, m, q, out, count);
    return hipGetLastError();
}
hipError_t launch_conv_offsets(const ConvProb& p, int kernel, int BM, int bk, int nw, const int64_t* m, const int64_t* q,
                               const int64_t* col, int64_t* in_off, int64_t* w_off, int64_t* out_off, int count, hipStream_t s) {
    if (count <= 0) return hipSuccess;
    hipLaunchKernelGGL(conv_offsets_kernel, dim3((count + 255) / 256), dim3(256), 0, s, p, kernel, BM, bk, nw, m, q, col,
                       in_off, w_off, out_off, count);
    return hipGetLastError();
}

}  // namespace lp
