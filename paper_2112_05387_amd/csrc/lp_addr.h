// Address arithmetic of the direct-to-LDS convolution kernels, written once as host+device functions: the kernels
// call them on the GPU, and the debug entry points of the C ABI call the very same functions on the host (bounds
// enumeration without a GPU) or from a one-thread-per-sample debug kernel (bit-exact comparison with the index
// function of the convolution's definition).
#pragma once
#include <hip/hip_runtime.h>

#include "lp_kernels.h"

#define LP_HD __host__ __device__ __forceinline__

namespace lp {
namespace addr {

constexpr unsigned kOOB = 0x80000000u;      // byte offset beyond any buffer: the hardware returns (and writes to LDS) zeros

// ---------------------------------------------------------------------------------------------------------------
// Filter (B operand) tiles.  A tile is BN filter rows of BK channels of one tap; it is fetched as 1 KiB wave-loads
// ("slabs" of RPS = 1024 / (2*BK) rows): wave w fetches slabs w, w + NW, w + 2*NW, ... (round j = 0, 1, ...); lane l
// of a slab fetches row l / CPR and the 16-byte chunk `kvg` of it.
// The range check of a raw buffer load covers the per-lane offset only, not the wave-uniform one that is added to
// it, so the per-lane offset must itself say "this row does not exist": rows of a ragged last column tile at or
// beyond Ncol get kOOB in every round, not only in round 0.
// ---------------------------------------------------------------------------------------------------------------
struct FilterRows {
    unsigned base0;      // per-lane byte offset of (row of round 0, chunk kvg)
    unsigned step;       // bytes between the rows of consecutive rounds (wave-uniform)
    int jmax;            // rounds whose row exists (row < Ncol); per lane
};
LP_HD FilterRows filter_rows(int n0, int rps, int nw, int wave, int lrow, int kvg, int ldw, int ncol) {
    FilterRows f;
    const int row0 = n0 + rps * wave + lrow;
    f.base0 = (unsigned)((row0 * ldw + kvg * 8) * 2);
    f.step = (unsigned)(rps * nw * ldw * 2);
    f.jmax = row0 >= ncol ? 0 : (ncol - row0 + rps * nw - 1) / (rps * nw);
    return f;
}
// per-lane offset of round j (kOOB: the load returns zeros) and the wave-uniform offset that goes with it
LP_HD unsigned filter_voffset(const FilterRows& f, int j, bool live) { return (live && j < f.jmax) ? f.base0 : kOOB; }
LP_HD unsigned filter_soffset(const FilterRows& f, unsigned tap_off, int j) { return tap_off + (unsigned)j * f.step; }
// byte offset of (tap, channel slab) inside a filter row: tap index (r0 + rs*tr, s0 + ss*ts) of an S-wide filter
LP_HD unsigned filter_tap_offset(const ConvProb& P, int tr, int ts, int ci0) {
    return (unsigned)((((P.r0 + P.rs * tr) * P.S + (P.s0 + P.ss * ts)) * P.Cin + ci0) * 2);
}
// chunk a lane fetches so that the LDS slot (row, l % CPR) holds the chunk the XOR swizzle of the fragment reads expects
LP_HD int filter_kvg(int bk, int lane, int wave) {
    return bk == 32 ? ((lane & 3) ^ ((lane >> 4) & 3)) : ((lane & 7) ^ (4 * (wave & 1) + (lane >> 4)));
}


// ---------------------------------------------------------------------------------------------------------------
// Activation (A operand) addresses.  GEMM row m is output pixel (n, a, b) of the row grid [N][OA][OB]; tap (tr, ts)
// reads input pixel (a*imul + dh0 + dhs*tr, b*imul + dw0 + dws*ts) of image n, zero outside the image.
// ---------------------------------------------------------------------------------------------------------------
struct RowGeom { int pix, ih0, iw0; };      // n*IH*IW, and the input coordinate tap (0, 0) reads
LP_HD RowGeom row_geom(const ConvProb& P, int m) {
    const int per = P.OA * P.OB;
    const int n = m / per, rem = m - n * per;
    const int a = rem / P.OB, b = rem - a * P.OB;
    RowGeom g;
    g.pix = n * P.IH * P.IW; g.ih0 = a * P.imul + P.dh0; g.iw0 = b * P.imul + P.dw0;
    return g;
}
LP_HD bool tap_inside(const ConvProb& P, const RowGeom& g, int tr, int ts, int& ih, int& iw) {
    ih = g.ih0 + P.dhs * tr; iw = g.iw0 + P.dws * ts;
    return (unsigned)ih < (unsigned)P.IH && (unsigned)iw < (unsigned)P.IW;
}
// general kernel: element offset of channel ci of input pixel (ih, iw)
LP_HD size_t elem_offset(const ConvProb& P, const RowGeom& g, int ih, int iw, int ci) {
    return (size_t)(g.pix + ih * P.IW + iw) * P.Cin + ci;
}
// output element offset of GEMM row m, column 0 (shared by every forward / data-gradient kernel)
LP_HD int out_row_offset(const ConvProb& P, int m) {
    const int per = P.OA * P.OB;
    const int n = m / per, rem = m - n * per;
    const int a = rem / P.OB, b = rem - a * P.OB;
    return ((n * P.OH + a * P.omul + P.ooh) * P.OW + b * P.omul + P.oow) * P.Ncol;
}

// implicit-GEMM wide-layer kernel: per-lane byte offset of (row m, tap (0,0), chunk kvg), the bit mask of the taps that
// fall inside the image, and the wave-uniform byte offset of (tap, channel slab); a load is base + tap offset when
// the tap's bit is set, kOOB otherwise
LP_HD int fast_row_base(const ConvProb& P, const RowGeom& g, int kvg) {
    return ((g.pix + g.ih0 * P.IW + g.iw0) * P.Cin + kvg * 8) * 2;
}
LP_HD unsigned fast_row_mask(const ConvProb& P, const RowGeom& g) {
    unsigned mk = 0u;
    for (int tr = 0; tr < P.ntr; ++tr)
        for (int ts = 0; ts < P.nts; ++ts) {
            int ih, iw;
            if (tap_inside(P, g, tr, ts, ih, iw)) mk |= 1u << (tr * P.nts + ts);
        }
    return mk;
}
LP_HD int fast_tap_offset(const ConvProb& P, int tr, int ts, int ci0) {
    return ((P.dhs * tr * P.IW + P.dws * ts) * P.Cin + ci0) * 2;
}

// window kernel: the tile's window is nseg segments (one per image, or one band of an image) of (SH + 2) x (W + 2)
// pixels; window pixel wp of the tile that starts at GEMM row m0 is fetched from the byte offset below (chunk lc of
// the 64-channel slab that starts at channel 0; kOOB-like 0xffffffff: padding; bit 31: upper half of a slab)
struct WinGeom { int H, W, per, TH, SH, nseg, WW, SEGP, NP; };
LP_HD WinGeom win_geom(const ConvProb& P, int BM) {
    WinGeom w;
    w.H = P.OA; w.W = P.OB; w.per = w.H * w.W;
    w.TH = BM / w.W; w.SH = w.TH < w.H ? w.TH : w.H; w.nseg = w.TH / w.SH;
    w.WW = w.W + 2; w.SEGP = (w.SH + 2) * w.WW; w.NP = w.nseg * w.SEGP;
    return w;
}
LP_HD unsigned win_slot_offset(const ConvProb& P, const WinGeom& w, int m0, int wp, int lc, int cpr) {
    if (wp >= w.NP) return 0xffffffffu;
    const int nimg = P.M / w.per;
    const int sg = wp / w.SEGP, rem = wp - sg * w.SEGP;
    const int wr = rem / w.WW, wc = rem - wr * w.WW;
    const int gr = m0 / w.W + sg * w.SH;                 // first image row of the segment, counted over all images
    const int n = gr / w.H, h0 = gr - n * w.H;
    const int ih = h0 + wr - 1, iw = wc - 1;
    if (!(n < nimg && (unsigned)ih < (unsigned)w.H && (unsigned)iw < (unsigned)w.W)) return 0xffffffffu;
    unsigned ab = (unsigned)((((n * w.H + ih) * w.W + iw) * P.Cin + lc * 8) * 2);
    if (lc >= cpr / 2) ab |= 0x80000000u;                // upper half: absent from a half slab
    return ab;
}
// window row (in pixels) that output pixel p of the tile reads at tap (tr, ts)
LP_HD int win_frag_row(const ConvProb& P, const WinGeom& w, int p, int tr, int ts) {
    const int hh_all = p / w.W, x = p - hh_all * w.W;
    const int sg = hh_all / w.SH, hh = hh_all - sg * w.SH;
    return sg * w.SEGP + hh * w.WW + x + (1 + P.dh0 + P.dhs * tr) * w.WW + (1 + P.dw0 + P.dws * ts);
}

}  // namespace addr
}  // namespace lp
