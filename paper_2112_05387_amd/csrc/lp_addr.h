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

}  // namespace addr
}  // namespace lp
