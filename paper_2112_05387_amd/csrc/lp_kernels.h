// Device-side problem descriptors and launch entry points of the local-step kernels (gfx950).
// Every kernel is a *grouped* launch: one grid covers the same operation of several modules, the
// per-module problems travel by value in the kernel arguments, and a workgroup finds its problem from
// a prefix table of tile counts.  That is how the K independent local steps of Sec. 4.1 share one GPU.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lp {

constexpr int kMaxGroup = 16;   // problems per grouped launch (bounded by the 4 KiB kernel-argument block)

// ---------------------------------------------------------------------------------------------------
// Implicit-GEMM convolution, forward and data-gradient:  OUT[m, col] = sum_q A[m, q] * WT[col, q]
//   m   -> (n, a, b) on a row grid [N][OA][OB];  q -> (tr, ts, ci) with ci fastest
//   A[m,q] = IN[n, a*imul + dh0 + dhs*tr, b*imul + dw0 + dws*ts, ci]      (zero outside the image)
//   WT[col,q] = wt[col*ldw + ((r0 + rs*tr)*S + (s0 + ss*ts))*Cin + ci]
//   OUT pixel = (n, a*omul + ooh, b*omul + oow) of an [N][OH][OW][Ncol] tensor
// Forward conv: imul = stride, dh0 = -pad, dhs = 1, full tap range, omul = 1.
// Data-gradient: IN = dY, wt = filters re-laid-out as [Cin][R][S][Cout]; stride 1: dh0 = pad, dhs = -1;
// stride 2: one problem per output parity class with the taps of matching parity (rs = 2).
struct ConvProb {
    const void* in;
    const void* wt;
    void* out;
    const void* add0;     // optional addends with the layout of out (skip-path gradients)
    const void* add1;
    double* stats;        // optional: [2*Ncol] per-column sum and sum of squares of the fp32 results
    int M, Ncol, Kg, Cin;
    int OA, OB, IH, IW, imul;
    int ntr, nts, dh0, dhs, dw0, dws;
    int r0, rs, s0, ss, S, ldw;
    int OH, OW, omul, ooh, oow;
    int tiles_m, tiles_n, tile_start;
};
struct ConvGroup {
    int nprob, total_tiles;
    ConvProb p[kMaxGroup];
};

// Weight gradient:  dW[co, (r,s,ci)] (+)= sum_m dY[m, co] * X[n, ho*stride - pad + r, wo*stride - pad + s, ci]
// split over `ksplit` slices of the reduction; partial results are added to dW with fp32 atomics.
struct WgradProb {
    const void* x;
    const void* dy;
    float* dw;
    int M, Cout, Kg, Cin;
    int Ho, Wo, IH, IW, stride, pad, R, S;
    int ksplit, kchunk;
    int tiles_m, tiles_n, tile_start;
    unsigned mulW, shW, mulH, shH;   // fast division by IW and IH (wide-layer kernel)
    // parameter update in the epilogue (w != NULL): the workgroup that adds the LAST partial sum of an output tile
    // (ticket from cnt[tile], zero before the launch) reads the finished gradient tile back and updates the filter
    void* w;                         // the filter itself, storage type of the activations, layout of dw
    float* vel;                      // momentum buffer (NULL: none)
    float* master;                   // fp32 copy of the filter (NULL: w is read)
    unsigned* cnt;                   // tiles_m * tiles_n tickets
};
struct WgradGroup {
    int nprob, total_tiles;
    float lr, momentum, wd;          // of the update in the epilogue
    int lowp;                        // the filters are bf16
    WgradProb p[kMaxGroup];
};

// filters [Cout][R][S][Cin] -> [Cin][R][S][Cout]
struct WtransProb {
    const void* w;
    void* wt;
    int Cout, RS, Cin;
    int block_start;
};
struct WtransGroup {
    int nprob, total_blocks;
    WtransProb p[kMaxGroup];
};

// out = act( bn(y) [+ skip] ),  bn(y) = gamma*(y-mean)*invstd + beta from the summed statistics.
// skip_mode 0: none, 1: plain tensor, 2: bn_s(skip) with its own statistics.
// Fused form (the pass that writes a module's output F_k(x_k), inside lp_local_step): with dy != NULL the same pass
// evaluates the local loss and terminal adjoint on the value it stores, as LossProb below describes (xn, lam, dy,
// lam_out, loss), so that F_k(x_k) is not read again.
struct BnApplyProb {
    const void* y; void* out;
    const double* stats; const float* gamma; const float* beta;
    const void* skip; const double* sstats; const float* sgamma; const float* sbeta;
    const void* xn; const void* lam; void* dy; void* lam_out; float* loss; float* r2;
    int M, C, relu, skip_mode;
    int block_start, nblocks;
};
struct BnApplyGroup {
    int nprob, total_blocks; float eps;
    int cmax;             // largest channel count of the group (sizes the coefficient arrays in LDS)
    float rho, scale, step;   // fused form: penalty coefficient, loss scale, multiplier step
    BnApplyProb p[kMaxGroup];
};

// Batch-norm backward.  g' = g * [gamma*yhat + beta > 0] when relu is set.
// reduce: red[0..C) += sum g', red[C..2C) += sum g'*yhat.   apply: dy = gamma*invstd*(g' - red0/M - yhat*red1/M),
// and the first workgroup of each problem writes dgamma = red1, dbeta = red0.
struct BnBwdProb {       // add: optional addend of the apply pass with the layout of dy (identity skip of a pre-activation block)
    const void* add;
    const void* g; const void* y; void* dy;
    const double* stats; const float* gamma; const float* beta;
    double* red; float* dgamma; float* dbeta;
    int M, C, relu;
    int block_start, nblocks;
};
struct BnBwdGroup {
    int nprob, total_blocks; float eps;
    int cmax;             // largest channel count of the group (sizes the coefficient arrays in LDS)
    BnBwdProb p[kMaxGroup];
};

// gm = g * [out > 0]: the gradient through a ReLU behind a residual sum, from the stored block output
struct MaskProb { const void* g; const void* out; void* gm; size_t numel; int block_start, nblocks; };
struct MaskGroup { int nprob, total_blocks; MaskProb p[kMaxGroup]; };

struct FillProb { void* ptr; size_t bytes; int block_start; };
struct FillGroup { int nprob, total_blocks; FillProb p[kMaxGroup]; };

// r = y - x_next;  dy = scale*(rho*r + lam);  loss += scale*(rho/2*sum r^2 + sum lam*r)
struct LossProb {
    const void* y; const void* xn; const void* lam; void* dy; float* loss;
    float* r2;               // != NULL: += sum r^2 (the constraint violation |F_k(x_k) - x_{k+1}|^2 of the interface)
    void* lam_out;           // != NULL: lam + step*(y - x_next) is written there (may be lam itself) after dy took the old lam
    size_t numel; int block_start, nblocks;
};
struct LossGroup { int nprob, total_blocks; float rho, scale, step; LossProb p[kMaxGroup]; };

// lam += step*(y - x_next)
struct MultProb { void* lam; const void* y; const void* xn; size_t numel; int block_start, nblocks; };
struct MultGroup { int nprob, total_blocks; float step; MultProb p[kMaxGroup]; };
// parameter update of one tensor: g' = g + wd*W; v = mu*v + g' (if v); W -= lr*(v or g'); master (fp32 copy) optional
struct SgdProb { void* p; const float* g; float* v; float* master; size_t numel; int lowp; int block_start, nblocks; };
struct SgdGroup { int nprob, total_blocks; float lr, momentum, wd; SgdProb p[kMaxGroup]; };
// correction of an auxiliary variable: x <- x - eta*(scale*(rho*(x - yprev) - lam) + dx), lam may be NULL
struct AuxVarProb {      // gout != NULL: the gradient scale*(rho*(x - yprev) - lam) + dx is written there and x is left as it is
    void* x; const void* yprev; const void* dx; const void* lam; void* gout; size_t numel; int block_start, nblocks;
};
struct AuxVarGroup { int nprob, total_blocks; float rho, scale, eta; AuxVarProb p[kMaxGroup]; };

struct PoolProb {        // max pooling R x R, stride, pad on NHWC
    const void* x; void* y; uint8_t* arg; const void* dy; void* dx;
    int N, H, W, C, Ho, Wo, R, stride, pad;
};

struct HeadProb {        // global average pool + linear
    const void* feat; float* pooled; const float* w; const float* b; float* logits;
    const float* dlogits; float* dw; float* db; void* dfeat;
    int N, HW, C, classes;
};

// ---- launchers (host side; return hipError_t of the launch) ----------------------------------------
// tile configuration ids of the implicit-GEMM kernels
enum ConvCfg { CFG_N16 = 0, CFG_N32, CFG_N64, CFG_N128, CFG_N160,
               CFG_N64S,                               // 64 x 64 tiles with twice the k-tile: 33..64 output channels, few pixels (forward / data-gradient only)
               CFG_COUNT,
               FAST_256x320 = 8, FAST_512x160 = 9,     // bf16 wide-layer kernel (lp_conv_fast.hip)
               FAST_128x320 = 10, FAST_128x160 = 11,   // ... its four- and two-wave variants, chosen per launch
               FAST64_256x320 = 12, FAST64_128x320 = 13, FAST64_128x160 = 14,   // ... with k-tiles of 64 channels
               FAST_256x160 = 15, FAST64_256x160 = 16,  // four-wave variants of the 160-wide family
               WIN64_512x160 = 21, WIN64_256x320 = 23,  // bf16 3x3 stride-1 kernel with the input window in LDS (lp_conv_win.hip)
               WGRAD_FAST = 8 };                       // bf16 wide-layer filter-gradient kernel (lp_wgrad_fast.hip)
struct CfgInfo { int BM, BN, BK; };
CfgInfo conv_cfg_info(int cfg, int dtype);
CfgInfo wgrad_cfg_info(int cfg, int dtype);
CfgInfo conv_fast_cfg_info(int cfg);
CfgInfo conv_win_cfg_info(int cfg);
// window slabs (1 KiB wave-loads) a wave of the window kernel can hold addresses for
constexpr int conv_win_max_slabs(int BM, int NW) { return BM == 512 ? 10 : 7; }

hipError_t launch_conv(const ConvGroup& g, int dtype, int cfg, bool vec, hipStream_t s);
hipError_t launch_conv_fast(const ConvGroup& g, int cfg, hipStream_t s);
hipError_t launch_conv_win(const ConvGroup& g, int cfg, hipStream_t s);
hipError_t launch_wgrad_fast(const WgradGroup& g, hipStream_t s);
int wgrad_fast_blocks(const WgradProb& p);
void fastdiv_make(unsigned d, unsigned* mul, unsigned* shift);
hipError_t launch_wgrad(const WgradGroup& g, int dtype, int cfg, bool vec, hipStream_t s);
hipError_t launch_wtrans(const WtransGroup& g, int dtype, hipStream_t s);
hipError_t launch_bn_apply(const BnApplyGroup& g, int dtype, bool fused_loss, hipStream_t s);
hipError_t launch_bn_bwd_reduce(const BnBwdGroup& g, int dtype, hipStream_t s);
hipError_t launch_bn_bwd_apply(const BnBwdGroup& g, int dtype, hipStream_t s);
hipError_t launch_fill(const FillGroup& g, hipStream_t s);
hipError_t launch_relu_mask(const MaskGroup& g, int dtype, hipStream_t s);
hipError_t launch_loss(const LossGroup& g, int dtype, hipStream_t s);
hipError_t launch_mult(const MultGroup& g, int dtype, hipStream_t s);
hipError_t launch_auxvar(const AuxVarGroup& g, int dtype, hipStream_t s);
hipError_t launch_sgd(const SgdGroup& g, hipStream_t s);
// per-channel sum and sum of squares of a stored tensor [M, C] (fields y, red, M, C of BnBwdProb), added to red[2C]
hipError_t launch_bn_stats(const BnBwdGroup& g, int dtype, hipStream_t s);
constexpr int kSgdElemsPerBlock = 4096;
hipError_t launch_maxpool_fwd(const PoolProb& p, int dtype, hipStream_t s);
hipError_t launch_maxpool_bwd(const PoolProb& p, int dtype, hipStream_t s);
hipError_t launch_head_fwd(const HeadProb& p, int dtype, hipStream_t s);
hipError_t launch_head_bwd(const HeadProb& p, int dtype, hipStream_t s);
hipError_t launch_ce(const float* logits, const int32_t* labels, float* loss, float* dlogits,
                     int N, int classes, hipStream_t s);
hipError_t launch_zero_selected(float* v, uint32_t mask, int n, hipStream_t s);
hipError_t launch_im2col_offsets(const ConvProb& p, const int64_t* m, const int64_t* q, int64_t* out, int count, hipStream_t s);
hipError_t launch_conv_offsets(const ConvProb& p, int kernel, int BM, int bk, int nw, const int64_t* m, const int64_t* q,
                               const int64_t* col, int64_t* in_off, int64_t* w_off, int64_t* out_off, int count, hipStream_t s);

hipError_t launch_mfma_peak(int mode, int blocks, int iters, unsigned long long* clk, float* sink, hipStream_t s);

constexpr int kElemBlock = 256;          // threads per workgroup of the elementwise kernels
// Per-channel sums (batch statistics, BN backward sums) are accumulated with fp64 atomics by every workgroup that holds
// a piece of the tensor.  Atomics on ONE address are performed one after another at the memory side (about 25 ns each
// on this device: 512 workgroups adding to the same 32 addresses cost 13 us), so a sum is kept as several partial sums
// ("stripes", layout [kStatStripes][2][C]); workgroup b adds to stripe b % stat_stripes(C) and readers add the stripes
// up in a fixed order.  Readers pay for every stripe in their prologue (C x stripes loads per workgroup), so the
// number of stripes in use falls with the channel count: narrow layers have many writers per address and cheap readers,
// wide layers the opposite (measured: ResNet-56 step 1.36 -> 1.27 ms with 4-8 stripes; 2048-channel layers lose with 4).
constexpr int kStatStripes = 8;
__host__ __device__ inline int stat_stripes(int C) { return C <= 64 ? 8 : (C <= 320 ? 4 : 1); }
__host__ __device__ inline size_t stat_bytes(int C) { return sizeof(double) * 2 * (size_t)C * kStatStripes; }
constexpr int kBnReduceBlock = 512;      // threads per workgroup of the BN backward reduction (measured: 256 -7 %, 1024 -20 %)
// ... and 256 for launches whose widest tensor has at most 64 channels (see launch_bn_bwd_reduce)
inline int bn_reduce_threads(int cmax) { return cmax <= 64 ? 256 : kBnReduceBlock; }
constexpr int kElemVecsPerBlock = 2048;  // 16-byte vectors handled by one workgroup

}  // namespace lp
