// Host side of the local-step library: descriptor validation, packed parameter layout, workspace layout,
// the per-module operation lists of the forward and backward passes, and the scheduler that merges the same
// operation of different modules into one grouped launch (the K local steps of Sec. 4.1 are independent, so
// they are advanced in lock-step on one GPU).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/lp.h"
#include "lp_addr.h"
#include "lp_kernels.h"

using namespace lp;

// ----------------------------------------------------------------------------------------------------
// errors
// ----------------------------------------------------------------------------------------------------
static thread_local std::string g_err;
static thread_local bool g_keep_gradients = false;   // lp_debug_keep_gradients: nets created on this thread keep every gradient

static lp_status fail(lp_status st, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    g_err = buf;
    return st;
}

// ----------------------------------------------------------------------------------------------------
// plan structures
// ----------------------------------------------------------------------------------------------------
namespace {

enum Space { SP_NONE = 0, SP_WS, SP_X, SP_Y, SP_PARAM, SP_DPARAM, SP_DY, SP_DX, SP_LOGITS, SP_DLOGITS,
             SP_AUXP, SP_XOUT, SP_IMAGE, SP_AUXG, SP_XTGT, SP_XNEXT, SP_LAM, SP_LOSS, SP_LABELS, SP_SCRATCH };
struct Ref { int space = SP_NONE; int idx = 0; size_t off = 0; };
static Ref mk(int sp, int idx, size_t off) { Ref r; r.space = sp; r.idx = idx; r.off = off; return r; }

struct Bindings {
    char* ws = nullptr;
    char* scratch = nullptr;               // the library's own device array (lp_auxnet_forward_static)
    const void* const* x = nullptr;
    void* const* y = nullptr;
    const void* const* params = nullptr;
    float* const* dparams = nullptr;
    const void* const* dy = nullptr;
    void* const* dx = nullptr;
    float* logits = nullptr;
    const float* dlogits = nullptr;
    const void* const* auxp = nullptr;
    void* const* xout = nullptr;
    const void* image = nullptr;
    float* const* auxg = nullptr;
    const void* const* xtgt = nullptr;     // corrected auxiliary variables (input of a chained AuxNet's distillation)
    // the fused local step: interface tensors, multipliers, losses, labels and the scalars of its loss / multiplier kernels
    const void* const* xnext = nullptr;
    void* const* lam = nullptr;
    float* loss = nullptr;
    const int32_t* labels = nullptr;
    float rho = 0.f, scale = 1.f, mstep = 0.f;
    // parameter update inside the backward pass (lp_net_set_fused_update): per module, layout of dparams
    float* const* vel = nullptr;
    float* const* master = nullptr;
};
static void* resolve(const Ref& r, const Bindings& b) {
    switch (r.space) {
        case SP_WS: return b.ws + r.off;
        case SP_SCRATCH: return b.scratch + r.off;
        case SP_X: return (char*)b.x[r.idx] + r.off;
        case SP_Y: return (char*)b.y[r.idx] + r.off;
        case SP_PARAM: return (char*)b.params[r.idx] + r.off;
        case SP_DPARAM: return (char*)b.dparams[r.idx] + r.off;
        case SP_DY: return (char*)b.dy[r.idx] + r.off;
        case SP_DX: return (char*)b.dx[r.idx] + r.off;
        case SP_LOGITS: return (char*)b.logits + r.off;
        case SP_DLOGITS: return (char*)b.dlogits + r.off;
        case SP_AUXP: return (char*)b.auxp[r.idx] + r.off;
        case SP_XOUT: return (char*)b.xout[r.idx] + r.off;
        case SP_IMAGE: return (char*)b.image + r.off;
        case SP_AUXG: return (char*)b.auxg[r.idx] + r.off;
        case SP_XTGT: return (char*)b.xtgt[r.idx] + r.off;
        case SP_XNEXT: return (char*)b.xnext[r.idx] + r.off;
        case SP_LAM: return (b.lam && b.lam[r.idx]) ? (char*)b.lam[r.idx] + r.off : nullptr;
        case SP_LOSS: return (char*)b.loss + r.off;
        case SP_LABELS: return (char*)b.labels + r.off;
        default: return nullptr;
    }
}

enum OpType { OP_FILL = 0, OP_WTRANS, OP_CONV, OP_BN_APPLY, OP_POOL_FWD, OP_HEAD_FWD, OP_HEAD_BWD, OP_POOL_BWD,
              OP_BN_BWD_REDUCE, OP_BN_BWD_APPLY, OP_WGRAD, OP_BN_STATS, OP_LOSS, OP_CE, OP_MULT_UNUSED, OP_RELU_MASK, OP_SGD_REST };

struct Op {
    int type = 0, cfg = 0;
    int phase = 0;                         // fused step: 0 forward, 1 loss, 2 backward, 3 multiplier update
    bool vec = true;
    Ref r[14];
    size_t fill_bytes = 0;
    size_t numel = 0;                      // OP_LOSS: elements of the interface tensor
    ConvProb conv;
    WgradProb wg;
    WtransProb wt;
    BnApplyProb bna;
    BnBwdProb bnb;
    PoolProb pool;
    HeadProb head;
    int key() const { return type * 64 + cfg * 2 + (vec ? 1 : 0); }
};
typedef std::vector<Op> Step;              // operations of one module that may run concurrently
typedef std::vector<Step> Program;         // steps run in order

// one conv + batch-norm unit
struct Unit {
    int R = 3, cin = 0, cout = 0, stride = 1, pad = 1;
    int N = 0, H = 0, W = 0, Ho = 0, Wo = 0;
    bool relu = false, need_dgrad = true;
    int t_w = -1, t_g = -1, t_b = -1;      // tensor table indices
    size_t ws_y = 0, ws_dy = 0, ws_stats = 0, ws_red = 0, ws_wt = 0;
    size_t out_elems() const { return (size_t)N * Ho * Wo * cout; }
    size_t in_elems() const { return (size_t)N * H * W * cin; }
};
struct BlockPlan {
    std::vector<Unit> main;                // 2 (basic) or 3 (bottleneck)
    bool has_proj = false;
    bool proj_plain = false, post_relu = false;   // options of the conv-BN-ReLU order: bare conv1x1 projection, ReLU behind the sum
    size_t ws_gmask = 0;                   // post_relu: the arriving gradient masked by (block output > 0)
    Ref graw_ref;                          // ... and the unmasked one
    Unit proj;
    std::vector<size_t> ws_act;            // activations between main convs
    Ref in, out;                           // block input / output tensors
    Ref gout;                              // pre-activation order: gradient with respect to the block output (kept for the filter gradients)
    size_t in_elems = 0, out_elems = 0;
    // conv-BN-ReLU order, backward pass: where the gradient on the block input, on the activation behind main[j]
    // (j < main.size()-1) and the projection's data-gradient go.  Normally buffers the blocks of a module share;
    // with lp_debug_keep_gradients every block has its own, so that all of them can be read after the pass.
    size_t ws_gin = 0, ws_gproj = 0;
    std::vector<size_t> ws_gact;
    Ref gin_ref, g_ref;                    // gradient on the block input / output as the backward program binds them
};
struct ModulePlan {
    lp_module_desc d;
    std::vector<lp_block_desc> blocks;
    std::vector<lp_tensor_info> tensors;
    size_t param_bytes = 0, grad_bytes = 0;
    bool has_stem = false;
    Unit stem;
    size_t ws_stem_act = 0;                // stem output (after ReLU; before pooling for stem 2)
    size_t ws_pool_out = 0, ws_pool_arg = 0;
    int pH = 0, pW = 0;                    // dims after the stem conv (pool input)
    std::vector<BlockPlan> bp;
    int oN = 0, oH = 0, oW = 0, oC = 0;    // F_k(x_k) shape
    size_t ws_feat = 0;                    // last module: F_k(x_k)
    size_t ws_pooled = 0, ws_dfeat = 0;
    int t_fcw = -1, t_fcb = -1;
    int t_hg = -1, t_hb = -1;              // pre-activation order: BN in front of the head
    size_t ws_hstats = 0, ws_hred = 0, ws_hf = 0, ws_ghead = 0, ws_gstem = 0;
    size_t ws_stats0 = 0, ws_stats_bytes = 0, ws_red0 = 0, ws_red_bytes = 0;
    size_t ws_cnt0 = 0, ws_cnt_bytes = 0;  // completion tickets of the filter-gradient tiles (update in the epilogue)
    std::vector<char> t_in_epilogue;       // per tensor: its update rides on a filter-gradient kernel
    size_t ws_G[2] = {0, 0}, ws_A = 0, ws_P = 0, ws_gpool = 0;
    Program fwd, bwd, bwd_dx0;             // bwd_dx0: variant that also produces dx for a stem-less module 0
    Program step, step_dx0;                // forward, loss / terminal adjoint, backward, multiplier update in one list
};
struct AuxPlan {
    lp_aux_desc d;
    std::vector<Unit> pre;                 // the blocks in front of the last one (conv - BN - ReLU each)
    Unit u;                                // the last block: its output is the auxiliary variable
    std::vector<size_t> ws_act, ws_gact;   // output of pre[i] and the gradient with respect to it
    std::vector<lp_tensor_info> tensors;
    size_t param_bytes = 0, grad_bytes = 0;
    size_t ws_out = 0, ws_g = 0;           // recomputed AuxNet output and the gradient on it (distillation)
    Program fwd, bwd_a, bwd_b;             // distillation: before / after the loss kernel
    Program fwd_static;                    // forward pass whose intermediates live in the library's own device array
    bool chained = false;                  // input = the previous auxiliary variable instead of the mini-batch
};

}  // namespace

struct lp_net {
    int K = 0, dtype = 0;
    float eps = 1e-5f;
    size_t esz = 4;
    std::vector<ModulePlan> mods;
    std::vector<AuxPlan> aux;
    size_t ws_bytes = 0;
    char* ws = nullptr;
    size_t ws_given = 0;
    uint32_t fwd_done = 0;
    bool aux_fwd_done = false;
    std::vector<const void*> saved_x;
    std::vector<void*> saved_y;            // y[k] of the last forward call (a ReLU behind the last block's sum is masked from it)
    // optional second stream: modules in side_mask are issued there, concurrently with the others
    std::vector<int> lane;                 // per module: 0 = the caller's stream, 1..3 = extra stream
    hipStream_t extra_stream[4] = {nullptr, nullptr, nullptr, nullptr};
    hipEvent_t ev_fork = nullptr, ev_join[4] = {nullptr, nullptr, nullptr, nullptr};
    bool lanes_ready = false;              // every extra stream and event above exists
    bool keep_gradients = false;           // debug layout: no gradient buffer is reused inside a backward pass
    bool deterministic = false;            // lp_net_set_deterministic: every reduction in a fixed order
    // lp_net_set_fused_update: the parameter update runs inside lp_module_backward / lp_local_step
    bool fused_update = false;
    float fu_lr = 0.f, fu_momentum = 0.f, fu_wd = 0.f;
    std::vector<float*> fu_vel, fu_master;
    float* r2 = nullptr;                   // optional device output [K-1]: |F_k(x_k) - x_{k+1}|^2 per interface (lp_net_set_residual_output)
    size_t scratch_bytes = 0;              // what the AuxNet forward passes need of the library's own device array
    // optional per-launch timing (hipEvents around every grouped launch)
    bool prof = false;
    int lanes_in_flight = 1;               // stream lanes of the call being enqueued (launch-time tile choice)
    bool prof_serial = false;              // issue every stream lane on the caller's stream (launches timed in isolation)
    struct ProfRec { hipEvent_t a, b; int type, cfg, nprob, blocks; double flops, bytes; };
    std::vector<ProfRec> prof_recs;
    std::vector<hipEvent_t> prof_pool;
};

namespace {

static_assert(kStatStripes == LP_STAT_STRIPES, "the header documents the layout of the per-channel sums");

static size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

// the wide-layer bf16 kernel applies when a k-tile of 32 channels lies inside one tap and offsets fit 31 bits
static bool conv_fast_ok(const lp_net* net, const ConvProb& c) {
    if (net->dtype != LP_BF16 || c.Cin % 32 != 0 || c.Ncol % 8 != 0) return false;
    if (c.ntr * c.nts > 32) return false;
    // output channels are tiled by 160 or 320: worth it when at least three quarters of the last tile are used
    const int tn = c.Ncol > 160 ? 320 : 160;
    if (4 * c.Ncol < 3 * ((c.Ncol + tn - 1) / tn) * tn) return false;
    const double in_bytes = (double)c.M / ((double)c.OA * c.OB) * c.IH * c.IW * c.Cin * 2.0;
    const double w_bytes = (double)c.Ncol * c.ldw * 2.0;
    return in_bytes < 2.0e9 && w_bytes < 2.0e9;
}

// pick the wide-layer configuration of a problem; returns false if the wide-layer kernel does not apply
static bool pick_fast_cfg(const lp_net* net, const ConvProb& c, int& cfg) {
    if (!conv_fast_ok(net, c)) return false;
    cfg = c.Ncol > 160 ? FAST_256x320 : FAST_512x160;
    return true;
}

// the window kernel: 3x3 taps at offsets -1..1, stride 1, same-size input and output, tiles that are bands of whole
// image rows (or whole images)
static bool pick_win_cfg(const lp_net* net, const ConvProb& c, int& cfg) {
    if (!conv_fast_ok(net, c)) return false;
    if (c.ntr != 3 || c.nts != 3 || c.imul != 1 || c.omul != 1 || c.IH != c.OA || c.IW != c.OB || c.OH != c.OA || c.OW != c.OB)
        return false;
    for (int t = 0; t < 3; ++t)
        if (std::abs(c.dh0 + c.dhs * t) > 1 || std::abs(c.dw0 + c.dws * t) > 1) return false;
    const int BN = c.Ncol > 160 ? 320 : 160, BK = 64, BM = c.Ncol > 160 ? 256 : 512, NW = 8;
    if (BM % c.OB != 0) return false;
    const int TH = BM / c.OB;
    if (c.OA % TH != 0 && TH % c.OA != 0) return false;
    const int SH = std::min(TH, c.OA), NP = (TH / SH) * (SH + 2) * (c.OB + 2), RPS = 1024 / (BK * 2);
    const int nslab = (NP + RPS - 1) / RPS;
    if ((nslab + NW - 1) / NW > conv_win_max_slabs(BM, NW)) return false;
    const size_t ring_end = (size_t)nslab * 1024 + (size_t)2 * BN * BK * 2;
    if (std::max(ring_end, (size_t)NW * 32 * 336) + BM * sizeof(int) + (size_t)conv_win_max_slabs(BM, NW) * NW * 64 * 4 > 160 * 1024)
        return false;
    cfg = c.Ncol > 160 ? WIN64_256x320 : WIN64_512x160;
    return true;
}

static int conv_cfg_for(int ncol, bool vec, int M) {
    int cfg;
    if (ncol % 160 == 0) cfg = CFG_N160;
    else if (ncol <= 16) cfg = CFG_N16;
    else if (ncol <= 32) cfg = CFG_N32;
    // few pixels (the 8 x 8 x 64 layers of the CIFAR networks: 64 tiles of 128 rows for 256 CUs): smaller tiles, longer
    // k-tiles (measured on ResNet-56 / ResNet-20: 0.27 -> 0.20 ms and 0.43 -> 0.28 ms per step for these layers)
    else if (ncol <= 64) cfg = M <= 16384 ? CFG_N64S : CFG_N64;
    else cfg = CFG_N128;
    if (!vec && (cfg == CFG_N128 || cfg == CFG_N160)) cfg = CFG_N64;
    return cfg;
}
static int wgrad_cfg_for(int cout, int kg, bool vec) {
    int cfg;
    if (cout % 160 == 0 && kg % 160 == 0) cfg = CFG_N160;
    else if (cout <= 16) cfg = CFG_N16;
    else if (cout <= 32) cfg = CFG_N32;
    else if (cout <= 64) cfg = CFG_N64;
    else cfg = CFG_N128;
    if (!vec && cfg > CFG_N64) cfg = CFG_N64;
    return cfg;
}

struct Builder {
    lp_net* net;
    int epv() const { return net->dtype == LP_BF16 ? 8 : 4; }

    // ---- op constructors ------------------------------------------------------------------------
    Op fill(Ref p, size_t bytes) const {
        Op o; o.type = OP_FILL; o.r[0] = p; o.fill_bytes = bytes; return o;
    }
    Op conv_fwd(const Unit& u, Ref in, Ref w, Ref out, Ref stats) const {
        Op o; o.type = OP_CONV;
        ConvProb& c = o.conv; memset(&c, 0, sizeof(c));
        c.M = u.N * u.Ho * u.Wo; c.Ncol = u.cout; c.Cin = u.cin; c.Kg = u.R * u.R * u.cin;
        c.OA = u.Ho; c.OB = u.Wo; c.IH = u.H; c.IW = u.W; c.imul = u.stride;
        c.ntr = u.R; c.nts = u.R; c.dh0 = -u.pad; c.dhs = 1; c.dw0 = -u.pad; c.dws = 1;
        c.r0 = 0; c.rs = 1; c.s0 = 0; c.ss = 1; c.S = u.R; c.ldw = c.Kg;
        c.OH = u.Ho; c.OW = u.Wo; c.omul = 1; c.ooh = 0; c.oow = 0;
        o.vec = (u.cin % epv()) == 0;
        o.cfg = conv_cfg_for(c.Ncol, o.vec, c.M);
        pick_fast_cfg(net, c, o.cfg);
        pick_win_cfg(net, c, o.cfg);
        o.r[0] = in; o.r[1] = w; o.r[2] = out; o.r[5] = stats;
        return o;
    }
    // data-gradient of unit u: dX[N,H,W,cin] from dY[N,Ho,Wo,cout] and the re-laid-out filters [cin][R][R][cout]
    void conv_dgrad(const Unit& u, Ref dy, Ref wt, Ref dx, Ref add0, Ref add1, Step& step) const {
        const int st = u.stride;
        for (int ph = 0; ph < st; ++ph)
            for (int pw = 0; pw < st; ++pw) {
                Op o; o.type = OP_CONV;
                ConvProb& c = o.conv; memset(&c, 0, sizeof(c));
                c.Ncol = u.cin; c.Cin = u.cout; c.S = u.R; c.ldw = u.R * u.R * u.cout;
                c.IH = u.Ho; c.IW = u.Wo; c.imul = 1;
                c.OH = u.H; c.OW = u.W; c.omul = st; c.ooh = ph; c.oow = pw;
                c.OA = u.H / st; c.OB = u.W / st;
                c.M = u.N * c.OA * c.OB;
                // taps r with (ph + pad - r) divisible by the stride; source row = a + (ph + pad - r)/stride
                c.r0 = (ph + u.pad) % st; c.rs = st;
                c.ntr = c.r0 < u.R ? (u.R - c.r0 + st - 1) / st : 0;
                c.dh0 = (ph + u.pad - c.r0) / st; c.dhs = -1;
                c.s0 = (pw + u.pad) % st; c.ss = st;
                c.nts = c.s0 < u.R ? (u.R - c.s0 + st - 1) / st : 0;
                c.dw0 = (pw + u.pad - c.s0) / st; c.dws = -1;
                if (c.ntr == 0 || c.nts == 0) { c.ntr = 0; c.nts = 1; }
                c.Kg = c.ntr * c.nts * c.Cin;
                o.vec = (u.cout % epv()) == 0;
                o.cfg = conv_cfg_for(c.Ncol, o.vec, c.M);
                pick_fast_cfg(net, c, o.cfg);
                pick_win_cfg(net, c, o.cfg);
                o.r[0] = dy; o.r[1] = wt; o.r[2] = dx; o.r[3] = add0; o.r[4] = add1;
                step.push_back(o);
            }
    }
    Op wgrad(const Unit& u, Ref x, Ref dy, Ref dw) const {
        Op o; o.type = OP_WGRAD;
        WgradProb& w = o.wg; memset(&w, 0, sizeof(w));
        w.M = u.N * u.Ho * u.Wo; w.Cout = u.cout; w.Cin = u.cin; w.Kg = u.R * u.R * u.cin;
        w.Ho = u.Ho; w.Wo = u.Wo; w.IH = u.H; w.IW = u.W; w.stride = u.stride; w.pad = u.pad; w.R = u.R; w.S = u.R;
        o.vec = (u.cin % epv()) == 0;
        // wide 3x3 stride-1 layers in bf16: the direct-to-LDS kernel with 160 x (3 taps x 160) tiles.  Widths that fill
        // 64 % of those tiles (128, 256, 512 channels) still gain: the three taps of a filter row share one window of
        // pixels, which the register-staged kernel fetches once per tap (ResNet-50 step 6.49 -> 6.39 ms); at 16 % (64
        // channels) the padded MFMA work costs more than the fetches save (6.53 ms).
        const int t160m = (u.cout + 159) / 160, t160n = (u.cin + 159) / 160;
        const double fill160 = (double)u.cout * u.cin / ((double)t160m * t160n * 160.0 * 160.0);
        const bool fast = net->dtype == LP_BF16 && u.R == 3 && u.stride == 1 && u.pad == 1 && u.Ho == u.H && u.Wo == u.W &&
                          u.cin % 8 == 0 && u.cout % 8 == 0 && fill160 >= 0.6 &&
                          (double)w.M * std::max(u.cin, u.cout) * 2.0 < 2.0e9;
        if (fast) {
            o.cfg = WGRAD_FAST;
            w.tiles_m = t160m; w.tiles_n = 3 * t160n;
            fastdiv_make((unsigned)u.W, &w.mulW, &w.shW);
            fastdiv_make((unsigned)u.H, &w.mulH, &w.shH);
            // one block per CU: as many pixel chunks as fill the chip once, but at least 512 pixels each
            int ks = std::max(1, 256 / (w.tiles_m * w.tiles_n));
            int chunk = std::max(512, (w.M + ks - 1) / ks);
            chunk = (chunk + 31) / 32 * 32;
            w.kchunk = chunk; w.ksplit = (w.M + chunk - 1) / chunk;
            o.r[0] = x; o.r[1] = dy; o.r[2] = dw;
            return o;
        }
        o.cfg = wgrad_cfg_for(u.cout, w.Kg, o.vec);
        const CfgInfo ci = wgrad_cfg_info(o.cfg, net->dtype);
        w.tiles_m = (w.Cout + ci.BM - 1) / ci.BM; w.tiles_n = (w.Kg + ci.BN - 1) / ci.BN;
        // split the pixel dimension: about 4096 pixels per block, more splits (down to 512 pixels) when the filter
        // has so few output tiles that the launch would not fill the chip
        int ks = (w.M + 4095) / 4096;
        const int want = (512 + w.tiles_m * w.tiles_n - 1) / (w.tiles_m * w.tiles_n);
        ks = std::max(ks, std::min(want, (w.M + 511) / 512));
        ks = std::max(1, std::min(ks, 256));
        int chunk = (w.M + ks - 1) / ks;
        chunk = (chunk + ci.BK - 1) / ci.BK * ci.BK;
        ks = (w.M + chunk - 1) / chunk;
        w.ksplit = ks; w.kchunk = chunk;
        o.r[0] = x; o.r[1] = dy; o.r[2] = dw;
        return o;
    }
    Op wtrans(const Unit& u, Ref w, Ref wt) const {
        Op o; o.type = OP_WTRANS;
        memset(&o.wt, 0, sizeof(o.wt));
        o.wt.Cout = u.cout; o.wt.RS = u.R * u.R; o.wt.Cin = u.cin;
        o.r[0] = w; o.r[1] = wt;
        return o;
    }
    Op bn_apply(int M, int C, Ref y, Ref out, Ref stats, Ref gamma, Ref beta, bool relu,
                int skip_mode = 0, Ref skip = Ref(), Ref sstats = Ref(), Ref sgamma = Ref(), Ref sbeta = Ref()) const {
        Op o; o.type = OP_BN_APPLY;
        memset(&o.bna, 0, sizeof(o.bna));
        o.bna.M = M; o.bna.C = C; o.bna.relu = relu; o.bna.skip_mode = skip_mode;
        o.r[0] = y; o.r[1] = out; o.r[2] = stats; o.r[3] = gamma; o.r[4] = beta;
        o.r[5] = skip; o.r[6] = sstats; o.r[7] = sgamma; o.r[8] = sbeta;
        return o;
    }
    Op bn_bwd(int type, int M, int C, Ref g, Ref y, Ref dy, Ref stats, Ref gamma, Ref beta, Ref red, Ref dgamma,
              Ref dbeta, bool relu) const {
        Op o; o.type = type;
        memset(&o.bnb, 0, sizeof(o.bnb));
        o.bnb.M = M; o.bnb.C = C; o.bnb.relu = relu;
        o.r[0] = g; o.r[1] = y; o.r[2] = dy; o.r[3] = stats; o.r[4] = gamma; o.r[5] = beta; o.r[6] = red;
        o.r[7] = dgamma; o.r[8] = dbeta;
        return o;
    }
    Op bn_stats(int M, int C, Ref y, Ref stats) const {
        Op o; o.type = OP_BN_STATS;
        memset(&o.bnb, 0, sizeof(o.bnb));
        o.bnb.M = M; o.bnb.C = C;
        o.r[1] = y; o.r[6] = stats;
        return o;
    }
};

static Ref param_ref(const ModulePlan& m, int k, int t) { return mk(SP_PARAM, k, m.tensors[t].offset); }
static Ref grad_ref(const ModulePlan& m, int k, int t) { return mk(SP_DPARAM, k, m.tensors[t].grad_offset); }

static void add_tensor(std::vector<lp_tensor_info>& v, size_t& poff, size_t& goff, int kind, int block, int slot,
                       int dtype, std::initializer_list<int> dims) {
    lp_tensor_info t;
    memset(&t, 0, sizeof(t));
    t.kind = kind; t.block = block; t.slot = slot; t.dtype = dtype; t.ndim = (int)dims.size();
    size_t n = 1; int i = 0;
    for (int d : dims) { t.dims[i++] = d; n *= (size_t)d; }
    t.numel = n;
    t.offset = poff; t.grad_offset = goff;
    poff = align_up(poff + n * (dtype == LP_BF16 ? 2 : 4));
    goff = align_up(goff + n * 4);
    v.push_back(t);
}
static void add_unit_tensors(std::vector<lp_tensor_info>& v, size_t& poff, size_t& goff, Unit& u, int block, int slot,
                             int dtype) {
    u.t_w = (int)v.size();
    add_tensor(v, poff, goff, LP_T_CONV, block, slot, dtype, {u.cout, u.R, u.R, u.cin});
    u.t_g = (int)v.size();
    add_tensor(v, poff, goff, LP_T_BN_GAMMA, block, slot, LP_F32, {u.cout});
    u.t_b = (int)v.size();
    add_tensor(v, poff, goff, LP_T_BN_BETA, block, slot, LP_F32, {u.cout});
}

static Unit make_unit(int R, int cin, int cout, int stride, int pad, int N, int H, int W, bool relu) {
    Unit u;
    u.R = R; u.cin = cin; u.cout = cout; u.stride = stride; u.pad = pad; u.N = N; u.H = H; u.W = W;
    u.Ho = (H + 2 * pad - R) / stride + 1; u.Wo = (W + 2 * pad - R) / stride + 1;
    u.relu = relu;
    return u;
}

struct WsAlloc {
    size_t off = 0;
    size_t take(size_t bytes) { const size_t o = off; off = align_up(off + std::max<size_t>(bytes, 16)); return o; }
};

// Parameter update inside the backward pass: every filter-gradient operation of module k that writes into dparams[k]
// gets the filter it belongs to (r[4]) and a run of completion tickets in the workspace (r[3], one per output tile;
// cleared by the step that clears the gradients); one last step updates the tensors no filter-gradient kernel owns
// (BN affine, head).  The operations carry these references always; they are bound only while the update is switched on.
static void attach_update(lp_net* net, int k, WsAlloc& ws) {
    ModulePlan& m = net->mods[k];
    m.t_in_epilogue.assign(m.tensors.size(), 0);
    std::vector<size_t> cnt_off(m.tensors.size(), 0);
    m.ws_cnt0 = ws.off;
    bool first = true;
    for (Program* P : {&m.bwd, &m.bwd_dx0}) {
        for (Step& st : *P)
            for (Op& o : st) {
                if (o.type != OP_WGRAD || o.r[2].space != SP_DPARAM) continue;
                int t = -1;
                for (size_t i = 0; i < m.tensors.size(); ++i)
                    if (m.tensors[i].kind == LP_T_CONV && m.tensors[i].grad_offset == o.r[2].off) t = (int)i;
                if (t < 0) continue;
                if (first) { cnt_off[t] = ws.take(sizeof(unsigned) * (size_t)o.wg.tiles_m * o.wg.tiles_n); m.t_in_epilogue[t] = 1; }
                if (!m.t_in_epilogue[t]) continue;
                o.r[3] = mk(SP_WS, 0, cnt_off[t]);
                o.r[4] = mk(SP_PARAM, k, m.tensors[t].offset);
            }
        first = false;
    }
    m.ws_cnt_bytes = ws.off - m.ws_cnt0;
    Builder B{net};
    for (Program* P : {&m.bwd, &m.bwd_dx0}) {
        if (P->empty()) continue;
        for (Step& st : *P) {
            bool clears_grads = false;
            for (const Op& o : st) clears_grads = clears_grads || (o.type == OP_FILL && o.r[0].space == SP_DPARAM);
            if (clears_grads) { if (m.ws_cnt_bytes) st.push_back(B.fill(mk(SP_WS, 0, m.ws_cnt0), m.ws_cnt_bytes)); break; }
        }
        Op o; o.type = OP_SGD_REST; o.r[0] = mk(SP_PARAM, k, 0);
        P->push_back(Step{o});
    }
}

// ---- build one module: units, tensors, workspace, programs ------------------------------------------------
static lp_status build_module(lp_net* net, int k, WsAlloc& ws) {
    ModulePlan& m = net->mods[k];
    const lp_module_desc& d = m.d;
    const int dt = net->dtype;
    const size_t esz = net->esz;
    const int epv = dt == LP_BF16 ? 8 : 4;
    const bool last = (k == net->K - 1);
    size_t poff = 0, goff = 0;
    int N = d.N, H = d.H, W = d.W, C = d.C;

    auto check_c = [&](int c, const char* what) -> lp_status {
        if (c <= 0 || c % epv != 0 || c > 2048)
            return fail(LP_ERR_SHAPE, "module %d: %s = %d must be a positive multiple of %d and at most 2048", k, what, c, epv);
        return LP_OK;
    };
    lp_status st;
    if (d.stem == 1 || d.stem == 2) {
        if ((st = check_c(d.stem_cout, "stem_cout")) != LP_OK) return st;
        m.has_stem = true;
        if (d.stem == 1) m.stem = make_unit(3, C, d.stem_cout, 1, 1, N, H, W, true);
        else {
            if (H % 4 || W % 4) return fail(LP_ERR_SHAPE, "module %d: stem 2 needs H and W divisible by 4", k);
            m.stem = make_unit(7, C, d.stem_cout, 2, 3, N, H, W, true);
        }
        m.stem.need_dgrad = false;
        add_unit_tensors(m.tensors, poff, goff, m.stem, -1, 0, dt);
        H = m.stem.Ho; W = m.stem.Wo; C = d.stem_cout;
        m.pH = H; m.pW = W;
        if (d.stem == 2) { H = (H + 2 - 3) / 2 + 1; W = (W + 2 - 3) / 2 + 1; }
    } else if (d.stem != 0) {
        return fail(LP_ERR_INVALID_ARG, "module %d: stem must be 0, 1 or 2", k);
    } else if ((st = check_c(C, "input channels C")) != LP_OK) return st;

    for (int i = 0; i < d.n_blocks; ++i) {
        const lp_block_desc& b = m.blocks[i];
        if (b.kind != LP_BLOCK_BASIC && b.kind != LP_BLOCK_BOTTLENECK)
            return fail(LP_ERR_INVALID_ARG, "module %d block %d: unknown kind %d", k, i, b.kind);
        if (b.cin != C) return fail(LP_ERR_SHAPE, "module %d block %d: cin %d does not match incoming %d channels", k, i, b.cin, C);
        if (b.stride != 1 && b.stride != 2) return fail(LP_ERR_SHAPE, "module %d block %d: stride %d (1 or 2)", k, i, b.stride);
        if (H % b.stride || W % b.stride) return fail(LP_ERR_SHAPE, "module %d block %d: %dx%d not divisible by stride", k, i, H, W);
        if ((b.stride != 1 || b.cin != b.cout) && !b.proj)
            return fail(LP_ERR_SHAPE, "module %d block %d: shape changes, projection required", k, i);
        if ((st = check_c(b.cout, "cout")) != LP_OK) return st;
        BlockPlan bp;
        if (b.kind == LP_BLOCK_BASIC) {
            bp.main.push_back(make_unit(3, b.cin, b.cout, b.stride, 1, N, H, W, true));
            bp.main.push_back(make_unit(3, b.cout, b.cout, 1, 1, N, H / b.stride, W / b.stride, false));
        } else {
            if ((st = check_c(b.width, "width")) != LP_OK) return st;
            bp.main.push_back(make_unit(1, b.cin, b.width, 1, 0, N, H, W, true));
            bp.main.push_back(make_unit(3, b.width, b.width, b.stride, 1, N, H, W, true));
            bp.main.push_back(make_unit(1, b.width, b.cout, 1, 0, N, H / b.stride, W / b.stride, false));
        }
        for (size_t j = 0; j < bp.main.size(); ++j) add_unit_tensors(m.tensors, poff, goff, bp.main[j], i, (int)j, dt);
        bp.post_relu = b.post_relu != 0;
        if (b.proj) {
            bp.has_proj = true;
            bp.proj_plain = b.proj_plain != 0;
            bp.proj = make_unit(1, b.cin, b.cout, b.stride, 0, N, H, W, false);
            if (bp.proj_plain) {
                bp.proj.t_w = (int)m.tensors.size();
                add_tensor(m.tensors, poff, goff, LP_T_CONV, i, 3, dt, {b.cout, 1, 1, b.cin});
            } else add_unit_tensors(m.tensors, poff, goff, bp.proj, i, 3, dt);
        }
        bp.in_elems = (size_t)N * H * W * C;
        H /= b.stride; W /= b.stride; C = b.cout;
        bp.out_elems = (size_t)N * H * W * C;
        if (bp.in_elems >= (1u << 31) || bp.out_elems >= (1u << 31))
            return fail(LP_ERR_SHAPE, "module %d block %d: tensor beyond 2^31 elements", k, i);
        m.bp.push_back(bp);
    }
    m.oN = N; m.oH = H; m.oW = W; m.oC = C;
    if (d.head != (last ? 1 : 0))
        return fail(LP_ERR_SHAPE, "module %d: head must be set on the last module and only there", k);
    if (last) {
        if (d.n_classes < 1) return fail(LP_ERR_INVALID_ARG, "module %d: n_classes %d", k, d.n_classes);
        m.t_fcw = (int)m.tensors.size();
        add_tensor(m.tensors, poff, goff, LP_T_FC_W, d.n_blocks, 0, LP_F32, {d.n_classes, C});
        m.t_fcb = (int)m.tensors.size();
        add_tensor(m.tensors, poff, goff, LP_T_FC_B, d.n_blocks, 0, LP_F32, {d.n_classes});
    }
    if (m.tensors.empty()) return fail(LP_ERR_SHAPE, "module %d has no layers", k);
    m.param_bytes = poff; m.grad_bytes = goff;

    // ---- workspace ------------------------------------------------------------------------------
    // module 0 without a stem: its first block skips the data-gradient unless dx[0] is requested
    const bool first_block_dx_optional = (k == 0 && !m.has_stem);
    std::vector<Unit*> units;
    if (m.has_stem) units.push_back(&m.stem);
    for (auto& bp : m.bp) {
        for (auto& u : bp.main) units.push_back(&u);
        if (bp.has_proj) units.push_back(&bp.proj);
    }
    m.ws_stats0 = ws.off;
    for (Unit* u : units) u->ws_stats = ws.take(stat_bytes(u->cout));
    m.ws_stats_bytes = ws.off - m.ws_stats0;
    m.ws_red0 = ws.off;
    for (Unit* u : units) u->ws_red = ws.take(stat_bytes(u->cout));
    m.ws_red_bytes = ws.off - m.ws_red0;
    size_t maxD = 0, maxA = 0, maxG = 0, maxP = 0;
    for (Unit* u : units) {
        u->ws_y = ws.take(u->out_elems() * esz);
        u->ws_dy = ws.take(u->out_elems() * esz);     // its own gradient buffer: the filter gradients run at the end
        if (u->need_dgrad) u->ws_wt = ws.take((size_t)u->cout * u->R * u->R * u->cin * esz);
        maxD = std::max(maxD, u->out_elems());
    }
    if (m.has_stem) {
        m.ws_stem_act = ws.take(m.stem.out_elems() * esz);
        maxG = std::max(maxG, m.stem.out_elems());
        if (d.stem == 2) {
            const int Hp = (m.pH + 2 - 3) / 2 + 1, Wp = (m.pW + 2 - 3) / 2 + 1;
            const size_t pn = (size_t)d.N * Hp * Wp * d.stem_cout;
            m.ws_pool_out = ws.take(pn * esz);
            m.ws_pool_arg = ws.take(pn);
            m.ws_gpool = ws.take(m.stem.out_elems() * esz);
        }
    }
    for (size_t i = 0; i < m.bp.size(); ++i) {
        BlockPlan& bp = m.bp[i];
        for (size_t j = 0; j + 1 < bp.main.size(); ++j) {
            bp.ws_act.push_back(ws.take(bp.main[j].out_elems() * esz));
            maxA = std::max(maxA, bp.main[j].out_elems());
        }
        // input
        if (i == 0) {
            if (m.has_stem) bp.in = mk(SP_WS, 0, d.stem == 2 ? m.ws_pool_out : m.ws_stem_act);
            else bp.in = mk(SP_X, k, 0);
        } else bp.in = m.bp[i - 1].out;
        // output
        if (i + 1 == m.bp.size() && !last) bp.out = mk(SP_Y, k, 0);
        else {
            const size_t o = ws.take(bp.out_elems * esz);
            bp.out = mk(SP_WS, 0, o);
            if (i + 1 == m.bp.size()) m.ws_feat = o;
        }
        maxG = std::max(maxG, std::max(bp.in_elems, bp.out_elems));
        if (bp.has_proj) maxP = std::max(maxP, bp.in_elems);
    }
    if (m.bp.empty()) return fail(LP_ERR_SHAPE, "module %d: at least one residual block is required", k);
    m.ws_G[0] = ws.take(maxG * esz); m.ws_G[1] = ws.take(maxG * esz);
    m.ws_A = ws.take(std::max<size_t>(maxA, 1) * esz);
    m.ws_P = ws.take(std::max<size_t>(maxP, 1) * esz);
    for (size_t i = 0; i < m.bp.size(); ++i) {
        BlockPlan& bp = m.bp[i];
        const bool keep = net->keep_gradients;
        bp.ws_gin = keep ? ws.take(bp.in_elems * esz) : m.ws_G[i & 1];
        bp.ws_gproj = (keep && bp.has_proj) ? ws.take(bp.in_elems * esz) : m.ws_P;
        for (size_t j = 0; j + 1 < bp.main.size(); ++j)
            bp.ws_gact.push_back(keep ? ws.take(bp.main[j].out_elems() * esz) : m.ws_A);
    }
    {   // ReLU behind the sum: one buffer for the masked gradient (per block when every gradient is kept)
        size_t maxO = 0, shared = 0;
        for (auto& bp : m.bp) if (bp.post_relu) maxO = std::max(maxO, bp.out_elems);
        if (maxO && !net->keep_gradients) shared = ws.take(maxO * esz);
        for (auto& bp : m.bp) if (bp.post_relu) bp.ws_gmask = net->keep_gradients ? ws.take(bp.out_elems * esz) : shared;
    }
    if (last) {
        m.ws_pooled = ws.take((size_t)N * C * 4);
        m.ws_dfeat = ws.take((size_t)N * H * W * C * esz);
    }

    // ---- forward program ----------------------------------------------------------------------------
    Builder B{net};
    auto stats = [&](const Unit& u) { return mk(SP_WS, 0, u.ws_stats); };
    auto redr = [&](const Unit& u) { return mk(SP_WS, 0, u.ws_red); };
    auto yref = [&](const Unit& u) { return mk(SP_WS, 0, u.ws_y); };
    auto wref = [&](const Unit& u) { return param_ref(m, k, u.t_w); };
    auto gref = [&](const Unit& u) { return param_ref(m, k, u.t_g); };
    auto bref = [&](const Unit& u) { return param_ref(m, k, u.t_b); };
    auto Mof = [&](const Unit& u) { return u.N * u.Ho * u.Wo; };

    Program& F = m.fwd;
    F.push_back(Step{B.fill(mk(SP_WS, 0, m.ws_stats0), m.ws_stats_bytes)});
    if (m.has_stem) {
        const Unit& u = m.stem;
        F.push_back(Step{B.conv_fwd(u, mk(SP_X, k, 0), wref(u), yref(u), stats(u))});
        F.push_back(Step{B.bn_apply(Mof(u), u.cout, yref(u), mk(SP_WS, 0, m.ws_stem_act), stats(u), gref(u), bref(u), true)});
        if (d.stem == 2) {
            Op o; o.type = OP_POOL_FWD;
            memset(&o.pool, 0, sizeof(o.pool));
            o.pool.N = d.N; o.pool.H = m.pH; o.pool.W = m.pW; o.pool.C = d.stem_cout;
            o.pool.Ho = (m.pH + 2 - 3) / 2 + 1; o.pool.Wo = (m.pW + 2 - 3) / 2 + 1;
            o.pool.R = 3; o.pool.stride = 2; o.pool.pad = 1;
            o.r[0] = mk(SP_WS, 0, m.ws_stem_act); o.r[1] = mk(SP_WS, 0, m.ws_pool_out); o.r[2] = mk(SP_WS, 0, m.ws_pool_arg);
            F.push_back(Step{o});
        }
    }
    for (auto& bp : m.bp) {
        Ref cur = bp.in;
        for (size_t j = 0; j < bp.main.size(); ++j) {
            const Unit& u = bp.main[j];
            Step s{B.conv_fwd(u, cur, wref(u), yref(u), stats(u))};
            if (j == 0 && bp.has_proj)
                s.push_back(B.conv_fwd(bp.proj, bp.in, wref(bp.proj), yref(bp.proj), bp.proj_plain ? Ref() : stats(bp.proj)));
            F.push_back(s);
            if (j + 1 < bp.main.size()) {
                Ref a = mk(SP_WS, 0, bp.ws_act[j]);
                F.push_back(Step{B.bn_apply(Mof(u), u.cout, yref(u), a, stats(u), gref(u), bref(u), true)});
                cur = a;
            } else if (bp.has_proj && !bp.proj_plain) {
                const Unit& p = bp.proj;
                F.push_back(Step{B.bn_apply(Mof(u), u.cout, yref(u), bp.out, stats(u), gref(u), bref(u), bp.post_relu, 2, yref(p),
                                            stats(p), gref(p), bref(p))});
            } else {      // identity skip, or the bare projection's result
                F.push_back(Step{B.bn_apply(Mof(u), u.cout, yref(u), bp.out, stats(u), gref(u), bref(u), bp.post_relu, 1,
                                            bp.has_proj ? yref(bp.proj) : bp.in)});
            }
        }
    }
    if (last) {
        Op o; o.type = OP_HEAD_FWD;
        memset(&o.head, 0, sizeof(o.head));
        o.head.N = N; o.head.HW = H * W; o.head.C = C; o.head.classes = d.n_classes;
        o.r[0] = mk(SP_WS, 0, m.ws_feat); o.r[1] = mk(SP_WS, 0, m.ws_pooled);
        o.r[2] = param_ref(m, k, m.t_fcw); o.r[3] = param_ref(m, k, m.t_fcb); o.r[4] = mk(SP_LOGITS, 0, 0);
        F.push_back(Step{o});
    }

    // ---- backward program (two variants when the data-gradient of the first block is optional) ----------
    for (int variant = 0; variant < (first_block_dx_optional ? 2 : 1); ++variant) {
        const bool want_dx_first = first_block_dx_optional ? (variant == 1) : true;
        Program& Bw = variant == 0 ? m.bwd : m.bwd_dx0;
        {
            Step s{B.fill(mk(SP_WS, 0, m.ws_red0), m.ws_red_bytes), B.fill(mk(SP_DPARAM, k, 0), m.grad_bytes)};
            Bw.push_back(s);
        }
        {   // filter re-layouts for every data-gradient of this pass
            Step s;
            for (size_t i = 0; i < m.bp.size(); ++i) {
                const bool need_in_grad = (i > 0) || m.has_stem || want_dx_first;
                BlockPlan& bp = m.bp[i];
                for (size_t j = 0; j < bp.main.size(); ++j)
                    if (j > 0 || need_in_grad) s.push_back(B.wtrans(bp.main[j], wref(bp.main[j]), mk(SP_WS, 0, bp.main[j].ws_wt)));
                if (bp.has_proj && need_in_grad) s.push_back(B.wtrans(bp.proj, wref(bp.proj), mk(SP_WS, 0, bp.proj.ws_wt)));
            }
            if (!s.empty()) Bw.push_back(s);
        }
        Ref g;                                      // gradient with respect to the current block output
        if (last) {
            Op o; o.type = OP_HEAD_BWD;
            memset(&o.head, 0, sizeof(o.head));
            o.head.N = N; o.head.HW = H * W; o.head.C = C; o.head.classes = d.n_classes;
            o.r[1] = mk(SP_WS, 0, m.ws_pooled); o.r[2] = param_ref(m, k, m.t_fcw); o.r[5] = mk(SP_DLOGITS, 0, 0);
            o.r[6] = grad_ref(m, k, m.t_fcw); o.r[7] = grad_ref(m, k, m.t_fcb); o.r[8] = mk(SP_WS, 0, m.ws_dfeat);
            Bw.push_back(Step{o});
            g = mk(SP_WS, 0, m.ws_dfeat);
        } else g = mk(SP_DY, k, 0);
        auto dyref = [&](const Unit& u) { return mk(SP_WS, 0, u.ws_dy); };
        // The filter gradients depend on nothing but a unit's input and its output gradient, and nothing depends on
        // them: they are collected and run as the last step, where the scheduler groups them into few large launches.
        Step wg_tail;
        for (int i = (int)m.bp.size() - 1; i >= 0; --i) {
            BlockPlan& bp = m.bp[i];
            const bool need_in_grad = (i > 0) || m.has_stem || want_dx_first;
            Ref gin;                                // where the gradient with respect to the block input goes
            if (i == 0 && !m.has_stem) gin = mk(SP_DX, k, 0);
            else gin = mk(SP_WS, 0, bp.ws_gin);
            const Ref Pp = mk(SP_WS, 0, bp.ws_gproj);
            bp.graw_ref = g;
            if (bp.post_relu) {                     // through the ReLU behind the sum: everything below sees the masked gradient
                Op o; o.type = OP_RELU_MASK; o.numel = bp.out_elems;
                o.r[0] = g; o.r[1] = bp.out; o.r[2] = mk(SP_WS, 0, bp.ws_gmask);
                Bw.push_back(Step{o});
                g = o.r[2];
            }
            bp.gin_ref = gin; bp.g_ref = g;
            const int nm = (int)bp.main.size();
            Ref gcur = g;                           // gradient arriving at the BN output of unit j
            for (int j = nm - 1; j >= 0; --j) {
                const Unit& u = bp.main[j];
                const bool lastu = (j == nm - 1);
                const Ref Dm = dyref(u), Dp = !bp.has_proj ? Ref() : bp.proj_plain ? g : dyref(bp.proj);   // bare projection: no BN to go through
                Step s1{B.bn_bwd(OP_BN_BWD_REDUCE, Mof(u), u.cout, gcur, yref(u), Dm, stats(u), gref(u), bref(u), redr(u),
                                 grad_ref(m, k, u.t_g), grad_ref(m, k, u.t_b), u.relu)};
                Step s2{B.bn_bwd(OP_BN_BWD_APPLY, Mof(u), u.cout, gcur, yref(u), Dm, stats(u), gref(u), bref(u), redr(u),
                                 grad_ref(m, k, u.t_g), grad_ref(m, k, u.t_b), u.relu)};
                if (lastu && bp.has_proj && !bp.proj_plain) {
                    const Unit& p = bp.proj;
                    s1.push_back(B.bn_bwd(OP_BN_BWD_REDUCE, Mof(p), p.cout, g, yref(p), Dp, stats(p), gref(p), bref(p), redr(p),
                                          grad_ref(m, k, p.t_g), grad_ref(m, k, p.t_b), false));
                    s2.push_back(B.bn_bwd(OP_BN_BWD_APPLY, Mof(p), p.cout, g, yref(p), Dp, stats(p), gref(p), bref(p), redr(p),
                                          grad_ref(m, k, p.t_g), grad_ref(m, k, p.t_b), false));
                }
                Bw.push_back(s1);
                Bw.push_back(s2);
                // weight gradients (and the projection's data-gradient) of this level
                Step s3;
                const Ref uin = (j == 0) ? bp.in : mk(SP_WS, 0, bp.ws_act[j - 1]);
                wg_tail.push_back(B.wgrad(u, uin, Dm, grad_ref(m, k, u.t_w)));
                if (lastu && bp.has_proj) {
                    // a bare projection's gradient operand is the block-output gradient itself, whose buffer the next
                    // block reuses: its filter gradient cannot wait for the tail and runs with this step
                    if (bp.proj_plain) s3.push_back(B.wgrad(bp.proj, bp.in, Dp, grad_ref(m, k, bp.proj.t_w)));
                    else wg_tail.push_back(B.wgrad(bp.proj, bp.in, Dp, grad_ref(m, k, bp.proj.t_w)));
                    if (need_in_grad) B.conv_dgrad(bp.proj, Dp, mk(SP_WS, 0, bp.proj.ws_wt), Pp, Ref(), Ref(), s3);
                }
                // data-gradient of this unit
                if (j > 0) {
                    const Ref A = mk(SP_WS, 0, bp.ws_gact[j - 1]);
                    B.conv_dgrad(u, Dm, mk(SP_WS, 0, u.ws_wt), A, Ref(), Ref(), s3);
                    Bw.push_back(s3);
                    gcur = A;
                } else {
                    if (!s3.empty()) Bw.push_back(s3);
                    if (need_in_grad) {
                        Step s4;
                        // skip path: identity adds the block-output gradient, projection adds its data-gradient.
                        // (a unit with one main conv would need the projection result of the same step: split)
                        B.conv_dgrad(u, Dm, mk(SP_WS, 0, u.ws_wt), gin, bp.has_proj ? Pp : g, Ref(), s4);
                        Bw.push_back(s4);
                    }
                }
            }
            g = gin;
        }
        if (m.has_stem) {
            const Unit& u = m.stem;
            Ref gs = g;
            if (d.stem == 2) {
                Op o; o.type = OP_POOL_BWD;
                memset(&o.pool, 0, sizeof(o.pool));
                o.pool.N = d.N; o.pool.H = m.pH; o.pool.W = m.pW; o.pool.C = d.stem_cout;
                o.pool.Ho = (m.pH + 2 - 3) / 2 + 1; o.pool.Wo = (m.pW + 2 - 3) / 2 + 1;
                o.pool.R = 3; o.pool.stride = 2; o.pool.pad = 1;
                o.r[2] = mk(SP_WS, 0, m.ws_pool_arg); o.r[3] = g; o.r[4] = mk(SP_WS, 0, m.ws_gpool);
                Bw.push_back(Step{o});
                gs = mk(SP_WS, 0, m.ws_gpool);
            }
            const Ref Dm = dyref(u);
            Bw.push_back(Step{B.bn_bwd(OP_BN_BWD_REDUCE, Mof(u), u.cout, gs, yref(u), Dm, stats(u), gref(u), bref(u), redr(u),
                                       grad_ref(m, k, u.t_g), grad_ref(m, k, u.t_b), true)});
            Bw.push_back(Step{B.bn_bwd(OP_BN_BWD_APPLY, Mof(u), u.cout, gs, yref(u), Dm, stats(u), gref(u), bref(u), redr(u),
                                       grad_ref(m, k, u.t_g), grad_ref(m, k, u.t_b), true)});
            wg_tail.push_back(B.wgrad(u, mk(SP_X, k, 0), Dm, grad_ref(m, k, u.t_w)));
        }
        Bw.push_back(wg_tail);
    }
    attach_update(net, k, ws);
    return LP_OK;
}

// ---- build one module in the pre-activation order (Fig. 2): every conv3x3 of a block is preceded by BN-ReLU, the
// skip is the block input (or a bare conv1x1 of the activated input), the stem is a bare conv3x3 and the head is
// BN-ReLU-avgpool-linear.  Unit fields: t_g/t_b and ws_stats/ws_red belong to the BN in FRONT of the conv (cin channels).
static lp_status build_module_pre(lp_net* net, int k, WsAlloc& ws) {
    ModulePlan& m = net->mods[k];
    const lp_module_desc& d = m.d;
    const int dt = net->dtype;
    const size_t esz = net->esz;
    const int epv = dt == LP_BF16 ? 8 : 4;
    const bool last = (k == net->K - 1);
    size_t poff = 0, goff = 0;
    int N = d.N, H = d.H, W = d.W, C = d.C;
    auto check_c = [&](int c, const char* what) -> lp_status {
        if (c <= 0 || c % epv != 0 || c > 2048)
            return fail(LP_ERR_SHAPE, "module %d: %s = %d must be a positive multiple of %d and at most 2048", k, what, c, epv);
        return LP_OK;
    };
    lp_status st;
    if (d.stem == 1) {
        if ((st = check_c(d.stem_cout, "stem_cout")) != LP_OK) return st;
        m.has_stem = true;
        m.stem = make_unit(3, C, d.stem_cout, 1, 1, N, H, W, false);
        m.stem.need_dgrad = false;
        m.stem.t_w = (int)m.tensors.size();
        add_tensor(m.tensors, poff, goff, LP_T_CONV, -1, 0, dt, {d.stem_cout, 3, 3, C});
        C = d.stem_cout;
    } else if (d.stem != 0) {
        return fail(LP_ERR_SHAPE, "module %d: the pre-activation order supports stem 0 or 1", k);
    } else if ((st = check_c(C, "input channels C")) != LP_OK) return st;

    for (int i = 0; i < d.n_blocks; ++i) {
        const lp_block_desc& b = m.blocks[i];
        if (b.kind != LP_BLOCK_BASIC) return fail(LP_ERR_SHAPE, "module %d block %d: the pre-activation order supports basic blocks", k, i);
        if (b.proj_plain || b.post_relu) return fail(LP_ERR_SHAPE, "module %d block %d: proj_plain / post_relu are options of the conv-BN-ReLU order", k, i);
        if (b.cin != C) return fail(LP_ERR_SHAPE, "module %d block %d: cin %d does not match incoming %d channels", k, i, b.cin, C);
        if (b.stride != 1 && b.stride != 2) return fail(LP_ERR_SHAPE, "module %d block %d: stride %d (1 or 2)", k, i, b.stride);
        if (H % b.stride || W % b.stride) return fail(LP_ERR_SHAPE, "module %d block %d: %dx%d not divisible by stride", k, i, H, W);
        if ((b.stride != 1 || b.cin != b.cout) && !b.proj)
            return fail(LP_ERR_SHAPE, "module %d block %d: shape changes, projection required", k, i);
        if ((st = check_c(b.cout, "cout")) != LP_OK) return st;
        BlockPlan bp;
        bp.main.push_back(make_unit(3, b.cin, b.cout, b.stride, 1, N, H, W, true));
        bp.main.push_back(make_unit(3, b.cout, b.cout, 1, 1, N, H / b.stride, W / b.stride, true));
        for (int j = 0; j < 2; ++j) {
            Unit& u = bp.main[j];
            u.t_g = (int)m.tensors.size();
            add_tensor(m.tensors, poff, goff, LP_T_BN_GAMMA, i, j, LP_F32, {u.cin});
            u.t_b = (int)m.tensors.size();
            add_tensor(m.tensors, poff, goff, LP_T_BN_BETA, i, j, LP_F32, {u.cin});
            u.t_w = (int)m.tensors.size();
            add_tensor(m.tensors, poff, goff, LP_T_CONV, i, j, dt, {u.cout, 3, 3, u.cin});
        }
        if (b.proj) {
            bp.has_proj = true;
            bp.proj = make_unit(1, b.cin, b.cout, b.stride, 0, N, H, W, false);
            bp.proj.t_w = (int)m.tensors.size();
            add_tensor(m.tensors, poff, goff, LP_T_CONV, i, 3, dt, {b.cout, 1, 1, b.cin});
        }
        bp.in_elems = (size_t)N * H * W * C;
        H /= b.stride; W /= b.stride; C = b.cout;
        bp.out_elems = (size_t)N * H * W * C;
        if (bp.in_elems >= (1u << 31) || bp.out_elems >= (1u << 31))
            return fail(LP_ERR_SHAPE, "module %d block %d: tensor beyond 2^31 elements", k, i);
        m.bp.push_back(bp);
    }
    if (m.bp.empty()) return fail(LP_ERR_SHAPE, "module %d: at least one residual block is required", k);
    m.oN = N; m.oH = H; m.oW = W; m.oC = C;
    if (d.head != (last ? 1 : 0))
        return fail(LP_ERR_SHAPE, "module %d: head must be set on the last module and only there", k);
    if (last) {
        if (d.n_classes < 1) return fail(LP_ERR_INVALID_ARG, "module %d: n_classes %d", k, d.n_classes);
        m.t_hg = (int)m.tensors.size();
        add_tensor(m.tensors, poff, goff, LP_T_BN_GAMMA, d.n_blocks, 0, LP_F32, {C});
        m.t_hb = (int)m.tensors.size();
        add_tensor(m.tensors, poff, goff, LP_T_BN_BETA, d.n_blocks, 0, LP_F32, {C});
        m.t_fcw = (int)m.tensors.size();
        add_tensor(m.tensors, poff, goff, LP_T_FC_W, d.n_blocks, 0, LP_F32, {d.n_classes, C});
        m.t_fcb = (int)m.tensors.size();
        add_tensor(m.tensors, poff, goff, LP_T_FC_B, d.n_blocks, 0, LP_F32, {d.n_classes});
    }
    m.param_bytes = poff; m.grad_bytes = goff;

    // ---- workspace ------------------------------------------------------------------------------
    const bool first_block_dx_optional = (k == 0 && !m.has_stem);
    const size_t nb = m.bp.size();
    m.ws_stats0 = ws.off;
    for (auto& bp : m.bp) for (auto& u : bp.main) u.ws_stats = ws.take(stat_bytes(u.cin));
    if (last) m.ws_hstats = ws.take(stat_bytes(C));
    m.ws_stats_bytes = ws.off - m.ws_stats0;
    m.ws_red0 = ws.off;
    for (auto& bp : m.bp) for (auto& u : bp.main) u.ws_red = ws.take(stat_bytes(u.cin));
    if (last) m.ws_hred = ws.take(stat_bytes(C));
    m.ws_red_bytes = ws.off - m.ws_red0;
    if (m.has_stem) {
        m.ws_stem_act = ws.take(m.stem.out_elems() * esz);      // the bare stem output = input of the first block
        m.ws_gstem = ws.take(m.stem.out_elems() * esz);
    }
    size_t maxIn = 0, maxMid = 0;
    for (size_t i = 0; i < nb; ++i) {
        BlockPlan& bp = m.bp[i];
        Unit& u0 = bp.main[0];
        Unit& u1 = bp.main[1];
        bp.ws_act.push_back(ws.take(bp.in_elems * esz));         // o1 = ReLU(BN1(block input))
        u0.ws_y = ws.take(u0.out_elems() * esz);                 // y1 = conv1(o1)
        bp.ws_act.push_back(ws.take(u0.out_elems() * esz));      // o2 = ReLU(BN2(y1))
        u0.ws_dy = ws.take(u0.out_elems() * esz);                // gradient on y1 (kept for the filter gradient)
        u0.ws_wt = ws.take((size_t)u0.cout * 9 * u0.cin * esz);
        u1.ws_wt = ws.take((size_t)u1.cout * 9 * u1.cin * esz);
        if (bp.has_proj) {
            bp.proj.ws_y = ws.take(bp.out_elems * esz);
            bp.proj.ws_wt = ws.take((size_t)bp.proj.cout * bp.proj.cin * esz);
        }
        if (i == 0) bp.in = m.has_stem ? mk(SP_WS, 0, m.ws_stem_act) : mk(SP_X, k, 0);
        else bp.in = m.bp[i - 1].out;
        if (i + 1 == nb && !last) bp.out = mk(SP_Y, k, 0);
        else {
            const size_t o = ws.take(bp.out_elems * esz);
            bp.out = mk(SP_WS, 0, o);
            if (i + 1 == nb) m.ws_feat = o;
        }
        if (i + 1 == nb) {
            if (last) { m.ws_ghead = ws.take(bp.out_elems * esz); bp.gout = mk(SP_WS, 0, m.ws_ghead); }
            else bp.gout = mk(SP_DY, k, 0);
        } else bp.gout = mk(SP_WS, 0, ws.take(bp.out_elems * esz));
        maxIn = std::max(maxIn, bp.in_elems);
        maxMid = std::max(maxMid, u0.out_elems());
    }
    m.ws_G[0] = ws.take(maxIn * esz);          // gradient on o1
    m.ws_G[1] = ws.take(maxIn * esz);          // unwanted dx of a stem-less module 0
    m.ws_A = ws.take(maxMid * esz);            // gradient on o2
    m.ws_P = ws.take(maxIn * esz);             // data-gradient of the projection
    if (last) {
        m.ws_hf = ws.take((size_t)N * H * W * C * esz);
        m.ws_pooled = ws.take((size_t)N * C * 4);
        m.ws_dfeat = ws.take((size_t)N * H * W * C * esz);
    }

    // ---- forward program ----------------------------------------------------------------------------
    Builder B{net};
    auto W_ = [&](size_t off) { return mk(SP_WS, 0, off); };
    auto wref = [&](const Unit& u) { return param_ref(m, k, u.t_w); };
    auto gref = [&](const Unit& u) { return param_ref(m, k, u.t_g); };
    auto bref = [&](const Unit& u) { return param_ref(m, k, u.t_b); };
    auto Min = [&](const Unit& u) { return u.N * u.H * u.W; };
    Program& F = m.fwd;
    F.push_back(Step{B.fill(W_(m.ws_stats0), m.ws_stats_bytes)});
    {
        const Unit& f0 = m.bp[0].main[0];
        if (m.has_stem) F.push_back(Step{B.conv_fwd(m.stem, mk(SP_X, k, 0), wref(m.stem), W_(m.ws_stem_act), W_(f0.ws_stats))});
        else F.push_back(Step{B.bn_stats(Min(f0), f0.cin, mk(SP_X, k, 0), W_(f0.ws_stats))});
    }
    for (size_t i = 0; i < nb; ++i) {
        BlockPlan& bp = m.bp[i];
        const Unit& u0 = bp.main[0];
        const Unit& u1 = bp.main[1];
        const Ref o1 = W_(bp.ws_act[0]), y1 = W_(u0.ws_y), o2 = W_(bp.ws_act[1]);
        F.push_back(Step{B.bn_apply(Min(u0), u0.cin, bp.in, o1, W_(u0.ws_stats), gref(u0), bref(u0), true)});
        Step s{B.conv_fwd(u0, o1, wref(u0), y1, W_(u1.ws_stats))};
        if (bp.has_proj) s.push_back(B.conv_fwd(bp.proj, o1, wref(bp.proj), W_(bp.proj.ws_y), Ref()));
        F.push_back(s);
        F.push_back(Step{B.bn_apply(Min(u1), u1.cin, y1, o2, W_(u1.ws_stats), gref(u1), bref(u1), true)});
        // the statistics of the block output belong to whoever normalises it next: the following block or the head
        Ref nstats;
        if (i + 1 < nb) nstats = W_(m.bp[i + 1].main[0].ws_stats);
        else if (last) nstats = W_(m.ws_hstats);
        Op c2 = B.conv_fwd(u1, o2, wref(u1), bp.out, nstats);
        c2.r[3] = bp.has_proj ? W_(bp.proj.ws_y) : bp.in;
        F.push_back(Step{c2});
    }
    const int Mout = N * H * W;
    if (last) {
        F.push_back(Step{B.bn_apply(Mout, C, W_(m.ws_feat), W_(m.ws_hf), W_(m.ws_hstats), param_ref(m, k, m.t_hg),
                                    param_ref(m, k, m.t_hb), true)});
        Op o; o.type = OP_HEAD_FWD;
        memset(&o.head, 0, sizeof(o.head));
        o.head.N = N; o.head.HW = H * W; o.head.C = C; o.head.classes = d.n_classes;
        o.r[0] = W_(m.ws_hf); o.r[1] = W_(m.ws_pooled);
        o.r[2] = param_ref(m, k, m.t_fcw); o.r[3] = param_ref(m, k, m.t_fcb); o.r[4] = mk(SP_LOGITS, 0, 0);
        F.push_back(Step{o});
    }

    // ---- backward program -----------------------------------------------------------------------------
    for (int variant = 0; variant < (first_block_dx_optional ? 2 : 1); ++variant) {
        const bool want_dx_first = first_block_dx_optional ? (variant == 1) : true;
        Program& Bw = variant == 0 ? m.bwd : m.bwd_dx0;
        Bw.push_back(Step{B.fill(W_(m.ws_red0), m.ws_red_bytes), B.fill(mk(SP_DPARAM, k, 0), m.grad_bytes)});
        {
            Step s;
            for (auto& bp : m.bp) {
                for (auto& u : bp.main) s.push_back(B.wtrans(u, wref(u), W_(u.ws_wt)));
                if (bp.has_proj) s.push_back(B.wtrans(bp.proj, wref(bp.proj), W_(bp.proj.ws_wt)));
            }
            Bw.push_back(s);
        }
        if (last) {
            Op o; o.type = OP_HEAD_BWD;
            memset(&o.head, 0, sizeof(o.head));
            o.head.N = N; o.head.HW = H * W; o.head.C = C; o.head.classes = d.n_classes;
            o.r[1] = W_(m.ws_pooled); o.r[2] = param_ref(m, k, m.t_fcw); o.r[5] = mk(SP_DLOGITS, 0, 0);
            o.r[6] = grad_ref(m, k, m.t_fcw); o.r[7] = grad_ref(m, k, m.t_fcb); o.r[8] = W_(m.ws_dfeat);
            Bw.push_back(Step{o});
            for (int type : {OP_BN_BWD_REDUCE, OP_BN_BWD_APPLY})
                Bw.push_back(Step{B.bn_bwd(type, Mout, C, W_(m.ws_dfeat), W_(m.ws_feat), W_(m.ws_ghead), W_(m.ws_hstats),
                                           param_ref(m, k, m.t_hg), param_ref(m, k, m.t_hb), W_(m.ws_hred),
                                           grad_ref(m, k, m.t_hg), grad_ref(m, k, m.t_hb), true)});
        }
        const Ref A = W_(m.ws_A), D1 = W_(m.ws_G[0]), Pp = W_(m.ws_P);
        Step wg_tail;
        for (int i = (int)nb - 1; i >= 0; --i) {
            BlockPlan& bp = m.bp[i];
            const Unit& u0 = bp.main[0];
            const Unit& u1 = bp.main[1];
            const Ref o1 = W_(bp.ws_act[0]), y1 = W_(u0.ws_y), o2 = W_(bp.ws_act[1]), dy1 = W_(u0.ws_dy);
            Ref gin;                                 // gradient with respect to the block input
            if (i > 0) gin = m.bp[i - 1].gout;
            else if (m.has_stem) gin = W_(m.ws_gstem);
            else gin = (k > 0 || want_dx_first) ? mk(SP_DX, k, 0) : W_(m.ws_G[1]);
            {   // through conv2 (and the projection) into the two activations
                Step s;
                B.conv_dgrad(u1, bp.gout, W_(u1.ws_wt), A, Ref(), Ref(), s);
                if (bp.has_proj) B.conv_dgrad(bp.proj, bp.gout, W_(bp.proj.ws_wt), Pp, Ref(), Ref(), s);
                Bw.push_back(s);
            }
            wg_tail.push_back(B.wgrad(u1, o2, bp.gout, grad_ref(m, k, u1.t_w)));
            if (bp.has_proj) wg_tail.push_back(B.wgrad(bp.proj, o1, bp.gout, grad_ref(m, k, bp.proj.t_w)));
            for (int type : {OP_BN_BWD_REDUCE, OP_BN_BWD_APPLY})
                Bw.push_back(Step{B.bn_bwd(type, Min(u1), u1.cin, A, y1, dy1, W_(u1.ws_stats), gref(u1), bref(u1), W_(u1.ws_red),
                                           grad_ref(m, k, u1.t_g), grad_ref(m, k, u1.t_b), true)});
            wg_tail.push_back(B.wgrad(u0, o1, dy1, grad_ref(m, k, u0.t_w)));
            {
                Step s;
                B.conv_dgrad(u0, dy1, W_(u0.ws_wt), D1, bp.has_proj ? Pp : Ref(), Ref(), s);
                Bw.push_back(s);
            }
            for (int type : {OP_BN_BWD_REDUCE, OP_BN_BWD_APPLY}) {
                Op o = B.bn_bwd(type, Min(u0), u0.cin, D1, bp.in, gin, W_(u0.ws_stats), gref(u0), bref(u0), W_(u0.ws_red),
                                grad_ref(m, k, u0.t_g), grad_ref(m, k, u0.t_b), true);
                if (type == OP_BN_BWD_APPLY && !bp.has_proj) o.r[9] = bp.gout;      // identity skip
                Bw.push_back(Step{o});
            }
        }
        if (m.has_stem) wg_tail.push_back(B.wgrad(m.stem, mk(SP_X, k, 0), W_(m.ws_gstem), grad_ref(m, k, m.stem.t_w)));
        Bw.push_back(wg_tail);
    }
    attach_update(net, k, ws);
    return LP_OK;
}

// the whole local step of module k as one list: forward, loss and terminal adjoint (with the multiplier update), backward
static void build_step_programs(lp_net* net, int k) {
    ModulePlan& m = net->mods[k];
    const bool last = (k == net->K - 1);
    Step loss_step;
    if (last) {
        Op o; o.type = OP_CE;
        memset(&o.head, 0, sizeof(o.head));
        o.head.N = m.oN; o.head.classes = m.d.n_classes;
        o.r[0] = mk(SP_LOGITS, 0, 0); o.r[1] = mk(SP_LABELS, 0, 0); o.r[2] = mk(SP_LOSS, 0, sizeof(float) * k);
        o.r[3] = mk(SP_DLOGITS, 0, 0);
        loss_step.push_back(o);
    } else {
        const size_t numel = (size_t)m.oN * m.oH * m.oW * m.oC;
        Op o; o.type = OP_LOSS; o.numel = numel;
        o.r[0] = mk(SP_Y, k, 0); o.r[1] = mk(SP_XNEXT, k, 0); o.r[2] = mk(SP_LAM, k, 0); o.r[3] = mk(SP_DY, k, 0);
        o.r[4] = mk(SP_LOSS, 0, sizeof(float) * k);
        loss_step.push_back(o);     // with a multiplier step bound, the same kernel also writes lam + step*(y - x_next)
    }
    for (int variant = 0; variant < 2; ++variant) {
        const Program& bw = variant == 0 ? m.bwd : m.bwd_dx0;
        Program& out = variant == 0 ? m.step : m.step_dx0;
        if (bw.empty()) continue;
        out = m.fwd;
        // The pass that writes F_k(x_k) (the BN apply + skip of the last block, conv-BN-ReLU order) also evaluates the
        // local loss and the terminal adjoint on the value it stores: F_k(x_k) is not read again.  Where the module
        // output is written by something else (the convolution epilogue of the pre-activation order) the loss keeps
        // its own pass.
        Op* last_apply = nullptr;
        if (!last && !out.empty() && out.back().size() == 1 && out.back()[0].type == OP_BN_APPLY &&
            out.back()[0].r[1].space == SP_Y)
            last_apply = &out.back()[0];
        if (last_apply) {
            last_apply->cfg = 1;
            last_apply->r[9] = mk(SP_XNEXT, k, 0); last_apply->r[10] = mk(SP_LAM, k, 0);
            last_apply->r[11] = mk(SP_DY, k, 0); last_apply->r[12] = mk(SP_LOSS, 0, sizeof(float) * k);
        } else {
            out.push_back(loss_step);
            for (Op& o : out.back()) o.phase = 1;
        }
        for (const Step& st : bw) {
            out.push_back(st);
            for (Op& o : out.back()) o.phase = 2;
        }
    }
}

static lp_status build_aux(lp_net* net, int j, WsAlloc& ws) {
    AuxPlan& a = net->aux[j];
    a.chained = a.d.from_prev != 0 && j > 0;
    const ModulePlan& m0 = net->mods[a.chained ? j : 0];      // whose input tensor the AuxNet reads: x_j or the mini-batch x_0
    const ModulePlan& mt = net->mods[j + 1];
    const int epv = net->dtype == LP_BF16 ? 8 : 4;
    const int depth = a.d.depth > 0 ? a.d.depth : 1;
    if (depth > LP_AUX_MAX_DEPTH) return fail(LP_ERR_INVALID_ARG, "aux %d: depth %d > %d", j, depth, LP_AUX_MAX_DEPTH);
    if (a.d.cin != m0.d.C) return fail(LP_ERR_SHAPE, "aux %d: cin %d != channels of its input (%d)", j, a.d.cin, m0.d.C);
    if (a.d.cout != mt.d.C || a.d.cout % epv) return fail(LP_ERR_SHAPE, "aux %d: cout %d != channels of x_%d (%d)", j, a.d.cout, j + 1, mt.d.C);
    // the stack: blocks 0..depth-2 end in ReLU, the last one maps to the shape of x_{j+1}
    int c = a.d.cin, H = m0.d.H, W = m0.d.W;
    for (int i = 0; i + 1 < depth; ++i) {
        const int co = a.d.mid_cout[i], sd = a.d.mid_stride[i];
        if (co < 1 || co % epv) return fail(LP_ERR_SHAPE, "aux %d: block %d has %d output channels (need a positive multiple of %d)", j, i, co, epv);
        if (sd < 1 || H % sd || W % sd) return fail(LP_ERR_SHAPE, "aux %d: stride %d of block %d does not divide %dx%d", j, sd, i, H, W);
        a.pre.push_back(make_unit(3, c, co, sd, 1, m0.d.N, H, W, true));
        c = co; H = a.pre.back().Ho; W = a.pre.back().Wo;
    }
    if (a.d.stride < 1 || H != mt.d.H * a.d.stride || W != mt.d.W * a.d.stride)
        return fail(LP_ERR_SHAPE, "aux %d: stride %d does not map %dx%d to %dx%d", j, a.d.stride, H, W, mt.d.H, mt.d.W);
    a.u = make_unit(3, c, a.d.cout, a.d.stride, 1, m0.d.N, H, W, a.d.relu != 0);
    if (a.u.Ho != mt.d.H || a.u.Wo != mt.d.W) return fail(LP_ERR_SHAPE, "aux %d: output %dx%d != %dx%d", j, a.u.Ho, a.u.Wo, mt.d.H, mt.d.W);
    size_t poff = 0, goff = 0;
    for (int i = 0; i + 1 < depth; ++i) add_unit_tensors(a.tensors, poff, goff, a.pre[i], -1, i, net->dtype);
    add_unit_tensors(a.tensors, poff, goff, a.u, -1, depth - 1, net->dtype);
    a.param_bytes = poff; a.grad_bytes = goff;
    std::vector<Unit*> us;
    for (Unit& p : a.pre) us.push_back(&p);
    us.push_back(&a.u);
    for (int i = 0; i < depth; ++i) {
        Unit& u = *us[i];
        u.ws_stats = ws.take(stat_bytes(u.cout));
        u.ws_red = ws.take(stat_bytes(u.cout));
        u.ws_y = ws.take(u.out_elems() * net->esz);
        u.ws_dy = ws.take(u.out_elems() * net->esz);
        if (i > 0) u.ws_wt = ws.take((size_t)u.cout * 9 * u.cin * net->esz);
        if (i + 1 < depth) {
            a.ws_act.push_back(ws.take(u.out_elems() * net->esz));
            a.ws_gact.push_back(ws.take(u.out_elems() * net->esz));
        }
    }
    a.ws_out = ws.take(a.u.out_elems() * net->esz);
    a.ws_g = ws.take(a.u.out_elems() * net->esz);

    Builder B{net};
    auto W_ = [&](size_t off) { return mk(SP_WS, 0, off); };
    auto P_ = [&](int t) { return mk(SP_AUXP, j, a.tensors[t].offset); };
    auto G_ = [&](int t) { return mk(SP_AUXG, j, a.tensors[t].grad_offset); };
    auto Mof = [](const Unit& u) { return u.N * u.Ho * u.Wo; };
    // forward pass of the stack from `in`, the last block writing to `out`
    auto forward = [&](Program& prog, Ref in, Ref out) {
        for (int i = 0; i < depth; ++i) {
            const Unit& u = *us[i];
            const Ref dst = i + 1 < depth ? W_(a.ws_act[i]) : out;
            prog.push_back(Step{B.conv_fwd(u, i == 0 ? in : W_(a.ws_act[i - 1]), P_(u.t_w), W_(u.ws_y), W_(u.ws_stats))});
            prog.push_back(Step{B.bn_apply(Mof(u), u.cout, W_(u.ws_y), dst, W_(u.ws_stats), P_(u.t_g), P_(u.t_b), u.relu)});
        }
    };
    auto fill_stats = [&](Step& s) {
        for (int i = 0; i < depth; ++i) s.push_back(B.fill(W_(us[i]->ws_stats), stat_bytes(us[i]->cout)));
    };
    const Ref in0 = a.chained ? mk(SP_XOUT, j - 1, 0) : mk(SP_IMAGE, 0, 0);
    {
        Step s0;
        fill_stats(s0);
        a.fwd.push_back(s0);
    }
    forward(a.fwd, in0, mk(SP_XOUT, j, 0));
    {   // the same pass with a compact layout of its intermediates (statistics, conv results, inner activations) in the
        // library's own device array: nothing of it is kept for the gradient calls
        WsAlloc sc; sc.off = net->scratch_bytes;
        std::vector<size_t> s_stats(depth), s_y(depth), s_act(depth, 0);
        for (int i = 0; i < depth; ++i) {
            s_stats[i] = sc.take(stat_bytes(us[i]->cout));
            s_y[i] = sc.take(us[i]->out_elems() * net->esz);
            if (i + 1 < depth) s_act[i] = sc.take(us[i]->out_elems() * net->esz);
        }
        net->scratch_bytes = sc.off;
        auto S_ = [&](size_t off) { return mk(SP_SCRATCH, 0, off); };
        Step s0;
        for (int i = 0; i < depth; ++i) s0.push_back(B.fill(S_(s_stats[i]), stat_bytes(us[i]->cout)));
        a.fwd_static.push_back(s0);
        for (int i = 0; i < depth; ++i) {
            const Unit& u = *us[i];
            const Ref dst = i + 1 < depth ? S_(s_act[i]) : mk(SP_XOUT, j, 0);
            a.fwd_static.push_back(Step{B.conv_fwd(u, i == 0 ? in0 : S_(s_act[i - 1]), P_(u.t_w), S_(s_y[i]), S_(s_stats[i]))});
            a.fwd_static.push_back(Step{B.bn_apply(Mof(u), u.cout, S_(s_y[i]), dst, S_(s_stats[i]), P_(u.t_g), P_(u.t_b), u.relu)});
        }
    }

    // Gradient through the stack.  First part (before the loss or correction kernel): the AuxNet output again, from the
    // saved pre-BN tensor of the last block; a chained AuxNet is distilled at the CORRECTED input x_j (Sec. 4.2), so
    // its whole forward pass is run again from there.
    const Ref din = a.chained ? mk(SP_XTGT, j - 1, 0) : mk(SP_IMAGE, 0, 0);
    {
        Step s0{B.fill(mk(SP_AUXG, j, 0), a.grad_bytes)};
        for (int i = 0; i < depth; ++i) s0.push_back(B.fill(W_(us[i]->ws_red), stat_bytes(us[i]->cout)));
        if (a.chained) fill_stats(s0);
        for (int i = 1; i < depth; ++i) s0.push_back(B.wtrans(*us[i], P_(us[i]->t_w), W_(us[i]->ws_wt)));
        a.bwd_a.push_back(s0);
    }
    if (a.chained) forward(a.bwd_a, din, W_(a.ws_out));
    else a.bwd_a.push_back(Step{B.bn_apply(Mof(a.u), a.u.cout, W_(a.u.ws_y), W_(a.ws_out), W_(a.u.ws_stats), P_(a.u.t_g), P_(a.u.t_b), a.u.relu)});
    // Second part: from the gradient on the output, block by block towards the input; the filter gradients last.
    Step wg_tail;
    Ref gcur = W_(a.ws_g);
    for (int i = depth - 1; i >= 0; --i) {
        const Unit& u = *us[i];
        const Ref y = W_(u.ws_y), dyc = W_(u.ws_dy), st = W_(u.ws_stats), red = W_(u.ws_red);
        a.bwd_b.push_back(Step{B.bn_bwd(OP_BN_BWD_REDUCE, Mof(u), u.cout, gcur, y, dyc, st, P_(u.t_g), P_(u.t_b), red, G_(u.t_g), G_(u.t_b), u.relu)});
        a.bwd_b.push_back(Step{B.bn_bwd(OP_BN_BWD_APPLY, Mof(u), u.cout, gcur, y, dyc, st, P_(u.t_g), P_(u.t_b), red, G_(u.t_g), G_(u.t_b), u.relu)});
        wg_tail.push_back(B.wgrad(u, i == 0 ? din : W_(a.ws_act[i - 1]), dyc, G_(u.t_w)));
        if (i > 0) {
            Step s;
            B.conv_dgrad(u, dyc, W_(u.ws_wt), W_(a.ws_gact[i - 1]), Ref(), Ref(), s);
            a.bwd_b.push_back(s);
            gcur = W_(a.ws_gact[i - 1]);
        }
    }
    a.bwd_b.push_back(wg_tail);
    return LP_OK;
}

// ----------------------------------------------------------------------------------------------------
// scheduler: advance the selected programs in lock-step, merging equal operations into grouped launches
// ----------------------------------------------------------------------------------------------------
static int elem_blocks(size_t nvec) { return (int)((nvec + kElemVecsPerBlock - 1) / kElemVecsPerBlock); }

// algorithmic work of one operation: flops of the contraction, minimum bytes each tensor moves once
static void op_work(const lp_net* net, const Op& o, double& flops, double& bytes) {
    const double e = (double)net->esz;
    flops = 0; bytes = 0;
    switch (o.type) {
        case OP_CONV: {
            const ConvProb& c = o.conv;
            flops = 2.0 * c.M * c.Ncol * c.Kg;
            const double nimg = (double)c.M / ((double)c.OA * c.OB);
            const double in_e = nimg * c.IH * c.IW * c.Cin / ((double)c.omul * c.omul);   // shared by the parity classes
            const double w_e = (double)c.Ncol * c.Kg;
            double out_e = (double)c.M * c.Ncol;
            if (o.r[3].space != SP_NONE) out_e += (double)c.M * c.Ncol;
            if (o.r[4].space != SP_NONE) out_e += (double)c.M * c.Ncol;
            bytes = (in_e + w_e + out_e) * e;
        } break;
        case OP_WGRAD: {
            const WgradProb& w = o.wg;
            flops = 2.0 * w.M * w.Cout * w.Kg;
            const double nimg = (double)w.M / ((double)w.Ho * w.Wo);
            bytes = (nimg * w.IH * w.IW * w.Cin + (double)w.M * w.Cout) * e + (double)w.Cout * w.Kg * 4.0;
        } break;
        case OP_WTRANS: bytes = 2.0 * o.wt.Cout * o.wt.RS * o.wt.Cin * e; break;
        case OP_FILL: bytes = (double)o.fill_bytes; break;
        case OP_BN_APPLY:      // fused with the loss / terminal adjoint: + x_next, lam, dy (the multiplier written back: + 1)
            bytes = (double)o.bna.M * o.bna.C * e * ((o.bna.skip_mode ? 3.0 : 2.0) + (o.cfg == 1 ? 3.0 : 0.0)); break;
        case OP_BN_BWD_REDUCE: bytes = (double)o.bnb.M * o.bnb.C * e * 2.0; break;
        case OP_BN_BWD_APPLY: bytes = (double)o.bnb.M * o.bnb.C * e * (o.r[9].space != SP_NONE ? 4.0 : 3.0); break;
        case OP_BN_STATS: bytes = (double)o.bnb.M * o.bnb.C * e; break;
        case OP_LOSS: bytes = (double)o.numel * e * 4.0; break;
        case OP_RELU_MASK: bytes = (double)o.numel * e * 3.0; break;
        case OP_POOL_FWD:
        case OP_POOL_BWD: bytes = ((double)o.pool.N * o.pool.H * o.pool.W + (double)o.pool.N * o.pool.Ho * o.pool.Wo) * o.pool.C * e; break;
        case OP_HEAD_FWD:
        case OP_HEAD_BWD: bytes = (double)o.head.N * o.head.HW * o.head.C * e; break;
        default: break;
    }
}

// Split-K of a grouped launch of the wide-layer filter-gradient kernel.  Every block has the same tile, so its time
// is its number of 32-pixel k-tiles plus a fixed epilogue (the atomic adds of its 160 x 480 partial sums, which
// cost about as much as 24 k-tiles); one block runs per CU.  Pick the common chunk length that minimises
// rounds x (chunk + epilogue).  The gradients were zeroed at the start of the backward pass and are accumulated
// atomically, so the split may differ from launch to launch.
static void plan_wgrad_fast_splits(WgradGroup& g) {
    const int kEpilogue = 24, kCUs = 256;
    int best_chunk = 16; double best_cost = 1e300;
    int max_kt = 1;
    for (int i = 0; i < g.nprob; ++i) max_kt = std::max(max_kt, (g.p[i].M + 31) / 32);
    for (int chunk = 16; chunk <= std::max(16, max_kt); ++chunk) {
        long blocks = 0;
        for (int i = 0; i < g.nprob; ++i) {
            const int kt = (g.p[i].M + 31) / 32;
            blocks += (long)g.p[i].tiles_m * g.p[i].tiles_n * ((kt + chunk - 1) / chunk);
        }
        const double cost = (double)((blocks + kCUs - 1) / kCUs) * (chunk + kEpilogue);
        if (cost < best_cost) { best_cost = cost; best_chunk = chunk; }
    }
    for (int i = 0; i < g.nprob; ++i) {
        WgradProb& p = g.p[i];
        const int kt = (p.M + 31) / 32;
        const int ks = (kt + best_chunk - 1) / best_chunk;
        p.ksplit = ks;
        p.kchunk = (kt + ks - 1) / ks * 32;          // equal chunks
    }
}

static hipError_t launch_group_impl(lp_net* net, std::vector<const Op*>& ops, size_t base, int n, const Bindings& b, hipStream_t s,
                                    int* used_cfg, int* used_blocks);

static hipError_t launch_group(lp_net* net, std::vector<const Op*>& ops, const Bindings& b, hipStream_t s) {
    hipError_t err = hipSuccess;
    for (size_t base = 0; base < ops.size() && err == hipSuccess; base += kMaxGroup) {
        const int n = (int)std::min<size_t>(kMaxGroup, ops.size() - base);
        if (ops[base]->type == OP_SGD_REST && !net->fused_update) continue;      // nothing to launch, nothing to record
        if (!net->prof) { err = launch_group_impl(net, ops, base, n, b, s, nullptr, nullptr); continue; }
        lp_net::ProfRec r;
        r.type = ops[base]->type; r.cfg = ops[base]->cfg; r.nprob = n; r.blocks = 0; r.flops = 0; r.bytes = 0;
        for (int i = 0; i < n; ++i) { double f, by; op_work(net, *ops[base + i], f, by); r.flops += f; r.bytes += by; }
        for (hipEvent_t* e : {&r.a, &r.b}) {
            if (!net->prof_pool.empty()) { *e = net->prof_pool.back(); net->prof_pool.pop_back(); }
            else if ((err = hipEventCreate(e)) != hipSuccess) return err;
        }
        if ((err = hipEventRecord(r.a, s)) != hipSuccess) return err;
        err = launch_group_impl(net, ops, base, n, b, s, &r.cfg, &r.blocks);
        if (err == hipSuccess) err = hipEventRecord(r.b, s);
        net->prof_recs.push_back(r);
    }
    return err;
}

static hipError_t launch_group_impl(lp_net* net, std::vector<const Op*>& ops, size_t base, int n, const Bindings& b, hipStream_t s,
                                    int* used_cfg, int* used_blocks) {
    const int type = ops[base]->type, dt = net->dtype;
    const int epv = dt == LP_BF16 ? 8 : 4;
    hipError_t err = hipSuccess;
    {
        switch (type) {
            case OP_FILL: {
                FillGroup g; g.nprob = n; int tot = 0;
                for (int i = 0; i < n; ++i) {
                    const Op& o = *ops[base + i];
                    g.p[i].ptr = resolve(o.r[0], b); g.p[i].bytes = o.fill_bytes; g.p[i].block_start = tot;
                    tot += elem_blocks(o.fill_bytes / 16);
                }
                g.total_blocks = tot;
                err = launch_fill(g, s);
            } break;
            case OP_WTRANS: {
                WtransGroup g; g.nprob = n; int tot = 0;
                for (int i = 0; i < n; ++i) {
                    const Op& o = *ops[base + i];
                    g.p[i] = o.wt;
                    g.p[i].w = resolve(o.r[0], b); g.p[i].wt = resolve(o.r[1], b); g.p[i].block_start = tot;
                    tot += ((o.wt.Cin + 63) / 64) * ((o.wt.Cout + 63) / 64) * o.wt.RS;
                }
                g.total_blocks = tot;
                err = launch_wtrans(g, dt, s);
            } break;
            case OP_CONV: {
                ConvGroup g; g.nprob = n; int tot = 0;
                int cfg = ops[base]->cfg;
                bool win = cfg >= WIN64_512x160;
                const bool fast = cfg >= FAST_256x320;
                if (win) {
                    // The window kernel needs its eight-wave tiles (two waves per SIMD keep the matrix core fed) and
                    // about one tile per compute unit; a launch with fewer tiles goes to the implicit-GEMM kernel,
                    // whose smaller tile variants fill the chip.
                    // (next to the launches of other stream lanes the idle compute units are not lost: keep it)
                    const int TW = net->lanes_in_flight > 1 ? 0 : 200;
                    long big = 0;
                    for (int i = 0; i < n; ++i) {
                        const ConvProb& c = ops[base + i]->conv;
                        big += cfg == WIN64_256x320 ? (long)((c.M + 255) / 256) * ((c.Ncol + 319) / 320)
                                                    : (long)((c.M + 511) / 512) * ((c.Ncol + 159) / 160);
                    }
                    if (big < TW) { cfg = cfg == WIN64_256x320 ? FAST_256x320 : FAST_512x160; win = false; }
                }
                if (cfg == FAST_256x320 || cfg == FAST_512x160) {
                    // Too few full-size tiles for the chip: the four-wave variants (and the two-wave one of the
                    // 320-wide family).  k-tiles of 64 channels where every problem allows them and the tile fits.
                    long big = 0, mid = 0;
                    bool k64 = true;
                    for (int i = 0; i < n; ++i) {
                        const ConvProb& c = ops[base + i]->conv;
                        if (cfg == FAST_256x320) {
                            big += (long)((c.M + 255) / 256) * ((c.Ncol + 319) / 320);
                            mid += (long)((c.M + 127) / 128) * ((c.Ncol + 319) / 320);
                        } else {
                            big += (long)((c.M + 511) / 512) * ((c.Ncol + 159) / 160);
                        }
                        k64 = k64 && (c.Cin % 64 == 0);
                    }
                    // alone on the device a launch wants at least 200 tiles; next to the launches of other stream lanes
                    // the idle compute units are not lost, and the larger tile's better operand reuse wins
                    const int T1 = net->lanes_in_flight > 1 ? 64 : 200, T2 = 200, T3 = 200;
                    if (cfg == FAST_256x320) {
                        if (big < T1) cfg = mid < T2 ? FAST_128x160 : FAST_128x320;
                        if (k64) cfg = cfg == FAST_256x320 ? FAST64_256x320 : cfg == FAST_128x320 ? FAST64_128x320 : FAST64_128x160;
                    } else if (big < T3) {
                        cfg = k64 ? FAST64_256x160 : FAST_256x160;
                    }
                }
                if (used_cfg) *used_cfg = cfg;
                const CfgInfo ci = win ? conv_win_cfg_info(cfg) : fast ? conv_fast_cfg_info(cfg) : conv_cfg_info(cfg, dt);
                // longest tiles first: the blocks of a launch are dispatched in order
                std::stable_sort(ops.begin() + base, ops.begin() + base + n,
                                 [](const Op* a, const Op* b2) { return a->conv.Kg > b2->conv.Kg; });
                BnBwdGroup sg; sg.nprob = 0; sg.total_blocks = 0; sg.eps = net->eps; sg.cmax = 0;
                for (int i = 0; i < n; ++i) {
                    const Op& o = *ops[base + i];
                    ConvProb& p = g.p[i]; p = o.conv;
                    p.in = resolve(o.r[0], b); p.wt = resolve(o.r[1], b); p.out = resolve(o.r[2], b);
                    p.add0 = resolve(o.r[3], b); p.add1 = resolve(o.r[4], b); p.stats = (double*)resolve(o.r[5], b);
                    if (net->deterministic && p.stats) {
                        // fixed summation order: no per-tile atomics from the epilogue; one workgroup per tensor sums
                        // the stored result afterwards (a single addition per channel onto the cleared statistics)
                        BnBwdProb& q = sg.p[sg.nprob]; memset(&q, 0, sizeof(q));
                        q.y = p.out; q.red = p.stats; q.M = p.M; q.C = p.Ncol;
                        q.block_start = sg.total_blocks; q.nblocks = 1; sg.total_blocks += 1;
                        sg.cmax = std::max(sg.cmax, q.C); ++sg.nprob;
                        p.stats = nullptr;
                    }
                    p.tiles_m = (p.M + ci.BM - 1) / ci.BM; p.tiles_n = (p.Ncol + ci.BN - 1) / ci.BN;
                    p.tile_start = tot; tot += p.tiles_m * p.tiles_n;
                }
                g.total_tiles = tot;
                if (used_blocks) *used_blocks = tot;
                err = win ? launch_conv_win(g, cfg, s) : fast ? launch_conv_fast(g, cfg, s) : launch_conv(g, dt, cfg, ops[base]->vec, s);
                if (err == hipSuccess && sg.nprob) err = launch_bn_stats(sg, dt, s);
            } break;
            case OP_WGRAD: {
                WgradGroup g; g.nprob = n; int tot = 0;
                for (int i = 0; i < n; ++i) g.p[i] = ops[base + i]->wg;
                if (net->deterministic) {       // one block per output tile runs through all pixels: no partial sums to add
                    const int bk = ops[base]->cfg == WGRAD_FAST ? 32 : wgrad_cfg_info(ops[base]->cfg, dt).BK;
                    for (int i = 0; i < n; ++i) { g.p[i].ksplit = 1; g.p[i].kchunk = (g.p[i].M + bk - 1) / bk * bk; }
                } else if (ops[base]->cfg == WGRAD_FAST) plan_wgrad_fast_splits(g);
                for (int i = 0; i < n; ++i) {
                    const Op& o = *ops[base + i];
                    WgradProb& p = g.p[i];
                    p.x = resolve(o.r[0], b); p.dy = resolve(o.r[1], b); p.dw = (float*)resolve(o.r[2], b);
                    p.w = nullptr; p.vel = nullptr; p.master = nullptr; p.cnt = nullptr;
                    if (net->fused_update && o.r[4].space == SP_PARAM) {
                        const int k = o.r[4].idx;
                        p.w = resolve(o.r[4], b); p.cnt = (unsigned*)resolve(o.r[3], b);
                        if (b.vel && b.vel[k]) p.vel = (float*)((char*)b.vel[k] + o.r[2].off);
                        if (b.master && b.master[k]) p.master = (float*)((char*)b.master[k] + o.r[2].off);
                    }
                    p.tile_start = tot;
                    tot += ops[base]->cfg == WGRAD_FAST ? wgrad_fast_blocks(p) : p.tiles_m * p.tiles_n * p.ksplit;
                }
                g.total_tiles = tot;
                g.lr = net->fu_lr; g.momentum = net->fu_momentum; g.wd = net->fu_wd; g.lowp = dt == LP_BF16;
                if (used_blocks) *used_blocks = tot;
                err = ops[base]->cfg == WGRAD_FAST ? launch_wgrad_fast(g, s) : launch_wgrad(g, dt, ops[base]->cfg, ops[base]->vec, s);
            } break;
            case OP_BN_APPLY: {
                BnApplyGroup g; g.nprob = n; g.eps = net->eps; g.cmax = 0; int tot = 0;
                const bool fused_loss = ops[base]->cfg == 1;
                g.rho = b.rho; g.scale = b.scale; g.step = b.mstep;
                for (int i = 0; i < n; ++i) g.cmax = std::max(g.cmax, ops[base + i]->bna.C);
                for (int i = 0; i < n; ++i) {
                    const Op& o = *ops[base + i];
                    BnApplyProb& p = g.p[i]; p = o.bna;
                    p.y = resolve(o.r[0], b); p.out = resolve(o.r[1], b); p.stats = (const double*)resolve(o.r[2], b);
                    p.gamma = (const float*)resolve(o.r[3], b); p.beta = (const float*)resolve(o.r[4], b);
                    p.skip = resolve(o.r[5], b); p.sstats = (const double*)resolve(o.r[6], b);
                    p.sgamma = (const float*)resolve(o.r[7], b); p.sbeta = (const float*)resolve(o.r[8], b);
                    p.xn = nullptr; p.lam = nullptr; p.dy = nullptr; p.lam_out = nullptr; p.loss = nullptr; p.r2 = nullptr;
                    if (fused_loss) {      // the local loss and terminal adjoint (and the multiplier update) ride on this pass
                        p.xn = resolve(o.r[9], b); p.lam = resolve(o.r[10], b); p.dy = resolve(o.r[11], b);
                        p.loss = (float*)resolve(o.r[12], b);
                        p.r2 = net->r2 ? net->r2 + (p.loss - b.loss) : nullptr;      // loss + k  ->  r2 + k
                        p.lam_out = b.mstep != 0.f ? const_cast<void*>(p.lam) : nullptr;
                    }
                    p.block_start = tot; p.nblocks = elem_blocks((size_t)p.M * p.C / epv); tot += p.nblocks;
                }
                g.total_blocks = tot;
                err = launch_bn_apply(g, dt, fused_loss, s);
            } break;
            case OP_BN_STATS:
            case OP_BN_BWD_REDUCE:
            case OP_BN_BWD_APPLY: {
                BnBwdGroup g; g.nprob = n; g.eps = net->eps; g.cmax = 0; int tot = 0;
                for (int i = 0; i < n; ++i) g.cmax = std::max(g.cmax, ops[base + i]->bnb.C);
                for (int i = 0; i < n; ++i) {
                    const Op& o = *ops[base + i];
                    BnBwdProb& p = g.p[i]; p = o.bnb;
                    p.g = resolve(o.r[0], b); p.y = resolve(o.r[1], b); p.dy = resolve(o.r[2], b);
                    p.stats = (const double*)resolve(o.r[3], b); p.gamma = (const float*)resolve(o.r[4], b);
                    p.beta = (const float*)resolve(o.r[5], b); p.red = (double*)resolve(o.r[6], b);
                    p.dgamma = (float*)resolve(o.r[7], b); p.dbeta = (float*)resolve(o.r[8], b);
                    p.add = resolve(o.r[9], b);
                    p.block_start = tot;
                    if (type == OP_BN_BWD_REDUCE) {
                        // at least 64 rows per workgroup, and (one trip of the reduction being four rows per row lane) no more
                        // workgroups than trips
                        const int rows_trip = 4 * std::max(1, bn_reduce_threads(g.cmax) / (p.C / epv));
                        p.nblocks = net->deterministic ? 1 : std::max(1, std::min(std::min(256, (p.M + 63) / 64), (p.M + rows_trip - 1) / rows_trip));
                    } else if (type != OP_BN_BWD_APPLY) p.nblocks = net->deterministic ? 1 : std::max(1, std::min(256, (p.M + 63) / 64));
                    else p.nblocks = elem_blocks((size_t)p.M * p.C / epv);
                    tot += p.nblocks;
                }
                g.total_blocks = tot;
                err = type == OP_BN_STATS ? launch_bn_stats(g, dt, s)
                      : type == OP_BN_BWD_REDUCE ? launch_bn_bwd_reduce(g, dt, s) : launch_bn_bwd_apply(g, dt, s);
            } break;
            case OP_SGD_REST: {
                if (!net->fused_update) break;
                SgdGroup g; g.nprob = 0; g.total_blocks = 0; g.lr = net->fu_lr; g.momentum = net->fu_momentum; g.wd = net->fu_wd;
                for (int i = 0; i < n && err == hipSuccess; ++i) {
                    const int k = ops[base + i]->r[0].idx;
                    const ModulePlan& m = net->mods[k];
                    for (size_t t = 0; t < m.tensors.size() && err == hipSuccess; ++t) {
                        if (m.t_in_epilogue[t]) continue;
                        const lp_tensor_info& ti = m.tensors[t];
                        SgdProb& p = g.p[g.nprob];
                        p.p = (char*)b.params[k] + ti.offset; p.lowp = ti.dtype == LP_BF16;
                        p.g = (const float*)((const char*)b.dparams[k] + ti.grad_offset);
                        p.v = (b.vel && b.vel[k]) ? (float*)((char*)b.vel[k] + ti.grad_offset) : nullptr;
                        p.master = (b.master && b.master[k]) ? (float*)((char*)b.master[k] + ti.grad_offset) : nullptr;
                        p.numel = ti.numel; p.block_start = g.total_blocks;
                        p.nblocks = (int)((ti.numel + kSgdElemsPerBlock - 1) / kSgdElemsPerBlock);
                        g.total_blocks += p.nblocks;
                        if (++g.nprob == kMaxGroup) { err = launch_sgd(g, s); g.nprob = 0; g.total_blocks = 0; }
                    }
                }
                if (g.nprob && err == hipSuccess) err = launch_sgd(g, s);
            } break;
            case OP_LOSS: {
                LossGroup g; g.nprob = n; g.rho = b.rho; g.scale = b.scale; g.step = b.mstep; int tot = 0;
                for (int i = 0; i < n; ++i) {
                    const Op& o = *ops[base + i];
                    LossProb& p = g.p[i];
                    p.y = resolve(o.r[0], b); p.xn = resolve(o.r[1], b); p.lam = resolve(o.r[2], b); p.dy = resolve(o.r[3], b);
                    // the multiplier update rides on the pass that has y, x_next and lam in registers anyway
                    p.lam_out = b.mstep != 0.f ? const_cast<void*>(p.lam) : nullptr;
                    p.loss = (float*)resolve(o.r[4], b); p.numel = o.numel;
                    p.r2 = net->r2 ? net->r2 + (p.loss - b.loss) : nullptr;
                    p.block_start = tot; p.nblocks = elem_blocks(o.numel / epv); tot += p.nblocks;
                }
                g.total_blocks = tot;
                err = launch_loss(g, dt, s);
            } break;
            case OP_RELU_MASK: {
                MaskGroup g; g.nprob = n; int tot = 0;
                for (int i = 0; i < n; ++i) {
                    const Op& o = *ops[base + i];
                    MaskProb& p = g.p[i];
                    p.g = resolve(o.r[0], b); p.out = resolve(o.r[1], b); p.gm = resolve(o.r[2], b); p.numel = o.numel;
                    p.block_start = tot; p.nblocks = elem_blocks(o.numel / epv); tot += p.nblocks;
                }
                g.total_blocks = tot;
                err = launch_relu_mask(g, dt, s);
            } break;
            case OP_CE:
                for (int i = 0; i < n && err == hipSuccess; ++i) {
                    const Op& o = *ops[base + i];
                    err = launch_ce((const float*)resolve(o.r[0], b), (const int32_t*)resolve(o.r[1], b), (float*)resolve(o.r[2], b),
                                    (float*)resolve(o.r[3], b), o.head.N, o.head.classes, s);
                }
                break;
            case OP_POOL_FWD:
            case OP_POOL_BWD:
                for (int i = 0; i < n && err == hipSuccess; ++i) {
                    const Op& o = *ops[base + i];
                    PoolProb p = o.pool;
                    p.x = resolve(o.r[0], b); p.y = resolve(o.r[1], b); p.arg = (uint8_t*)resolve(o.r[2], b);
                    p.dy = resolve(o.r[3], b); p.dx = resolve(o.r[4], b);
                    err = type == OP_POOL_FWD ? launch_maxpool_fwd(p, dt, s) : launch_maxpool_bwd(p, dt, s);
                }
                break;
            case OP_HEAD_FWD:
            case OP_HEAD_BWD:
                for (int i = 0; i < n && err == hipSuccess; ++i) {
                    const Op& o = *ops[base + i];
                    HeadProb p = o.head;
                    p.feat = resolve(o.r[0], b); p.pooled = (float*)resolve(o.r[1], b); p.w = (const float*)resolve(o.r[2], b);
                    p.b = (const float*)resolve(o.r[3], b); p.logits = (float*)resolve(o.r[4], b);
                    p.dlogits = (const float*)resolve(o.r[5], b); p.dw = (float*)resolve(o.r[6], b);
                    p.db = (float*)resolve(o.r[7], b); p.dfeat = resolve(o.r[8], b);
                    err = type == OP_HEAD_FWD ? launch_head_fwd(p, dt, s) : launch_head_bwd(p, dt, s);
                }
                break;
            default: err = hipErrorInvalidValue;
        }
    }
    return err;
}

// Order of the grouped launches of a set of independent programs (no launch happens here).
static void plan_programs(const std::vector<const Program*>& progs, std::vector<std::vector<const Op*>>& plan) {
    const size_t np = progs.size();
    std::vector<size_t> step(np, 0);
    std::vector<std::vector<char>> issued(np);
    for (size_t i = 0; i < np; ++i)
        if (!progs[i]->empty()) issued[i].assign((*progs[i])[0].size(), 0);
    std::vector<char> off(np, 0);
    for (;;) {
        // Programs of a fused step move through its phases together (a program that is ahead waits): the operations
        // of one phase merge into grouped launches, those of different phases would not.
        int min_phase = 1 << 30;
        for (size_t i = 0; i < np; ++i)
            if (step[i] < progs[i]->size()) min_phase = std::min(min_phase, (*progs[i])[step[i]][0].phase);
        for (size_t i = 0; i < np; ++i)
            off[i] = step[i] >= progs[i]->size() || (*progs[i])[step[i]][0].phase != min_phase;
        // candidate operations: everything not yet issued in the current step of every program
        int best_key = -1, best_cnt = 0;
        std::vector<std::pair<int, int>> keys;     // (key, count)
        bool any = false;
        for (size_t i = 0; i < np; ++i) {
            if (off[i]) continue;
            const Step& st = (*progs[i])[step[i]];
            for (size_t j = 0; j < st.size(); ++j) {
                if (issued[i][j]) continue;
                any = true;
                const int key = st[j].key();
                bool found = false;
                for (auto& kc : keys) if (kc.first == key) { ++kc.second; found = true; }
                if (!found) keys.push_back({key, 1});
            }
        }
        if (!any) break;
        // The program with the most steps left is the critical path: one of its pending operations goes next (the one
        // most programs share), and every other program with the same operation pending joins the launch.  Filter
        // gradients only when nothing else is ready, so that the tails of all programs meet and merge.
        bool only_wgrad = true;
        for (auto& kc : keys) only_wgrad = only_wgrad && (kc.first / 64 == OP_WGRAD);
        size_t lead = np, lead_left = 0;
        for (size_t i = 0; i < np; ++i) {
            if (off[i]) continue;
            const Step& st = (*progs[i])[step[i]];
            bool eligible = false;
            for (size_t j = 0; j < st.size(); ++j)
                eligible = eligible || (!issued[i][j] && (only_wgrad || st[j].key() / 64 != OP_WGRAD));
            const size_t left = progs[i]->size() - step[i];
            if (eligible && left > lead_left) { lead = i; lead_left = left; }
        }
        {
            const Step& st = (*progs[lead])[step[lead]];
            for (size_t j = 0; j < st.size(); ++j) {
                if (issued[lead][j]) continue;
                const int key = st[j].key();
                if (!only_wgrad && key / 64 == OP_WGRAD) continue;
                int cnt = 0;
                for (auto& kc : keys) if (kc.first == key) cnt = kc.second;
                if (cnt > best_cnt || (cnt == best_cnt && key < best_key)) { best_key = key; best_cnt = cnt; }
            }
        }
        std::vector<const Op*> ops;
        for (size_t i = 0; i < np; ++i) {
            if (off[i]) continue;
            const Step& st = (*progs[i])[step[i]];
            for (size_t j = 0; j < st.size(); ++j)
                if (!issued[i][j] && st[j].key() == best_key) { ops.push_back(&st[j]); issued[i][j] = 1; }
        }
        plan.push_back(ops);
        for (size_t i = 0; i < np; ++i) {
            if (off[i]) continue;
            bool done = true;
            for (char c : issued[i]) done = done && c;
            if (done) {
                ++step[i];
                if (step[i] < progs[i]->size()) issued[i].assign((*progs[i])[step[i]].size(), 0);
            }
        }
    }
}

static lp_status run_programs(lp_net* net, const std::vector<const Program*>& progs, const Bindings& b, hipStream_t s,
                              const std::vector<int>* lane = nullptr) {
    // lane[i]: 0 = program i is issued on the caller's stream, j > 0 = on the net's j-th extra stream, concurrently.
    // Programs of one lane are grouped with each other only.
    constexpr int kLanes = 4;
    std::vector<const Program*> set[kLanes];
    for (size_t i = 0; i < progs.size(); ++i) set[lane ? std::min(std::max((*lane)[i], 0), kLanes - 1) : 0].push_back(progs[i]);
    std::vector<std::vector<const Op*>> plan[kLanes];
    int used = 0;
    for (int l = 0; l < kLanes; ++l) if (!set[l].empty()) { plan_programs(set[l], plan[l]); ++used; }
    hipError_t err = hipSuccess;
    net->lanes_in_flight = std::max(used, 1);
    if (used <= 1) {
        for (int l = 0; l < kLanes; ++l)
            for (auto& ops : plan[l]) {
                err = launch_group(net, ops, b, s);
                if (err != hipSuccess) return fail(LP_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(err));
            }
        return LP_OK;
    }
    if (!net->lanes_ready) {
        // all handles into locals first: the net takes them only when every one exists, a partial set is destroyed
        hipEvent_t fork = nullptr, join[kLanes] = {nullptr, nullptr, nullptr, nullptr};
        hipStream_t extra[kLanes] = {nullptr, nullptr, nullptr, nullptr};
        err = hipEventCreateWithFlags(&fork, hipEventDisableTiming);
        for (int l = 1; l < kLanes && err == hipSuccess; ++l) {
            err = hipStreamCreateWithFlags(&extra[l], hipStreamNonBlocking);
            if (err == hipSuccess) err = hipEventCreateWithFlags(&join[l], hipEventDisableTiming);
        }
        if (err != hipSuccess) {
            if (fork) (void)hipEventDestroy(fork);
            for (int l = 1; l < kLanes; ++l) {
                if (extra[l]) (void)hipStreamDestroy(extra[l]);
                if (join[l]) (void)hipEventDestroy(join[l]);
            }
            return fail(LP_ERR_HIP, "extra streams: %s", hipGetErrorString(err));
        }
        net->ev_fork = fork;
        for (int l = 1; l < kLanes; ++l) { net->extra_stream[l] = extra[l]; net->ev_join[l] = join[l]; }
        net->lanes_ready = true;
    }
    if (net->prof && net->prof_serial) {
        size_t pos[kLanes] = {0, 0, 0, 0};
        for (bool more = true; more;) {
            more = false;
            for (int l = 0; l < kLanes; ++l)
                if (pos[l] < plan[l].size()) {
                    if ((err = launch_group(net, plan[l][pos[l]++], b, s)) != hipSuccess)
                        return fail(LP_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(err));
                    more = true;
                }
        }
        return LP_OK;
    }
    hipStream_t st[kLanes];
    st[0] = s;
    for (int l = 1; l < kLanes; ++l) st[l] = net->extra_stream[l];
    if ((err = hipEventRecord(net->ev_fork, s)) != hipSuccess) return fail(LP_ERR_HIP, "extra streams: %s", hipGetErrorString(err));
    for (int l = 1; l < kLanes; ++l)
        if (!plan[l].empty() && (err = hipStreamWaitEvent(st[l], net->ev_fork, 0)) != hipSuccess)
            return fail(LP_ERR_HIP, "extra streams: %s", hipGetErrorString(err));
    size_t pos[kLanes] = {0, 0, 0, 0};
    for (bool more = true; more && err == hipSuccess;) {
        more = false;
        for (int l = 0; l < kLanes && err == hipSuccess; ++l)
            if (pos[l] < plan[l].size()) { err = launch_group(net, plan[l][pos[l]++], b, st[l]); more = true; }
    }
    // join even after a failed launch: the caller's stream must not run ahead of what was enqueued on the others
    for (int l = 1; l < kLanes; ++l) {
        if (plan[l].empty()) continue;
        hipError_t e2 = hipEventRecord(net->ev_join[l], st[l]);
        if (e2 == hipSuccess) e2 = hipStreamWaitEvent(s, net->ev_join[l], 0);
        if (err == hipSuccess) err = e2;
    }
    if (err != hipSuccess) return fail(LP_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(err));
    return LP_OK;
}

// stream lane of every selected module, in the order the programs are collected
static std::vector<int> lanes_of(const lp_net* net, uint32_t module_mask) {
    std::vector<int> out;
    for (int k = 0; k < net->K; ++k)
        if ((module_mask >> k) & 1u) out.push_back(k < (int)net->lane.size() ? net->lane[k] : 0);
    return out;
}
static bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

}  // namespace

// ----------------------------------------------------------------------------------------------------
// The library's own device array (lp_auxnet_forward_static): intermediates of the AuxNet forward passes for callers
// that can lend no workspace.  Every GPU the library runs on holds its own copy until the process ends; in host code
// the array's name is only a handle, its device address comes from hipGetSymbolAddress, once per device.
// ----------------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[LP_STATIC_SCRATCH_BYTES];   // (the compiler gives it external linkage in the code object because host code names it below)

namespace {
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static char* g_scratch_ptr[kMaxDevices] = {nullptr};

static lp_status static_scratch(char** out) {
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return fail(LP_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(err));
    if (dev < 0 || dev >= kMaxDevices) return fail(LP_ERR_HIP, "device ordinal %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err != hipSuccess || !p) return fail(LP_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(err));
        g_scratch_ptr[dev] = (char*)p;
    }
    *out = g_scratch_ptr[dev];
    return LP_OK;
}
}  // namespace

// ----------------------------------------------------------------------------------------------------
// C ABI
// ----------------------------------------------------------------------------------------------------
extern "C" {

const char* lp_last_error(void) { return g_err.c_str(); }
const char* lp_version(void) { return "lp-gfx950 0.1"; }

lp_status lp_net_create(int K, const lp_module_desc* mods, const lp_aux_desc* aux, int dtype, float bn_eps,
                        struct lp_net** out) {
    if (!out) return fail(LP_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (K < 1 || K > 32) return fail(LP_ERR_INVALID_ARG, "K = %d outside [1, 32]", K);
    if (!mods) return fail(LP_ERR_INVALID_ARG, "mods is NULL");
    if (dtype != LP_F32 && dtype != LP_BF16) return fail(LP_ERR_DTYPE, "dtype %d is neither LP_F32 nor LP_BF16", dtype);
    if (!(bn_eps > 0.f)) return fail(LP_ERR_INVALID_ARG, "bn_eps must be positive");
    lp_net* net = new lp_net();
    net->K = K; net->dtype = dtype; net->eps = bn_eps; net->esz = dtype == LP_BF16 ? 2 : 4;
    net->keep_gradients = g_keep_gradients;
    net->mods.resize(K);
    net->saved_x.assign(K, nullptr);
    net->saved_y.assign(K, nullptr);
    WsAlloc ws;
    lp_status st = LP_OK;
    for (int k = 0; k < K && st == LP_OK; ++k) {
        ModulePlan& m = net->mods[k];
        m.d = mods[k];
        if (m.d.N < 1 || m.d.H < 1 || m.d.W < 1 || m.d.C < 1) { st = fail(LP_ERR_INVALID_ARG, "module %d: non-positive input shape", k); break; }
        if (m.d.n_blocks < 1 || m.d.n_blocks > 64 || !m.d.blocks) { st = fail(LP_ERR_INVALID_ARG, "module %d: n_blocks %d or blocks NULL", k, m.d.n_blocks); break; }
        m.blocks.assign(m.d.blocks, m.d.blocks + m.d.n_blocks);
        m.d.blocks = nullptr;
        if (m.d.order != LP_ORDER_POST && m.d.order != LP_ORDER_PRE) { st = fail(LP_ERR_INVALID_ARG, "module %d: unknown block order %d", k, m.d.order); break; }
        st = m.d.order == LP_ORDER_PRE ? build_module_pre(net, k, ws) : build_module(net, k, ws);
        if (st == LP_OK) build_step_programs(net, k);
        if (st == LP_OK && k > 0) {
            const ModulePlan& p = net->mods[k - 1];
            if (p.oN != m.d.N || p.oH != m.d.H || p.oW != m.d.W || p.oC != m.d.C)
                st = fail(LP_ERR_SHAPE, "module %d output [%d,%d,%d,%d] != module %d input [%d,%d,%d,%d]", k - 1, p.oN, p.oH,
                          p.oW, p.oC, k, m.d.N, m.d.H, m.d.W, m.d.C);
        }
    }
    if (st == LP_OK && aux) {
        net->aux.resize(K - 1);
        for (int j = 0; j < K - 1 && st == LP_OK; ++j) {
            net->aux[j].d = aux[j];
            st = build_aux(net, j, ws);
        }
    }
    if (st != LP_OK) { delete net; return st; }
    net->ws_bytes = ws.off;
    // Default stream lanes.  Up to four modules: a lane each, so that the memory-bound passes of one module overlap
    // the matrix-bound passes of another and launches fill each other's tails.  More modules: those of the same
    // output width run the same layer shapes and merge into full launches, so they share a lane (at most four lanes).
    net->lane.assign(K, 0);
    if (K <= 4) {
        for (int k = 0; k < K; ++k) net->lane[k] = k;
    } else {
        std::vector<int> widths;
        for (int k = 0; k < K; ++k) {
            const int w = net->mods[k].oC;
            size_t i = 0;
            while (i < widths.size() && widths[i] != w) ++i;
            if (i == widths.size()) widths.push_back(w);
            net->lane[k] = (int)std::min<size_t>(i, 3);
        }
    }
    *out = net;
    return LP_OK;
}

lp_status lp_net_destroy(struct lp_net* net) {
    if (net) {
        if (net->ev_fork) (void)hipEventDestroy(net->ev_fork);
        for (int l = 1; l < 4; ++l) {
            if (net->extra_stream[l]) (void)hipStreamDestroy(net->extra_stream[l]);
            if (net->ev_join[l]) (void)hipEventDestroy(net->ev_join[l]);
        }
        for (auto& r : net->prof_recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
        for (hipEvent_t e : net->prof_pool) (void)hipEventDestroy(e);
    }
    delete net;
    return LP_OK;
}

lp_status lp_net_set_stream_lanes(struct lp_net* net, const int* lanes) {
    if (!net) return fail(LP_ERR_INVALID_ARG, "net is NULL");
    if (!lanes) { net->lane.assign(net->K, 0); return LP_OK; }
    for (int k = 0; k < net->K; ++k)
        if (lanes[k] < 0 || lanes[k] > 3) return fail(LP_ERR_INVALID_ARG, "lanes[%d] = %d outside [0, 3]", k, lanes[k]);
    net->lane.assign(lanes, lanes + net->K);
    return LP_OK;
}

lp_status lp_net_set_deterministic(struct lp_net* net, int on) {
    if (!net) return fail(LP_ERR_INVALID_ARG, "net is NULL");
    net->deterministic = on != 0;
    return LP_OK;
}

lp_status lp_net_set_fused_update(struct lp_net* net, int on, float lr, float momentum, float weight_decay,
                                  float* const* velocity, float* const* master) {
    if (!net) return fail(LP_ERR_INVALID_ARG, "net is NULL");
    if (!on) { net->fused_update = false; return LP_OK; }
    if (momentum != 0.f && !velocity) return fail(LP_ERR_INVALID_ARG, "momentum != 0 needs velocity buffers");
    std::vector<float*> vel(net->K, nullptr), mas(net->K, nullptr);
    for (int k = 0; k < net->K; ++k) {
        if (momentum != 0.f) {
            if (!velocity[k]) return fail(LP_ERR_INVALID_ARG, "velocity[%d] is NULL", k);
            vel[k] = velocity[k];
        }
        if (master) mas[k] = master[k];
        if (misaligned(vel[k]) || misaligned(mas[k])) return fail(LP_ERR_INVALID_ARG, "parameter set %d: a buffer is not 16-byte aligned", k);
    }
    net->fu_vel = vel; net->fu_master = mas;
    net->fu_lr = lr; net->fu_momentum = momentum; net->fu_wd = weight_decay;
    net->fused_update = true;
    return LP_OK;
}

lp_status lp_net_set_residual_output(struct lp_net* net, float* r2) {
    if (!net) return fail(LP_ERR_INVALID_ARG, "net is NULL");
    if (r2 && (reinterpret_cast<uintptr_t>(r2) & 3u)) return fail(LP_ERR_INVALID_ARG, "r2 is not 4-byte aligned");
    net->r2 = r2;
    return LP_OK;
}

lp_status lp_profile_enable(struct lp_net* net, int on) {
    if (!net) return fail(LP_ERR_INVALID_ARG, "net is NULL");
    net->prof = on != 0;
    net->prof_serial = on == 2;
    return LP_OK;
}

lp_status lp_profile_fetch(struct lp_net* net, lp_profile_rec* out, int max_recs, int* n_out) {
    if (!net || !n_out) return fail(LP_ERR_INVALID_ARG, "NULL argument");
    const int n = (int)net->prof_recs.size();
    *n_out = n;
    if (!out) return LP_OK;                       // size query
    if (max_recs < n) return fail(LP_ERR_INVALID_ARG, "room for %d records, %d recorded", max_recs, n);
    for (int i = 0; i < n; ++i) {
        lp_net::ProfRec& r = net->prof_recs[i];
        hipError_t err = hipEventSynchronize(r.b);
        float ms = 0.f;
        if (err == hipSuccess) err = hipEventElapsedTime(&ms, r.a, r.b);
        if (err != hipSuccess) return fail(LP_ERR_HIP, "event timing failed: %s", hipGetErrorString(err));
        out[i].kind = r.type; out[i].cfg = r.cfg; out[i].nprob = r.nprob; out[i].blocks = r.blocks;
        out[i].ms = ms; out[i].flops = r.flops; out[i].bytes = r.bytes;
        net->prof_pool.push_back(r.a); net->prof_pool.push_back(r.b);
    }
    net->prof_recs.clear();
    return LP_OK;
}

static lp_status table_of(const lp_net* net, int aux, int k, const std::vector<lp_tensor_info>** t, size_t* pb, size_t* gb) {
    if (!net) return fail(LP_ERR_INVALID_ARG, "net is NULL");
    if (aux) {
        if (k < 0 || k >= (int)net->aux.size()) return fail(LP_ERR_INVALID_ARG, "aux block %d out of range", k);
        *t = &net->aux[k].tensors; *pb = net->aux[k].param_bytes; *gb = net->aux[k].grad_bytes;
    } else {
        if (k < 0 || k >= net->K) return fail(LP_ERR_INVALID_ARG, "module %d out of range", k);
        *t = &net->mods[k].tensors; *pb = net->mods[k].param_bytes; *gb = net->mods[k].grad_bytes;
    }
    return LP_OK;
}
lp_status lp_net_param_bytes(const struct lp_net* net, int aux, int k, size_t* param_bytes, size_t* grad_bytes) {
    const std::vector<lp_tensor_info>* t; size_t pb, gb;
    lp_status st = table_of(net, aux, k, &t, &pb, &gb);
    if (st != LP_OK) return st;
    if (param_bytes) *param_bytes = pb;
    if (grad_bytes) *grad_bytes = gb;
    return LP_OK;
}
lp_status lp_net_num_tensors(const struct lp_net* net, int aux, int k, int* n) {
    const std::vector<lp_tensor_info>* t; size_t pb, gb;
    lp_status st = table_of(net, aux, k, &t, &pb, &gb);
    if (st != LP_OK) return st;
    if (!n) return fail(LP_ERR_INVALID_ARG, "n is NULL");
    *n = (int)t->size();
    return LP_OK;
}
lp_status lp_net_tensor_info(const struct lp_net* net, int aux, int k, int i, lp_tensor_info* info) {
    const std::vector<lp_tensor_info>* t; size_t pb, gb;
    lp_status st = table_of(net, aux, k, &t, &pb, &gb);
    if (st != LP_OK) return st;
    if (!info || i < 0 || i >= (int)t->size()) return fail(LP_ERR_INVALID_ARG, "tensor index %d out of range", i);
    *info = (*t)[i];
    return LP_OK;
}

lp_status lp_net_workspace_bytes(const struct lp_net* net, size_t* bytes) {
    if (!net || !bytes) return fail(LP_ERR_INVALID_ARG, "NULL argument");
    *bytes = net->ws_bytes;
    return LP_OK;
}
lp_status lp_net_set_workspace(struct lp_net* net, void* dev_ptr, size_t bytes) {
    if (!net || !dev_ptr) return fail(LP_ERR_INVALID_ARG, "NULL argument");
    if (reinterpret_cast<uintptr_t>(dev_ptr) & 255u) return fail(LP_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    if (bytes < net->ws_bytes) return fail(LP_ERR_WORKSPACE, "workspace of %zu bytes, %zu needed", bytes, net->ws_bytes);
    net->ws = (char*)dev_ptr; net->ws_given = bytes; net->fwd_done = 0; net->aux_fwd_done = false;
    return LP_OK;
}

static lp_status check_common(const lp_net* net, uint32_t mask, bool need_mask) {
    if (!net) return fail(LP_ERR_INVALID_ARG, "net is NULL");
    if (!net->ws) return fail(LP_ERR_WORKSPACE, "no workspace set (lp_net_set_workspace)");
    if (need_mask) {
        if (mask == 0) return fail(LP_ERR_INVALID_ARG, "module_mask selects no module");
        if (net->K < 32 && (mask >> net->K) != 0) return fail(LP_ERR_INVALID_ARG, "module_mask 0x%x has bits beyond K = %d", mask, net->K);
    }
    return LP_OK;
}

lp_status lp_auxnet_forward(struct lp_net* net, void* stream, const void* image, const void* const* aux_params,
                            void* const* x_out) {
    lp_status st = check_common(net, 0, false);
    if (st != LP_OK) return st;
    if (net->aux.empty()) return fail(LP_ERR_STATE, "the net was created without AuxNet descriptors");
    if (!image || !aux_params || !x_out) return fail(LP_ERR_INVALID_ARG, "NULL argument");
    if (misaligned(image)) return fail(LP_ERR_INVALID_ARG, "image is not 16-byte aligned");
    std::vector<const Program*> progs;
    for (int j = 0; j < net->K - 1; ++j) {
        if (!aux_params[j] || !x_out[j]) return fail(LP_ERR_INVALID_ARG, "aux_params[%d] or x_out[%d] is NULL", j, j);
        if (misaligned(aux_params[j]) || misaligned(x_out[j])) return fail(LP_ERR_INVALID_ARG, "aux tensor %d is not 16-byte aligned", j);
        progs.push_back(&net->aux[j].fwd);
    }
    Bindings b; b.ws = net->ws; b.image = image; b.auxp = aux_params; b.xout = x_out;
    bool any_chained = false;
    for (const AuxPlan& a : net->aux) any_chained = any_chained || a.chained;
    if (!any_chained) st = run_programs(net, progs, b, (hipStream_t)stream);
    else   // x_{j+1} = AuxNet_j(x_j): one block after the other (the AuxNets are forward-locked, Sec. 4.2)
        for (size_t j = 0; j < progs.size() && st == LP_OK; ++j) st = run_programs(net, {progs[j]}, b, (hipStream_t)stream);
    if (st == LP_OK) net->aux_fwd_done = true;
    return st;
}

lp_status lp_auxnet_forward_static(struct lp_net* net, void* stream, const void* image, const void* const* aux_params,
                                   void* const* x_out) {
    if (!net) return fail(LP_ERR_INVALID_ARG, "net is NULL");
    if (net->aux.empty()) return fail(LP_ERR_STATE, "the net was created without AuxNet descriptors");
    if (!image || !aux_params || !x_out) return fail(LP_ERR_INVALID_ARG, "NULL argument");
    if (misaligned(image)) return fail(LP_ERR_INVALID_ARG, "image is not 16-byte aligned");
    if (net->scratch_bytes > LP_STATIC_SCRATCH_BYTES)
        return fail(LP_ERR_WORKSPACE, "the AuxNet forward passes need %zu bytes of intermediates, the library's own array holds %zu",
                    net->scratch_bytes, (size_t)LP_STATIC_SCRATCH_BYTES);
    std::vector<const Program*> progs;
    for (int j = 0; j < net->K - 1; ++j) {
        if (!aux_params[j] || !x_out[j]) return fail(LP_ERR_INVALID_ARG, "aux_params[%d] or x_out[%d] is NULL", j, j);
        if (misaligned(aux_params[j]) || misaligned(x_out[j])) return fail(LP_ERR_INVALID_ARG, "aux tensor %d is not 16-byte aligned", j);
        progs.push_back(&net->aux[j].fwd_static);
    }
    Bindings b; b.image = image; b.auxp = aux_params; b.xout = x_out;
    lp_status st = static_scratch(&b.scratch);
    if (st != LP_OK) return st;
    bool any_chained = false;
    for (const AuxPlan& a : net->aux) any_chained = any_chained || a.chained;
    if (!any_chained) return run_programs(net, progs, b, (hipStream_t)stream);
    for (size_t j = 0; j < progs.size() && st == LP_OK; ++j) st = run_programs(net, {progs[j]}, b, (hipStream_t)stream);
    return st;
}

lp_status lp_auxnet_distill_grad(struct lp_net* net, void* stream, const void* image, const void* const* aux_params,
                                 const void* const* x_target, float loss_scale, float* loss, float* const* daux_params) {
    lp_status st = check_common(net, 0, false);
    if (st != LP_OK) return st;
    if (net->aux.empty()) return fail(LP_ERR_STATE, "the net was created without AuxNet descriptors");
    if (!net->aux_fwd_done) return fail(LP_ERR_STATE, "lp_auxnet_forward has not run: no saved AuxNet activations");
    if (!image || !aux_params || !x_target || !loss || !daux_params) return fail(LP_ERR_INVALID_ARG, "NULL argument");
    if (misaligned(image)) return fail(LP_ERR_INVALID_ARG, "image is not 16-byte aligned");
    const int epv = net->dtype == LP_BF16 ? 8 : 4;
    hipStream_t s = (hipStream_t)stream;
    std::vector<const Program*> pa, pb;
    uint32_t mask = 0;
    LossGroup g; g.nprob = 0; g.total_blocks = 0; g.rho = 2.f; g.scale = loss_scale; g.step = 0.f;   // rho/2 * r^2 with rho = 2: |r|^2
    std::vector<LossGroup> groups;
    for (int j = 0; j < net->K - 1; ++j) {
        if (!daux_params[j]) continue;
        if (!aux_params[j] || !x_target[j]) return fail(LP_ERR_INVALID_ARG, "aux_params[%d] or x_target[%d] is NULL", j, j);
        if (misaligned(aux_params[j]) || misaligned(x_target[j]) || misaligned(daux_params[j]))
            return fail(LP_ERR_INVALID_ARG, "aux tensor %d is not 16-byte aligned", j);
        const AuxPlan& a = net->aux[j];
        if (a.chained && (!x_target[j - 1] || misaligned(x_target[j - 1])))
            return fail(LP_ERR_INVALID_ARG, "x_target[%d] (input of the chained AuxNet %d) is NULL or not 16-byte aligned", j - 1, j);
        pa.push_back(&a.bwd_a); pb.push_back(&a.bwd_b);
        mask |= 1u << j;
        LossProb& p = g.p[g.nprob];
        p.y = net->ws + a.ws_out; p.xn = x_target[j]; p.lam = nullptr; p.lam_out = nullptr; p.dy = net->ws + a.ws_g; p.loss = loss + j;
        p.r2 = nullptr;
        p.numel = a.u.out_elems();
        p.block_start = g.total_blocks; p.nblocks = elem_blocks(p.numel / epv); g.total_blocks += p.nblocks;
        if (++g.nprob == kMaxGroup) { groups.push_back(g); g.nprob = 0; g.total_blocks = 0; }
    }
    if (g.nprob) groups.push_back(g);
    if (!mask) return LP_OK;
    Bindings b; b.ws = net->ws; b.image = image; b.auxp = aux_params; b.auxg = daux_params; b.xtgt = x_target;
    st = run_programs(net, pa, b, s);
    if (st != LP_OK) return st;
    hipError_t err = launch_zero_selected(loss, mask, net->K - 1, s);
    for (size_t i = 0; i < groups.size() && err == hipSuccess; ++i) err = launch_loss(groups[i], net->dtype, s);
    if (err != hipSuccess) return fail(LP_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(err));
    return run_programs(net, pb, b, s);
}

lp_status lp_reauxnet_grad(struct lp_net* net, void* stream, const void* image, const void* const* aux_params,
                           const void* const* y_prev, const void* const* dx, const void* const* lam_prev, float rho,
                           float scale, float* const* daux_params) {
    lp_status st = check_common(net, 0, false);
    if (st != LP_OK) return st;
    if (net->aux.empty()) return fail(LP_ERR_STATE, "the net was created without AuxNet descriptors");
    if (!net->aux_fwd_done) return fail(LP_ERR_STATE, "lp_auxnet_forward has not run: no saved AuxNet activations");
    if (!image || !aux_params || !y_prev || !dx || !daux_params) return fail(LP_ERR_INVALID_ARG, "NULL argument");
    if (!(rho >= 0.f)) return fail(LP_ERR_INVALID_ARG, "rho must be non-negative");
    if (misaligned(image)) return fail(LP_ERR_INVALID_ARG, "image is not 16-byte aligned");
    const int epv = net->dtype == LP_BF16 ? 8 : 4;
    hipStream_t s = (hipStream_t)stream;
    std::vector<const Program*> pa, pb;
    AuxVarGroup g; g.nprob = 0; g.total_blocks = 0; g.rho = rho; g.scale = scale; g.eta = 0.f;
    std::vector<AuxVarGroup> groups;
    for (int j = 0; j < net->K - 1; ++j) {
        if (!daux_params[j]) continue;
        if (!aux_params[j] || !y_prev[j] || !dx[j + 1]) return fail(LP_ERR_INVALID_ARG, "aux_params[%d], y_prev[%d] or dx[%d] is NULL", j, j, j + 1);
        const void* lam = lam_prev ? lam_prev[j] : nullptr;
        if (misaligned(aux_params[j]) || misaligned(y_prev[j]) || misaligned(dx[j + 1]) || misaligned(lam) || misaligned(daux_params[j]))
            return fail(LP_ERR_INVALID_ARG, "aux tensor %d is not 16-byte aligned", j);
        AuxPlan& a = net->aux[j];
        if (a.chained) return fail(LP_ERR_STATE, "aux %d reads the previous auxiliary variable: the recursive-AuxNet update is defined for AuxNets fed by the mini-batch", j);
        pa.push_back(&a.bwd_a); pb.push_back(&a.bwd_b);
        AuxVarProb& p = g.p[g.nprob];
        p.x = net->ws + a.ws_out; p.yprev = y_prev[j]; p.dx = dx[j + 1]; p.lam = lam; p.gout = net->ws + a.ws_g;
        p.numel = a.u.out_elems();
        p.block_start = g.total_blocks; p.nblocks = elem_blocks(p.numel / epv); g.total_blocks += p.nblocks;
        if (++g.nprob == kMaxGroup) { groups.push_back(g); g.nprob = 0; g.total_blocks = 0; }
    }
    if (g.nprob) groups.push_back(g);
    if (pa.empty()) return LP_OK;
    Bindings b; b.ws = net->ws; b.image = image; b.auxp = aux_params; b.auxg = daux_params;
    st = run_programs(net, pa, b, s);          // recomputed AuxNet output x_k (BN apply of the saved conv output)
    if (st != LP_OK) return st;
    hipError_t err = hipSuccess;
    for (size_t i = 0; i < groups.size() && err == hipSuccess; ++i) err = launch_auxvar(groups[i], net->dtype, s);
    if (err != hipSuccess) return fail(LP_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(err));
    return run_programs(net, pb, b, s);        // [ReLU,] BN backward, filter gradient
}

lp_status lp_module_forward(struct lp_net* net, void* stream, uint32_t module_mask, const void* const* x,
                            const void* const* params, void* const* y, float* logits) {
    lp_status st = check_common(net, module_mask, true);
    if (st != LP_OK) return st;
    if (!x || !params) return fail(LP_ERR_INVALID_ARG, "x or params is NULL");
    std::vector<const Program*> progs;
    for (int k = 0; k < net->K; ++k) {
        if (!((module_mask >> k) & 1u)) continue;
        if (!x[k] || !params[k]) return fail(LP_ERR_INVALID_ARG, "x[%d] or params[%d] is NULL", k, k);
        if (misaligned(x[k]) || misaligned(params[k])) return fail(LP_ERR_INVALID_ARG, "x[%d] or params[%d] is not 16-byte aligned", k, k);
        if (k < net->K - 1) {
            if (!y || !y[k]) return fail(LP_ERR_INVALID_ARG, "y[%d] is NULL", k);
            if (misaligned(y[k])) return fail(LP_ERR_INVALID_ARG, "y[%d] is not 16-byte aligned", k);
        } else if (!logits) return fail(LP_ERR_INVALID_ARG, "logits is NULL");
        progs.push_back(&net->mods[k].fwd);
    }
    Bindings b; b.ws = net->ws; b.x = x; b.params = params; b.y = y; b.logits = logits;
    const std::vector<int> lanes = lanes_of(net, module_mask);
    st = run_programs(net, progs, b, (hipStream_t)stream, &lanes);
    if (st == LP_OK) {
        for (int k = 0; k < net->K; ++k)
            if ((module_mask >> k) & 1u) {
                net->saved_x[k] = x[k]; net->fwd_done |= (1u << k);
                net->saved_y[k] = (k < net->K - 1) ? y[k] : nullptr;
            }
    }
    return st;
}

lp_status lp_local_loss_grad(struct lp_net* net, void* stream, uint32_t module_mask, const void* const* y,
                             const void* const* x_next, const void* const* lam, float rho, float loss_scale,
                             const float* logits, const int32_t* labels, float* loss, void* const* dy, float* dlogits) {
    if (!net) return fail(LP_ERR_INVALID_ARG, "net is NULL");
    if (module_mask == 0) return fail(LP_ERR_INVALID_ARG, "module_mask selects no module");
    if (net->K < 32 && (module_mask >> net->K) != 0) return fail(LP_ERR_INVALID_ARG, "module_mask 0x%x has bits beyond K = %d", module_mask, net->K);
    if (!(rho >= 0.f)) return fail(LP_ERR_INVALID_ARG, "rho must be non-negative");
    if (!loss) return fail(LP_ERR_INVALID_ARG, "loss is NULL");
    hipStream_t s = (hipStream_t)stream;
    const int epv = net->dtype == LP_BF16 ? 8 : 4;
    LossGroup g; g.nprob = 0; g.total_blocks = 0; g.rho = rho; g.scale = loss_scale; g.step = 0.f;
    bool want_ce = false;
    for (int k = 0; k < net->K; ++k) {
        if (!((module_mask >> k) & 1u)) continue;
        if (k == net->K - 1) { want_ce = true; continue; }
        if (!y || !x_next || !dy || !y[k] || !x_next[k] || !dy[k]) return fail(LP_ERR_INVALID_ARG, "y/x_next/dy[%d] is NULL", k);
        if (misaligned(y[k]) || misaligned(x_next[k]) || misaligned(dy[k]) || (lam && lam[k] && misaligned(lam[k])))
            return fail(LP_ERR_INVALID_ARG, "interface tensor %d is not 16-byte aligned", k);
    }
    if (want_ce && (!logits || !labels || !dlogits)) return fail(LP_ERR_INVALID_ARG, "logits, labels or dlogits is NULL");
    // loss[k] = 0 for the selected modules (the kernels below accumulate with atomics)
    hipError_t err = launch_zero_selected(loss, module_mask, net->K, s);
    if (err == hipSuccess && net->r2 && net->K > 1) err = launch_zero_selected(net->r2, module_mask & ((1u << (net->K - 1)) - 1u), net->K - 1, s);
    if (err != hipSuccess) return fail(LP_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(err));
    for (int k = 0; k < net->K - 1; ++k) {
        if (!((module_mask >> k) & 1u)) continue;
        const ModulePlan& m = net->mods[k];
        LossProb& p = g.p[g.nprob];
        p.y = y[k]; p.xn = x_next[k]; p.lam = (lam ? lam[k] : nullptr); p.lam_out = nullptr; p.dy = dy[k]; p.loss = loss + k;
        p.r2 = net->r2 ? net->r2 + k : nullptr;
        p.numel = (size_t)m.oN * m.oH * m.oW * m.oC;
        p.block_start = g.total_blocks; p.nblocks = elem_blocks(p.numel / epv); g.total_blocks += p.nblocks;
        if (++g.nprob == kMaxGroup) {
            err = launch_loss(g, net->dtype, s);
            if (err != hipSuccess) return fail(LP_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(err));
            g.nprob = 0; g.total_blocks = 0;
        }
    }
    if (g.nprob) {
        err = launch_loss(g, net->dtype, s);
        if (err != hipSuccess) return fail(LP_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(err));
    }
    if (want_ce) {
        const ModulePlan& m = net->mods[net->K - 1];
        err = launch_ce(logits, labels, loss + (net->K - 1), dlogits, m.oN, m.d.n_classes, s);
        if (err != hipSuccess) return fail(LP_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(err));
    }
    return LP_OK;
}

lp_status lp_module_backward(struct lp_net* net, void* stream, uint32_t module_mask, const void* const* dy,
                             const float* dlogits, const void* const* params, float* const* dparams, void* const* dx) {
    lp_status st = check_common(net, module_mask, true);
    if (st != LP_OK) return st;
    if (!params || !dparams) return fail(LP_ERR_INVALID_ARG, "params or dparams is NULL");
    if ((net->fwd_done & module_mask) != module_mask)
        return fail(LP_ERR_STATE, "lp_module_backward without a matching lp_module_forward (mask 0x%x, forward done 0x%x)", module_mask, net->fwd_done);
    std::vector<const Program*> progs;
    for (int k = 0; k < net->K; ++k) {
        if (!((module_mask >> k) & 1u)) continue;
        const ModulePlan& m = net->mods[k];
        if (!params[k] || !dparams[k]) return fail(LP_ERR_INVALID_ARG, "params[%d] or dparams[%d] is NULL", k, k);
        if (misaligned(params[k]) || misaligned(dparams[k])) return fail(LP_ERR_INVALID_ARG, "params[%d] or dparams[%d] is not 16-byte aligned", k, k);
        if (k < net->K - 1) {
            if (!dy || !dy[k]) return fail(LP_ERR_INVALID_ARG, "dy[%d] is NULL", k);
            if (misaligned(dy[k])) return fail(LP_ERR_INVALID_ARG, "dy[%d] is not 16-byte aligned", k);
        } else if (!dlogits) return fail(LP_ERR_INVALID_ARG, "dlogits is NULL");
        const bool needs_dx = !m.has_stem && k > 0;
        const bool opt_dx = !m.has_stem && k == 0 && dx && dx[0];
        if (needs_dx && (!dx || !dx[k])) return fail(LP_ERR_INVALID_ARG, "dx[%d] is NULL", k);
        if ((needs_dx || opt_dx) && misaligned(dx[k])) return fail(LP_ERR_INVALID_ARG, "dx[%d] is not 16-byte aligned", k);
        progs.push_back(opt_dx ? &m.bwd_dx0 : &m.bwd);
    }
    Bindings b; b.ws = net->ws; b.x = net->saved_x.data(); b.params = params; b.dparams = dparams; b.dy = dy; b.dx = dx;
    if (net->fused_update) { b.vel = net->fu_vel.data(); b.master = net->fu_master.data(); }
    b.dlogits = dlogits; b.y = net->saved_y.data();
    const std::vector<int> lanes = lanes_of(net, module_mask);
    st = run_programs(net, progs, b, (hipStream_t)stream, &lanes);
    if (st == LP_OK) net->fwd_done &= ~module_mask;
    return st;
}

lp_status lp_local_step(struct lp_net* net, void* stream, uint32_t module_mask, const void* const* x,
                        const void* const* params, void* const* y, const void* const* x_next, void* const* lam, float rho,
                        float loss_scale, float mult_step, const int32_t* labels, float* loss, void* const* dy, float* logits,
                        float* dlogits, float* const* dparams, void* const* dx) {
    lp_status st = check_common(net, module_mask, true);
    if (st != LP_OK) return st;
    if (!x || !params || !dparams || !loss) return fail(LP_ERR_INVALID_ARG, "x, params, dparams or loss is NULL");
    if (!(rho >= 0.f)) return fail(LP_ERR_INVALID_ARG, "rho must be non-negative");
    std::vector<const Program*> progs;
    for (int k = 0; k < net->K; ++k) {
        if (!((module_mask >> k) & 1u)) continue;
        const ModulePlan& m = net->mods[k];
        if (!x[k] || !params[k] || !dparams[k]) return fail(LP_ERR_INVALID_ARG, "x[%d], params[%d] or dparams[%d] is NULL", k, k, k);
        if (misaligned(x[k]) || misaligned(params[k]) || misaligned(dparams[k]))
            return fail(LP_ERR_INVALID_ARG, "x[%d], params[%d] or dparams[%d] is not 16-byte aligned", k, k, k);
        if (k < net->K - 1) {
            if (!y || !x_next || !dy || !y[k] || !x_next[k] || !dy[k]) return fail(LP_ERR_INVALID_ARG, "y/x_next/dy[%d] is NULL", k);
            if (misaligned(y[k]) || misaligned(x_next[k]) || misaligned(dy[k]) || (lam && lam[k] && misaligned(lam[k])))
                return fail(LP_ERR_INVALID_ARG, "interface tensor %d is not 16-byte aligned", k);
        } else if (!logits || !labels || !dlogits) return fail(LP_ERR_INVALID_ARG, "logits, labels or dlogits is NULL");
        const bool needs_dx = !m.has_stem && k > 0;
        const bool opt_dx = !m.has_stem && k == 0 && dx && dx[0];
        if (needs_dx && (!dx || !dx[k])) return fail(LP_ERR_INVALID_ARG, "dx[%d] is NULL", k);
        if ((needs_dx || opt_dx) && misaligned(dx[k])) return fail(LP_ERR_INVALID_ARG, "dx[%d] is not 16-byte aligned", k);
        progs.push_back(opt_dx ? &m.step_dx0 : &m.step);
    }
    hipStream_t s = (hipStream_t)stream;
    // loss[k] = 0 for the selected modules, ahead of the fork (the loss kernels accumulate with atomics)
    hipError_t err = launch_zero_selected(loss, module_mask, net->K, s);
    if (err == hipSuccess && net->r2 && net->K > 1) err = launch_zero_selected(net->r2, module_mask & ((1u << (net->K - 1)) - 1u), net->K - 1, s);
    if (err != hipSuccess) return fail(LP_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(err));
    Bindings b; b.ws = net->ws; b.x = x; b.params = params; b.y = y; b.logits = logits;
    b.dparams = dparams; b.dy = dy; b.dx = dx; b.dlogits = dlogits;
    if (net->fused_update) { b.vel = net->fu_vel.data(); b.master = net->fu_master.data(); }
    b.xnext = x_next; b.lam = lam; b.loss = loss; b.labels = labels; b.rho = rho; b.scale = loss_scale; b.mstep = mult_step;
    const std::vector<int> lanes = lanes_of(net, module_mask);
    st = run_programs(net, progs, b, s, &lanes);
    if (st == LP_OK)
        for (int k = 0; k < net->K; ++k)
            if ((module_mask >> k) & 1u) { net->saved_x[k] = x[k]; net->fwd_done &= ~(1u << k); }
    return st;
}

lp_status lp_al_multiplier_update(struct lp_net* net, void* stream, void* const* lam, const void* const* y,
                                  const void* const* x_next, float step) {
    if (!net) return fail(LP_ERR_INVALID_ARG, "net is NULL");
    if (!lam || !y || !x_next) return fail(LP_ERR_INVALID_ARG, "NULL argument");
    const int epv = net->dtype == LP_BF16 ? 8 : 4;
    MultGroup g; g.nprob = 0; g.total_blocks = 0; g.step = step;
    hipError_t err = hipSuccess;
    for (int k = 0; k < net->K - 1; ++k) {
        if (!lam[k]) continue;
        if (!y[k] || !x_next[k]) return fail(LP_ERR_INVALID_ARG, "y[%d] or x_next[%d] is NULL", k, k);
        if (misaligned(lam[k]) || misaligned(y[k]) || misaligned(x_next[k])) return fail(LP_ERR_INVALID_ARG, "interface tensor %d is not 16-byte aligned", k);
        const ModulePlan& m = net->mods[k];
        MultProb& p = g.p[g.nprob];
        p.lam = lam[k]; p.y = y[k]; p.xn = x_next[k]; p.numel = (size_t)m.oN * m.oH * m.oW * m.oC;
        p.block_start = g.total_blocks; p.nblocks = elem_blocks(p.numel / epv); g.total_blocks += p.nblocks;
        if (++g.nprob == kMaxGroup) {
            err = launch_mult(g, net->dtype, (hipStream_t)stream);
            if (err != hipSuccess) return fail(LP_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(err));
            g.nprob = 0; g.total_blocks = 0;
        }
    }
    if (g.nprob) {
        err = launch_mult(g, net->dtype, (hipStream_t)stream);
        if (err != hipSuccess) return fail(LP_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(err));
    }
    return LP_OK;
}

lp_status lp_sgd_update(struct lp_net* net, void* stream, int aux, uint32_t mask, void* const* params,
                        const float* const* dparams, float* const* velocity, float* const* master, float lr,
                        float momentum, float weight_decay) {
    if (!net) return fail(LP_ERR_INVALID_ARG, "net is NULL");
    if (!params || !dparams) return fail(LP_ERR_INVALID_ARG, "params or dparams is NULL");
    if (momentum != 0.f && !velocity) return fail(LP_ERR_INVALID_ARG, "momentum != 0 needs velocity buffers");
    if (aux && net->aux.empty()) return fail(LP_ERR_STATE, "the net was created without an AuxNet");
    const int n = aux ? (int)net->aux.size() : net->K;
    if (mask == 0 || (n < 32 && (mask >> n) != 0)) return fail(LP_ERR_INVALID_ARG, "mask 0x%x does not fit %d parameter sets", mask, n);
    SgdGroup g; g.nprob = 0; g.total_blocks = 0; g.lr = lr; g.momentum = momentum; g.wd = weight_decay;
    hipError_t err = hipSuccess;
    for (int k = 0; k < n; ++k) {
        if (!((mask >> k) & 1u)) continue;
        const std::vector<lp_tensor_info>* t; size_t pb, gb;
        lp_status st = table_of(net, aux, k, &t, &pb, &gb);
        if (st != LP_OK) return st;
        if (!params[k] || !dparams[k]) return fail(LP_ERR_INVALID_ARG, "params[%d] or dparams[%d] is NULL", k, k);
        float* vel = (momentum != 0.f) ? velocity[k] : nullptr;
        if (momentum != 0.f && !vel) return fail(LP_ERR_INVALID_ARG, "velocity[%d] is NULL", k);
        float* mas = master ? master[k] : nullptr;
        if (misaligned(params[k]) || misaligned(dparams[k]) || misaligned(vel) || misaligned(mas))
            return fail(LP_ERR_INVALID_ARG, "parameter set %d: a buffer is not 16-byte aligned", k);
        for (const lp_tensor_info& ti : *t) {
            SgdProb& p = g.p[g.nprob];
            p.p = (char*)params[k] + ti.offset; p.lowp = ti.dtype == LP_BF16;
            p.g = (const float*)((const char*)dparams[k] + ti.grad_offset);
            p.v = vel ? (float*)((char*)vel + ti.grad_offset) : nullptr;
            p.master = mas ? (float*)((char*)mas + ti.grad_offset) : nullptr;
            p.numel = ti.numel;
            p.block_start = g.total_blocks;
            p.nblocks = (int)((ti.numel + kSgdElemsPerBlock - 1) / kSgdElemsPerBlock);
            g.total_blocks += p.nblocks;
            if (++g.nprob == kMaxGroup) {
                err = launch_sgd(g, (hipStream_t)stream);
                if (err != hipSuccess) return fail(LP_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(err));
                g.nprob = 0; g.total_blocks = 0;
            }
        }
    }
    if (g.nprob) {
        err = launch_sgd(g, (hipStream_t)stream);
        if (err != hipSuccess) return fail(LP_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(err));
    }
    return LP_OK;
}

lp_status lp_aux_variable_update(struct lp_net* net, void* stream, void* const* x, const void* const* y_prev,
                                 const void* const* dx, const void* const* lam_prev, float rho, float scale, float eta) {
    if (!net) return fail(LP_ERR_INVALID_ARG, "net is NULL");
    if (!x || !y_prev || !dx) return fail(LP_ERR_INVALID_ARG, "NULL argument");
    const int epv = net->dtype == LP_BF16 ? 8 : 4;
    AuxVarGroup g; g.nprob = 0; g.total_blocks = 0; g.rho = rho; g.scale = scale; g.eta = eta;
    hipError_t err = hipSuccess;
    for (int k = 1; k < net->K; ++k) {
        if (!x[k]) continue;
        if (!y_prev[k - 1] || !dx[k]) return fail(LP_ERR_INVALID_ARG, "y_prev[%d] or dx[%d] is NULL", k - 1, k);
        const void* lam = lam_prev ? lam_prev[k - 1] : nullptr;
        if (misaligned(x[k]) || misaligned(y_prev[k - 1]) || misaligned(dx[k]) || misaligned(lam))
            return fail(LP_ERR_INVALID_ARG, "interface tensor %d is not 16-byte aligned", k);
        const ModulePlan& m = net->mods[k];
        AuxVarProb& p = g.p[g.nprob];
        p.x = x[k]; p.yprev = y_prev[k - 1]; p.dx = dx[k]; p.lam = lam; p.gout = nullptr;
        p.numel = (size_t)m.d.N * m.d.H * m.d.W * m.d.C;
        p.block_start = g.total_blocks; p.nblocks = elem_blocks(p.numel / epv); g.total_blocks += p.nblocks;
        if (++g.nprob == kMaxGroup) {
            err = launch_auxvar(g, net->dtype, (hipStream_t)stream);
            if (err != hipSuccess) return fail(LP_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(err));
            g.nprob = 0; g.total_blocks = 0;
        }
    }
    if (g.nprob) {
        err = launch_auxvar(g, net->dtype, (hipStream_t)stream);
        if (err != hipSuccess) return fail(LP_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(err));
    }
    return LP_OK;
}

lp_status lp_debug_im2col_offsets(void* stream, int H, int W, int Cin, int R, int S, int stride, int pad,
                                  const int64_t* m, const int64_t* q, int64_t* out, int count) {
    if (!m || !q || !out || count < 0) return fail(LP_ERR_INVALID_ARG, "NULL argument or negative count");
    if (H < 1 || W < 1 || Cin < 1 || R < 1 || S < 1 || stride < 1 || pad < 0) return fail(LP_ERR_INVALID_ARG, "bad geometry");
    if (R != S) return fail(LP_ERR_INVALID_ARG, "square filters only");
    lp_net tmp; tmp.dtype = LP_F32;
    Builder B{&tmp};
    const Unit u = make_unit(R, Cin, 8, stride, pad, 1, H, W, false);           // the row index alone fixes the image
    const Op o = B.conv_fwd(u, Ref(), Ref(), Ref(), Ref());
    const hipError_t err = launch_im2col_offsets(o.conv, m, q, out, count, (hipStream_t)stream);
    if (err != hipSuccess) return fail(LP_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(err));
    return LP_OK;
}

// the descriptor the library builds for a forward convolution or one parity class of its data-gradient, and the tile
// shape of the kernel asked for
static lp_status debug_conv_prob(int kernel, int mode, int parity, int N, int H, int W, int Cin, int Cout, int R, int stride,
                                 int pad, ConvProb& P, int& BM, int& bk, int& nw) {
    if (kernel < 0 || kernel > 2 || (mode != 0 && mode != 1)) return fail(LP_ERR_INVALID_ARG, "kernel %d / mode %d", kernel, mode);
    if (N < 1 || H < 1 || W < 1 || Cin < 1 || Cout < 1 || R < 1 || stride < 1 || pad < 0) return fail(LP_ERR_INVALID_ARG, "bad geometry");
    if (parity < 0 || parity >= stride * stride) return fail(LP_ERR_INVALID_ARG, "parity class %d of a stride-%d data-gradient", parity, stride);
    lp_net tmp; tmp.dtype = LP_BF16;
    Builder B{&tmp};
    Unit u = make_unit(R, Cin, Cout, stride, pad, N, H, W, false);
    Op o;
    if (mode == 0) o = B.conv_fwd(u, Ref(), Ref(), Ref(), Ref());
    else {
        if (H % stride || W % stride) return fail(LP_ERR_SHAPE, "%dx%d not divisible by the stride", H, W);
        Step st;
        B.conv_dgrad(u, Ref(), Ref(), Ref(), Ref(), Ref(), st);
        o = st[parity];
    }
    P = o.conv;
    BM = 128; bk = bk == 64 ? 64 : 32; nw = 8;
    int cfg = 0;
    if (kernel == 1) {
        if (!pick_fast_cfg(&tmp, P, cfg)) return fail(LP_ERR_SHAPE, "the implicit-GEMM wide-layer kernel does not take this layer");
        if (P.Cin % bk) return fail(LP_ERR_SHAPE, "k-tiles of %d channels do not divide %d", bk, P.Cin);
        BM = cfg == FAST_256x320 ? 256 : 512;
    } else if (kernel == 2) {
        if (!pick_win_cfg(&tmp, P, cfg)) return fail(LP_ERR_SHAPE, "the window kernel does not take this layer");
        BM = cfg == WIN64_256x320 ? 256 : 512; bk = 64;
    }
    return LP_OK;
}

lp_status lp_debug_conv_geometry(int kernel, int mode, int parity, int N, int H, int W, int Cin, int Cout, int R, int stride,
                                 int pad, int bk, int* geom) {
    if (!geom) return fail(LP_ERR_INVALID_ARG, "geom is NULL");
    ConvProb P; int BM, nw;
    const lp_status st = debug_conv_prob(kernel, mode, parity, N, H, W, Cin, Cout, R, stride, pad, P, BM, bk, nw);
    if (st != LP_OK) return st;
    const int g[12] = {P.M, P.Ncol, P.Cin, P.ntr, P.nts, P.r0, P.rs, P.s0, P.ss, P.ldw, BM, bk};
    memcpy(geom, g, sizeof(g));
    return LP_OK;
}

lp_status lp_debug_conv_offsets(void* stream, int kernel, int mode, int parity, int N, int H, int W, int Cin, int Cout, int R,
                                int stride, int pad, int bk, const int64_t* m, const int64_t* q, const int64_t* col,
                                int64_t* in_off, int64_t* w_off, int64_t* out_off, int count) {
    if (!m || !q || !col || !in_off || !w_off || !out_off || count < 0) return fail(LP_ERR_INVALID_ARG, "NULL argument or negative count");
    ConvProb P; int BM, nw;
    const lp_status st = debug_conv_prob(kernel, mode, parity, N, H, W, Cin, Cout, R, stride, pad, P, BM, bk, nw);
    if (st != LP_OK) return st;
    const hipError_t err = launch_conv_offsets(P, kernel, BM, bk, nw, m, q, col, in_off, w_off, out_off, count, (hipStream_t)stream);
    if (err != hipSuccess) return fail(LP_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(err));
    return LP_OK;
}

lp_status lp_debug_mfma_peak(void* stream, int mode, int blocks, int iters, uint64_t* clk, float* sink) {
    if ((mode != 0 && mode != 1) || blocks < 1 || iters < 1 || !sink) return fail(LP_ERR_INVALID_ARG, "bad argument");
    const hipError_t err = launch_mfma_peak(mode, blocks, iters, (unsigned long long*)clk, sink, (hipStream_t)stream);
    if (err != hipSuccess) return fail(LP_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(err));
    return LP_OK;
}

lp_status lp_debug_keep_gradients(int on) {
    g_keep_gradients = on != 0;
    return LP_OK;
}

static lp_debug_ref dref(const Ref& r) {
    lp_debug_ref d; d.space = LP_REF_NONE; d.idx = r.idx; d.off = r.off;
    switch (r.space) {
        case SP_WS: d.space = LP_REF_WORKSPACE; break;
        case SP_X: d.space = LP_REF_X; break;
        case SP_Y: d.space = LP_REF_Y; break;
        case SP_DY: d.space = LP_REF_DY; break;
        case SP_DX: d.space = LP_REF_DX; break;
        default: d.idx = 0; d.off = 0; break;
    }
    return d;
}
static lp_debug_ref dws(size_t off) { return dref(mk(SP_WS, 0, off)); }

// the conv+BN units of module k in forward order: stem, then per block main[0..], projection
static void collect_units(const ModulePlan& m, std::vector<lp_debug_unit>& out, int k) {
    auto base = [&](const Unit& u, int block, int slot) {
        lp_debug_unit d; memset(&d, 0, sizeof(d));
        d.block = block; d.slot = slot; d.R = u.R; d.stride = u.stride; d.pad = u.pad; d.cin = u.cin; d.cout = u.cout;
        d.N = u.N; d.H = u.H; d.W = u.W; d.Ho = u.Ho; d.Wo = u.Wo; d.relu = u.relu ? 1 : 0;
        d.t_w = u.t_w; d.t_gamma = u.t_g; d.t_beta = u.t_b; d.skip_unit = -1;
        d.graw.space = LP_REF_NONE;
        d.y = dws(u.ws_y); d.stats = dws(u.ws_stats); d.dy = dws(u.ws_dy); d.red = dws(u.ws_red);
        return d;
    };
    if (m.has_stem) {
        lp_debug_unit d = base(m.stem, -1, 0);
        d.in = dref(mk(SP_X, k, 0));
        d.out = dws(m.ws_stem_act);
        d.gout = m.d.stem == 2 ? dws(m.ws_gpool) : dref(m.bp[0].gin_ref);
        out.push_back(d);
    }
    for (size_t i = 0; i < m.bp.size(); ++i) {
        const BlockPlan& bp = m.bp[i];
        const bool need_in_grad = (i > 0) || m.has_stem;       // the backward program without dx[0]
        const int nm = (int)bp.main.size();
        const int first = (int)out.size();
        for (int j = 0; j < nm; ++j) {
            lp_debug_unit d = base(bp.main[j], (int)i, j);
            d.in = j == 0 ? dref(bp.in) : dws(bp.ws_act[j - 1]);
            if (j + 1 < nm) {
                d.out = dws(bp.ws_act[j]);
                d.gout = dws(bp.ws_gact[j]);
            } else {
                d.out = dref(bp.out);
                d.gout = dref(bp.g_ref);
                d.post_relu = bp.post_relu ? 1 : 0;
                if (bp.post_relu) d.graw = dref(bp.graw_ref);
                if (bp.has_proj) { d.skip_kind = 2; d.skip_unit = first + nm; }
                else { d.skip_kind = 1; d.skip = dref(bp.in); }
            }
            if (j > 0) { d.has_dgrad = 1; d.din = dws(bp.ws_gact[j - 1]); }
            else if (need_in_grad) {
                d.has_dgrad = 1; d.din = dref(bp.gin_ref);
                d.din_add = bp.has_proj ? dws(bp.ws_gproj) : dref(bp.g_ref);
            }
            out.push_back(d);
        }
        if (bp.has_proj) {
            lp_debug_unit d = base(bp.proj, (int)i, 3);
            d.in = dref(bp.in);
            d.gout = dref(bp.g_ref);
            if (bp.proj_plain) { d.plain = 1; d.dy = dref(bp.g_ref); d.stats = d.red = dref(Ref()); }
            if (need_in_grad) { d.has_dgrad = 1; d.din = dws(bp.ws_gproj); }
            out.push_back(d);
        }
    }
}

lp_status lp_debug_unit_count(const struct lp_net* net, int k, int* n) {
    if (!net || !n) return fail(LP_ERR_INVALID_ARG, "NULL argument");
    if (k < 0 || k >= net->K) return fail(LP_ERR_INVALID_ARG, "module %d out of range", k);
    if (net->mods[k].d.order != LP_ORDER_POST) return fail(LP_ERR_INVALID_ARG, "module %d: unit views describe the conv-BN-ReLU order only", k);
    std::vector<lp_debug_unit> u;
    collect_units(net->mods[k], u, k);
    *n = (int)u.size();
    return LP_OK;
}

lp_status lp_debug_unit_info(const struct lp_net* net, int k, int i, lp_debug_unit* info) {
    if (!net || !info) return fail(LP_ERR_INVALID_ARG, "NULL argument");
    if (k < 0 || k >= net->K) return fail(LP_ERR_INVALID_ARG, "module %d out of range", k);
    if (net->mods[k].d.order != LP_ORDER_POST) return fail(LP_ERR_INVALID_ARG, "module %d: unit views describe the conv-BN-ReLU order only", k);
    std::vector<lp_debug_unit> u;
    collect_units(net->mods[k], u, k);
    if (i < 0 || i >= (int)u.size()) return fail(LP_ERR_INVALID_ARG, "unit %d out of range", i);
    *info = u[i];
    return LP_OK;
}

lp_status lp_debug_module_info(const struct lp_net* net, int k, lp_debug_module* info) {
    if (!net || !info) return fail(LP_ERR_INVALID_ARG, "NULL argument");
    if (k < 0 || k >= net->K) return fail(LP_ERR_INVALID_ARG, "module %d out of range", k);
    const ModulePlan& m = net->mods[k];
    if (m.d.order != LP_ORDER_POST) return fail(LP_ERR_INVALID_ARG, "module %d: unit views describe the conv-BN-ReLU order only", k);
    memset(info, 0, sizeof(*info));
    info->keep_gradients = net->keep_gradients ? 1 : 0;
    info->oN = m.oN; info->oH = m.oH; info->oW = m.oW; info->oC = m.oC;
    if (m.d.stem == 2) {
        info->pool_in = dws(m.ws_stem_act); info->pool_out = dws(m.ws_pool_out); info->pool_arg = dws(m.ws_pool_arg);
        info->g_pool_out = dref(m.bp[0].gin_ref); info->g_pool_in = dws(m.ws_gpool);
        info->pH = m.pH; info->pW = m.pW; info->pC = m.d.stem_cout;
    }
    if (k == net->K - 1) {
        info->feat = dws(m.ws_feat); info->pooled = dws(m.ws_pooled); info->dfeat = dws(m.ws_dfeat);
        info->t_fc_w = m.t_fcw; info->t_fc_b = m.t_fcb;
    }
    return LP_OK;
}

lp_status lp_debug_filter_load_extent(int kernel, int bk, int bn, int nw, int Ncol, int Cin, int R, size_t* max_end,
                                      size_t* n_live) {
    if (!max_end || !n_live) return fail(LP_ERR_INVALID_ARG, "NULL argument");
    if ((kernel != 0 && kernel != 1) || (bk != 32 && bk != 64) || bn < 1 || nw < 1 || Ncol < 1 || Cin < 1 || R < 1)
        return fail(LP_ERR_INVALID_ARG, "bad geometry");
    if (kernel == 0 ? (Cin % bk != 0) : (bk != 64 || Cin % 32 != 0))
        return fail(LP_ERR_SHAPE, "Cin = %d does not fit channel slabs of %d", Cin, bk);
    // the filter loads exactly as conv_igemm_fast_kernel (kernel 0) and conv_win_kernel (kernel 1) form them
    ConvProb P; memset(&P, 0, sizeof(P));
    P.Ncol = Ncol; P.Cin = Cin; P.S = R; P.rs = 1; P.ss = 1; P.ldw = R * R * Cin;
    const int rps = 1024 / (bk * 2), cpr = bk * 2 / 16;
    const int nsbt = bn / rps, nsb = (nsbt + nw - 1) / nw;
    const int nslabc = (Cin + bk - 1) / bk;
    const bool half_last = (Cin % bk) != 0;
    size_t worst = 0, live = 0;
    for (int tile_n = 0; tile_n * bn < Ncol; ++tile_n)
        for (int wave = 0; wave < nw; ++wave) {
            const bool last_b = (wave + nw * (nsb - 1)) < nsbt;
            for (int lane = 0; lane < 64; ++lane) {
                const int kvg = addr::filter_kvg(bk, lane, wave);
                const addr::FilterRows f = addr::filter_rows(tile_n * bn, rps, nw, wave, lane / cpr, kvg, P.ldw, Ncol);
                const bool b_hi = kvg >= cpr / 2;
                for (int j = 0; j < nsb; ++j) {
                    if (!(j + 1 < nsb || last_b)) continue;
                    for (int sc = 0; sc < nslabc; ++sc)
                        for (int tr = 0; tr < R; ++tr)
                            for (int ts = 0; ts < R; ++ts) {
                                const int ci0 = sc * bk;
                                const bool t_live = !(kernel == 1 && b_hi && half_last && ci0 + bk > Cin);
                                const unsigned vo = addr::filter_voffset(f, j, t_live);
                                if (vo == addr::kOOB) continue;
                                const size_t end = (size_t)vo + addr::filter_soffset(f, addr::filter_tap_offset(P, tr, ts, ci0), j) + 16;
                                worst = std::max(worst, end);
                                ++live;
                            }
                }
            }
        }
    *max_end = worst; *n_live = live;
    return LP_OK;
}

lp_status lp_debug_saved_tensor(const struct lp_net* net, int k, int which, const void** ptr, size_t* numel) {
    if (!net || !ptr || !numel) return fail(LP_ERR_INVALID_ARG, "NULL argument");
    if (k < 0 || k >= net->K) return fail(LP_ERR_INVALID_ARG, "module %d out of range", k);
    if (!net->ws) return fail(LP_ERR_WORKSPACE, "no workspace set");
    const ModulePlan& m = net->mods[k];
    if (m.d.order != LP_ORDER_POST) return fail(LP_ERR_INVALID_ARG, "module %d: the saved-tensor ids describe the conv-BN-ReLU order only", k);
    if (which == 0) {
        if (!m.has_stem) return fail(LP_ERR_INVALID_ARG, "module %d has no stem", k);
        *ptr = net->ws + (m.d.stem == 2 ? m.ws_pool_out : m.ws_stem_act);
        *numel = m.bp[0].in_elems;
        return LP_OK;
    }
    if (which < 0) return fail(LP_ERR_INVALID_ARG, "tensor id %d is negative", which);
    const int bi = (which - 1) / 8, sub = (which - 1) % 8;
    if (bi >= (int)m.bp.size()) return fail(LP_ERR_INVALID_ARG, "block %d out of range", bi);
    const BlockPlan& bp = m.bp[bi];
    if (sub < 3) {
        if (sub >= (int)bp.main.size()) return fail(LP_ERR_INVALID_ARG, "conv slot %d out of range", sub);
        *ptr = net->ws + bp.main[sub].ws_y; *numel = bp.main[sub].out_elems();
    } else if (sub == 3) {
        if (!bp.has_proj) return fail(LP_ERR_INVALID_ARG, "block %d has no projection", bi);
        *ptr = net->ws + bp.proj.ws_y; *numel = bp.proj.out_elems();
    } else if (sub == 4) {
        if (bp.out.space != SP_WS) return fail(LP_ERR_INVALID_ARG, "block %d writes to the caller's y", bi);
        *ptr = net->ws + bp.out.off; *numel = bp.out_elems;
    } else return fail(LP_ERR_INVALID_ARG, "unknown tensor id %d", which);
    return LP_OK;
}

}  // extern "C"
