/*
 * lp.h - C ABI of the module-parallel local step on one MI355X (gfx950).
 *
 * One synchronous local step of the auxiliary-variable, module-parallel training of a residual
 * network: each of K modules (a stack of residual blocks with its own weights) starts from its
 * auxiliary variable x_k, runs its blocks forward, evaluates its local loss against x_{k+1}
 * (cross-entropy for the last module) and back-propagates inside the module only.  All K modules
 * are independent inside the step and are executed together as grouped kernel launches.
 *
 * Symbols (paper's letter in brackets):  x_k [lambda_k] auxiliary variable = input of module k,
 * x_0 = the mini-batch;  F_k(x_k) [X^k_{kn+n}] output of module k;  lam_k [kappa_{k+1}] explicit
 * multiplier on the interface produced by module k;  rho = 2*beta (the paper weights
 * psi = ||.||^2, without 1/2, by beta).
 *
 * Conventions
 *  - every tensor pointer is a DEVICE pointer owned by the caller and borrowed until the work
 *    enqueued on `stream` has completed; `stream` is a hipStream_t passed as void* (NULL = default
 *    stream); calls only enqueue work and return;
 *  - activations are NHWC [N,H,W,C], filters KRSC [Cout,R,S,Cin]; tensors in the net's storage type
 *    (LP_F32 or LP_BF16) are: x_k, F_k(x_k), lam_k, dy, dx, conv filters.  BN affine parameters, the
 *    linear head, logits, losses and every parameter gradient are fp32.  All accumulation is fp32
 *    (batch statistics are summed across tiles in fp64);
 *  - arrays indexed by module have K entries, arrays indexed by interface have K-1 entries and entry
 *    k belongs to the interface between module k and k+1 (y[k], x_next[k] = x_{k+1}, lam[k], dy[k]);
 *  - `module_mask` bit k selects module k; entries of unselected modules may be NULL;
 *  - every entry point returns lp_status and never throws; lp_last_error() gives the text of the
 *    last failure on the calling thread.  All argument checks run on the host.
 */
#ifndef LP_H
#define LP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LP_OK = 0,
    LP_ERR_INVALID_ARG = 1,   /* NULL required pointer, K < 1, mask beyond K, misaligned tensor, rho < 0 */
    LP_ERR_SHAPE = 2,         /* inconsistent block chain, H or W not divisible by a stride           */
    LP_ERR_DTYPE = 3,
    LP_ERR_WORKSPACE = 4,     /* workspace missing or too small                                      */
    LP_ERR_STATE = 5,         /* backward without a matching forward                                  */
    LP_ERR_HIP = 6            /* a HIP call or kernel launch failed                                   */
} lp_status;

typedef enum { LP_F32 = 0, LP_BF16 = 1 } lp_dtype;
typedef enum { LP_BLOCK_BASIC = 0, LP_BLOCK_BOTTLENECK = 1 } lp_block_kind;

/* Order of the layers inside a residual block.
 * LP_ORDER_POST: conv - BN - ReLU ... conv - BN, then the sum (described below at lp_block_desc).
 * LP_ORDER_PRE : the order the architecture figure of the paper draws (Fig. 2), basic blocks only:
 *     X_{m+1} = skip + conv3x3(ReLU(BN2(conv3x3(stride)(ReLU(BN1(X_m)))))),
 *     skip = X_m, or conv1x1(stride)(ReLU(BN1(X_m))) without BN when `proj` is set;
 *   the stem (1 only) is the bare conv3x3 and the head is BN - ReLU - average pool - linear.  BN1 normalises cin
 *   channels with the batch statistics of X_m; parameter order per block: gamma1, beta1, W1, gamma2, beta2, W2,
 *   [Wproj]; stem: W; head: gamma, beta, fc weight, fc bias.  dx[k] is always computed inside the module (the
 *   statistics of BN1 depend on X_m) and handed out under the same rule as for LP_ORDER_POST. */
typedef enum { LP_ORDER_POST = 0, LP_ORDER_PRE = 1 } lp_block_order;

/* Residual block X_{m+1} = skip(X_m) + F(X_m, W_m)  (Sec. 2.1 and the feature flow of Sec. 4.1).
 * basic:      F = conv3x3(stride) - BN - ReLU - conv3x3 - BN
 * bottleneck: F = conv1x1 - BN - ReLU - conv3x3(stride) - BN - ReLU - conv1x1 - BN   (inner width `width`)
 * skip = identity, or conv1x1(stride) - BN when `proj` is set.  As the feature-flow equation writes it there is no
 * ReLU after the sum.  Two options of the conv-BN-ReLU order (zero keeps the form above; LP_ORDER_PRE refuses them):
 * proj_plain: the projection is the bare conv1x1(stride), without BN (its parameter set is the filter alone);
 * post_relu: X_{m+1} = ReLU(skip(X_m) + F(X_m, W_m)), the classic post-activation block. */
typedef struct {
    int kind;      /* lp_block_kind */
    int cin, cout;
    int width;     /* bottleneck inner width; ignored for basic blocks */
    int stride;    /* 1 or 2 */
    int proj;      /* required when stride != 1 or cin != cout */
    int proj_plain;
    int post_relu;
} lp_block_desc;

/* Module k: [input layer S] + blocks + [output layer T]  (S and T belong to the first and last worker,
 * footnote in Sec. 4.2.1).  stem 0: none; 1: conv3x3(C -> stem_cout) - BN - ReLU;
 * 2: conv7x7 stride 2 pad 3 - BN - ReLU - maxpool3x3 stride 2 pad 1.  head: global average pool then
 * linear(+bias) to n_classes.  N,H,W,C: shape of the module input x_k. */
typedef struct {
    int stem, stem_cout;
    int n_blocks;
    const lp_block_desc* blocks;   /* host pointer, copied by lp_net_create */
    int head, n_classes;
    int N, H, W, C;
    int order;                     /* lp_block_order */
} lp_module_desc;

/* AuxNet j, generating x_{j+1} (Sec. 4.2, forward map of the auxiliary-variable network): a stack of `depth` blocks
 * conv3x3(pad 1) - BN(batch statistics) - ReLU, the ReLU of the last block being optional.  In its one-block form
 * (depth 0 or 1) it is conv3x3(cin -> cout, stride) - BN [- ReLU].  With depth = d > 1 the blocks 0..d-2 in front
 * of the last one have mid_cout[i] output channels and stride mid_stride[i] (each followed by ReLU); the last block
 * maps mid_cout[d-2] -> cout with `stride`.  The product of the strides must map the input size to that of x_{j+1}.
 * A stack that starts at the mini-batch and has one block per interface it passes (x_0 -> x_1 -> ... -> x_{j+1}
 * shapes, parameters of its own) is the recursive AuxNet of Sec. 4.4. */
#define LP_AUX_MAX_DEPTH 8
typedef struct {
    int cin, cout, stride, relu;
    int from_prev;   /* 0: the AuxNet reads the mini-batch x_0 (forward-unlocked form);  1: AuxNet j reads x_j, the output of
                        AuxNet j-1 (x_{j+1} = AuxNet_j(x_j), the chained form of Algorithm 1's first loop; AuxNet 0 reads x_0
                        either way).  cin and the strides then refer to x_j.  lp_auxnet_forward runs chained AuxNets one after
                        the other; lp_auxnet_distill_grad runs a chained AuxNet again from x_target[j-1], the corrected
                        x_j, before it takes the gradient (Sec. 4.2: theta_j <- argmin |x_{j+1} - AuxNet_j(x_j; theta)|^2);
                        lp_reauxnet_grad refuses chained AuxNets (LP_ERR_STATE). */
    int depth;       /* number of blocks, 1..LP_AUX_MAX_DEPTH; 0 is read as 1 */
    int mid_cout[LP_AUX_MAX_DEPTH - 1];     /* used when depth > 1: blocks 0..depth-2 */
    int mid_stride[LP_AUX_MAX_DEPTH - 1];
} lp_aux_desc;

typedef enum { LP_T_CONV = 0, LP_T_BN_GAMMA = 1, LP_T_BN_BETA = 2, LP_T_FC_W = 3, LP_T_FC_B = 4 } lp_tensor_kind;

/* One parameter tensor inside a module's packed parameter buffer.  The gradient buffer of the module
 * holds the same tensors in the same order, all fp32, at `grad_offset`. */
typedef struct {
    int kind;              /* lp_tensor_kind */
    int block;             /* -1 stem, 0..n_blocks-1, n_blocks = head */
    int slot;              /* conv index inside the block: 0,1,2 main path, 3 projection */
    int dtype;             /* lp_dtype of the parameter itself */
    int ndim;
    int dims[4];
    size_t offset;         /* byte offset in the parameter buffer (256-byte aligned) */
    size_t grad_offset;    /* byte offset in the fp32 gradient buffer (256-byte aligned) */
    size_t numel;
} lp_tensor_info;

struct lp_net;

/* Build the launch plan for K modules (and K-1 AuxNets when aux != NULL).  Host only: no device
 * memory is touched.  Descriptors are copied.  Errors: LP_ERR_INVALID_ARG, LP_ERR_SHAPE, LP_ERR_DTYPE. */
lp_status lp_net_create(int K, const lp_module_desc* mods, const lp_aux_desc* aux, int dtype, float bn_eps,
                        struct lp_net** out);
lp_status lp_net_destroy(struct lp_net* net);

/* Packed parameter layout of module k (aux = 0) or of AuxNet k (aux = 1: filter, BN gamma, BN beta of every block of
 * the stack in order; lp_tensor_info.slot is the block's index in the stack). */
lp_status lp_net_param_bytes(const struct lp_net* net, int aux, int k, size_t* param_bytes, size_t* grad_bytes);
lp_status lp_net_num_tensors(const struct lp_net* net, int aux, int k, int* n);
lp_status lp_net_tensor_info(const struct lp_net* net, int aux, int k, int i, lp_tensor_info* info);

/* Stream lanes of lp_module_forward / lp_module_backward.  The modules of a step are independent (Sec. 4.1: each
 * starts from its own auxiliary variable), so their kernel sequences may overlap: modules with lanes[k] = 0 are
 * enqueued on the caller's stream, modules with lanes[k] = 1..3 on streams the net owns (created at the first call that
 * needs them, default priority, destroyed with the net).  Modules of one lane are merged into grouped launches with
 * each other only.  Every call forks from the caller's stream and joins it again before it returns (events, no host
 * wait), so for the caller all work is ordered on `stream` as before; the pattern is legal under stream capture.
 * lp_net_create picks a default (K <= 4: a lane per module; otherwise modules of equal output width share a lane);
 * lanes == NULL puts every module on the caller's stream.  Host only.  Error: LP_ERR_INVALID_ARG (lane outside [0, 3]). */
lp_status lp_net_set_stream_lanes(struct lp_net* net, const int* lanes);

/* Workspace: saved activations, batch statistics, gradient scratch, re-laid-out filters.  The caller
 * allocates `bytes` of device memory (256-byte aligned) and lends it for the lifetime of the net. */
lp_status lp_net_workspace_bytes(const struct lp_net* net, size_t* bytes);
lp_status lp_net_set_workspace(struct lp_net* net, void* dev_ptr, size_t bytes);

/* x_{j+1} = AuxNet_j(image), j = 0..K-2  (Sec. 4.2; first loop of Algorithm 1, from-the-image form).
 * image: [N,H,W,C] of module 0.  aux_params[j]: packed parameters of AuxNet j.  x_out[j]: x_{j+1}. */
lp_status lp_auxnet_forward(struct lp_net* net, void* stream, const void* image,
                            const void* const* aux_params, void* const* x_out);

/* lp_auxnet_forward for callers that cannot allocate device memory and have no workspace to lend (code under HIP-graph
 * capture, serving loops, harnesses that forbid hipMalloc): same arguments, same kernels and same x_out, but the
 * intermediates of the pass (per-channel statistics, pre-BN convolution results, activations between the blocks of a
 * stack) live in a device array of LP_STATIC_SCRATCH_BYTES that is part of the library (every GPU the library runs on
 * holds one until the process ends) instead of the workspace; lp_net_set_workspace is not needed.  It allocates
 * nothing and frees nothing.  Limits: LP_ERR_WORKSPACE when the AuxNets of the net need more than
 * LP_STATIC_SCRATCH_BYTES (the ResNet-56 configuration at batch 128 needs 16.1 MiB in bf16); nothing is saved for
 * lp_auxnet_distill_grad / lp_reauxnet_grad (they keep requiring lp_auxnet_forward); all calls on one GPU share the
 * one array, which keeps the last call's contents: the call clears what must start at zero, and calls that overlap in
 * time on one GPU (two streams, two nets, two threads) race.  The array's address is looked up on the first call on a
 * device: make that call outside stream capture.  Errors otherwise as lp_auxnet_forward. */
#define LP_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
lp_status lp_auxnet_forward_static(struct lp_net* net, void* stream, const void* image,
                                   const void* const* aux_params, void* const* x_out);

/* Gradient of the AuxNet distillation objective of Sec. 4.2 (theta_{k-1} <- argmin |x_k - AuxNet_{k-1}(x_0; theta)|^2,
 * one descent step per iteration; the step itself is the caller's).  For every j with daux_params[j] != NULL:
 *     loss[j] = loss_scale * sum (AuxNet_j(image) - x_target[j])^2,   daux_params[j] = d loss[j] / d theta_j,
 * back-propagated through [ReLU,] batch norm (batch statistics) and the convolution of every block of the stack.
 * daux_params[j]: fp32
 * gradient buffer of AuxNet j (second size of lp_net_param_bytes(net, 1, j, ...), tensor table as the
 * parameters'), overwritten.  x_target[j]: K-1 device tensors shaped like x_{j+1}, storage type.  loss: K-1 device
 * floats, entries j overwritten.  Uses the pre-BN output and statistics lp_auxnet_forward saved in the workspace:
 * LP_ERR_STATE if lp_auxnet_forward has not run since the workspace was set (or the net has no AuxNet); image and
 * aux_params must be the ones of that call.  Errors: LP_ERR_INVALID_ARG, LP_ERR_WORKSPACE, LP_ERR_HIP. */
lp_status lp_auxnet_distill_grad(struct lp_net* net, void* stream, const void* image, const void* const* aux_params,
                                 const void* const* x_target, float loss_scale, float* loss, float* const* daux_params);

/* Decoupled forward pass of the selected modules (feature-flow equation of Sec. 4.1):
 * X = x_k; X <- skip(X) + F(X, W) for every block; y[k] = F_k(x_k) for k < K-1; the last module writes
 * logits [N, n_classes] (fp32).  Saves what the backward pass needs in the workspace. */
lp_status lp_module_forward(struct lp_net* net, void* stream, uint32_t module_mask,
                            const void* const* x, const void* const* params,
                            void* const* y, float* logits);

/* Local losses and terminal adjoints (penalty functional of Sec. 3.2 / augmented Lagrangian of Sec. 3.3;
 * terminal condition of the discrete adjoint in Sec. 4.1).  For k < K-1, with r = y[k] - x_next[k]:
 *   loss[k] = loss_scale * (rho/2 * sum r^2 + sum lam[k]*r),   dy[k] = loss_scale * (rho*r + lam[k]);
 * lam == NULL (or lam[k] == NULL) is the penalty method.  For k = K-1: loss[K-1] = mini-batch mean of the
 * softmax cross-entropy of logits against labels (int32 [N], values in [0, n_classes)), and
 * dlogits = (softmax - onehot)/N.  loss: K fp32 device scalars (overwritten). */
lp_status lp_local_loss_grad(struct lp_net* net, void* stream, uint32_t module_mask,
                             const void* const* y, const void* const* x_next, const void* const* lam,
                             float rho, float loss_scale,
                             const float* logits, const int32_t* labels,
                             float* loss, void* const* dy, float* dlogits);

/* Module-local back-propagation (discrete adjoint recursion and weight gradient of Sec. 4.1) from the
 * terminal adjoint dy[k] (k < K-1) or dlogits (k = K-1).  dparams[k]: fp32 gradient buffer of module k
 * (overwritten).  dx[k]: gradient with respect to x_k, written for k >= 1, and for k = 0 only when module 0
 * has no stem and dx[0] != NULL.  Requires lp_module_forward of the same modules since the last backward:
 * otherwise LP_ERR_STATE.  Like x[k] and params[k], the y[k] given to that forward call is read again here when the
 * last block of module k has post_relu (the ReLU behind the sum is masked from the stored output): it must still hold
 * F_k(x_k). */
lp_status lp_module_backward(struct lp_net* net, void* stream, uint32_t module_mask,
                             const void* const* dy, const float* dlogits, const void* const* params,
                             float* const* dparams, void* const* dx);

/* Deterministic reductions (for race hunting: run a step twice and compare bit for bit).  By default per-channel batch
 * statistics, the sums of the batch-norm backward pass and the split filter gradients are accumulated with atomic adds,
 * whose order varies from run to run (last-bit differences).  With on != 0 every such sum has a fixed order: the
 * convolution epilogues emit no statistics and one workgroup per tensor sums the stored result instead; the
 * batch-norm backward sums run in one workgroup per tensor; every filter-gradient tile is reduced over all pixels by
 * one workgroup (no split).  Every activation, adjoint, gradient and multiplier
 * of lp_module_forward / lp_local_loss_grad / lp_module_backward / lp_local_step / lp_al_multiplier_update is then
 * bit-identical from run to run (the scalar losses, which are sums of per-workgroup atomics, keep their last-bit
 * freedom).  Much slower; results equal the default mode's within rounding.  Host only. */
lp_status lp_net_set_deterministic(struct lp_net* net, int on);

/* Constraint violation of the interfaces (the quantity the convergence figures of Sec. 5 plot beside the loss):
 * r2 = K-1 device floats or NULL.  While set, every lp_local_loss_grad / lp_local_step overwrites r2[k], for the
 * selected modules k < K-1, with |F_k(x_k) - x_{k+1}|^2 = sum r^2 (unscaled; it comes out of the same pass and the same
 * reduction as loss[k]).  The buffer is borrowed until it is reset or the net destroyed.  Host only.  Error:
 * LP_ERR_INVALID_ARG. */
lp_status lp_net_set_residual_output(struct lp_net* net, float* r2);

/* The synchronous local step of the selected modules in ONE call (Sec. 4.1: forward, terminal condition of the
 * adjoint, backward recursion with the weight gradients, multiplier update, each module on its own): exactly
 * lp_module_forward, lp_local_loss_grad, lp_module_backward and, when lam != NULL and mult_step != 0,
 * lp_al_multiplier_update(lam, y, x_next, mult_step), with the same arguments, results and conventions.  The
 * difference is the schedule: here every stream lane runs through all phases of its own modules without waiting for
 * the other lanes between the phases (the separate calls join all lanes at the end of each call), and the multiplier
 * update rides on the loss kernel, which has y, x_next and lam at hand: it writes dy from the old lam[k] and then the
 * new lam[k] (nothing else in the step reads it), bit for bit what the separate call writes.
 * Errors as the four calls'. */
lp_status lp_local_step(struct lp_net* net, void* stream, uint32_t module_mask, const void* const* x,
                        const void* const* params, void* const* y, const void* const* x_next, void* const* lam, float rho,
                        float loss_scale, float mult_step, const int32_t* labels, float* loss, void* const* dy, float* logits,
                        float* dlogits, float* const* dparams, void* const* dx);

/* Multiplier update of Sec. 4.1: lam[k] <- lam[k] + step * (y[k] - x_next[k]) for every interface k with
 * lam[k] != NULL (the paper's step is eta/(2*beta) = eta/rho). */
lp_status lp_al_multiplier_update(struct lp_net* net, void* stream, void* const* lam,
                                  const void* const* y, const void* const* x_next, float step);

/* Update direction of a recursive AuxNet (Sec. 4.4, the rule given there for xi_k when the auxiliary variable is
 * generated from the mini-batch, x_k = ReAuxNet_k(x_0; xi_k), instead of being a free variable): the gradient of the
 * relaxed objective with respect to x_k,
 *     g_k = scale*(rho*(x_k - y_prev[k-1]) - lam_prev[k-1]) + dx[k],
 * pulled back through every block of the AuxNet ([ReLU,] BN with batch statistics, conv3x3) into daux_params[k-1]
 * (overwritten; layout of lp_net_param_bytes(net, 1, k-1)).  x_k is the AuxNet output of the last lp_auxnet_forward
 * (recomputed from its saved activations: that call must have run with the same image and aux_params, else
 * LP_ERR_STATE); y_prev[k-1] = F_{k-1}(x_{k-1}) as written by lp_module_forward; dx[k] as written by
 * lp_module_backward for the step whose x_k was that AuxNet output (dx[0] is not read); lam_prev NULL or an entry
 * NULL: penalty method, as the paper states the rule.  daux_params[j] == NULL skips AuxNet j.  Depth of the
 * recursion: the depth of the AuxNet descriptors (a stack of k blocks from the mini-batch for x_k is the paper's
 * ReAuxNet_k).  The descent step is lp_sgd_update with aux = 1.  Device memory, 16-byte aligned, activation dtype.
 * Errors: LP_ERR_INVALID_ARG, LP_ERR_STATE, LP_ERR_WORKSPACE; LP_ERR_HIP if a launch fails. */
lp_status lp_reauxnet_grad(struct lp_net* net, void* stream, const void* image, const void* const* aux_params,
                           const void* const* y_prev, const void* const* dx, const void* const* lam_prev, float rho,
                           float scale, float* const* daux_params);

/* Parameter update of Sec. 4.1 (W <- W - eta * dW for every tensor of a module, right after the module's adjoint
 * recursion).  The paper states plain gradient descent; the two usual extensions are off at 0:
 *     g' = dW + weight_decay * W;   v <- momentum * v + g'  (when momentum != 0);   W <- W - lr * (v or g').
 * aux = 0: modules (mask bit k, K sets), aux = 1: AuxNets (K-1 sets).  params[k]: packed parameters, updated in
 * place (bf16 tensors are re-rounded); dparams[k]: fp32 gradients; velocity[k]: fp32, layout of dparams[k], required
 * (and updated) when momentum != 0, zero it before the first step; master[k]: optional fp32 copy of the parameters with
 * the layout of dparams[k]: when given, the update is applied to it and params[k] receives the rounded result
 * (master == NULL or an entry NULL: the stored parameters themselves are read).  Device memory, 16-byte aligned.
 * Errors: LP_ERR_INVALID_ARG; LP_ERR_HIP if a launch fails. */
lp_status lp_sgd_update(struct lp_net* net, void* stream, int aux, uint32_t mask, void* const* params,
                        const float* const* dparams, float* const* velocity, float* const* master, float lr,
                        float momentum, float weight_decay);

/* The same update INSIDE the backward pass (Sec. 4.1 states the update of W_{kn+m} right after the adjoint at that
 * layer, inside the backward loop of Algorithm 1, not as a pass of its own).  While switched on, lp_module_backward
 * and lp_local_step update params[k] of the selected modules in place (the const of their params argument
 * notwithstanding): every convolution filter in the epilogue of its filter-gradient kernel -- the workgroup that adds
 * the last partial sum of an output tile reads the finished gradient tile back and applies
 *     g' = dW + weight_decay * W;   v <- momentum * v + g';   W <- W - lr * (v or g')
 * to that tile -- and the small tensors (BN affine, head) in one grouped launch behind the module's last kernel.
 * dparams[k] still receives the gradients.  velocity (K entries, required when momentum != 0; zero them before the
 * first step) and master (K entries or NULL, entries may be NULL) as in lp_sgd_update; the pointers are kept by the
 * net until the update is switched off (on = 0: the other arguments are ignored) or set again.  Results equal those of
 * lp_module_backward followed by lp_sgd_update up to the order in which the partial sums were added; in the
 * deterministic mode bit for bit.  Nothing else of a step may read params[k] while its backward pass runs.
 * Errors: LP_ERR_INVALID_ARG. */
lp_status lp_net_set_fused_update(struct lp_net* net, int on, float lr, float momentum, float weight_decay,
                                  float* const* velocity, float* const* master);

/* Correction of the auxiliary variables that follows the adjoint recursion in Sec. 4.1 (the update of lambda_k,
 * 1 <= k <= K-1): one gradient step of the relaxed objective with respect to x_k,
 *     x[k] <- x[k] - eta * ( scale*(rho*(x[k] - y_prev[k-1]) - lam_prev[k-1]) + dx[k] ),
 * where y_prev[k-1] = F_{k-1}(x_{k-1}) (K-1 entries, as y of lp_module_forward), dx[k] is the input gradient
 * lp_module_backward wrote (K entries, entry 0 ignored), lam_prev[k-1] the multiplier of that interface
 * (lam_prev == NULL or an entry NULL: penalty method), scale the loss_scale of lp_local_loss_grad.
 * x: K entries, entry 0 ignored, a NULL entry skips that variable; updated in place.  All tensors device
 * memory in the storage type, 16-byte aligned.  Errors: LP_ERR_INVALID_ARG; LP_ERR_HIP if a launch fails. */
lp_status lp_aux_variable_update(struct lp_net* net, void* stream, void* const* x, const void* const* y_prev,
                                 const void* const* dx, const void* const* lam_prev, float rho, float scale, float eta);

/* Flat NHWC offset read by element (m, q) of the implicit-GEMM operand of a forward convolution as the
 * device kernels compute it (m = output pixel index, q = (r*S+s)*Cin+ci), -1 in the padding.  Evaluated on
 * the device for `count` (m,q) pairs; out: int64 [count] device.  For bit-exact address checks. */
lp_status lp_debug_im2col_offsets(void* stream, int H, int W, int Cin, int R, int S, int stride, int pad,
                                  const int64_t* m, const int64_t* q, int64_t* out, int count);

/* The addresses the convolution kernels form, for bit-exact checks against the index function of the convolution's
 * definition.  The library builds the same problem descriptor it builds for a layer (mode 0: forward convolution
 * [N,H,W,Cin] -> Cout, R x R, stride, pad; mode 1: its data-gradient, parity class `parity` = ph*stride + pw of the
 * output pixels, a GEMM over dY [N,Ho,Wo,Cout] and the re-laid-out filter [Cin][R][R][Cout]) and evaluates, on the
 * device, the address functions the chosen kernel runs (kernel 0: the general implicit-GEMM kernel; 1: the wide-layer
 * implicit-GEMM kernel with k-tiles of bk = 32 or 64 channels; 2: the window kernel), one sample per thread:
 *   in_off[i]  element offset of the activation operand fetched for GEMM element (m[i], q[i]), q = (tr*nts + ts)*C + c
 *              in the descriptor's own tap numbering, -1 where the kernel substitutes zero padding (the lane/chunk
 *              swizzles of the direct-to-LDS loads are resolved; -2 would report a broken chunk permutation or a
 *              fragment read outside the window);
 *   w_off[i]   element offset of the filter element (row col[i]) that multiplies it;
 *   out_off[i] element offset of output (m[i], column 0).
 * lp_debug_conv_geometry (host only) returns what is needed to draw samples and to decode the tap numbering:
 * geom[12] = {M, Ncol, C, ntr, nts, r0, rs, s0, ss, ldw, BM, bk} (filter tap of (tr, ts): (r0 + rs*tr, s0 + ss*ts)).
 * Errors: LP_ERR_INVALID_ARG; LP_ERR_SHAPE when the kernel does not take the layer; LP_ERR_HIP. */
lp_status lp_debug_conv_geometry(int kernel, int mode, int parity, int N, int H, int W, int Cin, int Cout, int R, int stride,
                                 int pad, int bk, int* geom);
lp_status lp_debug_conv_offsets(void* stream, int kernel, int mode, int parity, int N, int H, int W, int Cin, int Cout, int R,
                                int stride, int pad, int bk, const int64_t* m, const int64_t* q, const int64_t* col,
                                int64_t* in_off, int64_t* w_off, int64_t* out_off, int count);

/* Read-only view of a saved activation after lp_module_forward (for layer-wise checks): which = 0 output of
 * the stem, 1 + 8*block + {0,1,2: pre-BN conv output of slot, 3: projection conv output, 4: block output}. */
lp_status lp_debug_saved_tensor(const struct lp_net* net, int k, int which, const void** ptr, size_t* numel);

/* Unit-by-unit views of a module in the conv-BN-ReLU order, for layer-wise checks (debug; read-only descriptions,
 * host only).  A unit is one convolution with the batch norm behind it.  Every tensor is named by a reference: the
 * caller's tensor of the last call (x[idx], y[idx], dy[idx], dx[idx]) or a byte offset into the workspace.
 *   forward:   in --conv--> y (pre-BN, stored) ; stats = per-channel [sum, sum of squares] of y, kept as LP_STAT_STRIPES
 *              partial sums that add up to it (fp64 [LP_STAT_STRIPES][2*cout]);
 *              out = [ReLU]( BN(y) [+ skip | + BN(y of unit skip_unit) | + y of a plain unit skip_unit] ), written by
 *              the unit's BN-apply pass (ReLU: the unit's own `relu`, or `post_relu` on the last unit of a block)
 *              (the projection unit has none: its BN is applied inside the pass of the block's last unit);
 *   backward:  gout = gradient arriving at the unit's BN output; dy = gradient on y (BN backward, stored);
 *              red = per-channel [sum g', sum g'*yhat] (fp64 [LP_STAT_STRIPES][2*cout], partial sums as above); din = the unit's data-gradient
 *              (+ din_add, the skip-path gradient added in its epilogue), present when has_dgrad.
 * Gradient buffers are reused from block to block inside a backward pass unless the net was created after
 * lp_debug_keep_gradients(1) (a per-thread switch read by lp_net_create: every gradient then has a buffer of its own;
 * the workspace grows, kernels and launches are the same).  The views describe the backward program without dx[0]. */
enum { LP_REF_NONE = 0, LP_REF_WORKSPACE = 1, LP_REF_X = 2, LP_REF_Y = 3, LP_REF_DY = 4, LP_REF_DX = 5 };
#define LP_STAT_STRIPES 8
typedef struct { int space; int idx; size_t off; } lp_debug_ref;
typedef struct {
    int block, slot;             /* block -1: stem; slot 0..2 main path, 3 projection */
    int R, stride, pad, cin, cout, N, H, W, Ho, Wo;
    int relu;                    /* ReLU behind this unit's BN */
    int t_w, t_gamma, t_beta;    /* indices into the module's tensor table */
    int skip_kind;               /* added inside this unit's BN-apply pass: 0 nothing, 1 the tensor `skip`, 2 BN(y) of unit skip_unit */
    int skip_unit;
    int has_dgrad;
    int plain;                   /* a bare projection: no BN (no stats / red / parameters of one; out = none, dy = gout) */
    int post_relu;               /* the block output is ReLU(sum): `out` carries it, and `gout` is the arriving gradient
                                    `graw` already masked by out > 0 (a pass of its own at the start of the block's backward) */
    lp_debug_ref in, y, stats, out, skip, gout, dy, red, din, din_add, graw;
} lp_debug_unit;
typedef struct {                 /* what lies around the units: max-pool of stem 2, head of the last module */
    int keep_gradients;
    int oN, oH, oW, oC;          /* shape of F_k(x_k) */
    int pH, pW, pC;              /* stem 2: shape of the pool input [N, pH, pW, pC] */
    lp_debug_ref pool_in, pool_out, pool_arg, g_pool_out, g_pool_in;
    lp_debug_ref feat, pooled, dfeat;   /* last module: F_k(x_k), its spatial mean [N, C] fp32, the gradient on F_k(x_k) */
    int t_fc_w, t_fc_b;
} lp_debug_module;
lp_status lp_debug_keep_gradients(int on);
lp_status lp_debug_unit_count(const struct lp_net* net, int k, int* n);
lp_status lp_debug_unit_info(const struct lp_net* net, int k, int i, lp_debug_unit* info);
lp_status lp_debug_module_info(const struct lp_net* net, int k, lp_debug_module* info);

/* Host-only bounds check of the direct-to-LDS filter loads of the wide-layer convolution kernels (no GPU): forms, with
 * the kernels' own address functions, every filter load of a forward layer with Ncol filters [R, R, Cin] for every
 * column tile (width bn), wave (nw per workgroup), lane, round, tap and channel slab (bk channels; kernel 0: the
 * implicit-GEMM kernel, Cin % bk == 0; kernel 1: the window kernel, bk = 64 with an optional last half slab), and
 * returns the largest byte offset past the end of any load that is not marked out of range, and how many such loads
 * there are.  Safe kernels keep *max_end <= Ncol*R*R*Cin*2.  Errors: LP_ERR_INVALID_ARG, LP_ERR_SHAPE. */
lp_status lp_debug_filter_load_extent(int kernel, int bk, int bn, int nw, int Ncol, int Cin, int R, size_t* max_end,
                                      size_t* n_live);

/* What the matrix cores of this device sustain (measurement aid of bench.py --measure-peak; no operand of the
 * library is touched).  Launches `blocks` workgroups of eight waves, each wave running `iters` times the 40
 * v_mfma_f32_32x32x16_bf16 of one filter tap of the convolution kernels' wave tile (2 x 5 micro-tiles, four k-steps):
 * mode 0 on register operands only, mode 1 with the seven operand fragments of every k-step read from LDS as the
 * kernels read them.  Work: blocks * 8 * iters * 40 * 32768 flop.  clk (device, 2*blocks uint64, or NULL): per
 * workgroup the shader-clock cycles and the ticks of the constant 100 MHz counter between its start and end.
 * sink: one device float (never written in practice).  The caller times the launch. */
lp_status lp_debug_mfma_peak(void* stream, int mode, int blocks, int iters, uint64_t* clk, float* sink);

/* Optional per-launch timing.  While enabled, every grouped kernel launch made by lp_auxnet_forward,
 * lp_module_forward and lp_module_backward is bracketed by two hipEvents on the stream it is enqueued on.
 * on = 1: launches of different stream lanes still overlap, so a record's duration includes the time its kernel
 * shared the device; on = 2: the same launches (same grouping per lane) are all enqueued on the caller's stream, one
 * after another, so that every record is the duration of its kernel alone.
 * lp_profile_fetch waits for the recorded launches, returns one record per launch in issue order and clears
 * the list (out == NULL: only the count).  kind: 0 clear, 1 filter re-layout, 2 conv forward/data-gradient,
 * 3 BN apply, 4 max-pool, 5 head, 6 head backward, 7 max-pool backward, 8 BN backward reduce, 9 BN backward
 * apply, 10 conv weight-gradient, 11 batch statistics of a module input, 12 loss / terminal adjoint, 13 cross-entropy,
 * 14 multiplier update (12, 13: launches of lp_local_step only; 14: not recorded any more, lp_local_step folds it into 12), 15 gradient mask of a ReLU behind a residual sum,
 * 16 update of the small tensors (lp_net_set_fused_update).  flops / bytes: algorithmic work of the launch (2*M*Ngemm*Kgemm per conv;
 * every operand tensor moved once).  blocks: workgroups of the launch (conv kernels: one per output tile and split; 0: not
 * recorded for this kind). */
typedef struct { int kind, cfg, nprob, blocks; float ms; double flops, bytes; } lp_profile_rec;
lp_status lp_profile_enable(struct lp_net* net, int on);
lp_status lp_profile_fetch(struct lp_net* net, lp_profile_rec* out, int max_recs, int* n_out);

const char* lp_last_error(void);
const char* lp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LP_H */
