"""CPU oracle, part 2 of 2: the synchronous local step in float64.  TEST INFRASTRUCTURE ONLY.

Plain, slow, definition-level implementation of what the HIP library computes; it shares no
code with it.  Pinned by tests/test_oracle_*.py (finite differences, closed forms, the
invariants of the relaxed problem); nothing here is pinned by a value printed in the paper,
because the paper prints none for the local step.

Notation (the paper's symbol in brackets): x_k [lambda_k] is the auxiliary variable that module
k takes as input; lam_k [kappa_{k+1}] the explicit multiplier on the interface that module k
produces; rho = 2*beta because the paper weights psi = ||.||^2 (no 1/2) by beta.

What follows what:
  module_forward     - decoupled feature flow of Sec. 4.1: X_{kn} = x_k, X_{m+1} = X_m + F(X_m, W_m)
  local_loss_grad    - per-interface term of the penalty functional (Sec. 3.2) / augmented Lagrangian
                       (Sec. 3.3, expanded in App. C) and the terminal condition of the discrete
                       adjoint (Sec. 4.1, second line of the backward dynamic)
  ce_loss_grad       - terminal loss phi, mini-batch mean (Sec. 2.1) and its terminal adjoint
  module_backward    - discrete adjoint recursion P_m = P_{m+1} dX_{m+1}/dX_m and the weight
                       gradient P_{m+1} dF/dW of Sec. 4.1
  auxnet_forward     - AuxNet forward map of Sec. 4.2 in its one-block, from-the-image form
  multiplier_update  - multiplier update rule of Sec. 4.1

Storage rounding (a DIAGNOSTIC mode, not the definition).  Every routine that composes layers takes `q`, a
callable applied where a low-precision implementation stores a tensor: going forward the convolution result
before BN, the activation after BN+ReLU and the block output; going backward the gradient of each of those
tensors, and the data-gradient of a projection branch before it is added.  Batch statistics are those of the
tensor that is normalised, i.e. of the stored (rounded) convolution result: batch norm is defined on the tensor it
receives, and that choice keeps its two identities (zero mean / unit variance of what it outputs, zero sums of the
backward result) exact for the stored values.  q=None (the default) is the plain float64 definition: it is what every
pin of the primitives and of the step exercises and what the unit-by-unit device tests compare against.  The
placement of the roundings is pinned separately (tests/test_oracle_step.py::test_storage_rounding_placement:
the same mode built from a library's layers and its reverse-mode differentiation).  The mode exists for end-to-end
comparisons of a whole bf16 backward pass, where decisions taken from stored values (ReLU masks, pooling argmax)
must be taken from values of the same precision on both sides.
"""
import ctypes
import os

import numpy as np

from workloads.configs import ModuleDesc, AuxDesc, NetDesc, Block, block_convs, aux_blocks

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        path = os.path.join(_HERE, "liblpref.so")
        if not os.path.exists(path):
            from .build import build
            build()
        L = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int64)
        ints = [ctypes.c_int] * 9
        L.lpref_conv_fwd.argtypes = [dp, dp, dp] + ints
        L.lpref_conv_dgrad.argtypes = [dp, dp, dp] + ints
        L.lpref_conv_wgrad.argtypes = [dp, dp, dp] + ints
        L.lpref_conv_fwd_at.argtypes = [dp, dp] + ints + [ctypes.c_int] * 4
        L.lpref_conv_fwd_at.restype = ctypes.c_double
        L.lpref_im2col_index.argtypes = [ctypes.c_int64, ctypes.c_int64] + [ctypes.c_int] * 7
        L.lpref_im2col_index.restype = ctypes.c_int64
        L.lpref_maxpool_fwd.argtypes = [dp, dp, ip] + [ctypes.c_int] * 7
        L.lpref_maxpool_bwd.argtypes = [dp, ip, dp, ctypes.c_int64, ctypes.c_int64]
        L.lpref_num_threads.restype = ctypes.c_int
        _LIB = L
    return _LIB


def num_threads() -> int:
    return int(_lib().lpref_num_threads())


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _c64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _out_hw(H, W, R, stride, pad):
    return (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1


# ----------------------------------------------------------------------------- primitives
def conv_fwd(x, w, stride, pad):
    x, w = _c64(x), _c64(w)
    N, H, W, Cin = x.shape
    Cout, R, S, Cin2 = w.shape
    assert Cin == Cin2
    Ho, Wo = _out_hw(H, W, R, stride, pad)
    y = np.empty((N, Ho, Wo, Cout))
    _lib().lpref_conv_fwd(_dp(x), _dp(w), _dp(y), N, H, W, Cin, Cout, R, S, stride, pad)
    return y


def conv_fwd_at(x, w, stride, pad, n, ho, wo, co):
    """A single output element of conv_fwd (x, w must already be contiguous float64)."""
    N, H, W, Cin = x.shape
    Cout, R, S, _ = w.shape
    return _lib().lpref_conv_fwd_at(_dp(x), _dp(w), N, H, W, Cin, Cout, R, S, stride, pad, n, ho, wo, co)


def conv_dgrad(dy, w, x_shape, stride, pad):
    dy, w = _c64(dy), _c64(w)
    N, H, W, Cin = x_shape
    Cout, R, S, _ = w.shape
    dx = np.empty(x_shape)
    _lib().lpref_conv_dgrad(_dp(dy), _dp(w), _dp(dx), N, H, W, Cin, Cout, R, S, stride, pad)
    return dx


def conv_wgrad(x, dy, w_shape, stride, pad):
    x, dy = _c64(x), _c64(dy)
    N, H, W, Cin = x.shape
    Cout, R, S, _ = w_shape
    dw = np.empty(w_shape)
    _lib().lpref_conv_wgrad(_dp(x), _dp(dy), _dp(dw), N, H, W, Cin, Cout, R, S, stride, pad)
    return dw


def im2col_index(m, q, H, W, Cin, R, S, stride, pad):
    return int(_lib().lpref_im2col_index(int(m), int(q), H, W, Cin, R, S, stride, pad))


def maxpool_fwd(x, R=3, stride=2, pad=1):
    x = _c64(x)
    N, H, W, C = x.shape
    Ho, Wo = _out_hw(H, W, R, stride, pad)
    y = np.empty((N, Ho, Wo, C))
    idx = np.empty((N, Ho, Wo, C), dtype=np.int64)
    _lib().lpref_maxpool_fwd(_dp(x), _dp(y), idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                             N, H, W, C, R, stride, pad)
    return y, idx


def maxpool_bwd(dy, idx, x_shape):
    dy = _c64(dy)
    dx = np.empty(x_shape)
    _lib().lpref_maxpool_bwd(_dp(dy), idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), _dp(dx),
                             dy.size, dx.size)
    return dx


def _id(a):
    return a


def bn_fwd(y, gamma, beta, eps, q=None):
    """Training-mode batch norm: per-channel mean and biased variance over N*H*W.
    With storage rounding q everything refers to the stored tensor q(y)."""
    if q is not None:
        y = q(y)
    mean = y.mean(axis=(0, 1, 2))
    var = ((y - mean) ** 2).mean(axis=(0, 1, 2))
    invstd = 1.0 / np.sqrt(var + eps)
    yhat = (y - mean) * invstd
    return gamma * yhat + beta, (yhat, invstd)


def bn_bwd(dz, cache, gamma):
    """Exact gradient through the batch statistics."""
    yhat, invstd = cache
    M = dz.shape[0] * dz.shape[1] * dz.shape[2]
    dbeta = dz.sum(axis=(0, 1, 2))
    dgamma = (dz * yhat).sum(axis=(0, 1, 2))
    dy = gamma * invstd * (dz - dbeta / M - yhat * (dgamma / M))
    return dy, dgamma, dbeta


# ----------------------------------------------------------------------------- conv+BN unit
def _cbr_fwd(x, w, gamma, beta, stride, pad, relu, eps, q=None):
    """conv -> BN(batch statistics) [-> ReLU].  The result is NOT rounded here (the caller stores it)."""
    y = conv_fwd(x, w, stride, pad)
    z, bc = bn_fwd(y, gamma, beta, eps, q)
    a = np.maximum(z, 0.0) if relu else z
    return a, (x, w, gamma, bc, z if relu else None, stride, pad)


def _cbr_bwd(da, cache, need_dx=True, q=None):
    """Returns the unrounded data-gradient (the caller stores it) and [dW, dgamma, dbeta]."""
    q = q or _id
    x, w, gamma, bc, z, stride, pad = cache
    dz = da * (z > 0.0) if z is not None else da          # ReLU gradient is 0 at exactly 0
    dy, dgamma, dbeta = bn_bwd(dz, bc, gamma)
    dy = q(dy)
    dw = conv_wgrad(x, dy, w.shape, stride, pad)
    dx = conv_dgrad(dy, w, x.shape, stride, pad) if need_dx else None
    return dx, [dw, dgamma, dbeta]


# ----------------------------------------------------------------------------- residual block
def block_forward(x, p, b: Block, eps, q=None):
    """X_{m+1} = skip(X_m) + F(X_m, W_m); F = conv-BN-ReLU ... conv-BN.  As the feature-flow equation of Sec. 4.1 writes
    it there is no ReLU after the sum; b.post_relu is the variant with one, X_{m+1} = ReLU(skip + F) (the classic
    post-activation block).  skip = X_m, or BN(conv1x1_stride(X_m)), or the bare conv1x1_stride(X_m) when b.proj_bn
    is off."""
    qq = q or _id
    convs = block_convs(b)
    main = [c for c in convs if c[0] != 3]
    caches, a, i = [], x, 0
    for j, (_, r, ci, co, st, pad) in enumerate(main):
        inner = j < len(main) - 1
        a, c = _cbr_fwd(a, p[i], p[i + 1], p[i + 2], st, pad, relu=inner, eps=eps, q=q)
        if inner:
            a = qq(a)                      # activation between two convolutions is stored
        caches.append(c)
        i += 3
    if b.proj and b.proj_bn:
        _, r, ci, co, st, pad = convs[-1]
        s, pc = _cbr_fwd(x, p[i], p[i + 1], p[i + 2], st, pad, relu=False, eps=eps, q=q)
    elif b.proj:
        _, r, ci, co, st, pad = convs[-1]
        s = qq(conv_fwd(x, p[i], st, pad))                 # the bare projection's result is stored
        pc = ("plain", x, p[i], st, pad)
    else:
        s, pc = x, None
    pre = s + a
    out = np.maximum(pre, 0.0) if b.post_relu else pre
    return qq(out), (caches, pc, pre if b.post_relu else None)         # the block output is stored


def block_backward(dout, cache, need_dx=True, q=None):
    qq = q or _id
    caches, pc, pre = cache
    if pre is not None:
        dout = dout * (pre > 0.0)          # ReLU behind the sum (its gradient is 0 at exactly 0)
    grads = []
    da = dout
    for j in range(len(caches) - 1, -1, -1):
        da, g = _cbr_bwd(da, caches[j], need_dx=(need_dx or j > 0), q=q)
        if j > 0:
            da = qq(da)                    # gradient of a stored activation is stored
        grads = g + grads
    dx = da
    if pc is not None and isinstance(pc[0], str):          # bare projection: no BN between the sum and the conv1x1
        _, px, pw, pst, ppad = pc
        grads = grads + [conv_wgrad(px, dout, pw.shape, pst, ppad)]
        if need_dx:
            dx = qq(dx + qq(conv_dgrad(dout, pw, px.shape, pst, ppad)))
    elif pc is not None:
        dxp, g = _cbr_bwd(dout, pc, need_dx=need_dx, q=q)
        grads = grads + g
        if need_dx:
            dx = qq(dx + qq(dxp))          # the projection's data-gradient is stored, then added
    elif need_dx:
        dx = qq(dx + dout)
    return dx, grads


# ----------------------------------------------------------------------------- pre-activation order
def _bn_relu_fwd(x, gamma, beta, eps, q=None):
    """ReLU(BN(x)) with batch statistics of the stored x.  Not rounded here."""
    z, bc = bn_fwd(x, gamma, beta, eps, q)
    return np.maximum(z, 0.0), (bc, z, gamma)


def _bn_relu_bwd(do, cache):
    bc, z, gamma = cache
    return bn_bwd(do * (z > 0.0), bc, gamma)


def block_forward_pre(x, p, b: Block, eps, q=None):
    """Residual block in the order the paper's architecture figure draws (Fig. 2):
    X_{m+1} = skip + conv2(ReLU(BN2(conv1(ReLU(BN1(X_m)))))), skip = X_m or conv1x1(ReLU(BN1(X_m))).
    p = [gamma1, beta1, W1, gamma2, beta2, W2, (Wproj)]."""
    qq = q or _id
    o1, c1 = _bn_relu_fwd(x, p[0], p[1], eps, q)
    o1 = qq(o1)
    y1 = qq(conv_fwd(o1, p[2], b.stride, 1))
    o2, c2 = _bn_relu_fwd(y1, p[3], p[4], eps, q)
    o2 = qq(o2)
    z = conv_fwd(o2, p[5], 1, 1)
    skip = qq(conv_fwd(o1, p[6], b.stride, 0)) if b.proj else x
    return qq(z + skip), (x.shape, o1, o2, c1, c2, p[2], p[5], p[6] if b.proj else None, b.stride)


def block_backward_pre(dout, cache, q=None):
    """Always returns the input gradient: the statistics of BN1 depend on X_m, and gamma1, beta1 need the gradient
    that reaches BN1's output."""
    qq = q or _id
    xshape, o1, o2, c1, c2, w1, w2, wp, stride = cache
    dw2 = conv_wgrad(o2, dout, w2.shape, 1, 1)
    do2 = qq(conv_dgrad(dout, w2, o2.shape, 1, 1))
    dy1, dg2, db2 = _bn_relu_bwd(do2, c2)
    dy1 = qq(dy1)
    dw1 = conv_wgrad(o1, dy1, w1.shape, stride, 1)
    do1 = conv_dgrad(dy1, w1, o1.shape, stride, 1)
    grads_p = []
    if wp is not None:
        grads_p = [conv_wgrad(o1, dout, wp.shape, stride, 0)]
        do1 = do1 + qq(conv_dgrad(dout, wp, o1.shape, stride, 0))
    do1 = qq(do1)
    dx, dg1, db1 = _bn_relu_bwd(do1, c1)
    if wp is None:
        dx = dx + dout
    return qq(dx), [dg1, db1, dw1, dg2, db2, dw2] + grads_p


def _module_forward_pre(m: ModuleDesc, x, params, eps, q):
    qq = q or _id
    p = [_c64(t) for t in params]
    a = _c64(x)
    cache = {"stem": None, "blocks": [], "head": None, "in_shape": a.shape, "order": "pre"}
    i = 0
    if m.stem == 1:
        cache["stem"] = (a, p[0])
        a = qq(conv_fwd(a, p[0], 1, 1))
        i = 1
    elif m.stem != 0:
        raise ValueError("pre-activation order: stem 0 or 1")
    for b in m.blocks:
        n = 7 if b.proj else 6
        a, c = block_forward_pre(a, p[i:i + n], b, eps, q)
        cache["blocks"].append(c)
        i += n
    logits = None
    if m.head:
        f, hc = _bn_relu_fwd(a, p[i], p[i + 1], eps, q)
        f = qq(f)
        pooled = f.mean(axis=(1, 2))
        logits = pooled @ p[i + 2].T + p[i + 3]
        cache["head"] = (pooled, p[i + 2], f.shape, hc)
    return a, logits, cache


def _module_backward_pre(m: ModuleDesc, cache, dy, dlogits, need_dx, q):
    qq = q or _id
    tail = []
    if m.head:
        pooled, wfc, shp, hc = cache["head"]
        dwfc = dlogits.T @ pooled
        dbfc = dlogits.sum(axis=0)
        df = qq(np.broadcast_to((dlogits @ wfc)[:, None, None, :] / (shp[1] * shp[2]), shp).copy())
        g, dgh, dbh = _bn_relu_bwd(df, hc)
        g = qq(g)
        tail = [dgh, dbh, dwfc, dbfc]
    else:
        g = _c64(dy)
    grads = []
    for j in range(len(cache["blocks"]) - 1, -1, -1):
        g, bg = block_backward_pre(g, cache["blocks"][j], q=q)
        grads = bg + grads
    if cache["stem"] is not None:
        img, w = cache["stem"]
        grads = [conv_wgrad(img, g, w.shape, 1, 1)] + grads
        g = qq(conv_dgrad(g, w, img.shape, 1, 1)) if need_dx else None
    return grads + tail, (g if need_dx else None)


# ----------------------------------------------------------------------------- module
def module_forward(m: ModuleDesc, x, params, eps=1e-5, q=None):
    """Returns (F_k(x_k), logits or None, cache).  params: list in workloads.module_tensor_specs order."""
    if m.order == "pre":
        return _module_forward_pre(m, x, params, eps, q)
    qq = q or _id
    p = [_c64(t) for t in params]
    a = _c64(x)
    cache = {"stem": None, "blocks": [], "head": None, "in_shape": a.shape}
    i = 0
    if m.stem == 1:
        a, c = _cbr_fwd(a, p[0], p[1], p[2], 1, 1, True, eps, q)
        a = qq(a)
        cache["stem"] = (c, None)
        i = 3
    elif m.stem == 2:
        a, c = _cbr_fwd(a, p[0], p[1], p[2], 2, 3, True, eps, q)
        a = qq(a)
        pre_shape = a.shape
        a, idx = maxpool_fwd(a, 3, 2, 1)
        cache["stem"] = (c, (idx, pre_shape))
        i = 3
    for b in m.blocks:
        n = 3 * len(block_convs(b)) - (2 if (b.proj and not b.proj_bn) else 0)
        a, c = block_forward(a, p[i:i + n], b, eps, q)
        cache["blocks"].append(c)
        i += n
    logits = None
    if m.head:
        pooled = a.mean(axis=(1, 2))
        logits = pooled @ p[i].T + p[i + 1]
        cache["head"] = (pooled, p[i], a.shape)
    return a, logits, cache


def module_backward(m: ModuleDesc, cache, dy=None, dlogits=None, need_dx=True, q=None):
    """Module-local back-propagation from the terminal adjoint: dy (on F_k(x_k)) or dlogits (last module).

    Returns (dparams list in packing order, dx_k or None)."""
    if cache.get("order") == "pre":
        return _module_backward_pre(m, cache, dy, dlogits, need_dx, q)
    qq = q or _id
    tail = []
    if m.head:
        pooled, wfc, shp = cache["head"]
        dwfc = dlogits.T @ pooled
        dbfc = dlogits.sum(axis=0)
        dpooled = dlogits @ wfc
        g = qq(np.broadcast_to(dpooled[:, None, None, :] / (shp[1] * shp[2]), shp).copy())
        tail = [dwfc, dbfc]
    else:
        g = _c64(dy)
    grads = []
    nb = len(cache["blocks"])
    for j in range(nb - 1, -1, -1):
        first = (j == 0 and cache["stem"] is None)
        g, bg = block_backward(g, cache["blocks"][j], need_dx=(need_dx or not first), q=q)
        grads = bg + grads
    if cache["stem"] is not None:
        c, mp = cache["stem"]
        if mp is not None:
            g = qq(maxpool_bwd(g, mp[0], mp[1]))
        g, sg = _cbr_bwd(g, c, need_dx=need_dx, q=q)
        if g is not None:
            g = qq(g)
        grads = sg + grads
    return grads + tail, (g if need_dx else None)


# ----------------------------------------------------------------------------- losses
def local_loss_grad(y, x_next, lam, rho, scale=1.0):
    """loss_k = s*(rho/2*sum r^2 + sum lam*r), dy = s*(rho*r + lam), r = F_k(x_k) - x_{k+1}; lam=None: penalty."""
    r = _c64(y) - _c64(x_next)
    loss = 0.5 * rho * np.sum(r * r)
    dy = rho * r
    if lam is not None:
        lam = _c64(lam)
        loss = loss + np.sum(lam * r)
        dy = dy + lam
    return scale * loss, scale * dy


def residual_norm2(y, x_next):
    """Constraint violation of an interface, |F_k(x_k) - x_{k+1}|^2 (the quantity Sec. 5 plots beside the loss)."""
    r = _c64(y) - _c64(x_next)
    return float(np.sum(r * r))


def ce_loss_grad(logits, labels):
    """Mini-batch mean of softmax cross-entropy and its gradient w.r.t. the logits."""
    z = _c64(logits)
    N = z.shape[0]
    zmax = z.max(axis=1, keepdims=True)
    e = np.exp(z - zmax)
    se = e.sum(axis=1, keepdims=True)
    lse = np.log(se) + zmax
    loss = float(np.mean(lse[:, 0] - z[np.arange(N), labels]))
    dz = e / se
    dz[np.arange(N), labels] -= 1.0
    return loss, dz / N


def multiplier_update(lam, y, x_next, step):
    """lam_k <- lam_k + step * (F_k(x_k) - x_{k+1})   (paper: step = eta/(2*beta) = eta/rho)."""
    return _c64(lam) + step * (_c64(y) - _c64(x_next))


def sgd_update(p, g, lr, v=None, momentum=0.0, weight_decay=0.0):
    """Parameter update of Sec. 4.1, W <- W - eta * dW, applied right after a module's adjoint recursion.  The paper
    states plain gradient descent; the two usual extensions are off at 0:  g' = g + weight_decay*W,
    v <- momentum*v + g' (v starts at 0), W <- W - lr*v.  Returns (W_new, v_new); v_new is None without momentum."""
    p = _c64(p)
    gg = _c64(g) + weight_decay * p
    if momentum != 0.0:
        v = gg if v is None else momentum * _c64(v) + gg
        return p - lr * v, v
    return p - lr * gg, None


def aux_variable_update(x, y_prev, dx, lam_prev, rho, eta, scale=1.0):
    """Correction of the auxiliary variable x_k, 1 <= k <= K-1 (Sec. 4.1, the update of lambda_k that follows the
    adjoint recursion): a gradient step on the relaxed objective with respect to x_k.  x_k enters the term of
    interface k-1, scale*(rho/2*|y_{k-1} - x_k|^2 + <lam_{k-1}, y_{k-1} - x_k>), whose derivative is
    scale*(rho*(x_k - y_{k-1}) - lam_{k-1}), and the local loss of module k, whose derivative dx_k the
    module-local backward pass returns:
        x_k <- x_k - eta * ( scale*(rho*(x_k - y_{k-1}) - lam_{k-1}) + dx_k ).
    lam_prev=None: penalty method."""
    x = _c64(x)
    g = rho * (x - _c64(y_prev))
    if lam_prev is not None:
        g = g - _c64(lam_prev)
    return x - eta * (scale * g + _c64(dx))


def _aux_stack_fwd(a: AuxDesc, x, params, eps, q):
    """The AuxNet as the stack its descriptor lists: block i = conv3x3(stride_i, pad 1) -> BN(batch statistics)
    [-> ReLU], parameters (filter, gamma, beta) at params[3i:3i+3]; blocks in front of the last end in ReLU and their
    outputs are stored (rounded by q).  Returns the unrounded output of the last block and one cache per block."""
    qq = q or _id
    caches = []
    blocks = aux_blocks(a)
    h = _c64(x)
    for i, (_, _, stride, relu) in enumerate(blocks):
        h, c = _cbr_fwd(h, _c64(params[3 * i]), _c64(params[3 * i + 1]), _c64(params[3 * i + 2]), stride, 1, relu, eps, q)
        caches.append(c)
        if i + 1 < len(blocks):
            h = qq(h)
    return h, caches


def _aux_stack_bwd(g, caches, q):
    """Pull the gradient g on the AuxNet output back through the stack; returns the parameter gradients in the order
    of the parameters."""
    qq = q or _id
    grads = [None] * len(caches)
    for i in range(len(caches) - 1, -1, -1):
        dx, grads[i] = _cbr_bwd(g, caches[i], need_dx=i > 0, q=q)
        if i > 0:
            g = qq(dx)
    return [t for gr in grads for t in gr]


def auxnet_forward(a: AuxDesc, image, params, eps=1e-5, q=None):
    """x = AuxNet(image): every block of the stack is [ReLU](BN(conv3x3_stride(.)))."""
    out, _ = _aux_stack_fwd(a, image, params, eps, q)
    return out if q is None else q(out)


def auxnet_distill_grad(a: AuxDesc, image, params, target, eps=1e-5, scale=1.0, q=None):
    """Distillation objective of an AuxNet (Sec. 4.2: theta <- argmin |x_k - AuxNet(x_0; theta)|^2, one descent step
    per iteration; the step is the caller's):  loss = scale * sum (AuxNet(image) - target)^2  and its gradient with
    respect to theta = (filter, gamma, beta) of every block, back-propagated through [ReLU,] BN (batch statistics) and
    the conv.  Returns (loss, [dW, dgamma, dbeta] per block, flat)."""
    qq = q or _id
    out, caches = _aux_stack_fwd(a, image, params, eps, q)
    out = qq(out)
    r = out - _c64(target)
    loss = scale * float(np.sum(r * r))
    g = qq(2.0 * scale * r)
    return loss, _aux_stack_bwd(g, caches, q)


def reauxnet_grad(a: AuxDesc, image, params, y_prev, dx, lam_prev, rho, scale=1.0, eps=1e-5, q=None):
    """Update direction of a recursive AuxNet (Sec. 4.4, the rule that replaces the separate correction and
    distillation when x_k = ReAuxNet_k(x_0; xi_k) is generated from the mini-batch): the gradient of the relaxed
    objective with respect to x_k,
        g = scale*(rho*(x_k - F_{k-1}(x_{k-1})) - lam_{k-1}) + dx_k,        x_k = ReAuxNet_k(x_0; xi_k),
    (interface term k-1 plus the local loss of module k, whose input gradient dx_k the module-local backward pass
    returns) pulled back through the AuxNet: d/d xi_k = g * dReAuxNet_k/d xi_k.  The paper states the rule for the
    penalty method; lam_prev=None is that case, a multiplier enters as in the correction of x_k.  ReAuxNet_k is the
    stack the descriptor lists (k blocks from the mini-batch in the paper's form).
    Returns [dW, dgamma, dbeta] per block, flat."""
    qq = q or _id
    out, caches = _aux_stack_fwd(a, image, params, eps, q)
    out = qq(out)
    g = rho * (out - _c64(y_prev))
    if lam_prev is not None:
        g = g - _c64(lam_prev)
    g = qq(scale * g + _c64(dx))
    return _aux_stack_bwd(g, caches, q)


# ----------------------------------------------------------------------------- whole step / serial net
def local_step(net: NetDesc, xs, params, labels, lams=None, scale=1.0, need_dx0=False, q=None):
    """One synchronous local step of all K modules.

    xs: [x_0 (image), x_1, ..., x_{K-1}]; lams: K-1 multipliers or None (penalty).
    Returns dict with y (K-1 interface outputs + last-module features), logits, loss[K], dy, dlogits,
    dparams[K], dx[K] (dx[0] None unless need_dx0)."""
    K = net.K
    out = {"y": [], "loss": [], "dy": [], "dparams": [], "dx": [], "logits": None, "dlogits": None}
    for k in range(K):
        m = net.modules[k]
        y, logits, cache = module_forward(m, xs[k], params[k], net.bn_eps, q)
        out["y"].append(y)
        if k < K - 1:
            lam = None if lams is None else lams[k]
            loss, dy = local_loss_grad(y, xs[k + 1], lam, net.rho, scale)
            if q is not None:
                dy = q(dy)
            out["dy"].append(dy)
            dp, dx = module_backward(m, cache, dy=dy, need_dx=(k > 0 or need_dx0), q=q)
        else:
            loss, dz = ce_loss_grad(logits, labels)
            out["logits"], out["dlogits"] = logits, dz
            dp, dx = module_backward(m, cache, dlogits=dz, need_dx=(k > 0 or need_dx0), q=q)
        out["loss"].append(loss)
        out["dparams"].append(dp)
        out["dx"].append(dx)
    return out


def serial_forward(net: NetDesc, image, params):
    """Layer-serial forward (K=1 reading): states [x_0, X at every module boundary], logits, caches."""
    xs, caches, a, logits = [_c64(image)], [], _c64(image), None
    for k in range(net.K):
        a, logits, c = module_forward(net.modules[k], a, params[k], net.bn_eps)
        caches.append(c)
        if k < net.K - 1:
            xs.append(a)
    return xs, logits, caches


def serial_backward(net: NetDesc, caches, logits, labels, need_dx0=False):
    """End-to-end back-propagation of the classification loss: (loss, dparams[K], adjoints at interfaces).

    adjoint[k] = d phi / d X at the input of module k (k >= 1)."""
    loss, dz = ce_loss_grad(logits, labels)
    K = net.K
    dparams, adj = [None] * K, [None] * K
    g = None
    for k in range(K - 1, -1, -1):
        if k == K - 1:
            dp, g = module_backward(net.modules[k], caches[k], dlogits=dz, need_dx=(k > 0 or need_dx0))
        else:
            dp, g = module_backward(net.modules[k], caches[k], dy=g, need_dx=(k > 0 or need_dx0))
        dparams[k], adj[k] = dp, g
    return loss, dparams, adj
