"""ctypes binding of the C ABI declared in include/lp.h: same names, argument marshalling only."""
import ctypes
import os
from ctypes import POINTER, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_uint32, c_void_p

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblp.so")

LP_OK = 0
LP_ERR_INVALID_ARG, LP_ERR_SHAPE, LP_ERR_DTYPE, LP_ERR_WORKSPACE, LP_ERR_STATE, LP_ERR_HIP = 1, 2, 3, 4, 5, 6
LP_F32, LP_BF16 = 0, 1
LP_ORDER_POST, LP_ORDER_PRE = 0, 1
LP_T_CONV, LP_T_BN_GAMMA, LP_T_BN_BETA, LP_T_FC_W, LP_T_FC_B = 0, 1, 2, 3, 4

EXPORTS = ["lp_net_create", "lp_net_destroy", "lp_net_param_bytes", "lp_net_num_tensors", "lp_net_tensor_info",
           "lp_net_workspace_bytes", "lp_net_set_workspace", "lp_auxnet_forward", "lp_auxnet_forward_static", "lp_module_forward",
           "lp_local_loss_grad", "lp_module_backward", "lp_al_multiplier_update", "lp_aux_variable_update", "lp_auxnet_distill_grad", "lp_sgd_update", "lp_reauxnet_grad", "lp_net_set_stream_lanes", "lp_local_step", "lp_net_set_residual_output", "lp_net_set_deterministic",
           "lp_debug_im2col_offsets", "lp_debug_keep_gradients", "lp_debug_unit_count", "lp_debug_unit_info",
           "lp_debug_module_info", "lp_debug_filter_load_extent", "lp_debug_conv_geometry", "lp_debug_conv_offsets", "lp_debug_mfma_peak",
           "lp_debug_saved_tensor", "lp_net_set_fused_update", "lp_profile_enable", "lp_profile_fetch", "lp_last_error", "lp_version"]

KIND_NAMES = {0: "fill", 1: "filter_relayout", 2: "conv_igemm(fwd/dgrad)", 3: "bn_apply", 4: "maxpool_fwd", 5: "head_fwd",
              6: "head_bwd", 7: "maxpool_bwd", 8: "bn_bwd_reduce", 9: "bn_bwd_apply", 10: "conv_wgrad", 11: "bn_stats", 12: "loss", 13: "cross_entropy", 14: "multiplier_update",
              15: "relu_mask", 16: "sgd(small tensors)"}


class lp_block_desc(ctypes.Structure):
    _fields_ = [("kind", c_int), ("cin", c_int), ("cout", c_int), ("width", c_int), ("stride", c_int), ("proj", c_int),
                ("proj_plain", c_int), ("post_relu", c_int)]


class lp_module_desc(ctypes.Structure):
    _fields_ = [("stem", c_int), ("stem_cout", c_int), ("n_blocks", c_int), ("blocks", POINTER(lp_block_desc)),
                ("head", c_int), ("n_classes", c_int), ("N", c_int), ("H", c_int), ("W", c_int), ("C", c_int),
                ("order", c_int)]


LP_AUX_MAX_DEPTH = 8
LP_STAT_STRIPES = 8          # per-channel sums are kept as this many partial sums (debug views)


class lp_aux_desc(ctypes.Structure):
    _fields_ = [("cin", c_int), ("cout", c_int), ("stride", c_int), ("relu", c_int), ("from_prev", c_int),
                ("depth", c_int), ("mid_cout", c_int * (LP_AUX_MAX_DEPTH - 1)),
                ("mid_stride", c_int * (LP_AUX_MAX_DEPTH - 1))]


class lp_tensor_info(ctypes.Structure):
    _fields_ = [("kind", c_int), ("block", c_int), ("slot", c_int), ("dtype", c_int), ("ndim", c_int),
                ("dims", c_int * 4), ("offset", c_size_t), ("grad_offset", c_size_t), ("numel", c_size_t)]


LP_REF_NONE, LP_REF_WORKSPACE, LP_REF_X, LP_REF_Y, LP_REF_DY, LP_REF_DX = 0, 1, 2, 3, 4, 5


class lp_debug_ref(ctypes.Structure):
    _fields_ = [("space", c_int), ("idx", c_int), ("off", c_size_t)]


class lp_debug_unit(ctypes.Structure):
    _fields_ = [(n, c_int) for n in ("block", "slot", "R", "stride", "pad", "cin", "cout", "N", "H", "W", "Ho", "Wo", "relu",
                                     "t_w", "t_gamma", "t_beta", "skip_kind", "skip_unit", "has_dgrad", "plain", "post_relu")] + \
               [(n, lp_debug_ref) for n in ("in_", "y", "stats", "out", "skip", "gout", "dy", "red", "din", "din_add", "graw")]


class lp_debug_module(ctypes.Structure):
    _fields_ = [(n, c_int) for n in ("keep_gradients", "oN", "oH", "oW", "oC", "pH", "pW", "pC")] + \
               [(n, lp_debug_ref) for n in ("pool_in", "pool_out", "pool_arg", "g_pool_out", "g_pool_in", "feat", "pooled", "dfeat")] + \
               [("t_fc_w", c_int), ("t_fc_b", c_int)]


class lp_profile_rec(ctypes.Structure):
    _fields_ = [("kind", c_int), ("cfg", c_int), ("nprob", c_int), ("blocks", c_int), ("ms", c_float), ("flops", ctypes.c_double),
                ("bytes", ctypes.c_double)]


class LpError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"lp status {status}: {text}")
        self.status = status


_lib = None


def lib():
    """Load liblp.so (built in-tree by build.py).  Raises if it is missing: there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not found: build it with `python -m paper_2112_05387_amd.build` "
                               "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vpp = POINTER(c_void_p)
        L.lp_net_create.argtypes = [c_int, POINTER(lp_module_desc), POINTER(lp_aux_desc), c_int, c_float, POINTER(c_void_p)]
        L.lp_net_destroy.argtypes = [c_void_p]
        L.lp_net_param_bytes.argtypes = [c_void_p, c_int, c_int, POINTER(c_size_t), POINTER(c_size_t)]
        L.lp_net_num_tensors.argtypes = [c_void_p, c_int, c_int, POINTER(c_int)]
        L.lp_net_tensor_info.argtypes = [c_void_p, c_int, c_int, c_int, POINTER(lp_tensor_info)]
        L.lp_net_workspace_bytes.argtypes = [c_void_p, POINTER(c_size_t)]
        L.lp_net_set_workspace.argtypes = [c_void_p, c_void_p, c_size_t]
        L.lp_auxnet_forward.argtypes = [c_void_p, c_void_p, c_void_p, vpp, vpp]
        L.lp_auxnet_forward_static.argtypes = [c_void_p, c_void_p, c_void_p, vpp, vpp]
        L.lp_auxnet_distill_grad.argtypes = [c_void_p, c_void_p, c_void_p, vpp, vpp, c_float, c_void_p, vpp]
        L.lp_module_forward.argtypes = [c_void_p, c_void_p, c_uint32, vpp, vpp, vpp, c_void_p]
        L.lp_local_loss_grad.argtypes = [c_void_p, c_void_p, c_uint32, vpp, vpp, vpp, c_float, c_float, c_void_p,
                                         c_void_p, c_void_p, vpp, c_void_p]
        L.lp_module_backward.argtypes = [c_void_p, c_void_p, c_uint32, vpp, c_void_p, vpp, vpp, vpp]
        L.lp_al_multiplier_update.argtypes = [c_void_p, c_void_p, vpp, vpp, vpp, c_float]
        L.lp_local_step.argtypes = [c_void_p, c_void_p, c_uint32, vpp, vpp, vpp, vpp, vpp, c_float, c_float, c_float, c_void_p,
                                    c_void_p, vpp, c_void_p, c_void_p, vpp, vpp]
        L.lp_net_set_stream_lanes.argtypes = [c_void_p, POINTER(c_int)]
        L.lp_net_set_residual_output.argtypes = [c_void_p, c_void_p]
        L.lp_net_set_deterministic.argtypes = [c_void_p, c_int]
        L.lp_reauxnet_grad.argtypes = [c_void_p, c_void_p, c_void_p, vpp, vpp, vpp, vpp, c_float, c_float, vpp]
        L.lp_sgd_update.argtypes = [c_void_p, c_void_p, c_int, c_uint32, vpp, vpp, vpp, vpp, c_float, c_float, c_float]
        L.lp_net_set_fused_update.argtypes = [c_void_p, c_int, c_float, c_float, c_float, vpp, vpp]
        L.lp_aux_variable_update.argtypes = [c_void_p, c_void_p, vpp, vpp, vpp, vpp, c_float, c_float, c_float]
        L.lp_debug_im2col_offsets.argtypes = [c_void_p] + [c_int] * 7 + [c_void_p, c_void_p, c_void_p, c_int]
        L.lp_debug_saved_tensor.argtypes = [c_void_p, c_int, c_int, POINTER(c_void_p), POINTER(c_size_t)]
        L.lp_debug_conv_geometry.argtypes = [c_int] * 12 + [POINTER(c_int)]
        L.lp_debug_conv_offsets.argtypes = [c_void_p] + [c_int] * 12 + [c_void_p] * 6 + [c_int]
        L.lp_debug_mfma_peak.argtypes = [c_void_p, c_int, c_int, c_int, c_void_p, c_void_p]
        L.lp_debug_keep_gradients.argtypes = [c_int]
        L.lp_debug_unit_count.argtypes = [c_void_p, c_int, POINTER(c_int)]
        L.lp_debug_unit_info.argtypes = [c_void_p, c_int, c_int, POINTER(lp_debug_unit)]
        L.lp_debug_module_info.argtypes = [c_void_p, c_int, POINTER(lp_debug_module)]
        L.lp_debug_filter_load_extent.argtypes = [c_int] * 7 + [POINTER(c_size_t), POINTER(c_size_t)]
        L.lp_profile_enable.argtypes = [c_void_p, c_int]
        L.lp_profile_fetch.argtypes = [c_void_p, POINTER(lp_profile_rec), c_int, POINTER(c_int)]
        L.lp_last_error.restype = c_char_p
        L.lp_version.restype = c_char_p
        for name in EXPORTS:
            if name not in ("lp_last_error", "lp_version"):
                getattr(L, name).restype = c_int
        _lib = L
    return _lib


def _check(status):
    if status != LP_OK:
        raise LpError(status, lib().lp_last_error().decode())


def _ptr_array(ptrs):
    """Python list of ints/None -> (void*)[n]; None stays NULL."""
    if ptrs is None:
        return None
    arr = (c_void_p * len(ptrs))()
    for i, p in enumerate(ptrs):
        arr[i] = p if p else None
    return arr


def lp_version():
    return lib().lp_version().decode()


def lp_last_error():
    return lib().lp_last_error().decode()


def lp_net_create(modules, aux, dtype, bn_eps):
    """modules: objects with stem, stem_cout, blocks[kind,cin,cout,width,stride,proj], head, n_classes, N, H, W, C."""
    K = len(modules)
    mods = (lp_module_desc * max(K, 1))()
    keep = []
    for k, m in enumerate(modules):
        nb = len(m.blocks)
        blks = (lp_block_desc * max(nb, 1))()
        for i, b in enumerate(m.blocks):
            kind = b.kind if isinstance(b.kind, int) else {"basic": 0, "bottleneck": 1}[b.kind]
            blks[i] = lp_block_desc(kind, b.cin, b.cout, b.width, b.stride, int(b.proj),
                                    int(not getattr(b, "proj_bn", True)), int(getattr(b, "post_relu", False)))
        keep.append(blks)
        mods[k] = lp_module_desc(int(m.stem), int(m.stem_cout), nb, blks, int(m.head), int(m.n_classes), m.N, m.H, m.W, m.C,
                                 {"post": LP_ORDER_POST, "pre": LP_ORDER_PRE}[getattr(m, "order", "post")])
    auxp = None
    if aux is not None:
        auxp = (lp_aux_desc * max(len(aux), 1))()
        for j, a in enumerate(aux):
            mid = tuple(getattr(a, "mid", ()))
            if len(mid) > LP_AUX_MAX_DEPTH - 1:
                raise ValueError(f"AuxNet {j}: {len(mid) + 1} blocks, at most {LP_AUX_MAX_DEPTH}")
            d = lp_aux_desc(a.cin, a.cout, a.stride, int(a.relu), int(getattr(a, "from_prev", False)), len(mid) + 1)
            for i, (co, sd) in enumerate(mid):
                d.mid_cout[i] = co
                d.mid_stride[i] = sd
            auxp[j] = d
    out = c_void_p()
    dt = dtype if isinstance(dtype, int) else {"f32": LP_F32, "bf16": LP_BF16}[dtype]
    _check(lib().lp_net_create(K, mods, auxp, dt, float(bn_eps), ctypes.byref(out)))
    return out


def lp_net_destroy(net):
    _check(lib().lp_net_destroy(net))


def lp_net_param_bytes(net, aux, k):
    pb, gb = c_size_t(), c_size_t()
    _check(lib().lp_net_param_bytes(net, aux, k, ctypes.byref(pb), ctypes.byref(gb)))
    return pb.value, gb.value


def lp_net_num_tensors(net, aux, k):
    n = c_int()
    _check(lib().lp_net_num_tensors(net, aux, k, ctypes.byref(n)))
    return n.value


def lp_net_tensor_info(net, aux, k, i):
    info = lp_tensor_info()
    _check(lib().lp_net_tensor_info(net, aux, k, i, ctypes.byref(info)))
    return info


def lp_net_workspace_bytes(net):
    b = c_size_t()
    _check(lib().lp_net_workspace_bytes(net, ctypes.byref(b)))
    return b.value


def lp_net_set_workspace(net, dev_ptr, nbytes):
    _check(lib().lp_net_set_workspace(net, dev_ptr, nbytes))


def lp_auxnet_forward(net, stream, image, aux_params, x_out):
    _check(lib().lp_auxnet_forward(net, stream, image, _ptr_array(aux_params), _ptr_array(x_out)))


def lp_auxnet_forward_static(net, stream, image, aux_params, x_out):
    _check(lib().lp_auxnet_forward_static(net, stream, image, _ptr_array(aux_params), _ptr_array(x_out)))


def lp_module_forward(net, stream, module_mask, x, params, y, logits):
    _check(lib().lp_module_forward(net, stream, module_mask, _ptr_array(x), _ptr_array(params), _ptr_array(y), logits))


def lp_local_loss_grad(net, stream, module_mask, y, x_next, lam, rho, loss_scale, logits, labels, loss, dy, dlogits):
    _check(lib().lp_local_loss_grad(net, stream, module_mask, _ptr_array(y), _ptr_array(x_next), _ptr_array(lam),
                                    float(rho), float(loss_scale), logits, labels, loss, _ptr_array(dy), dlogits))


def lp_module_backward(net, stream, module_mask, dy, dlogits, params, dparams, dx):
    _check(lib().lp_module_backward(net, stream, module_mask, _ptr_array(dy), dlogits, _ptr_array(params),
                                    _ptr_array(dparams), _ptr_array(dx)))


def lp_auxnet_distill_grad(net, stream, image, aux_params, x_target, loss_scale, loss, daux_params):
    _check(lib().lp_auxnet_distill_grad(net, stream, image, _ptr_array(aux_params), _ptr_array(x_target), float(loss_scale),
                                        loss, _ptr_array(daux_params)))


def lp_local_step(net, stream, mask, x, params, y, x_next, lam, rho, scale, mult_step, labels, loss, dy, logits, dlogits,
                  dparams, dx):
    _check(lib().lp_local_step(net, stream, mask, _ptr_array(x), _ptr_array(params), _ptr_array(y), _ptr_array(x_next),
                               None if lam is None else _ptr_array(lam), float(rho), float(scale), float(mult_step), labels,
                               loss, _ptr_array(dy), logits, dlogits, _ptr_array(dparams), _ptr_array(dx)))


def lp_net_set_stream_lanes(net, lanes):
    arr = None if lanes is None else (c_int * len(lanes))(*[int(v) for v in lanes])
    _check(lib().lp_net_set_stream_lanes(net, arr))


def lp_net_set_deterministic(net, on):
    _check(lib().lp_net_set_deterministic(net, int(on)))


def lp_net_set_residual_output(net, r2):
    _check(lib().lp_net_set_residual_output(net, r2))


def lp_reauxnet_grad(net, stream, image, aux_params, y_prev, dx, lam_prev, rho, scale, daux_params):
    _check(lib().lp_reauxnet_grad(net, stream, image, _ptr_array(aux_params), _ptr_array(y_prev), _ptr_array(dx),
                                  None if lam_prev is None else _ptr_array(lam_prev), float(rho), float(scale),
                                  _ptr_array(daux_params)))


def lp_sgd_update(net, stream, aux, mask, params, dparams, velocity, master, lr, momentum, weight_decay):
    _check(lib().lp_sgd_update(net, stream, int(aux), mask, _ptr_array(params), _ptr_array(dparams),
                               None if velocity is None else _ptr_array(velocity),
                               None if master is None else _ptr_array(master), float(lr), float(momentum), float(weight_decay)))


def lp_net_set_fused_update(net, on, lr=0.0, momentum=0.0, weight_decay=0.0, velocity=None, master=None):
    _check(lib().lp_net_set_fused_update(net, int(on), float(lr), float(momentum), float(weight_decay),
                                         None if velocity is None else _ptr_array(velocity),
                                         None if master is None else _ptr_array(master)))


def lp_aux_variable_update(net, stream, x, y_prev, dx, lam_prev, rho, scale, eta):
    _check(lib().lp_aux_variable_update(net, stream, _ptr_array(x), _ptr_array(y_prev), _ptr_array(dx),
                                        None if lam_prev is None else _ptr_array(lam_prev), float(rho), float(scale), float(eta)))


def lp_al_multiplier_update(net, stream, lam, y, x_next, step):
    _check(lib().lp_al_multiplier_update(net, stream, _ptr_array(lam), _ptr_array(y), _ptr_array(x_next), float(step)))


def lp_debug_im2col_offsets(stream, H, W, Cin, R, S, stride, pad, m, q, out, count):
    _check(lib().lp_debug_im2col_offsets(stream, H, W, Cin, R, S, stride, pad, m, q, out, count))


def lp_debug_saved_tensor(net, k, which):
    p, n = c_void_p(), c_size_t()
    _check(lib().lp_debug_saved_tensor(net, k, which, ctypes.byref(p), ctypes.byref(n)))
    return p.value, n.value


def lp_debug_conv_geometry(kernel, mode, parity, N, H, W, Cin, Cout, R, stride, pad, bk):
    g = (c_int * 12)()
    _check(lib().lp_debug_conv_geometry(kernel, mode, parity, N, H, W, Cin, Cout, R, stride, pad, bk, g))
    return dict(zip(("M", "Ncol", "C", "ntr", "nts", "r0", "rs", "s0", "ss", "ldw", "BM", "bk"), list(g)))


def lp_debug_conv_offsets(stream, kernel, mode, parity, N, H, W, Cin, Cout, R, stride, pad, bk, m, q, col, in_off, w_off,
                          out_off, count):
    _check(lib().lp_debug_conv_offsets(stream, kernel, mode, parity, N, H, W, Cin, Cout, R, stride, pad, bk, m, q, col,
                                       in_off, w_off, out_off, count))


def lp_debug_mfma_peak(stream, mode, blocks, iters, clk, sink):
    _check(lib().lp_debug_mfma_peak(stream, mode, blocks, iters, clk, sink))


def lp_debug_keep_gradients(on):
    _check(lib().lp_debug_keep_gradients(int(on)))


def lp_debug_unit_count(net, k):
    n = c_int()
    _check(lib().lp_debug_unit_count(net, k, ctypes.byref(n)))
    return n.value


def lp_debug_unit_info(net, k, i):
    u = lp_debug_unit()
    _check(lib().lp_debug_unit_info(net, k, i, ctypes.byref(u)))
    return u


def lp_debug_module_info(net, k):
    m = lp_debug_module()
    _check(lib().lp_debug_module_info(net, k, ctypes.byref(m)))
    return m


def lp_debug_filter_load_extent(kernel, bk, bn, nw, ncol, cin, r):
    end, live = c_size_t(), c_size_t()
    _check(lib().lp_debug_filter_load_extent(kernel, bk, bn, nw, ncol, cin, r, ctypes.byref(end), ctypes.byref(live)))
    return end.value, live.value


def lp_profile_enable(net, on):
    _check(lib().lp_profile_enable(net, int(on)))


def lp_profile_fetch(net):
    n = c_int()
    _check(lib().lp_profile_fetch(net, None, 0, ctypes.byref(n)))
    if n.value == 0:
        return []
    recs = (lp_profile_rec * n.value)()
    _check(lib().lp_profile_fetch(net, recs, n.value, ctypes.byref(n)))
    return [dict(kind=r.kind, cfg=r.cfg, nprob=r.nprob, blocks=r.blocks, ms=r.ms, flops=r.flops, bytes=r.bytes) for r in recs]
