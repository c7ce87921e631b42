"""GPU-side test plumbing: run one local step through the C ABI and compare with the oracle."""
import sys

import numpy as np

import workloads as wl
from oracle import lpref
from tests.helpers import rel_err, step_inputs
from workloads import configs as cfg
from workloads.configs import Block

TOL = {"f32": 1e-4, "bf16": 2e-2}   # max|gpu-ref| / max|ref| per tensor


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def gpu_mini_basic(batch=3, dtype="f32", serial=False):
    """K=3, channels multiple of 8, ragged M (6x6 images): stem, stride-2 projection block, head.
    serial=True: the same network as one module (K=1, ordinary back-propagation)."""
    blocks = [Block("basic", 8, 8, 8, 1, False), Block("basic", 8, 16, 16, 2, True),
              Block("basic", 16, 16, 16, 1, False), Block("basic", 16, 16, 16, 1, False)]
    per_module = [blocks] if serial else [blocks[:2], blocks[2:3], blocks[3:]]
    net = cfg._assemble("gpu_mini_basic", per_module, batch, 6, 6, 3, 1, 8, 5, seed=21)
    net.dtype = dtype
    return net


def gpu_mini_basic_flags(batch=3, dtype="f32"):
    """gpu_mini_basic with ReLU behind the residual sum in three of its four blocks and a bare conv1x1 projection."""
    net = gpu_mini_basic(batch, dtype)
    net.name = "gpu_mini_basic_flags"
    blocks = [b for m in net.modules for b in m.blocks]
    for i in (0, 1, 3):
        blocks[i].post_relu = True
    blocks[1].proj_bn = False
    return net


def gpu_mini_bottleneck(batch=2, dtype="f32"):
    blocks = [Block("bottleneck", 8, 16, 8, 1, True), Block("bottleneck", 16, 32, 8, 2, True),
              Block("bottleneck", 32, 32, 8, 1, False)]
    net = cfg._assemble("gpu_mini_bottleneck", [blocks[:1], blocks[1:]], batch, 24, 24, 3, 2, 8, 6, seed=22)
    net.dtype = dtype
    return net


def gpu_mini_wide(batch=3):
    """bf16, widths 136 and 296 on 6x10 images: the wide-layer filter-gradient kernel with ragged channel tiles
    (136 of 160; 296 = 160 + 136), a ragged last k-tile (180 pixels) and image sizes that are not powers of two."""
    blocks = [Block("basic", 136, 136, 136, 1, False), Block("basic", 136, 296, 296, 1, True),
              Block("basic", 296, 296, 296, 1, False)]
    net = cfg._assemble("gpu_mini_wide", [blocks[:1], blocks[1:]], batch, 6, 10, 3, 1, 136, 7, seed=23)
    net.dtype = "bf16"
    return net


def gpu_mini_wide_strided(batch=5, side=(12, 20), widths=(136, 296)):
    """bf16, a stride-2 block between two wide widths (the shape of the 160->320 and 320->640 layers of WRN-28-10):
    ragged channel tiles, an output width that is not a power of two (10, or 5 with side (12, 10)) and a pixel count
    that is no multiple of a k-tile (batch 5: 300 or 150 output pixels)."""
    a, b = widths
    blocks = [Block("basic", a, a, a, 1, False), Block("basic", a, b, b, 2, True), Block("basic", b, b, b, 1, False)]
    net = cfg._assemble("gpu_mini_wide_strided", [blocks[:1], blocks[1:]], batch, side[0], side[1], 3, 1, a, 7, seed=29)
    net.dtype = "bf16"
    return net


def load_step(ls, net, inp):
    for k in range(net.K):
        ls.set_params(k, inp["params"][k])
        ls.set_x(k, inp["xs"][k])
    if inp.get("aux_params"):
        for j in range(net.K - 1):
            ls.set_aux_params(j, inp["aux_params"][j])
    ls.set_lams(inp["lams"])
    ls.set_labels(inp["labels"])


class _PerturbedRounding:
    """bf16 storage rounding preceded by a seeded relative perturbation of size 1e-6: a second, equally valid
    bf16 evaluation (it differs from the first the way another fp32 summation order would)."""

    def __init__(self, seed):
        self.seed, self.n = seed, 0

    def __call__(self, a):
        self.n += 1
        a = np.asarray(a, dtype=np.float64)
        return wl.round_bf16(a * (1.0 + 1e-6 * wl.normal(self.seed, f"perturb{self.n}", a.shape)))


def _oracle_pieces(net, inp, scale, want_dx0, q):
    """Oracle run entry point by entry point: forward; loss/adjoint from the stored forward outputs;
    backward from the stored adjoints."""
    from tests.helpers import store
    K = net.K
    fwd = [lpref.module_forward(net.modules[k], inp["xs"][k], inp["params"][k], net.bn_eps, q) for k in range(K)]
    o = {"y": [fwd[k][0] for k in range(K - 1)], "logits": fwd[K - 1][1], "fwd": fwd}
    o["y_in"] = [store(net, y) for y in o["y"]]
    o["logits_in"] = o["logits"].astype(np.float32).astype(np.float64)
    o["lg"] = [lpref.local_loss_grad(o["y_in"][k], inp["xs"][k + 1], None if inp["lams"] is None else inp["lams"][k],
                                     net.rho, scale) for k in range(K - 1)]
    o["ce_loss"], o["dz"] = lpref.ce_loss_grad(o["logits_in"], inp["labels"])
    o["dy_in"] = [store(net, g[1]) for g in o["lg"]]
    o["dz_in"] = o["dz"].astype(np.float32).astype(np.float64)
    o["bwd"] = []
    for k in range(K):
        need_dx = (k > 0) or want_dx0
        if k < K - 1:
            o["bwd"].append(lpref.module_backward(net.modules[k], fwd[k][2], dy=o["dy_in"][k], need_dx=need_dx, q=q))
        else:
            o["bwd"].append(lpref.module_backward(net.modules[k], fwd[k][2], dlogits=o["dz_in"], need_dx=need_dx, q=q))
    return o


def compare_step(net, scale=1.0, want_dx0=False, tol=None, check_aux=True, lanes="default", max_uncovered=None):
    """End-to-end parity of the whole local step on identical seeded inputs (the bar for the backward pass of the
    bf16 kernels is the unit-by-unit test of tests/gpu_unitwise.py; this is the whole-network check beside it).

    fp32 mode: the oracle is the plain float64 definition, tolerance 1e-4 on every tensor.

    bf16 mode: forward outputs, losses and terminal adjoints are compared with the plain float64 definition (2e-2).
    A backward pass through several layers takes decisions from stored bf16 values (ReLU masks), so end to end it is
    compared with the oracle's diagnostic storage-rounding mode at the same flat 2e-2.  Such a pass is chaotic where
    it is deep or where a gradient sums few pixels (a 1e-6 difference in front of a rounding flips a mask bit, and one
    flipped bit moves a filter gradient summed over M pixels by about 1/sqrt(M) of its norm): the oracle therefore
    measures its own spread (two more runs with a 1e-6 relative perturbation in front of every rounding), and a
    tensor that misses the tolerance while the oracle's own spread reaches a third of it is reported as NOT COVERED
    by this test -- it is never passed at a wider tolerance (its kernels are covered unit by unit).  max_uncovered,
    when given, bounds the number of such tensors.

    Pass 1 (entry point by entry point): the loss/terminal-adjoint call and the backward call are each fed the
    ORACLE's value of their input (rounded to the storage type) on both sides.
    Pass 2 (the fused call, as the product runs it): lp_local_step runs on the device; its y is compared with the
    oracle's, its loss and terminal adjoint with the oracle's evaluated AT the device's stored y (so the cancellation
    in r = F_k(x_k) - x_{k+1} amplifies nothing), and its backward results with the oracle's backward pass from the
    device's stored adjoint.  One tolerance for both passes.
    """
    import torch
    from paper_2112_05387_amd import LocalStep
    tol = TOL[net.dtype] if tol is None else tol
    K = net.K
    inp = step_inputs(net, lpref)
    specs = [wl.module_tensor_specs(m) for m in net.modules]
    bf16 = net.dtype == "bf16"
    q = wl.round_bf16 if bf16 else None
    plain_fwd = [lpref.module_forward(net.modules[k], inp["xs"][k], inp["params"][k], net.bn_eps) for k in range(K)] if bf16 else None
    o = _oracle_pieces(net, inp, scale, want_dx0, q)
    spread = {}
    if bf16:
        for trial in range(2):          # two perturbed evaluations; the spread of a tensor is the larger deviation
            o2 = _oracle_pieces(net, inp, scale, want_dx0, _PerturbedRounding(net.seed + 7919 * trial))
            for k in range(K):
                for sp, a, b in zip(specs[k], o2["bwd"][k][0], o["bwd"][k][0]):
                    key = f"m{k}.{sp.name}"
                    spread[key] = max(spread.get(key, 0.0), rel_err(a, b))
                if o["bwd"][k][1] is not None:
                    spread[f"dx{k}"] = max(spread.get(f"dx{k}", 0.0), rel_err(o2["bwd"][k][1], o["bwd"][k][1]))
    y_ref, logits_ref, lg, bwd = o["y"], o["logits"], o["lg"], o["bwd"]

    def check(errs, label):
        bad, uncovered = {}, {}
        for name, v in errs.items():
            sp = spread.get(name.replace("fused.", ""), 0.0)
            if v <= tol:
                continue
            if 3.0 * sp > tol:
                uncovered[name] = (v, sp)           # chaotic in bf16 end to end: reported as not covered, never passed
            else:
                bad[name] = (v, tol)
        top = sorted(((k, v) for k, v in errs.items() if k not in uncovered), key=lambda kv: -kv[1])[:5]
        say(f"[{net.name} {net.dtype} N={net.modules[0].N}] {label}: {len(errs) - len(uncovered)} tensors within {tol:g}, worst: "
            + ", ".join(f"{k}={v:.2e}" for k, v in top))
        if uncovered:
            wt = sorted(uncovered.items(), key=lambda kv: -kv[1][0])[:4]
            say(f"    NOT COVERED here ({len(uncovered)} backward tensors beyond {tol:g} whose own bf16 spread in the oracle exceeds {tol / 3:.1e}; "
                "the unit-wise test covers their kernels), e.g. " + ", ".join(f"{k}: err {v:.1e} spread {s_:.1e}" for k, (v, s_) in wt))
        assert not bad, f"{label}: beyond tolerance (error, allowed): {bad}"
        assert max_uncovered is None or len(uncovered) <= max_uncovered, f"{label}: {len(uncovered)} tensors not covered"

    ls = LocalStep(net)
    worst = {}
    try:
        if lanes != "default":
            ls.set_stream_lanes(lanes)
        load_step(ls, net, inp)
        if net.aux is not None and check_aux:
            ls.auxnet_forward()
            torch.cuda.synchronize()
            for j in range(K - 1):
                want = lpref.auxnet_forward(net.aux[j], inp["image"], inp["aux_params"][j], net.bn_eps)
                worst[f"aux{j}"] = rel_err(ls.to_host(ls.x[j + 1]), want)
            for k in range(1, K):          # the step itself starts from the oracle-side x_k (already rounded)
                ls.set_x(k, inp["xs"][k])
        # ---- pass 1
        ls.module_forward()
        torch.cuda.synchronize()
        for k in range(K - 1):
            worst[f"y{k}"] = rel_err(ls.to_host(ls.y[k]), plain_fwd[k][0] if bf16 else y_ref[k])
        worst["logits"] = rel_err(ls.to_host(ls.logits), plain_fwd[K - 1][1] if bf16 else logits_ref)
        for k in range(K - 1):
            ls.y[k].copy_(ls.to_dev(o["y_in"][k]))
        ls.logits.copy_(ls.to_dev(o["logits_in"], low=False))
        ls.local_loss_grad(net.rho, scale)
        torch.cuda.synchronize()
        for k in range(K - 1):
            worst[f"dy{k}"] = rel_err(ls.to_host(ls.dy[k]), lg[k][1])
            worst[f"loss{k}"] = abs(float(ls.loss[k].item()) - lg[k][0]) / max(abs(lg[k][0]), 1e-30)
            r2 = lpref.residual_norm2(o["y_in"][k], inp["xs"][k + 1])
            worst[f"r2_{k}"] = abs(float(ls.r2[k].item()) - r2) / max(r2, 1e-30)
        worst[f"loss{K - 1}"] = abs(float(ls.loss[K - 1].item()) - o["ce_loss"]) / abs(o["ce_loss"])
        worst["dlogits"] = rel_err(ls.to_host(ls.dlogits), o["dz"])
        for k in range(K - 1):
            ls.dy[k].copy_(ls.to_dev(o["dy_in"][k]))
        ls.dlogits.copy_(ls.to_dev(o["dz_in"], low=False))
        ls.module_backward(want_dx0=want_dx0)
        torch.cuda.synchronize()
        for k in range(K):
            for sp, g, r in zip(specs[k], ls.get_grads(k), bwd[k][0]):
                worst[f"m{k}.{sp.name}"] = rel_err(g, r)
            if bwd[k][1] is not None:
                worst[f"dx{k}"] = rel_err(ls.to_host(ls.dx[k]), bwd[k][1])
        if net.al:
            ls.al_multiplier_update(net.step)
            torch.cuda.synchronize()
            for k in range(K - 1):
                want = lpref.multiplier_update(inp["lams"][k], o["y_in"][k], inp["xs"][k + 1], net.step)
                worst[f"lam{k}"] = rel_err(ls.to_host(ls.lam[k]), want)
            ls.set_lams(inp["lams"])
        check(worst, "entry-point pass")
        # ---- pass 2: the fused entry point, every stream lane through all phases on its own
        ls.local_step(net.rho, scale, want_dx0=want_dx0)
        torch.cuda.synchronize()
        cw = {}
        fwd = o["fwd"]
        for k in range(K):
            need_dx = (k > 0) or want_dx0
            if k < K - 1:
                y_dev, dy_dev = ls.to_host(ls.y[k]), ls.to_host(ls.dy[k])
                cw[f"fused.y{k}"] = rel_err(y_dev, plain_fwd[k][0] if bf16 else y_ref[k])
                loss, dy = lpref.local_loss_grad(y_dev, inp["xs"][k + 1], None if inp["lams"] is None else inp["lams"][k], net.rho, scale)
                cw[f"fused.dy{k}"] = rel_err(dy_dev, dy)
                cw[f"fused.loss{k}"] = abs(float(ls.loss[k].item()) - loss) / max(abs(loss), 1e-30)
                r2 = lpref.residual_norm2(y_dev, inp["xs"][k + 1])
                cw[f"fused.r2_{k}"] = abs(float(ls.r2[k].item()) - r2) / max(r2, 1e-30)
                dp, dx = lpref.module_backward(net.modules[k], fwd[k][2], dy=dy_dev, need_dx=need_dx, q=q)
            else:
                z_dev, dz_dev = ls.to_host(ls.logits), ls.to_host(ls.dlogits)
                cw["fused.logits"] = rel_err(z_dev, plain_fwd[k][1] if bf16 else logits_ref)
                loss, dz = lpref.ce_loss_grad(z_dev, inp["labels"])
                cw["fused.dlogits"] = rel_err(dz_dev, dz)
                cw[f"fused.loss{k}"] = abs(float(ls.loss[k].item()) - loss) / abs(loss)
                dp, dx = lpref.module_backward(net.modules[k], fwd[k][2], dlogits=dz_dev, need_dx=need_dx, q=q)
            for sp, g, r in zip(specs[k], ls.get_grads(k), dp):
                cw[f"fused.m{k}.{sp.name}"] = rel_err(g, r)
            if dx is not None:
                cw[f"fused.dx{k}"] = rel_err(ls.to_host(ls.dx[k]), dx)
        check(cw, "fused pass")
        worst.update(cw)
    finally:
        ls.close()
    return worst
