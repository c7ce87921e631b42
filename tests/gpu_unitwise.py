"""Unit-by-unit parity of a local step at a FIXED tolerance.

The device runs one whole local step (all K modules, the launch configuration of the benchmark).  Then every
conv+BN unit is checked on its own: its INPUT tensors are read back from the device (the workspace layout that keeps
every gradient, `LocalStep(net, keep_gradients=True)`), every EXPECTED value is computed from them by the oracle's
plain float64 primitives (no storage rounding mode), and the device's outputs of that unit are compared with it:

  forward   y = conv(in, W)                          pre-BN result as stored
            per-channel mean / variance              from the device's [sum, sum of squares]
            out = [ReLU](BN(y) [+ skip | + BN_p(y_p)])
  backward  dgamma, dbeta                            BN backward sums
            dy  = BN backward of the arriving gradient (through ReLU)
            din = dgrad(dy, W) [+ skip-path gradient]
            dW  = wgrad(in, dy)

Every comparison is one layer deep, so nothing depends on a decision (ReLU mask) that an EARLIER rounding could have
flipped, and the tolerance is flat: max|dev - ref| / max|ref| <= tol.  The one decision inside a unit is its own ReLU
mask z > 0, which the device takes in fp32 and the oracle in fp64: elements whose |z| is within a few fp32 roundings
of zero may fall either way, both results are valid there, and the check accepts either (their number is printed and
must stay a vanishing fraction of the tensor).
"""
import numpy as np

import workloads as wl
from oracle import lpref
from tests.gpu_common import say
from tests.helpers import rel_err, store

TOL = {"f32": 1e-4, "bf16": 2e-2}
STAT_TOL = 1e-4           # batch statistics are accumulated in fp32 / fp64 in both modes
AMBIGUOUS = 1e-5          # |z| <= AMBIGUOUS * (|gamma*yhat| + |beta|): the ReLU decision may differ between fp32 and fp64


def _rel_floor(a, ref, floor):
    """max|a - ref| / max(max|ref|, floor).  `floor` is 1 % of the size of the TERMS a sum is made of: where the sum
    cancels exactly (the BN backward of a gradient that is constant over the pixels, which is what the head hands to
    the last unit of a one-sample mini-batch: d gamma = g * sum yhat = 0, d y = 0), the reference is rounding noise of
    float64 and an error relative to it means nothing; relative to the terms the bar is still 100 x tighter than tol."""
    d = float(np.max(np.abs(np.asarray(a, np.float64) - ref))) if ref.size else 0.0
    s = max(float(np.max(np.abs(ref))) if ref.size else 0.0, floor)
    return d / s if s > 0 else d


def _rel(d, ref):
    s = float(np.max(np.abs(ref))) if ref.size else 0.0
    return float(np.max(np.abs(d))) / s if s > 0 else float(np.max(np.abs(d))) if d.size else 0.0


def seeded_step_inputs(net):
    """Seeded inputs of one local step without an oracle forward pass: the auxiliary variables are free inputs of the
    step, so N(0,1) tensors of the module-input shapes serve (values change no kernel's work)."""
    K = net.K
    params = [wl.make_params(net, k) for k in range(K)]
    image, labels = wl.make_image(net), wl.make_labels(net)
    xs = [image] + [store(net, wl.normal(net.seed, f"unit_x{k}", (m.N, m.H, m.W, m.C)))
                    for k, m in enumerate(net.modules) if k > 0]
    lams = None
    if net.al:
        lams = [store(net, wl.normal(net.seed, f"unit_lam{k}", xs[k + 1].shape, net.lam_sigma)) for k in range(K - 1)]
    return params, image, labels, xs, lams


def check_units(net, tol=None, fused=True, modules=None, note="", scale=1.0):
    """Run one local step on the device and check every unit of the selected modules.  Returns {name: error}.
    scale: the caller's loss scale (losses and terminal adjoints are multiplied by it)."""
    import torch
    from paper_2112_05387_amd import LocalStep
    from paper_2112_05387_amd import binding as B
    tol = TOL[net.dtype] if tol is None else tol
    K = net.K
    params, image, labels, xs, lams = seeded_step_inputs(net)
    specs = [wl.module_tensor_specs(m) for m in net.modules]
    errs, n_amb, n_elems = {}, 0, 0
    ls = LocalStep(net, keep_gradients=True)
    try:
        for k in range(K):
            ls.set_params(k, params[k])
            ls.set_x(k, xs[k])
        ls.set_lams(lams)
        ls.set_labels(labels)
        say(f"unit-wise {net.name} N={net.modules[0].N} {net.dtype}{note}: device step ({'one call' if fused else 'four calls'})")
        if fused:
            ls.local_step(net.rho, scale)
        else:
            ls.module_forward()
            ls.local_loss_grad(net.rho, scale)
            ls.module_backward()
        torch.cuda.synchronize()
        for k in (range(K) if modules is None else modules):
            m = net.modules[k]
            units = ls.units(k)
            minfo = B.lp_debug_module_info(ls.net, k)
            grads = ls.get_grads(k)
            P = params[k]
            for ui, u in enumerate(units):
                tag = f"m{k}.{'stem' if u.block < 0 else 'b%d' % u.block}.{'proj' if u.slot == 3 else 'c%d' % u.slot}"
                in_shape, out_shape = (u.N, u.H, u.W, u.cin), (u.N, u.Ho, u.Wo, u.cout)
                Mpix = u.N * u.Ho * u.Wo
                w = P[u.t_w]
                x_in = ls.fetch(u.in_, in_shape)
                y_dev = ls.fetch(u.y, out_shape)
                # ---- forward: convolution
                errs[f"{tag}.y"] = rel_err(y_dev, lpref.conv_fwd(x_in, w, u.stride, u.pad))
                if u.plain:
                    # a bare projection: no BN; the gradient on its result is the (masked) gradient on the block output
                    g = ls.fetch(u.gout, out_shape)
                    if u.has_dgrad:
                        errs[f"{tag}.din"] = rel_err(ls.fetch(u.din, in_shape), lpref.conv_dgrad(g, w, in_shape, u.stride, u.pad))
                    errs[f"{tag}.dW"] = rel_err(grads[u.t_w], lpref.conv_wgrad(x_in, g, w.shape, u.stride, u.pad))
                    say(f"  {tag:16s} [{u.N}x{u.H}x{u.W}x{u.cin} -> {u.cout}, {u.R}x{u.R}/{u.stride}, no BN]")
                    continue
                gamma, beta = P[u.t_gamma], P[u.t_beta]
                # ---- forward: batch statistics of the stored tensor
                st = ls.fetch(u.stats, (B.LP_STAT_STRIPES, 2, u.cout), "f64").sum(axis=0)      # kept as partial sums
                mean_ref = y_dev.mean(axis=(0, 1, 2))
                var_ref = ((y_dev - mean_ref) ** 2).mean(axis=(0, 1, 2))
                mean_dev = st[0] / Mpix
                var_dev = st[1] / Mpix - mean_dev ** 2
                errs[f"{tag}.mean"] = float(np.max(np.abs(mean_dev - mean_ref)) / np.sqrt(np.max(var_ref)))
                errs[f"{tag}.var"] = float(np.max(np.abs(var_dev - var_ref)) / np.max(var_ref))
                # ---- forward: BN (+ skip) (+ ReLU), the oracle's own statistics of the tensor it normalises
                z, (yhat, invstd) = lpref.bn_fwd(y_dev, gamma, beta, net.bn_eps)
                if u.slot != 3:
                    pre = z
                    if u.skip_kind == 1:
                        pre = z + ls.fetch(u.skip, out_shape)
                    elif u.skip_kind == 2:
                        pu = units[u.skip_unit]
                        yp = ls.fetch(pu.y, out_shape)
                        zp = yp if pu.plain else lpref.bn_fwd(yp, P[pu.t_gamma], P[pu.t_beta], net.bn_eps)[0]
                        pre = z + zp
                    want = np.maximum(pre, 0.0) if (u.relu or u.post_relu) else pre
                    out_dev = ls.fetch(u.out, out_shape)
                    errs[f"{tag}.out"] = rel_err(out_dev, want)
                    if u.post_relu:          # the mask pass: the arriving gradient where the stored block output is positive
                        errs[f"{tag}.gmask"] = rel_err(ls.fetch(u.gout, out_shape), ls.fetch(u.graw, out_shape) * (out_dev > 0.0))
                # ---- backward: BN (through the unit's own ReLU)
                g = ls.fetch(u.gout, out_shape)
                amb = None
                if u.relu:
                    mask = z > 0.0
                    amb = np.abs(z) <= AMBIGUOUS * (np.abs(gamma * yhat) + np.abs(beta))
                    dz = g * mask
                else:
                    dz = g
                dy_ref, dgamma, dbeta = lpref.bn_bwd(dz, (yhat, invstd), gamma)
                errs[f"{tag}.dgamma"] = _rel_floor(grads[u.t_gamma], dgamma, 1e-2 * float(np.max(np.abs(dz * yhat).sum(axis=(0, 1, 2)))))
                errs[f"{tag}.dbeta"] = _rel_floor(grads[u.t_beta], dbeta, 1e-2 * float(np.max(np.abs(dz).sum(axis=(0, 1, 2)))))
                dy_dev = ls.fetch(u.dy, out_shape)
                d = np.abs(dy_dev - dy_ref)
                if amb is not None and amb.any():
                    # the other valid value of an element whose mask bit is undecided: the bit flipped for that element alone
                    alt = gamma * invstd * (np.where(mask, 0.0, g) - dbeta / Mpix - yhat * (dgamma / Mpix))
                    d = np.where(amb, np.minimum(d, np.abs(dy_dev - alt)), d)
                    n_amb += int(amb.sum())
                n_elems += d.size
                dy_floor = 1e-2 * float(np.max(np.abs(gamma * invstd)) * np.max(np.abs(dz)))
                dy_den = max(float(np.max(np.abs(dy_ref))), dy_floor) if d.size else 0.0
                errs[f"{tag}.dy"] = (float(np.max(d)) / dy_den if dy_den > 0 else float(np.max(d))) if d.size else 0.0
                # ---- backward: data- and filter-gradient from the stored dy
                if u.has_dgrad:
                    want = lpref.conv_dgrad(dy_dev, w, in_shape, u.stride, u.pad)
                    if u.din_add.space != B.LP_REF_NONE:
                        want = want + ls.fetch(u.din_add, in_shape)
                    errs[f"{tag}.din"] = rel_err(ls.fetch(u.din, in_shape), want)
                errs[f"{tag}.dW"] = rel_err(grads[u.t_w], lpref.conv_wgrad(x_in, dy_dev, w.shape, u.stride, u.pad))
                worst = max((v, n) for n, v in errs.items() if n.startswith(tag + "."))
                say(f"  {tag:16s} [{u.N}x{u.H}x{u.W}x{u.cin} -> {u.cout}, {u.R}x{u.R}/{u.stride}]  worst {worst[1].split('.')[-1]} = {worst[0]:.2e}")
            # ---- what lies around the units
            if m.stem == 2:
                pin = ls.fetch(minfo.pool_in, (m.N, minfo.pH, minfo.pW, minfo.pC))
                pout, idx = lpref.maxpool_fwd(pin, 3, 2, 1)
                errs[f"m{k}.pool.out"] = rel_err(ls.fetch(minfo.pool_out, pout.shape), pout)
                gp = ls.fetch(minfo.g_pool_out, pout.shape)
                errs[f"m{k}.pool.din"] = rel_err(ls.fetch(minfo.g_pool_in, pin.shape), lpref.maxpool_bwd(gp, idx, pin.shape))
            oshape = (minfo.oN, minfo.oH, minfo.oW, minfo.oC)
            if k < K - 1:
                y_dev = ls.to_host(ls.y[k])
                loss, dy = lpref.local_loss_grad(y_dev, xs[k + 1], None if lams is None else lams[k], net.rho, scale)
                errs[f"m{k}.loss"] = abs(float(ls.loss[k].item()) - loss) / abs(loss)
                errs[f"m{k}.adjoint"] = rel_err(ls.to_host(ls.dy[k]), dy)
            else:
                feat = ls.fetch(minfo.feat, oshape)
                wfc, bfc = P[minfo.t_fc_w], P[minfo.t_fc_b]
                pooled = feat.mean(axis=(1, 2))
                logits = pooled @ wfc.T + bfc
                logits_dev = ls.to_host(ls.logits)
                errs[f"m{k}.logits"] = rel_err(logits_dev, logits)
                ce, dz = lpref.ce_loss_grad(logits_dev, labels)
                errs[f"m{k}.ce"] = abs(float(ls.loss[k].item()) - ce) / abs(ce)
                dz_dev = ls.to_host(ls.dlogits)
                errs[f"m{k}.dlogits"] = rel_err(dz_dev, dz)
                errs[f"m{k}.fc_w"] = rel_err(grads[minfo.t_fc_w], dz_dev.T @ pooled)
                errs[f"m{k}.fc_b"] = rel_err(grads[minfo.t_fc_b], dz_dev.sum(axis=0))
                dfeat = np.broadcast_to((dz_dev @ wfc)[:, None, None, :] / (oshape[1] * oshape[2]), oshape)
                errs[f"m{k}.dfeat"] = rel_err(ls.fetch(minfo.dfeat, oshape), dfeat)
    finally:
        ls.close()
    top = sorted(errs.items(), key=lambda kv: -kv[1])
    say(f"unit-wise {net.name} N={net.modules[0].N} {net.dtype}{note}: {len(errs)} tensors, worst " +
        ", ".join(f"{n}={v:.2e}" for n, v in top[:6]))
    say(f"    ReLU decisions within fp32 rounding of zero (either value accepted): {n_amb} of {n_elems} elements")
    assert n_amb <= 1e-3 * max(n_elems, 1), f"{n_amb} undecided mask elements of {n_elems}"
    bad = {}
    for n, v in errs.items():
        t = STAT_TOL if n.endswith((".mean", ".var")) else tol
        if not v <= t:
            bad[n] = (v, t)
    assert not bad, f"beyond tolerance (error, allowed): {bad}"
    return errs
