"""Full-size parity: WideResNet-28-10, batch 128, bf16, augmented Lagrangian, in the launch configuration
`bench.py` times (every call covers all K modules, the filter gradients run as the grouped last launches).

What the oracle can afford at this size in about a minute of CPU time:
  * the forward pass of every module, element by element (plain float64 definition, tolerance 2e-2);
  * loss / terminal adjoint and multiplier update, element by element;
  * the backward pass through the LAST conv+BN unit of every module (and the projection of its block, and the
    classification head): dW, dgamma, dbeta.  That unit sees the terminal adjoint directly -- there is no ReLU
    between the module output and it -- so its gradients do not depend on decisions taken from rounded values,
    and they exercise the BN-backward kernels and both filter-gradient kernels at full size.  The expected values
    are the plain float64 definition (no storage rounding on the oracle's side).
Every other unit of the backward pass is covered at this size by tests/test_gpu_unitwise.py.
Auxiliary variables are seeded N(0,1) tensors (they are free inputs of the step)."""
import numpy as np
import pytest

import workloads as wl
from oracle import lpref
from tests.gpu_common import say
from tests.helpers import rel_err, store

pytestmark = pytest.mark.gpu

TOL = 2e-2


def test_wrn28_10_full_size():
    import torch
    from paper_2112_05387_amd import LocalStep
    net = wl.make_config("wrn28_10")
    K, scale = net.K, 1.0
    params = [wl.make_params(net, k) for k in range(K)]
    image, labels = wl.make_image(net), wl.make_labels(net)
    xs = [image] + [store(net, wl.normal(net.seed, f"full_x{k}", (m.N, m.H, m.W, m.C)))
                    for k, m in enumerate(net.modules) if k > 0]
    lams = [store(net, wl.normal(net.seed, f"full_lam{k}", xs[k + 1].shape, net.lam_sigma)) for k in range(K - 1)]
    specs = [wl.module_tensor_specs(m) for m in net.modules]

    ls = LocalStep(net)
    errs = {}
    try:
        for k in range(K):
            ls.set_params(k, params[k])
            ls.set_x(k, xs[k])
        ls.set_lams(lams)
        ls.set_labels(labels)
        say("full size: device forward")
        ls.module_forward()
        torch.cuda.synchronize()
        dev_y = [ls.to_host(ls.y[k]) for k in range(K - 1)]
        dev_logits = ls.to_host(ls.logits)

        # ---- oracle, module by module (the caches are large: keep only what the last unit needs)
        y_in, dy_in, want = [], [], {}
        for k in range(K):
            m = net.modules[k]
            say(f"full size: oracle forward of module {k}")
            y, logits, cache = lpref.module_forward(m, xs[k], params[k], net.bn_eps)
            unit_caches, proj_cache, _ = cache["blocks"][-1]
            last = unit_caches[-1]
            if k < K - 1:
                errs[f"y{k}"] = rel_err(dev_y[k], y)
                y_in.append(store(net, y))
                loss, dy = lpref.local_loss_grad(y_in[k], xs[k + 1], lams[k], net.rho, scale)
                want[f"loss{k}"] = loss
                want[f"dy{k}"] = dy
                dy_in.append(store(net, dy))
                g = dy_in[k]
                n_tail = 0
            else:
                errs["logits"] = rel_err(dev_logits, logits)
                logits_in = logits.astype(np.float32).astype(np.float64)
                ce, dz = lpref.ce_loss_grad(logits_in, labels)
                want["ce"], want["dz"] = ce, dz
                dz_in = dz.astype(np.float32).astype(np.float64)
                pooled, wfc, shp = cache["head"]
                want["fc_w"], want["fc_b"] = dz_in.T @ pooled, dz_in.sum(axis=0)
                g = store(net, np.broadcast_to((dz_in @ wfc)[:, None, None, :] / (shp[1] * shp[2]), shp).copy())
                n_tail = 2
            _, (dw, dgamma, dbeta) = lpref._cbr_bwd(g, last, need_dx=False)
            n_proj = 3 if proj_cache is not None else 0
            i_last = len(specs[k]) - n_tail - n_proj - 3
            want[f"m{k}.last"] = (i_last, dw, dgamma, dbeta)
            if proj_cache is not None:
                _, (pw, pg, pb) = lpref._cbr_bwd(g, proj_cache, need_dx=False)
                want[f"m{k}.proj"] = (i_last + 3, pw, pg, pb)
            del cache, unit_caches, proj_cache, last, y

        # ---- loss / terminal adjoint on the oracle's stored forward outputs
        for k in range(K - 1):
            ls.y[k].copy_(ls.to_dev(y_in[k]))
        ls.logits.copy_(ls.to_dev(logits_in, low=False))
        ls.local_loss_grad(net.rho, scale)
        torch.cuda.synchronize()
        for k in range(K - 1):
            errs[f"dy{k}"] = rel_err(ls.to_host(ls.dy[k]), want[f"dy{k}"])
            errs[f"loss{k}"] = abs(float(ls.loss[k].item()) - want[f"loss{k}"]) / abs(want[f"loss{k}"])
        errs["ce"] = abs(float(ls.loss[K - 1].item()) - want["ce"]) / abs(want["ce"])
        errs["dlogits"] = rel_err(ls.to_host(ls.dlogits), want["dz"])

        # ---- backward from the oracle's stored adjoints
        for k in range(K - 1):
            ls.dy[k].copy_(ls.to_dev(dy_in[k]))
        ls.dlogits.copy_(ls.to_dev(dz_in, low=False))
        say("full size: device backward")
        ls.module_backward()
        torch.cuda.synchronize()
        for k in range(K):
            grads = ls.get_grads(k)
            for tag in ("last", "proj"):
                if f"m{k}.{tag}" not in want:
                    continue
                i, dw, dgamma, dbeta = want[f"m{k}.{tag}"]
                assert specs[k][i].shape == tuple(dw.shape), (specs[k][i].name, specs[k][i].shape, dw.shape)
                errs[f"m{k}.{tag}.dW"] = rel_err(grads[i], dw)
                errs[f"m{k}.{tag}.dgamma"] = rel_err(grads[i + 1], dgamma)
                errs[f"m{k}.{tag}.dbeta"] = rel_err(grads[i + 2], dbeta)
        gl = ls.get_grads(K - 1)
        errs["fc_w"] = rel_err(gl[-2], want["fc_w"])
        errs["fc_b"] = rel_err(gl[-1], want["fc_b"])

        # ---- multiplier update
        ls.al_multiplier_update(net.step)
        torch.cuda.synchronize()
        for k in range(K - 1):
            errs[f"lam{k}"] = rel_err(ls.to_host(ls.lam[k]), lpref.multiplier_update(lams[k], y_in[k], xs[k + 1], net.step))
    finally:
        ls.close()
    top = sorted(errs.items(), key=lambda kv: -kv[1])
    say("full size, worst: " + ", ".join(f"{k}={v:.2e}" for k, v in top[:8]))
    bad = {k: v for k, v in errs.items() if not v <= TOL}
    assert not bad, f"beyond {TOL}: {bad}"
