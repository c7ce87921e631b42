"""Shared test helpers: small custom networks, oracle-side input recipes and error norms."""
import numpy as np

import workloads as wl
from workloads import configs as cfg
from workloads.configs import Block


def mini_basic(batch=3, dtype="f32"):
    """K=3: [stem + basic(4->4) + basic(4->8, stride 2, proj)], [basic(8->8)], [basic(8->8) + head(5)]."""
    blocks = [Block("basic", 4, 4, 4, 1, False), Block("basic", 4, 8, 8, 2, True),
              Block("basic", 8, 8, 8, 1, False), Block("basic", 8, 8, 8, 1, False)]
    net = cfg._assemble("mini_basic", [blocks[:2], blocks[2:3], blocks[3:]], batch, 6, 6, 3, 1, 4, 5, seed=11)
    net.dtype = dtype
    return net


def mini_basic_flags(batch=3, dtype="f32"):
    """mini_basic with the two block options of the conv-BN-ReLU order switched on: ReLU after the residual sum in
    blocks 0, 1 and 3, and a bare conv1x1 projection (no BN) on the stride-2 block."""
    net = mini_basic(batch, dtype)
    net.name = "mini_basic_flags"
    blocks = [b for m in net.modules for b in m.blocks]
    for i in (0, 1, 3):
        blocks[i].post_relu = True
    blocks[1].proj_bn = False
    return net


def mini_basic_pre(batch=3, dtype="f32"):
    """mini_basic in the pre-activation order: bare conv stem, BN-ReLU-conv blocks, BN-ReLU in front of the head."""
    return cfg.with_order(mini_basic(batch, dtype), "pre")


def mini_bottleneck(batch=2, dtype="f32"):
    """K=2 with the 7x7 stride-2 stem + maxpool and bottleneck blocks (one strided with projection)."""
    blocks = [Block("bottleneck", 4, 8, 2, 1, True), Block("bottleneck", 8, 16, 4, 2, True),
              Block("bottleneck", 16, 16, 4, 1, False)]
    net = cfg._assemble("mini_bottleneck", [blocks[:1], blocks[1:]], batch, 16, 16, 3, 2, 4, 6, seed=12)
    net.dtype = dtype
    return net


def store(net, a, low=True):
    """Round to what the device holds (bf16 for activations/filters in bf16 mode, else fp32)."""
    if net.dtype == "bf16" and low:
        return wl.round_bf16(a)
    return np.asarray(a, dtype=np.float32).astype(np.float64)


def step_inputs(net, lpref, consistent=False):
    """Oracle-side recipe of one local step's inputs.

    image, params, labels seeded; auxiliary variables = oracle serial forward states + N(0, sigma^2)
    (or AuxNet outputs when the config has an AuxNet); multipliers N(0, lam_sigma^2) or None."""
    params = [wl.make_params(net, k) for k in range(net.K)]
    image = wl.make_image(net)
    labels = wl.make_labels(net)
    aux_params = None
    if net.aux is not None:
        aux_params = [wl.make_aux_params(net, j) for j in range(net.K - 1)]
        xs = [image] + [store(net, lpref.auxnet_forward(net.aux[j], image, aux_params[j], net.bn_eps))
                        for j in range(net.K - 1)]
    else:
        states, _, _ = lpref.serial_forward(net, image, params)
        xs = [image]
        for k in range(1, net.K):
            noise = 0.0 if consistent else wl.make_noise(net, f"noise{k}", states[k].shape, net.noise_sigma)
            xs.append(store(net, states[k] + noise))
    lams = None
    if net.al:
        lams = [store(net, wl.make_noise(net, f"lam{k}", xs[k + 1].shape, net.lam_sigma)) for k in range(net.K - 1)]
    return dict(image=image, params=params, labels=labels, xs=xs, lams=lams, aux_params=aux_params)


def rel_err(a, ref):
    """max|a-ref| / max|ref| (infinity-norm relative error of a whole tensor)."""
    a = np.asarray(a, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    d = float(np.max(np.abs(a - ref))) if ref.size else 0.0
    s = float(np.max(np.abs(ref))) if ref.size else 0.0
    return d / s if s > 0 else d
