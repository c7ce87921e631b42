"""Pins of the oracle's local step: finite differences and the invariants the relaxed problem implies."""
import numpy as np
import pytest

import workloads as wl
from oracle import lpref
from tests.helpers import mini_basic, mini_basic_flags, mini_basic_pre, mini_bottleneck, step_inputs, rel_err


def _local_loss(net, k, x, params, x_next, lam, labels, scale):
    m = net.modules[k]
    y, logits, _ = lpref.module_forward(m, x, params, net.bn_eps)
    if k < net.K - 1:
        return lpref.local_loss_grad(y, x_next, lam, net.rho, scale)[0]
    return lpref.ce_loss_grad(logits, labels)[0]


@pytest.mark.parametrize("mk", [mini_basic, mini_bottleneck, mini_basic_pre, mini_basic_flags])
def test_module_backward_finite_differences(mk):
    """Every parameter tensor and the module input: directional derivatives, one tensor at a time,
    plus single coordinates, against central differences of the local loss (float64)."""
    net = mk()
    net.rho, net.al = 1.3, True
    net.lam_sigma = 0.5
    inp = step_inputs(net, lpref)
    rng = np.random.default_rng(7)
    scale = 0.7
    out = lpref.local_step(net, inp["xs"], inp["params"], inp["labels"], inp["lams"], scale, need_dx0=True)
    h = 1e-6
    for k in range(net.K):
        x, p = inp["xs"][k], inp["params"][k]
        xn = inp["xs"][k + 1] if k < net.K - 1 else None
        lam = inp["lams"][k] if k < net.K - 1 else None
        f = lambda xx, pp: _local_loss(net, k, xx, pp, xn, lam, inp["labels"], scale)
        specs = wl.module_tensor_specs(net.modules[k])
        assert len(specs) == len(p) == len(out["dparams"][k])
        for i, sp in enumerate(specs):
            assert out["dparams"][k][i].shape == tuple(sp.shape)
            d = rng.standard_normal(p[i].shape)
            pp, pm = list(p), list(p)
            pp[i], pm[i] = p[i] + h * d, p[i] - h * d
            fd = (f(x, pp) - f(x, pm)) / (2 * h)
            an = float(np.sum(out["dparams"][k][i] * d))
            assert abs(fd - an) <= 2e-6 * max(1.0, abs(an)), (k, sp.name, fd, an)
            j = tuple(rng.integers(0, s) for s in p[i].shape)
            e = np.zeros_like(p[i]); e[j] = h
            pp[i], pm[i] = p[i] + e, p[i] - e
            fd = (f(x, pp) - f(x, pm)) / (2 * h)
            assert abs(fd - out["dparams"][k][i][j]) <= 2e-6 * max(1.0, abs(fd)), (k, sp.name, j)
        d = rng.standard_normal(x.shape)
        fd = (f(x + h * d, p) - f(x - h * d, p)) / (2 * h)
        an = float(np.sum(out["dx"][k] * d))
        assert abs(fd - an) <= 2e-6 * max(1.0, abs(an)), (k, "dx", fd, an)


@pytest.mark.parametrize("mk", [mini_basic, mini_bottleneck, mini_basic_pre, mini_basic_flags])
def test_vanish_invariant(mk):
    """x_{k+1} = F_k(x_k) and zero multipliers: every penalty term, its terminal adjoint, every weight
    gradient and every dx of modules 0..K-2 vanish exactly (the relaxed problem reduces to the original)."""
    net = mk()
    inp = step_inputs(net, lpref, consistent=True)
    states, _, _ = lpref.serial_forward(net, inp["image"], inp["params"])
    xs = [inp["image"]] + states[1:]
    out = lpref.local_step(net, xs, inp["params"], inp["labels"], None, 1.0, need_dx0=True)
    for k in range(net.K - 1):
        assert out["loss"][k] == 0.0
        assert not out["dy"][k].any()
        assert all(not g.any() for g in out["dparams"][k])
        assert not out["dx"][k].any()
    assert out["loss"][-1] > 0.0


@pytest.mark.parametrize("mk", [mini_basic, mini_bottleneck, mini_basic_pre, mini_basic_flags])
def test_last_module_equals_end_to_end_and_serial_fd(mk):
    """With consistent auxiliary variables the last module's local gradients are those of end-to-end
    back-propagation; the end-to-end gradients themselves are pinned by finite differences of the
    serial network's loss."""
    net = mk()
    inp = step_inputs(net, lpref, consistent=True)
    states, logits, caches = lpref.serial_forward(net, inp["image"], inp["params"])
    loss, dps, adj = lpref.serial_backward(net, caches, logits, inp["labels"], need_dx0=True)
    xs = [inp["image"]] + states[1:]
    out = lpref.local_step(net, xs, inp["params"], inp["labels"], None, 1.0, need_dx0=True)
    assert out["loss"][-1] == loss
    for a, b in zip(out["dparams"][-1], dps[-1]):
        np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(out["dx"][-1], adj[-1])

    def serial_loss(params, image):
        _, lg, _ = lpref.serial_forward(net, image, params)
        return lpref.ce_loss_grad(lg, inp["labels"])[0]

    rng = np.random.default_rng(3)
    h = 1e-6
    for k in range(net.K):
        for i in range(len(inp["params"][k])):
            d = rng.standard_normal(inp["params"][k][i].shape)
            pp = [list(p) for p in inp["params"]]; pm = [list(p) for p in inp["params"]]
            pp[k][i] = pp[k][i] + h * d; pm[k][i] = pm[k][i] - h * d
            fd = (serial_loss(pp, inp["image"]) - serial_loss(pm, inp["image"])) / (2 * h)
            an = float(np.sum(dps[k][i] * d))
            assert abs(fd - an) <= 2e-6 * max(1.0, abs(an)), (k, i, fd, an)
    d = rng.standard_normal(inp["image"].shape)
    fd = (serial_loss(inp["params"], inp["image"] + h * d) - serial_loss(inp["params"], inp["image"] - h * d)) / (2 * h)
    assert abs(fd - float(np.sum(adj[0] * d))) <= 2e-6


@pytest.mark.parametrize("mk", [mini_basic, mini_bottleneck, mini_basic_pre, mini_basic_flags])
def test_multiplier_equal_to_adjoint_reproduces_end_to_end(mk):
    """Consistent auxiliary variables, arbitrary rho, multiplier on each interface := end-to-end adjoint
    there: every module's weight gradients and dx equal end-to-end back-propagation."""
    net = mk()
    net.rho = 3.7
    inp = step_inputs(net, lpref, consistent=True)
    states, logits, caches = lpref.serial_forward(net, inp["image"], inp["params"])
    _, dps, adj = lpref.serial_backward(net, caches, logits, inp["labels"], need_dx0=True)
    xs = [inp["image"]] + states[1:]
    lams = [adj[k + 1] for k in range(net.K - 1)]
    out = lpref.local_step(net, xs, inp["params"], inp["labels"], lams, 1.0, need_dx0=True)
    for k in range(net.K):
        for a, b in zip(out["dparams"][k], dps[k]):
            assert rel_err(a, b) < 1e-12
        assert rel_err(out["dx"][k], adj[k]) < 1e-12
    # zero multipliers reproduce the penalty method bit for bit
    zero = [np.zeros_like(l) for l in lams]
    noisy = step_inputs(net, lpref)
    o1 = lpref.local_step(net, noisy["xs"], noisy["params"], noisy["labels"], zero, 1.0)
    o2 = lpref.local_step(net, noisy["xs"], noisy["params"], noisy["labels"], None, 1.0)
    for k in range(net.K):
        assert o1["loss"][k] == o2["loss"][k]
        for a, b in zip(o1["dparams"][k], o2["dparams"][k]):
            np.testing.assert_array_equal(a, b)


def test_module_zero_has_no_incoming_penalty_and_split_matches_serial():
    """Module k's forward from the serial state equals the serial network's next state (the split
    changes nothing when the constraints hold), and the local step never touches a multiplier for the
    last module."""
    net = mini_basic()
    inp = step_inputs(net, lpref, consistent=True)
    states, logits, _ = lpref.serial_forward(net, inp["image"], inp["params"])
    for k in range(net.K):
        y, lg, _ = lpref.module_forward(net.modules[k], states[k], inp["params"][k], net.bn_eps)
        if k < net.K - 1:
            np.testing.assert_array_equal(y, states[k + 1])
        else:
            np.testing.assert_array_equal(lg, logits)


def test_auxnet_forward_definition():
    net = wl.make_config("resnet56", batch=2)
    a = net.aux[3]                      # stride 2, 32 channels
    img = wl.make_image(net)
    p = wl.make_aux_params(net, 3)
    x = lpref.auxnet_forward(a, img, p, net.bn_eps)
    assert x.shape == (2, 16, 16, 32) == (net.modules[4].N, net.modules[4].H, net.modules[4].W, net.modules[4].C)
    y = lpref.conv_fwd(img, p[0], 2, 1)
    mu, var = y.mean(axis=(0, 1, 2)), y.var(axis=(0, 1, 2))
    np.testing.assert_allclose(x, p[1] * (y - mu) / np.sqrt(var + net.bn_eps) + p[2], rtol=1e-12, atol=1e-12)
    a.relu = True
    np.testing.assert_array_equal(lpref.auxnet_forward(a, img, p, net.bn_eps), np.maximum(x, 0.0))


def test_workload_descriptors():
    """Shapes of the five workloads (module inputs/outputs, block split, conv FLOPs per sample)."""
    from workloads import configs as cfg
    expect = {"tiny": ([1, 1], 0.0012), "resnet20": ([3, 2, 2, 2], 0.0816),
              "resnet56": ([4, 4, 4, 3, 3, 3, 3, 3], 0.2515), "wrn28_10": ([3, 3, 3, 3], 10.49),
              "resnet50": ([3, 4, 6, 3], 8.17)}
    for name, (split, gf) in expect.items():
        net = wl.make_config(name)
        assert [len(m.blocks) for m in net.modules] == split
        assert abs(cfg.conv_flops_forward(net) / net.modules[0].N / 1e9 - gf) < 0.006 * max(gf, 0.1) + 1e-4
        for k in range(net.K - 1):
            nx = net.modules[k + 1]
            assert net.modules[k].out_shape() == (nx.N, nx.H, nx.W, nx.C)
    w = wl.make_config("wrn28_10")
    assert [(m.H, m.C) for m in w.modules] == [(32, 3), (32, 160), (16, 320), (8, 640)]
    r = wl.make_config("resnet50")
    assert [(m.H, m.C) for m in r.modules] == [(224, 3), (56, 256), (28, 512), (14, 1024)]


def test_storage_rounding_hook():
    """q = identity reproduces the plain definition bit for bit; q = bf16 rounding stays close to it; the
    bf16 rounding itself is round-to-nearest-even on the 8-bit significand."""
    net = mini_basic()
    net.al, net.lam_sigma = True, 0.1
    inp = step_inputs(net, lpref)
    a = lpref.local_step(net, inp["xs"], inp["params"], inp["labels"], inp["lams"], 1.0)
    b = lpref.local_step(net, inp["xs"], inp["params"], inp["labels"], inp["lams"], 1.0, q=lambda t: t)
    c = lpref.local_step(net, inp["xs"], inp["params"], inp["labels"], inp["lams"], 1.0, q=wl.round_bf16)
    for k in range(net.K):
        for x, y, z in zip(a["dparams"][k], b["dparams"][k], c["dparams"][k]):
            np.testing.assert_array_equal(x, y)
            assert z.shape == x.shape and np.all(np.isfinite(z))
        assert a["loss"][k] == b["loss"][k]
    for k in range(net.K - 1):
        assert rel_err(c["y"][k], a["y"][k]) < 0.02
        np.testing.assert_array_equal(c["y"][k], wl.round_bf16(c["y"][k]))      # stored values are bf16 values
    v = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -7, -(1.0 + 2.0 ** -8 + 2.0 ** -20), 3.0e38, 0.0])
    want = np.array([1.0, 1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -(1.0 + 2.0 ** -7), 3.0e38, 0.0])
    got = wl.round_bf16(v)
    np.testing.assert_array_equal(got[:5], want[:5])
    assert got[6] == 0.0 and abs(got[5] - 3.0e38) <= 3.0e38 * 2.0 ** -8
    r = np.random.default_rng(0).standard_normal(10000) * 10
    assert np.max(np.abs(wl.round_bf16(r) - r) / np.abs(r)) <= 2.0 ** -8
    np.testing.assert_array_equal(wl.round_bf16(wl.round_bf16(r)), wl.round_bf16(r))


def test_aux_variable_update_is_a_gradient_step_of_the_relaxed_objective():
    """(x_k - x_k_new)/eta equals the central-difference gradient of the whole relaxed objective
    sum_k loss_k with respect to x_k (x_k appears in the terms of interface k-1 and of module k), and the two
    fixed-point cases: consistent variables with zero multipliers and zero dx do not move; the penalty-only
    step pulls x_k towards F_{k-1}(x_{k-1}) by the factor eta*scale*rho."""
    net = mini_basic()
    net.rho, net.al, net.lam_sigma = 1.7, True, 0.4
    inp = step_inputs(net, lpref)
    scale, eta, h = 0.6, 0.05, 1e-6
    rng = np.random.default_rng(3)
    out = lpref.local_step(net, inp["xs"], inp["params"], inp["labels"], inp["lams"], scale)

    def objective(xs):
        return sum(_local_loss(net, k, xs[k], inp["params"][k], xs[k + 1] if k < net.K - 1 else None,
                               inp["lams"][k] if k < net.K - 1 else None, inp["labels"], scale) for k in range(net.K))

    for k in range(1, net.K):
        new = lpref.aux_variable_update(inp["xs"][k], out["y"][k - 1], out["dx"][k], inp["lams"][k - 1], net.rho, eta, scale)
        grad = (inp["xs"][k] - new) / eta
        for _ in range(3):
            d = rng.standard_normal(inp["xs"][k].shape)
            xp, xm = list(inp["xs"]), list(inp["xs"])
            xp[k], xm[k] = inp["xs"][k] + h * d, inp["xs"][k] - h * d
            fd = (objective(xp) - objective(xm)) / (2 * h)
            an = float(np.sum(grad * d))
            assert abs(fd - an) <= 2e-6 * max(1.0, abs(an)), (k, fd, an)
    x = rng.standard_normal((2, 3, 3, 4))
    assert np.array_equal(lpref.aux_variable_update(x, x, np.zeros_like(x), np.zeros_like(x), 2.0, 0.1), x)
    y = rng.standard_normal(x.shape)
    got = lpref.aux_variable_update(x, y, np.zeros_like(x), None, 2.0, 0.1, 0.5)
    np.testing.assert_allclose(got - y, (1 - 0.1 * 0.5 * 2.0) * (x - y), rtol=1e-13)


@pytest.mark.parametrize("relu", [False, True])
def test_auxnet_distill_grad_finite_differences(relu):
    """loss = scale*|AuxNet(image) - target|^2 by its definition, and d loss / d(filter, gamma, beta) against central
    differences (directional and single coordinates); at target = AuxNet(image) loss and gradients vanish."""
    import copy
    net = wl.make_config("resnet56", batch=2)
    a = copy.copy(net.aux[3])           # stride 2, 3 -> 32 channels
    a.relu = relu
    img = wl.make_image(net)
    p = wl.make_aux_params(net, 3)
    out = lpref.auxnet_forward(a, img, p, net.bn_eps)
    target = out + wl.normal(5, "distill_target", out.shape, 0.3)
    scale, h = 0.25, 1e-6
    loss, grads = lpref.auxnet_distill_grad(a, img, p, target, net.bn_eps, scale)
    assert abs(loss - scale * np.sum((out - target) ** 2)) <= 1e-12 * abs(loss)
    f = lambda pp: scale * np.sum((lpref.auxnet_forward(a, img, pp, net.bn_eps) - target) ** 2)
    rng = np.random.default_rng(11)
    for i in range(3):
        assert grads[i].shape == p[i].shape
        d = rng.standard_normal(p[i].shape)
        pp, pm = list(p), list(p)
        pp[i], pm[i] = p[i] + h * d, p[i] - h * d
        fd = (f(pp) - f(pm)) / (2 * h)
        an = float(np.sum(grads[i] * d))
        assert abs(fd - an) <= 5e-6 * max(1.0, abs(an)), (i, fd, an)
        j = tuple(rng.integers(0, s) for s in p[i].shape)
        e = np.zeros_like(p[i]); e[j] = h
        pp[i], pm[i] = p[i] + e, p[i] - e
        fd = (f(pp) - f(pm)) / (2 * h)
        assert abs(fd - grads[i][j]) <= 5e-6 * max(1.0, abs(fd)), (i, j, fd, grads[i][j])
    loss0, g0 = lpref.auxnet_distill_grad(a, img, p, out, net.bn_eps, scale)
    assert loss0 == 0.0 and all(np.all(g == 0.0) for g in g0)


def test_chained_auxnet_distill_finite_differences():
    """A chained AuxNet block reads the previous auxiliary variable (here: 8 channels at 3x3) instead of the
    mini-batch; its distillation gradient against central differences, the input held fixed."""
    from workloads import configs as cfg
    net = cfg.chain_aux(mini_basic(), relu=True)
    a = net.aux[1]
    assert a.from_prev and a.cin == net.modules[1].C and a.stride == 1
    m = net.modules[1]
    x_in = wl.normal(9, "chain_in", (m.N, m.H, m.W, m.C))
    p = wl.make_aux_params(net, 1)
    out = lpref.auxnet_forward(a, x_in, p, net.bn_eps)
    target = out + wl.normal(9, "chain_target", out.shape, 0.3)
    scale, h = 0.5, 1e-6
    loss, grads = lpref.auxnet_distill_grad(a, x_in, p, target, net.bn_eps, scale)
    f = lambda pp: scale * np.sum((lpref.auxnet_forward(a, x_in, pp, net.bn_eps) - target) ** 2)
    assert abs(loss - f(p)) <= 1e-12 * abs(loss)
    rng = np.random.default_rng(13)
    for i in range(3):
        d = rng.standard_normal(p[i].shape)
        pp, pm = list(p), list(p)
        pp[i], pm[i] = p[i] + h * d, p[i] - h * d
        fd = (f(pp) - f(pm)) / (2 * h)
        an = float(np.sum(grads[i] * d))
        assert abs(fd - an) <= 5e-6 * max(1.0, abs(an)), (i, fd, an)


def _three_block_aux():
    """An AuxNet of three blocks from a 3-channel 8x8 mini-batch: 3 -> 4 (stride 2, ReLU) -> 8 (stride 1, ReLU) -> 8
    (stride 2, the AuxNet's own ReLU flag off)."""
    from workloads.configs import AuxDesc, NetDesc, aux_blocks, aux_tensor_specs
    a = AuxDesc(cin=3, cout=8, stride=2, relu=False, mid=((4, 2), (8, 1)))
    assert aux_blocks(a) == [(3, 4, 2, True), (4, 8, 1, True), (8, 8, 2, False)]
    assert [sp.shape for sp in aux_tensor_specs(a)][::3] == [(4, 3, 3, 3), (8, 3, 3, 4), (8, 3, 3, 8)]
    net = NetDesc(name="aux3", K=2, modules=[], aux=[a], dtype="f32", seed=21)
    return net, a, wl.normal(21, "aux3_image", (2, 8, 8, 3)), wl.make_aux_params(net, 0)


def test_deep_auxnet_against_library_layers():
    """A three-block AuxNet re-composed from a library's float64 layers: pins the order of the blocks, the stride of
    each, ReLU after the blocks in front of the last and none after the last, and which parameters each block uses."""
    import torch
    import torch.nn.functional as F
    net, a, img, p = _three_block_aux()
    t = lambda v: torch.from_numpy(np.ascontiguousarray(v, dtype=np.float64))
    h = t(img).permute(0, 3, 1, 2)
    for i, (stride, relu) in enumerate([(2, True), (1, True), (2, False)]):
        h = F.conv2d(h, t(p[3 * i]).permute(0, 3, 1, 2), stride=stride, padding=1)
        h = F.batch_norm(h, None, None, t(p[3 * i + 1]), t(p[3 * i + 2]), True, 0.0, net.bn_eps)
        h = F.relu(h) if relu else h
    got = lpref.auxnet_forward(a, img, p, net.bn_eps)
    assert got.shape == (2, 2, 2, 8) and np.any(got < 0)
    np.testing.assert_allclose(got, h.permute(0, 2, 3, 1).numpy(), rtol=1e-10, atol=1e-12)


def test_deep_auxnet_distill_finite_differences():
    """Distillation gradient of the three-block AuxNet with respect to all nine parameter tensors against central
    differences along random directions."""
    net, a, img, p = _three_block_aux()
    out = lpref.auxnet_forward(a, img, p, net.bn_eps)
    target = out + wl.normal(22, "aux3_target", out.shape, 0.4)
    scale, h = 0.3, 1e-6
    loss, grads = lpref.auxnet_distill_grad(a, img, p, target, net.bn_eps, scale)
    f = lambda pp: scale * np.sum((lpref.auxnet_forward(a, img, pp, net.bn_eps) - target) ** 2)
    assert abs(loss - f(p)) <= 1e-12 * abs(loss) and len(grads) == 9
    rng = np.random.default_rng(23)
    for i in range(9):
        assert grads[i].shape == p[i].shape
        d = rng.standard_normal(p[i].shape)
        pp, pm = list(p), list(p)
        pp[i], pm[i] = p[i] + h * d, p[i] - h * d
        fd = (f(pp) - f(pm)) / (2 * h)
        an = float(np.sum(grads[i] * d))
        assert abs(an) > 1e-6, i            # every block's parameters take part (BN's shift-invariance aside)
        assert abs(fd - an) <= 5e-6 * max(1.0, abs(an)), (i, fd, an)


@pytest.mark.parametrize("order", ["post", "pre", "post_flags"])
def test_module_forward_against_library_layers(order):
    """The forward pass of every module, re-composed from a library's float64 layers (conv2d, training-mode
    batch_norm, relu, adaptive average pool, linear) in NCHW: pins the sequencing of both block orders (where BN
    sits, what the projection reads, no ReLU after the sum, the head)."""
    import torch
    import torch.nn.functional as F
    net = {"pre": mini_basic_pre, "post": mini_basic, "post_flags": mini_basic_flags}[order]()
    inp = step_inputs(net, lpref)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64))
    act = lambda a: t(a).permute(0, 3, 1, 2)
    filt = lambda w: t(w).permute(0, 3, 1, 2)
    bn = lambda a, g, b: F.batch_norm(a, None, None, t(g), t(b), True, 0.0, net.bn_eps)
    for k, m in enumerate(net.modules):
        p = inp["params"][k]
        a = act(inp["xs"][k])
        i = 0
        if order == "pre":
            if m.stem:
                a = F.conv2d(a, filt(p[0]), padding=1); i = 1
            for b in m.blocks:
                o1 = F.relu(bn(a, p[i], p[i + 1]))
                y1 = F.conv2d(o1, filt(p[i + 2]), stride=b.stride, padding=1)
                o2 = F.relu(bn(y1, p[i + 3], p[i + 4]))
                z = F.conv2d(o2, filt(p[i + 5]), padding=1)
                skip = F.conv2d(o1, filt(p[i + 6]), stride=b.stride) if b.proj else a
                a = z + skip
                i += 7 if b.proj else 6
            feat = a
            if m.head:
                a = F.relu(bn(a, p[i], p[i + 1])); i += 2
        else:
            if m.stem:
                a = F.relu(bn(F.conv2d(a, filt(p[0]), padding=1), p[1], p[2])); i = 3
            for b in m.blocks:
                y = F.relu(bn(F.conv2d(a, filt(p[i]), stride=b.stride, padding=1), p[i + 1], p[i + 2]))
                z = bn(F.conv2d(y, filt(p[i + 3]), padding=1), p[i + 4], p[i + 5])
                if b.proj and b.proj_bn:
                    skip = bn(F.conv2d(a, filt(p[i + 6]), stride=b.stride), p[i + 7], p[i + 8])
                elif b.proj:
                    skip = F.conv2d(a, filt(p[i + 6]), stride=b.stride)          # bare projection
                else:
                    skip = a
                a = F.relu(z + skip) if b.post_relu else z + skip
                i += 6 + ((3 if b.proj_bn else 1) if b.proj else 0)
            feat = a
        y, logits, _ = lpref.module_forward(m, inp["xs"][k], p, net.bn_eps)
        np.testing.assert_allclose(y, feat.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-11)
        if m.head:
            want = F.linear(F.adaptive_avg_pool2d(a, 1).flatten(1), t(p[i]), t(p[i + 1]))
            np.testing.assert_allclose(logits, want.numpy(), rtol=0, atol=1e-11)
        assert i + (2 if m.head else 0) == len(p)


@pytest.mark.parametrize("al,relu,stack", [(True, False, False), (False, True, False), (True, True, True), (False, False, True)])
def test_reauxnet_grad_finite_differences(al, relu, stack):
    """With x_k = AuxNet(image; xi) substituted, the relaxed objective depends on xi through the interface term k-1
    and through the local loss of module k.  reauxnet_grad (fed with the oracle's dx_k at that x_k) must equal the
    central-difference gradient of that composite, for the middle module (interface loss below it) and for the
    last one (cross-entropy below it).  stack: x_k comes from k blocks of its own (the recursion of Sec. 4.4 at its
    full depth), else from one block."""
    from workloads import configs as cfg
    from workloads.configs import AuxDesc
    net = mini_basic()
    net.rho, net.al, net.lam_sigma = 1.4, al, 0.3
    if stack:
        cfg.reaux(net, relu)
        assert [len(a.mid) for a in net.aux] == [0, 1] and net.aux[1].mid == ((8, 2),) and net.aux[1].stride == 1
    else:
        net.aux = [AuxDesc(cin=3, cout=m.C, stride=net.modules[0].H // m.H, relu=relu) for m in net.modules[1:]]
    inp = step_inputs(net, lpref)
    scale, h = 0.7, 1e-6
    rng = np.random.default_rng(17)
    for k in range(1, net.K):          # the exact AuxNet outputs (the shared recipe rounds them to the storage type)
        inp["xs"][k] = lpref.auxnet_forward(net.aux[k - 1], inp["image"], inp["aux_params"][k - 1], net.bn_eps)
    out = lpref.local_step(net, inp["xs"], inp["params"], inp["labels"], inp["lams"], scale)
    for k in range(1, net.K):
        a, theta = net.aux[k - 1], inp["aux_params"][k - 1]
        lam_prev = inp["lams"][k - 1] if al else None
        grads = lpref.reauxnet_grad(a, inp["image"], theta, out["y"][k - 1], out["dx"][k], lam_prev, net.rho, scale, net.bn_eps)

        def objective(th):
            x = lpref.auxnet_forward(a, inp["image"], th, net.bn_eps)
            below = lpref.local_loss_grad(out["y"][k - 1], x, lam_prev, net.rho, scale)[0]
            return below + _local_loss(net, k, x, inp["params"][k], inp["xs"][k + 1] if k < net.K - 1 else None,
                                       inp["lams"][k] if (al and k < net.K - 1) else None, inp["labels"], scale)

        assert len(grads) == len(theta) == 3 * (len(a.mid) + 1)
        for i in range(len(theta)):
            assert grads[i].shape == theta[i].shape
            d = rng.standard_normal(theta[i].shape)
            tp, tm = list(theta), list(theta)
            tp[i], tm[i] = theta[i] + h * d, theta[i] - h * d
            fd = (objective(tp) - objective(tm)) / (2 * h)
            an = float(np.sum(grads[i] * d))
            assert abs(fd - an) <= 5e-6 * max(1.0, abs(an)), (k, i, fd, an)


def test_sgd_update_closed_forms():
    """Plain descent on f = 1/2 |W|^2 (gradient W) contracts by (1 - lr) per step; weight decay on a zero gradient
    contracts by (1 - lr*wd); momentum on a constant gradient accumulates the geometric series; and a small enough
    step on the mini network's local loss decreases it (descent direction)."""
    rng = np.random.default_rng(5)
    w = rng.standard_normal((3, 4))
    a = w
    for _ in range(5):
        a, v = lpref.sgd_update(a, a, 0.1)
        assert v is None
    np.testing.assert_allclose(a, w * 0.9 ** 5, rtol=1e-14)
    b, _ = lpref.sgd_update(w, np.zeros_like(w), 0.1, weight_decay=0.5)
    np.testing.assert_allclose(b, w * (1 - 0.05), rtol=1e-14)
    g = rng.standard_normal(w.shape)
    c, v = w, None
    for n in range(1, 5):
        c, v = lpref.sgd_update(c, g, 0.2, v, momentum=0.5)
        np.testing.assert_allclose(v, g * (1 - 0.5 ** n) / (1 - 0.5), rtol=1e-14)
    np.testing.assert_allclose(c, w - 0.2 * g * sum((1 - 0.5 ** n) / 0.5 for n in range(1, 5)), rtol=1e-13)
    net = mini_basic()
    inp = step_inputs(net, lpref)
    out = lpref.local_step(net, inp["xs"], inp["params"], inp["labels"], None, 1.0)
    k = net.K - 1
    before = _local_loss(net, k, inp["xs"][k], inp["params"][k], None, None, inp["labels"], 1.0)
    stepped = [lpref.sgd_update(p, g, 1e-3)[0] for p, g in zip(inp["params"][k], out["dparams"][k])]
    after = _local_loss(net, k, inp["xs"][k], stepped, None, None, inp["labels"], 1.0)
    gn2 = sum(float(np.sum(g * g)) for g in out["dparams"][k])
    assert after < before and abs((before - after) - 1e-3 * gn2) <= 0.05 * 1e-3 * gn2


@pytest.mark.parametrize("order", ["post", "pre", "post_flags"])
def test_storage_rounding_placement(order):
    """Where the diagnostic storage-rounding mode rounds (`q` of the composing routines).  The mode is defined as:
    every STORED tensor is rounded once -- convolution results, activations, block outputs going forward; the gradient
    of each of those tensors going backward, the data-gradient of a projection branch before it is added -- and
    batch statistics are those of the stored tensor.  Here that definition is built a second time from a library's
    float64 layers and its reverse-mode differentiation: a `store` node rounds the value in the forward direction and
    the gradient in the backward direction, and one is placed on every stored tensor.  With a coarse rounding grid
    (2^-5) a rounding that the oracle puts anywhere else (or leaves out) moves results by 1e-2; agreement is 1e-9."""
    import torch
    import torch.nn.functional as F
    grid = 32.0
    q = lambda a: np.round(np.asarray(a, dtype=np.float64) * grid) / grid
    tq = lambda a: torch.round(a * grid) / grid

    class Store(torch.autograd.Function):          # value and gradient are both stored (rounded)
        @staticmethod
        def forward(ctx, a):
            return tq(a)

        @staticmethod
        def backward(ctx, g):
            return tq(g)

    class StoreGrad(torch.autograd.Function):      # only the gradient is stored (a branch reading an already stored tensor)
        @staticmethod
        def forward(ctx, a):
            return a.clone()

        @staticmethod
        def backward(ctx, g):
            return tq(g)

    store, store_grad = Store.apply, StoreGrad.apply
    net = {"pre": mini_basic_pre, "post": mini_basic, "post_flags": mini_basic_flags}[order]()
    net.al, net.lam_sigma = True, 0.1
    inp = step_inputs(net, lpref)
    xs = [q(x) for x in inp["xs"]]
    lams = [q(l) for l in inp["lams"]]
    want = lpref.local_step(net, xs, inp["params"], inp["labels"], lams, 1.0, need_dx0=False, q=q)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64))
    filt = lambda w: w.permute(0, 3, 1, 2)
    bn = lambda a, g, b: F.batch_norm(a, None, None, g, b, True, 0.0, net.bn_eps)
    for k, m in enumerate(net.modules):
        p = [t(a).requires_grad_(True) for a in inp["params"][k]]
        x = t(xs[k]).requires_grad_(True)
        a = store(x.permute(0, 3, 1, 2))           # x_k is a stored tensor: its gradient dx_k is stored
        i = 0
        if order == "pre":
            if m.stem:
                a = store(F.conv2d(a, filt(p[0]), padding=1)); i = 1
            for b in m.blocks:
                o1 = store(F.relu(bn(a, p[i], p[i + 1])))
                y1 = store(F.conv2d(o1, filt(p[i + 2]), stride=b.stride, padding=1))
                o2 = store(F.relu(bn(y1, p[i + 3], p[i + 4])))
                z = F.conv2d(o2, filt(p[i + 5]), padding=1)
                skip = store(F.conv2d(store_grad(o1), filt(p[i + 6]), stride=b.stride)) if b.proj else a
                a = store(z + skip)
                i += 7 if b.proj else 6
            feat = a
            if m.head:
                a = store(F.relu(bn(a, p[i], p[i + 1]))); i += 2
        else:
            if m.stem:
                a = store(F.relu(bn(store(F.conv2d(a, filt(p[0]), padding=1)), p[1], p[2]))); i = 3
            for b in m.blocks:
                y = store(F.relu(bn(store(F.conv2d(a, filt(p[i]), stride=b.stride, padding=1)), p[i + 1], p[i + 2])))
                z = bn(store(F.conv2d(y, filt(p[i + 3]), padding=1)), p[i + 4], p[i + 5])
                if b.proj and b.proj_bn:
                    skip = bn(store(F.conv2d(store_grad(a), filt(p[i + 6]), stride=b.stride)), p[i + 7], p[i + 8])
                elif b.proj:
                    skip = store(F.conv2d(store_grad(a), filt(p[i + 6]), stride=b.stride))
                else:
                    skip = a
                a = store(F.relu(z + skip) if b.post_relu else z + skip)
                i += 6 + ((3 if b.proj_bn else 1) if b.proj else 0)
            feat = a
        if m.head:
            logits = F.linear(F.adaptive_avg_pool2d(a, 1).flatten(1), p[i], p[i + 1])
            np.testing.assert_allclose(want["logits"], logits.detach().numpy(), rtol=0, atol=1e-9)
            logits.backward(t(want["dlogits"]))
        else:
            y_out = feat.permute(0, 2, 3, 1)
            np.testing.assert_allclose(want["y"][k], y_out.detach().numpy(), rtol=0, atol=1e-9)
            y_out.backward(t(want["dy"][k]))        # the stored terminal adjoint of the oracle's own run
        for j, (g, w) in enumerate(zip(p, want["dparams"][k])):
            np.testing.assert_allclose(w, g.grad.numpy(), rtol=0, atol=1e-9 * max(1.0, float(np.max(np.abs(w)))),
                                       err_msg=f"module {k} tensor {j}")
        if want["dx"][k] is not None:
            np.testing.assert_allclose(want["dx"][k], x.grad.numpy(), rtol=0, atol=1e-9)
