"""Host-side checks of the C ABI: exported symbols, descriptor validation, packed layouts, error paths.
No kernel is launched here (no GPU needed)."""
import ctypes
import os
import re
import subprocess
import sys

import pytest

import workloads as wl
from paper_2112_05387_amd import binding as B
from workloads.configs import Block, ModuleDesc, AuxDesc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_PTR = 0x10000000      # aligned, never dereferenced: every check below fails or returns before a launch


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "lp.h")).read()
    declared = set(re.findall(r"\b(lp_[a-z0-9_]+)\s*\(", hdr))
    assert {"lp_module_forward", "lp_local_loss_grad", "lp_module_backward", "lp_auxnet_forward",
            "lp_al_multiplier_update", "lp_aux_variable_update", "lp_auxnet_distill_grad", "lp_sgd_update", "lp_reauxnet_grad", "lp_net_set_stream_lanes", "lp_local_step"} <= declared
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), f"{name} declared in lp.h but not exported"
    assert set(B.EXPORTS) == declared
    assert B.lp_version().startswith("lp-gfx950")


def test_binding_refuses_missing_library(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/liblp.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        B.lib()


@pytest.mark.parametrize("name", wl.CONFIG_NAMES)
def test_tensor_table_matches_workload_specs(name):
    net = wl.make_config(name)
    h = B.lp_net_create(net.modules, net.aux, net.dtype, net.bn_eps)
    try:
        kinds = {"conv": B.LP_T_CONV, "bn_gamma": B.LP_T_BN_GAMMA, "bn_beta": B.LP_T_BN_BETA, "fc_w": B.LP_T_FC_W, "fc_b": B.LP_T_FC_B}
        for k, m in enumerate(net.modules):
            specs = wl.module_tensor_specs(m)
            assert B.lp_net_num_tensors(h, 0, k) == len(specs)
            pb, gb = B.lp_net_param_bytes(h, 0, k)
            prev_end = prev_gend = 0
            for i, sp in enumerate(specs):
                t = B.lp_net_tensor_info(h, 0, k, i)
                assert t.kind == kinds[sp.kind] and t.block == sp.block and t.slot == sp.slot
                assert tuple(t.dims[j] for j in range(t.ndim)) == tuple(sp.shape)
                want_dt = B.LP_BF16 if (sp.kind == "conv" and net.dtype == "bf16") else B.LP_F32
                assert t.dtype == want_dt
                assert t.offset % 256 == 0 and t.grad_offset % 256 == 0
                assert t.offset >= prev_end and t.grad_offset >= prev_gend
                prev_end = t.offset + t.numel * (2 if t.dtype == B.LP_BF16 else 4)
                prev_gend = t.grad_offset + t.numel * 4
            assert prev_end <= pb and prev_gend <= gb
        if net.aux is not None:
            for j, a in enumerate(net.aux):
                assert B.lp_net_num_tensors(h, 1, j) == 3
                t = B.lp_net_tensor_info(h, 1, j, 0)
                assert tuple(t.dims[i] for i in range(4)) == (a.cout, 3, 3, a.cin)
        assert B.lp_net_workspace_bytes(h) > 0
    finally:
        B.lp_net_destroy(h)


@pytest.mark.parametrize("form", ["reaux", "deep", "chained_deep"])
def test_aux_stack_tensor_table(form):
    """AuxNets of several blocks: the parameter table lists filter, gamma, beta of every block in order, slot = index
    of the block, and matches the shared tensor specs."""
    from workloads import configs as cfg
    net = wl.make_config("resnet56")
    ws0 = None
    h = B.lp_net_create(net.modules, net.aux, net.dtype, net.bn_eps)
    try:
        ws0 = B.lp_net_workspace_bytes(h)
    finally:
        B.lp_net_destroy(h)
    if form == "reaux":
        cfg.reaux(net)
        assert [len(a.mid) for a in net.aux] == list(range(net.K - 1))
        assert cfg.aux_blocks(net.aux[2]) == [(3, 16, 1, True), (16, 16, 1, True), (16, 32, 2, False)]
    elif form == "deep":
        cfg.deepen_aux(net, 2)
    else:
        cfg.deepen_aux(cfg.chain_aux(net), 1)
    kinds = {"conv": B.LP_T_CONV, "bn_gamma": B.LP_T_BN_GAMMA, "bn_beta": B.LP_T_BN_BETA}
    h = B.lp_net_create(net.modules, net.aux, net.dtype, net.bn_eps)
    try:
        for j, a in enumerate(net.aux):
            specs = wl.aux_tensor_specs(a)
            assert len(specs) == 3 * (len(a.mid) + 1) and B.lp_net_num_tensors(h, 1, j) == len(specs)
            pb, gb = B.lp_net_param_bytes(h, 1, j)
            end = gend = 0
            for i, sp in enumerate(specs):
                t = B.lp_net_tensor_info(h, 1, j, i)
                assert t.kind == kinds[sp.kind] and t.block == -1 and t.slot == sp.slot == i // 3
                assert tuple(t.dims[d] for d in range(t.ndim)) == tuple(sp.shape)
                assert t.offset % 256 == 0 and t.offset >= end and t.grad_offset >= gend
                end = t.offset + t.numel * (2 if t.dtype == B.LP_BF16 else 4)
                gend = t.grad_offset + t.numel * 4
            assert end <= pb and gend <= gb
        assert B.lp_net_workspace_bytes(h) > ws0
    finally:
        B.lp_net_destroy(h)


def _mod(blocks, N=2, H=8, W=8, C=8, stem=0, stem_cout=0, head=True, n_classes=4):
    return ModuleDesc(stem=stem, stem_cout=stem_cout, blocks=blocks, head=head, n_classes=n_classes, N=N, H=H, W=W, C=C)


def _expect(status, fn, *a):
    with pytest.raises(B.LpError) as e:
        fn(*a)
    assert e.value.status == status, str(e.value)
    assert B.lp_last_error() != ""


def test_create_rejects_bad_descriptors():
    ok = Block("basic", 8, 8, 8, 1, False)
    _expect(B.LP_ERR_INVALID_ARG, B.lp_net_create, [], None, "f32", 1e-5)                      # K = 0
    _expect(B.LP_ERR_DTYPE, B.lp_net_create, [_mod([ok])], None, 7, 1e-5)
    _expect(B.LP_ERR_INVALID_ARG, B.lp_net_create, [_mod([ok])], None, "f32", 0.0)              # eps
    _expect(B.LP_ERR_INVALID_ARG, B.lp_net_create, [_mod([])], None, "f32", 1e-5)               # no blocks
    _expect(B.LP_ERR_SHAPE, B.lp_net_create, [_mod([Block("basic", 16, 16, 16, 1, False)])], None, "f32", 1e-5)   # cin != C
    _expect(B.LP_ERR_SHAPE, B.lp_net_create, [_mod([Block("basic", 8, 16, 16, 1, False)])], None, "f32", 1e-5)    # proj missing
    _expect(B.LP_ERR_SHAPE, B.lp_net_create, [_mod([Block("basic", 8, 8, 8, 2, False)])], None, "f32", 1e-5)      # stride w/o proj
    _expect(B.LP_ERR_SHAPE, B.lp_net_create, [_mod([Block("basic", 8, 8, 8, 3, True)])], None, "f32", 1e-5)       # stride 3
    _expect(B.LP_ERR_SHAPE, B.lp_net_create, [_mod([Block("basic", 8, 8, 8, 2, True)], H=7)], None, "f32", 1e-5)  # H % stride
    _expect(B.LP_ERR_SHAPE, B.lp_net_create, [_mod([Block("basic", 8, 12, 12, 1, True)])], None, "bf16", 1e-5)    # 12 % 8
    _expect(B.LP_ERR_SHAPE, B.lp_net_create, [_mod([ok], head=False)], None, "f32", 1e-5)       # last module needs the head
    _expect(B.LP_ERR_SHAPE, B.lp_net_create, [_mod([ok]), _mod([ok])], None, "f32", 1e-5)       # head on a non-last module
    _expect(B.LP_ERR_SHAPE, B.lp_net_create, [_mod([ok], head=False), _mod([Block("basic", 16, 16, 16, 1, False)], C=16)],
            None, "f32", 1e-5)                                                                     # interface mismatch
    _expect(B.LP_ERR_INVALID_ARG, B.lp_net_create, [_mod([Block(5, 8, 8, 8, 1, False)])], None, "f32", 1e-5)     # kind
    _expect(B.LP_ERR_INVALID_ARG, B.lp_net_create, [_mod([ok], stem=3)], None, "f32", 1e-5)
    two = [_mod([ok], head=False), _mod([ok])]
    _expect(B.LP_ERR_SHAPE, B.lp_net_create, two, [AuxDesc(3, 8, 1, False)], "f32", 1e-5)       # aux cin != image channels
    _expect(B.LP_ERR_SHAPE, B.lp_net_create, two, [AuxDesc(8, 16, 1, False)], "f32", 1e-5)      # aux cout
    _expect(B.LP_ERR_SHAPE, B.lp_net_create, two, [AuxDesc(8, 8, 2, False)], "f32", 1e-5)       # aux stride
    _expect(B.LP_ERR_SHAPE, B.lp_net_create, two, [AuxDesc(8, 8, 1, False, mid=((6, 1),))], "f32", 1e-5)   # width of a block in front: 6 % 4
    _expect(B.LP_ERR_SHAPE, B.lp_net_create, two, [AuxDesc(8, 8, 1, False, mid=((8, 2),))], "f32", 1e-5)   # strides do not multiply to 1
    _expect(B.LP_ERR_SHAPE, B.lp_net_create, two, [AuxDesc(8, 8, 1, False, mid=((8, 3),))], "f32", 1e-5)   # 8 % 3
    with pytest.raises(ValueError):
        B.lp_net_create(two, [AuxDesc(8, 8, 1, False, mid=((8, 1),) * 8)], "f32", 1e-5)                    # nine blocks
    h = B.lp_net_create(two, [AuxDesc(8, 8, 1, False, mid=((16, 1), (8, 1)))], "f32", 1e-5)
    B.lp_net_destroy(h)
    h = B.lp_net_create(two, [AuxDesc(8, 8, 1, True)], "f32", 1e-5)
    B.lp_net_destroy(h)


def test_call_time_errors_without_touching_the_gpu():
    net = wl.make_config("tiny")
    h = B.lp_net_create(net.modules, None, "f32", 1e-5)
    try:
        K = net.K
        ptrs = [FAKE_PTR] * K
        _expect(B.LP_ERR_WORKSPACE, B.lp_module_forward, h, None, 3, ptrs, ptrs, ptrs[:1], FAKE_PTR)     # no workspace yet
        need = B.lp_net_workspace_bytes(h)
        _expect(B.LP_ERR_WORKSPACE, B.lp_net_set_workspace, h, FAKE_PTR, need - 1)
        _expect(B.LP_ERR_INVALID_ARG, B.lp_net_set_workspace, h, FAKE_PTR + 8, need)
        B.lp_net_set_workspace(h, FAKE_PTR, need)
        _expect(B.LP_ERR_INVALID_ARG, B.lp_module_forward, h, None, 0, ptrs, ptrs, ptrs[:1], FAKE_PTR)   # empty mask
        _expect(B.LP_ERR_INVALID_ARG, B.lp_module_forward, h, None, 1 << K, ptrs, ptrs, ptrs[:1], FAKE_PTR)
        _expect(B.LP_ERR_INVALID_ARG, B.lp_module_forward, h, None, 3, [None, FAKE_PTR], ptrs, ptrs[:1], FAKE_PTR)
        _expect(B.LP_ERR_INVALID_ARG, B.lp_module_forward, h, None, 3, [FAKE_PTR + 4, FAKE_PTR], ptrs, ptrs[:1], FAKE_PTR)
        _expect(B.LP_ERR_INVALID_ARG, B.lp_module_forward, h, None, 3, ptrs, ptrs, ptrs[:1], None)       # logits
        _expect(B.LP_ERR_INVALID_ARG, B.lp_module_forward, h, None, 1, ptrs, ptrs, [None], FAKE_PTR)     # y[0]
        _expect(B.LP_ERR_STATE, B.lp_module_backward, h, None, 3, ptrs[:1], FAKE_PTR, ptrs, ptrs, ptrs)  # no forward
        _expect(B.LP_ERR_INVALID_ARG, B.lp_local_loss_grad, h, None, 3, ptrs[:1], ptrs[:1], None, -1.0, 1.0, FAKE_PTR,
                FAKE_PTR, FAKE_PTR, ptrs[:1], FAKE_PTR)                                                   # rho < 0
        _expect(B.LP_ERR_INVALID_ARG, B.lp_local_loss_grad, h, None, 3, ptrs[:1], ptrs[:1], None, 1.0, 1.0, FAKE_PTR,
                FAKE_PTR, None, ptrs[:1], FAKE_PTR)                                                       # loss NULL
        _expect(B.LP_ERR_INVALID_ARG, B.lp_local_loss_grad, h, None, 2, ptrs[:1], ptrs[:1], None, 1.0, 1.0, None,
                FAKE_PTR, FAKE_PTR, ptrs[:1], FAKE_PTR)                                                   # logits NULL
        _expect(B.LP_ERR_STATE, B.lp_auxnet_forward, h, None, FAKE_PTR, ptrs[:1], ptrs[:1])              # net has no AuxNet
        _expect(B.LP_ERR_INVALID_ARG, B.lp_al_multiplier_update, h, None, None, ptrs[:1], ptrs[:1], 0.1)
        _expect(B.LP_ERR_STATE, B.lp_auxnet_distill_grad, h, None, FAKE_PTR, ptrs[:1], ptrs[:1], 1.0, FAKE_PTR, ptrs[:1])   # no AuxNet
        _expect(B.LP_ERR_INVALID_ARG, B.lp_aux_variable_update, h, None, None, ptrs[:1], ptrs, None, 1.0, 1.0, 0.1)   # x NULL
        _expect(B.LP_ERR_INVALID_ARG, B.lp_aux_variable_update, h, None, ptrs, ptrs[:1], [FAKE_PTR, None], None, 1.0, 1.0, 0.1)   # dx[1]
        _expect(B.LP_ERR_INVALID_ARG, B.lp_aux_variable_update, h, None, [None, FAKE_PTR + 2], ptrs[:1], ptrs, None, 1.0, 1.0, 0.1)   # alignment
        _expect(B.LP_ERR_STATE, B.lp_reauxnet_grad, h, None, FAKE_PTR, ptrs[:1], ptrs[:1], ptrs, None, 1.0, 1.0, ptrs[:1])   # no AuxNet
        _expect(B.LP_ERR_INVALID_ARG, B.lp_sgd_update, h, None, 0, 1, None, ptrs, None, None, 0.1, 0.0, 0.0)            # params NULL
        _expect(B.LP_ERR_INVALID_ARG, B.lp_sgd_update, h, None, 0, 1, ptrs, ptrs, None, None, 0.1, 0.9, 0.0)            # momentum, no velocity
        _expect(B.LP_ERR_INVALID_ARG, B.lp_sgd_update, h, None, 0, 0, ptrs, ptrs, None, None, 0.1, 0.0, 0.0)            # empty mask
        _expect(B.LP_ERR_INVALID_ARG, B.lp_sgd_update, h, None, 0, 1, [FAKE_PTR + 4, None], ptrs, None, None, 0.1, 0.0, 0.0)   # alignment
        _expect(B.LP_ERR_STATE, B.lp_sgd_update, h, None, 1, 1, ptrs, ptrs, None, None, 0.1, 0.0, 0.0)                  # no AuxNet
        _expect(B.LP_ERR_INVALID_ARG, B.lp_net_set_stream_lanes, h, [0, 7])
        _expect(B.LP_ERR_INVALID_ARG, B.lp_net_set_fused_update, h, 1, 0.1, 0.9, 0.0, None, None)          # momentum, no velocity
        _expect(B.LP_ERR_INVALID_ARG, B.lp_net_set_fused_update, h, 1, 0.1, 0.9, 0.0, [FAKE_PTR, None], None)   # velocity[1]
        _expect(B.LP_ERR_INVALID_ARG, B.lp_net_set_fused_update, h, 1, 0.1, 0.0, 0.0, None, [FAKE_PTR + 4, None])   # alignment
        B.lp_net_set_fused_update(h, 1, 0.1, 0.9, 5e-4, ptrs, [FAKE_PTR, None])
        B.lp_net_set_fused_update(h, 0)
        _expect(B.LP_ERR_INVALID_ARG, B.lp_local_step, h, None, 3, ptrs, ptrs, ptrs[:1], ptrs[:1], None, 1.0, 1.0, 0.0, None,
                FAKE_PTR, ptrs[:1], FAKE_PTR, FAKE_PTR, ptrs, ptrs)                                               # labels NULL
        _expect(B.LP_ERR_INVALID_ARG, B.lp_local_step, h, None, 0, ptrs, ptrs, ptrs[:1], ptrs[:1], None, 1.0, 1.0, 0.0, FAKE_PTR,
                FAKE_PTR, ptrs[:1], FAKE_PTR, FAKE_PTR, ptrs, ptrs)                                               # empty mask
        _expect(B.LP_ERR_INVALID_ARG, B.lp_local_step, h, None, 3, ptrs, ptrs, ptrs[:1], ptrs[:1], None, -1.0, 1.0, 0.0, FAKE_PTR,
                FAKE_PTR, ptrs[:1], FAKE_PTR, FAKE_PTR, ptrs, ptrs)                                               # rho < 0
        _expect(B.LP_ERR_INVALID_ARG, B.lp_net_tensor_info, h, 0, 0, 99)
        _expect(B.LP_ERR_INVALID_ARG, B.lp_net_param_bytes, h, 0, 5)
        _expect(B.LP_ERR_INVALID_ARG, B.lp_debug_saved_tensor, h, 0, 0)                                   # tiny has no stem
    finally:
        B.lp_net_destroy(h)


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


@pytest.mark.parametrize("kernel,bk,bn,nw,ncol,cin,r", [
    (0, 64, 320, 8, 296, 320, 3), (0, 64, 320, 4, 296, 64, 3), (0, 64, 160, 2, 136, 128, 3), (0, 32, 160, 8, 136, 160, 3),
    (0, 32, 320, 8, 520, 32, 1), (0, 64, 320, 8, 2048, 512, 1), (0, 32, 160, 4, 128, 96, 3), (1, 64, 320, 8, 296, 160, 3),
    (1, 64, 160, 8, 136, 136 - 8, 3), (1, 64, 320, 8, 640, 640, 3), (1, 64, 160, 8, 160, 160, 3)])
def test_filter_loads_stay_inside_the_filter_buffer(kernel, bk, bn, nw, ncol, cin, r):
    """Every direct-to-LDS filter load the wide-layer kernels form (their own address functions, enumerated on the
    host over column tiles, waves, lanes, rounds, taps and channel slabs) either is marked out of range or ends inside
    the filter tensor, ragged last column tile included (136 of 160, 296 = 160 + 136, 520 = 320 + 200 ...)."""
    end, live = B.lp_debug_filter_load_extent(kernel, bk, bn, nw, ncol, cin, r)
    size = ncol * r * r * cin * 2
    assert live > 0
    assert end <= size, f"a live load ends at byte {end} of a {size}-byte filter tensor"
    # every 16-byte chunk of the tensor is fetched exactly once per pass over it
    assert live * 16 == size


def test_unit_views_describe_every_conv_of_a_module():
    net = wl.make_config("wrn28_10", batch=4)
    B.lp_debug_keep_gradients(1)
    try:
        h = B.lp_net_create(net.modules, net.aux, net.dtype, net.bn_eps)
    finally:
        B.lp_debug_keep_gradients(0)
    try:
        for k, m in enumerate(net.modules):
            specs = wl.module_tensor_specs(m)
            n = B.lp_debug_unit_count(h, k)
            assert n == sum(1 for s in specs if s.kind == "conv")
            refs = set()
            for i in range(n):
                u = B.lp_debug_unit_info(h, k, i)
                assert specs[u.t_w].shape == (u.cout, u.R, u.R, u.cin)
                assert specs[u.t_gamma].kind == "bn_gamma" and specs[u.t_beta].kind == "bn_beta"
                assert u.y.space == B.LP_REF_WORKSPACE and u.dy.space == B.LP_REF_WORKSPACE
                for r in (u.y, u.dy, u.stats, u.red) + ((u.din,) if u.has_dgrad and u.din.space == B.LP_REF_WORKSPACE else ()):
                    assert (r.space, r.off) not in refs, "with kept gradients no buffer is shared between units"
                    refs.add((r.space, r.off))
                assert (u.skip_kind == 2) == (u.skip_unit >= 0)
            assert B.lp_debug_module_info(h, k).keep_gradients == 1
        with pytest.raises(B.LpError):
            B.lp_debug_unit_info(h, 0, 99)
    finally:
        B.lp_net_destroy(h)


def test_static_auxnet_forward_rejects_what_does_not_fit():
    """Size and argument checks of the entry point that allocates nothing come before any device call."""
    net = wl.make_config("wrn28_10", batch=128)
    m0 = net.modules[0]
    net.aux = [AuxDesc(cin=m0.C, cout=m.C, stride=m0.H // m.H, relu=False) for m in net.modules[1:]]
    h = B.lp_net_create(net.modules, net.aux, net.dtype, net.bn_eps)      # 40 + 20 + 10 MiB of pre-BN results alone
    try:
        _expect(B.LP_ERR_WORKSPACE, B.lp_auxnet_forward_static, h, None, FAKE_PTR, [FAKE_PTR] * 3, [FAKE_PTR] * 3)
        _expect(B.LP_ERR_INVALID_ARG, B.lp_auxnet_forward_static, h, None, None, [FAKE_PTR] * 3, [FAKE_PTR] * 3)
    finally:
        B.lp_net_destroy(h)
    net = wl.make_config("resnet20", batch=4)
    h = B.lp_net_create(net.modules, None, net.dtype, net.bn_eps)
    try:
        _expect(B.LP_ERR_STATE, B.lp_auxnet_forward_static, h, None, FAKE_PTR, [FAKE_PTR] * 3, [FAKE_PTR] * 3)
    finally:
        B.lp_net_destroy(h)


def test_block_options_tensor_table_and_refusals():
    from tests.helpers import mini_basic_flags, mini_basic_pre
    net = mini_basic_flags()
    for m in net.modules:                   # channel counts of the CPU-sized net are too small for the device: widen
        m.C = m.C * 2 if m.stem == 0 else m.C
        m.stem_cout *= 2
        for b in m.blocks:
            b.cin, b.cout, b.width = b.cin * 2, b.cout * 2, b.width * 2
    h = B.lp_net_create(net.modules, None, "f32", net.bn_eps)
    try:
        for k, m in enumerate(net.modules):
            specs = wl.module_tensor_specs(m)
            assert B.lp_net_num_tensors(h, 0, k) == len(specs)
            for i, sp in enumerate(specs):
                info = B.lp_net_tensor_info(h, 0, k, i)
                assert tuple(info.dims[j] for j in range(info.ndim)) == tuple(sp.shape), (k, sp.name)
        assert sum(1 for sp in wl.module_tensor_specs(net.modules[0]) if sp.name.startswith("block1.proj")) == 1
    finally:
        B.lp_net_destroy(h)
    pre = mini_basic_pre()
    for m in pre.modules:
        m.C = m.C * 2 if m.stem == 0 else m.C
        m.stem_cout *= 2
        for b in m.blocks:
            b.cin, b.cout, b.width = b.cin * 2, b.cout * 2, b.width * 2
    pre.modules[1].blocks[0].post_relu = True
    _expect(B.LP_ERR_SHAPE, B.lp_net_create, pre.modules, None, "f32", pre.bn_eps)
