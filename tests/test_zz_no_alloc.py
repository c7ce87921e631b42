"""The entry point that allocates nothing: lp_auxnet_forward_static keeps the intermediates of the AuxNet forward
passes in a device array that is part of the library, instead of the caller's workspace.  Its x_out must equal
lp_auxnet_forward's (same kernels; the per-channel statistics are summed with atomics, so equality is up to the
order of a handful of fp64 additions: checked against the storage type's tolerance and printed), on two calls in a row,
the second with a smaller input that shares the array with what the first call left there."""
import numpy as np
import pytest

import workloads as wl
from tests.gpu_common import say
from tests.helpers import rel_err
from workloads import configs as cfg

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def _both_ways(net):
    import torch
    from paper_2112_05387_amd import LocalStep
    from paper_2112_05387_amd import binding as B
    ls = LocalStep(net)
    try:
        ls.set_x(0, wl.make_image(net))
        for j in range(net.K - 1):
            ls.set_aux_params(j, wl.make_aux_params(net, j))
        ls.auxnet_forward()
        torch.cuda.synchronize()
        want = [ls.to_host(t) for t in ls.x[1:]]
        for t in ls.x[1:]:
            t.fill_(float("nan"))
        B.lp_auxnet_forward_static(ls.net, torch.cuda.current_stream().cuda_stream, ls.x[0].data_ptr(),
                                   ls._p(ls.aux_params), ls._p(ls.x[1:]))
        torch.cuda.synchronize()
        got = [ls.to_host(t) for t in ls.x[1:]]
    finally:
        ls.close()
    errs = {f"x{j + 1}": rel_err(g, w) for j, (g, w) in enumerate(zip(got, want))}
    exact = sum(int(np.array_equal(g, w)) for g, w in zip(got, want))
    say(f"static AuxNet forward, {net.name} N={net.modules[0].N} {net.dtype}: worst {max(errs.values()):.2e}, "
        f"{exact} of {len(want)} tensors bit-identical")
    for g in got:
        assert np.all(np.isfinite(g))
    bad = {k: v for k, v in errs.items() if not v <= TOL[net.dtype]}
    assert not bad, bad
    return errs


def test_static_auxnet_forward_two_calls_in_a_row():
    big = cfg.deepen_aux(wl.make_config("resnet56", batch=32), 2)          # K = 8, stacks of three blocks, bf16
    small = wl.make_config("resnet56", batch=4)                            # one block per AuxNet, a smaller input
    small.dtype = "f32"
    _both_ways(big)
    _both_ways(small)
    _both_ways(cfg.chain_aux(wl.make_config("resnet56", batch=8)))         # chained AuxNets run one after the other
