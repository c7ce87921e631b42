"""Backward (and forward) parity unit by unit at a fixed tolerance: see tests/gpu_unitwise.py for what is compared.

Cases: small networks that cover every kernel family (general fp32 / bf16 kernels, 7x7 stem with max-pool, bottleneck
blocks, stride-2 projections, ragged wide layers), then the configurations at their full sizes in the launch
configuration the benchmark times: ResNet-20 (fp32, batch 128), ResNet-56 (bf16, K = 8, batch 128), WideResNet-28-10
(bf16, batch 128: every one of its 25 conv+BN units, wide kernels at their full-size tiles) and the ImageNet-shaped
ResNet-50 (bf16, 224 x 224, batch 64)."""
import pytest

import workloads as wl
from tests.gpu_common import gpu_mini_basic, gpu_mini_basic_flags, gpu_mini_bottleneck, gpu_mini_wide, gpu_mini_wide_strided
from tests.gpu_unitwise import check_units

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_units_mini_basic(dtype):
    check_units(gpu_mini_basic(batch=3, dtype=dtype))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_units_mini_bottleneck(dtype):
    check_units(gpu_mini_bottleneck(batch=2, dtype=dtype))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_units_block_options(dtype):
    """ReLU behind the residual sum and a bare conv1x1 projection (the two options of the conv-BN-ReLU order)."""
    check_units(gpu_mini_basic_flags(batch=3, dtype=dtype))


def test_units_mini_wide():
    check_units(gpu_mini_wide(batch=3))
    check_units(gpu_mini_wide_strided(batch=5))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_units_edge_cases(dtype):
    """Degenerate sizes and coefficients: a mini-batch of ONE sample (batch statistics over 36 and 9 pixels, every tile
    ragged), images of 2 x 2 pixels (every 3x3 window hangs over the border on all sides; the stride-2 block leaves 1 x 1),
    rho = 0 with multipliers (the loss is the multiplier term alone) and a loss scale other than 1."""
    from workloads import configs as cfg
    from workloads.configs import Block
    check_units(gpu_mini_basic(batch=1, dtype=dtype), note=" [batch 1]")
    blocks = [Block("basic", 8, 8, 8, 1, False), Block("basic", 8, 16, 16, 2, True), Block("basic", 16, 16, 16, 1, False)]
    net = cfg._assemble("gpu_edge_2x2", [blocks[:1], blocks[1:]], 5, 2, 2, 3, 1, 8, 4, seed=31)
    net.dtype = dtype
    check_units(net, note=" [2 x 2 images]")
    net = gpu_mini_basic(batch=3, dtype=dtype)
    net.al, net.rho, net.lam_sigma = True, 0.0, 0.5
    check_units(net, note=" [rho = 0, multipliers]", scale=0.37)


def test_units_separate_calls():
    check_units(gpu_mini_basic(batch=3, dtype="bf16"), fused=False)


def test_units_wrn28_10_batch_8():
    check_units(wl.make_config("wrn28_10", batch=8))


def test_units_resnet20_full_size():
    check_units(wl.make_config("resnet20"))


def test_units_resnet56_full_size():
    check_units(wl.make_config("resnet56"))


def test_units_wrn28_10_full_size():
    check_units(wl.make_config("wrn28_10"))


def test_units_resnet50_full_size():
    check_units(wl.make_config("resnet50"))
