"""Workload definitions shared by the CPU oracle's tests and the HIP path's tests.

Holds only (i) network *descriptors* of the synthetic workloads (shapes, block
lists, which module owns the stem and the head) and (ii) seeded, counter-based
input generators.  None of the method's arithmetic (convolution, batch-norm,
losses, gradients) lives here.
"""
from .configs import (Block, ModuleDesc, AuxDesc, NetDesc, TensorSpec, CONFIG_NAMES,
                      make_config, module_tensor_specs, aux_tensor_specs,
                      block_convs, module_conv_shapes, conv_flops_forward)
from .synth import (normal, uniform_int, round_bf16, f32_to_bf16_bits, bf16_bits_to_f32,
                    make_params, make_aux_params, make_image, make_labels, make_noise)
