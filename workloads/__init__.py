"""Seeded synthetic workloads: network blobs, input pools and arrival traces.

This package only *generates data* (random tensors, layer lists, time stamps).
It contains none of the arithmetic of the early-exit forward pass or of the
scheduler, so that both the CPU oracle and the GPU library can be fed from it
without sharing any code of the method itself.
"""
from .rng import splitmix64, uniform_bytes, uniform_u01, normal_f64  # noqa: F401
from .blob import (HEADER_DT, STAGE_DT, OP_DT, EXIT_DT, Blob, OP_CONV, OP_DWCONV,  # noqa: F401
                   OP_MAXPOOL, OP_AVGPOOL, DT_I8, DT_BF16, f32_to_bf16_bits, bf16_bits_to_f32)
from .nets import build_net, load_net, apply_calibration, random_net, single_layer_net, inverted_residual_net, bottleneck_net, stem_net, CONFIGS  # noqa: F401
from .inputs import input_pool, poisson_trace, spiky_trace  # noqa: F401
