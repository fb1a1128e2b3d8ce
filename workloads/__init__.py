"""Seeded synthetic inputs and workload descriptions shared by the oracle and the HIP path.

This package holds no arithmetic of the method: only a counter-based random
generator, the one-time rounding of generated values to the storage type, and
plain-data descriptions (layer lists, shapes) of the synthetic workloads that
stand in for the paper's ResNet-50 and 3DUnet experiments (Section 6).
"""
from .rng import normal, uniform_int, round_to_bf16, bf16_bits, bits_to_f32  # noqa: F401
from .configs import (  # noqa: F401
    tiny_chain, bottleneck_stage, resnet50, unet3d, pool_net, updown_net, make_tensors, tensor_seed, infer_shapes,
)
