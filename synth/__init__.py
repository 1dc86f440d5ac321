"""Seeded synthetic inputs shared by the CPU oracle tests and the GPU path.

This package only *draws numbers and arranges them in tensors*: pools of
class-mean Gaussian images, uniform labels, initial network weights, perturbed
parameter replicas and loss arrays for selection tests.  It contains none of the
method's arithmetic (no forward pass, loss, selection, update or aggregation).
"""
from .rng import uniform01, normal, randint            # noqa: F401
from .inputs import (                                   # noqa: F401
    WORKLOADS, workload, image_pool, mlp_init, resnet_init, resnet_tensor_specs,
    mlp_tensor_specs, wrn_tensor_specs, wrn_init, transformer_tensor_specs, transformer_init, token_pool, replicas, loss_array, LOSS_ARRAY_KINDS,
)
