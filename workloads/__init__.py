"""Seeded synthetic workloads shared by the CPU oracle's tests and the HIP path.

This package describes shapes and draws random tensors. It holds none of the
method's arithmetic: no forward pass, no gradient, no loss.
"""
from .configs import CONFIGS, get_config, unit_count, depth_sweep, resnet_layout  # noqa: F401
from .gen import tensor_specs, make_params, make_batch, make_worker_grads, make_velocity  # noqa: F401
