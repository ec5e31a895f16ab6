"""Seeded synthetic workloads shared by the CPU oracle's tests and the HIP path's tests.

This package holds plain data only: layer lists of the split CNNs, DSP(p; m)
schedules, and seeded generators for parameters, mini-batches and labels.
None of the method's arithmetic (layers, gradients, queues, updates) lives here.
"""
from .configs import (  # noqa: F401
    CONFIGS,
    get_config,
    infer_shapes,
    param_shapes,
    count_macs,
)
from .gen import make_params, make_batch, make_error_gradient, flatten_params, unflatten_params  # noqa: F401
