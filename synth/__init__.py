"""Seeded synthetic inputs for the shadow-update path.

This package only produces inputs (tensor lists, hyper-parameters, initial
parameters, per-worker gradients, bucket arrival orders).  It contains none of
the method's arithmetic: no reduce, no clipping, no optimizer update, no bucket
assignment.  Both the CPU oracle's tests and the GPU path's tests draw their
inputs from here so that the two sides see identical bits.
"""
from .rng import (  # noqa: F401
    GAMMA,
    splitmix64_scalar,
    stream_base,
    uniform_u64,
    normal_f32,
    student_t3_f32,
    f32_to_bf16_bits,
    grad_values,
    param_values,
    tiled,
    arrival_order,
)
from .workloads import Workload, TensorSpec, get_workload, WORKLOADS  # noqa: F401
from .inputs import Inputs, TILE_PERIOD  # noqa: F401
