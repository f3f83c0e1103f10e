"""CPU oracle of the shadow update.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package; the product path never does.
"""
from .layout import Bucket, Layout, Segment, build_layout  # noqa: F401
from .shadow import (  # noqa: F401
    HParams,
    OracleShadow,
    SumSq,
    adam_f32,
    adam_f64,
    adamw_f32,
    adamw_f64,
    sgd_f32,
    sgd_f64,
    clip_coef,
    fold,
    get_threads,
    lib,
    set_threads,
    step_scalars,
    widen_bf16,
)
