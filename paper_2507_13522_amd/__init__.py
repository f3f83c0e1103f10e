"""MI355X-native shadow update (Checkmate, arxiv 2507.13522, sections 4.2.2-4.2.4).

The package is a thin ctypes binding over ``libshadow.so`` (hand-written HIP
kernels for gfx950 behind the C ABI of ``include/shadow.h``).  Every step of
the update runs in those kernels; there is no CPU or PyTorch fallback: if the
library cannot be loaded, importing ``binding`` functions raises.
"""
from .binding import (  # noqa: F401
    GRAD_BF16,
    GRAD_F32,
    K_ADAMW,
    K_FOLD_ADAMW,
    K_FOLD_SUMSQ,
    K_NORM,
    K_SNAPSHOT,
    LaunchShape,
    OPT_ADAM,
    OPT_ADAMW,
    OPT_SGD,
    REDUCE_MEAN,
    REDUCE_SUM,
    HParams,
    Layout,
    Shadow,
    ShadowError,
    TensorDesc,
    lib,
    shadow_apply_iteration_static,
    shadow_copy_probe,
    shadow_stream_probe,
    shadow_strerror,
)
