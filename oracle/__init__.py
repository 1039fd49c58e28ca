"""CPU oracle for the binary-convolution hot path (test infrastructure only).

Thin ctypes access to ``bcnn_oracle.c``, ``bcnn_branches_oracle.c`` and ``bcnn_pool_oracle.c``: argument marshalling between numpy
arrays and the C functions, no arithmetic of its own.  Only ``tests/``, the
smoke check and the benchmark's ``cpu_baseline`` leg import this package; the
product library never does.
"""
from .binding import (  # noqa: F401
    avgpool_nhwc,
    branches_pm1,
    branches_real,
    build,
    conv2d_pm1,
    conv2d_pm1_at,
    load_bf16,
    module_epilogue,
    module_tail,
    num_threads,
    out_dim,
    pack_channels,
    replicate_channels,
    sign_bias_f32,
    sign_f32,
    store_bf16,
    store_f16,
    threshold_sign,
    unpack_channels,
)
