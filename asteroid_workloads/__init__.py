"""Seeded synthetic workloads for the stage-training hot path.

This package serves both the CPU oracle's tests and the HIP library's tests and
benchmark.  It holds layer lists (the "stage model" of Sec. 3.2: a run of
consecutive layers), tensor shapes and seeded random draws only.  None of the
method's arithmetic (no layer forward/backward, no optimizer) lives here.
"""
from .configs import (  # noqa: F401
    CONFIGS,
    StageConfig,
    get_config,
    irb,
    mobilenetv2_layers,
    encoder_layer,
)
from .gen import (  # noqa: F401
    param_specs,
    num_params,
    make_params,
    make_inputs,
    round_to_bf16,
    out_shape,
)
