"""MI355X-native stage-training library: Python binding of the C ABI in include/asteroid.h.

Argument marshalling only; every step of the stage's forward, backward and update runs
in the HIP kernels of libasteroid_stage.so.  There is no CPU fallback: importing the
binding without the built library raises.
"""
from .binding import (  # noqa: F401
    Stage,
    AsteroidError,
    kp,
    plan_memory,
    lib_path,
    load_library,
    stream_create,
    stream_destroy,
)
