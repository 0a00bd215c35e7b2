"""CPU fp64 oracle of the stage-training hot path.  Test infrastructure: only tests,
the smoke check and the benchmark's cpu_baseline leg may import it."""
from .stage import OracleStage, run_round  # noqa: F401
from . import layers  # noqa: F401
