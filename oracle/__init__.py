"""CPU fp64 oracle for the ScatterMoE hot path (test infrastructure only).

Nothing in the product path may import this package: it exists so that the
tests, the smoke check and the bench's cpu_baseline leg have an independent,
slow, plainly-correct definition to compare the HIP kernels with.
"""
from .smoe_oracle import *  # noqa: F401,F403
from .momha_oracle import *  # noqa: F401,F403
