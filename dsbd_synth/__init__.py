"""Seeded synthetic inputs for the forest-verification path.

This package only *generates inputs* (random tensors, forest topologies,
uniform draws).  It holds none of the method's arithmetic, so both the CPU
oracle's tests and the HIP path's tests may import it.
"""
from .philox import philox4x32_10, uniform01_f32            # noqa: F401
from .bf16 import f32_to_bf16_bits, bf16_bits_to_f32       # noqa: F401
from .workloads import CONFIGS, make_workload, Workload    # noqa: F401
from .models import SyntheticModels                        # noqa: F401
