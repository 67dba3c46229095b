"""Seeded synthetic inputs shaped like the workloads the compression path is measured on.

This package holds shapes, seeds and value distributions only: none of the method's
arithmetic (no masks, no keep counts, no compaction).  Inputs are generated once and the
same bytes are handed to the GPU library and to the CPU oracle.
"""
from .shapes import TensorSpec, config_shapes, flat_size, seg_offsets  # noqa: F401
from .gen import CONFIGS, Workload, make_workload  # noqa: F401
