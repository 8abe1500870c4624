"""Seeded synthetic inputs shared by the CPU oracle, the tests and the benchmark.

This package only *describes* inputs: model shapes, which (holder, reader)
layouts a workload pairs up, seeded tensor values, and - for the scattered
sweep - the caller-supplied segment list.  It contains none of the method's
arithmetic: no shard/layout math, no wire-offset rule, no dtype narrowing.
The oracle and the HIP library each derive those on their own.
"""
from .models import MODELS, WORKLOADS, layout, workload  # noqa: F401
from .values import weight_values, id_pattern_values, to_bits, from_bits  # noqa: F401
from .scatter import scatter_description, scatter_values  # noqa: F401
