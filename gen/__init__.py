"""Seeded synthetic workloads for the LRQK decode step.

This package only *draws inputs*: low-rank keys, values, queries, planted heavy
tokens and their drift.  It holds none of the arithmetic of the method (scores,
selection, cache, attention) and is imported by the tests and the benchmark to
feed the same bits to the CPU oracle and to the HIP library.
"""
from .configs import CONFIGS, WorkloadConfig, get_config  # noqa: F401
from .workload import (LayerData, QueryStream, make_layer, make_prefill_inputs,  # noqa: F401
                       bf16_bits, as_numpy)
