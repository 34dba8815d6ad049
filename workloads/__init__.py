"""Seeded synthetic inputs shared by the HIP path's tests, the benchmark and the oracle's tests.

This package holds data recipes only (shapes, distributions, seeds).  It contains none of
the method's arithmetic and imports neither the oracle nor the HIP binding.
"""
from .synth import (Workload, WORKLOADS, layer_params, token_stream, hidden_stream, BASE_SEED)  # noqa: F401
