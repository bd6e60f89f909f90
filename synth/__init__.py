"""Seeded synthetic inputs shared by the oracle tests, the GPU parity tests and the benchmark.

This package holds model *shapes*, parameter *names* and random input generators only.  It contains
none of the method's arithmetic (no forward pass, no loss, no optimiser, no dropout hash), so that the
CPU oracle and the HIP path can both be fed from it without sharing any computation.
"""
from .shapes import ModelShape, PRESETS, param_specs, count_params          # noqa: F401
from .params import init_params                                             # noqa: F401
from .batches import Batch, make_batches, zipf_ids, WORKLOADS               # noqa: F401
