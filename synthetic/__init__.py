"""Seeded synthetic inputs for the multi-turn rollout path.

This package only *draws* inputs (random weights, token ids, turn lengths) and
serialises them; it contains none of the decoder's or the sampler's arithmetic.
Both the CPU oracle and the HIP library consume the bytes produced here, so
neither needs to reproduce the other's random number generation.
"""
from .shapes import ModelShape, SHAPES  # noqa: F401
from .weights import make_weight_blob, BLOB_HEADER_BYTES  # noqa: F401
from .workloads import Workload, make_workload  # noqa: F401
