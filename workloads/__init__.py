"""Seeded synthetic inputs for the PQT query path.

This module produces vectors and queries only.  It holds none of the method's
arithmetic (no quantisers, no distances, no sorting of candidates): both the
CPU oracle's tests and the HIP path's tests/bench draw their inputs from here
so that the two sides see byte-identical data.
"""
from .configs import CONFIGS, WorkloadConfig, get_config  # noqa: F401
from .synth import (  # noqa: F401
    tiny_mixture,
    sift_like,
    sift_like_tables,
    sift_like_torch,
    gist_like,
    gist_like_torch,
    small_integer_vectors,
)
