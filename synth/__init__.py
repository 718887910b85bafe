"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package only *draws inputs* (feature keys, bag offsets, upstream gradients,
prefill key ranges).  It contains none of the pull/push arithmetic and imports
neither the oracle nor the HIP binding.
"""
from . import ctr  # noqa: F401
from .ctr import (  # noqa: F401
    Batch,
    Config,
    CONFIGS,
    BatchStream,
    mix64,
    prefill_keys,
    resident_split,
    scaled,
    zipf_ranks,
)
