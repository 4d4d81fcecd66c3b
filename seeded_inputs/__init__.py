"""Seeded synthetic inputs for the weight-reshard path.

This module serves both the CPU oracle and the HIP library's tests/bench.  It holds
NO layout or resharding arithmetic: it only turns (seed, stream id, element index)
into a 16-bit pattern, and fills a caller-described list of regions with such
patterns.  Which region is which tensor, and where it lives, is always told to it
by the caller (the oracle's tables in tests, the library's tensor queries in bench).
"""
from .bits import (  # noqa: F401
    KIND_IDS,
    bits16_numpy,
    bits16_scalar,
    bits16_torch,
    config_seed,
    fill_regions_numpy,
    fill_regions_torch,
    stream_key,
    tensor_uid,
)
