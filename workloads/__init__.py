"""Seeded synthetic inputs shared by the tests, the oracle checks and the benchmark.

This package draws lengths and random bit patterns only.  It contains none of
the attention arithmetic and none of the region bookkeeping, so both the CPU
oracle and the HIP path can consume its arrays without sharing any code with
each other.
"""

from .gen import (  # noqa: F401
    CONFIGS,
    Config,
    base_seed,
    draw_lengths,
    normal_bits,
    decode_inputs,
    prefill_inputs,
    step_inputs,
    checksum64,
)
