"""CPU oracle for attention over per-request contiguous KV caches.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; it is
used by tests/, by the smoke check and by the benchmark's CPU-baseline leg.  It
shares no code with the HIP path.
"""

from .attention import widen, softmax_rows, decode, prefix_prefill  # noqa: F401
from . import meta  # noqa: F401
