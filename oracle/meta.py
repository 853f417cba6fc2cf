"""Integer metadata of virtually contiguous K/V regions and of the decode split plan (CPU oracle).

TEST INFRASTRUCTURE ONLY; shares no code with the library.

Region arithmetic follows the paper's vTensor description (Section 4.1 and the
Allocation paragraph of Section 4.3): a request gets a virtual range sized for
the maximum sequence length, physical memory is attached in fixed-size chunks
(2 MiB), and only as many chunks are mapped as the current length needs.

The decode split plan is this library's own rule (the paper is silent about the
kernel's work decomposition): every request's keys are cut into spans of P
tokens, P being the smallest power of two >= 128 for which the number of
(request, kv head, span) work units does not exceed a fixed target.
"""

from __future__ import annotations

from typing import List, Sequence, Tuple

ELEM_BYTES = 2                 # fp16 and bf16
CHUNK_BYTES = 2 * 1024 * 1024  # "2 MB" physical chunk of the paper, read as 2 MiB
PLAN_MIN_SPAN = 128
PLAN_MAX_SPAN = 1 << 20
PLAN_TARGET_UNITS = 32768


def row_bytes(n_kv_heads: int, head_dim: int) -> int:
    return n_kv_heads * head_dim * ELEM_BYTES


def capacity_bytes(max_tokens: int, n_kv_heads: int, head_dim: int, chunk: int = CHUNK_BYTES) -> int:
    need = max_tokens * row_bytes(n_kv_heads, head_dim)
    return (need + chunk - 1) // chunk * chunk


def chunks_for_len(length: int, n_kv_heads: int, head_dim: int, chunk: int = CHUNK_BYTES) -> int:
    """Chunks that must be mapped (per region, K or V) to back `length` token rows."""
    return (length * row_bytes(n_kv_heads, head_dim) + chunk - 1) // chunk


def decode_plan(kv_lens: Sequence[int], n_kv_heads: int,
                target_units: int = PLAN_TARGET_UNITS) -> Tuple[int, List[int], int, int]:
    """Returns (span P, n_splits per request, max_splits, n_units)."""
    span = PLAN_MIN_SPAN
    while True:
        n_splits = [(int(L) + span - 1) // span for L in kv_lens]
        units = sum(n_splits) * n_kv_heads
        if units <= target_units or span >= PLAN_MAX_SPAN:
            break
        span *= 2
    return span, n_splits, (max(n_splits) if n_splits else 0), units


def split_range(length: int, span: int, s: int) -> Tuple[int, int]:
    """Token range [begin, end) of split s of a request of `length` tokens."""
    return s * span, min((s + 1) * span, int(length))


# --- accounting used by reports (what the method must move / compute) ---------------------------

def decode_kv_bytes(kv_lens: Sequence[int], n_kv_heads: int, head_dim: int) -> int:
    """K and V bytes one decode step must read: every cached row once per KV head."""
    return sum(int(L) for L in kv_lens) * 2 * row_bytes(n_kv_heads, head_dim)


def decode_flops(kv_lens: Sequence[int], n_q_heads: int, head_dim: int) -> int:
    return sum(int(L) for L in kv_lens) * 4 * n_q_heads * head_dim


def prefill_flops(prefix_lens: Sequence[int], new_lens: Sequence[int], n_q_heads: int, head_dim: int) -> int:
    """Multiply-adds x2 over the unmasked (query, key) pairs only."""
    pairs = sum(int(n) * int(p) + int(n) * (int(n) + 1) // 2 for p, n in zip(prefix_lens, new_lens))
    return 4 * n_q_heads * head_dim * pairs
