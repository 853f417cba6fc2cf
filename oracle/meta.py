"""Integer metadata of virtually contiguous K/V regions and of the decode split plan (CPU oracle).

TEST INFRASTRUCTURE ONLY; shares no code with the library.

Region arithmetic follows the paper's vTensor description (Section 4.1 and the
Allocation paragraph of Section 4.3): a request gets a virtual range sized for
the maximum sequence length, physical memory is attached in fixed-size chunks
(2 MiB), and only as many chunks are mapped as the current length needs.

The decode split plan is this library's own rule (the paper is silent about the
kernel's work decomposition): per KV head the requests' tokens laid end to end
form a tape that is cut into equal segments, one per wavefront slot; a request
is covered by as many "pieces" as segments it touches.
"""

from __future__ import annotations

from typing import List, Sequence, Tuple

ELEM_BYTES = 2                 # fp16 and bf16
CHUNK_BYTES = 2 * 1024 * 1024  # "2 MB" physical chunk of the paper, read as 2 MiB
PLAN_WAVE_SLOTS = 2048         # 256 CUs x 2 workgroups x 4 wavefronts


def row_bytes(n_kv_heads: int, head_dim: int) -> int:
    return n_kv_heads * head_dim * ELEM_BYTES


def capacity_bytes(max_tokens: int, n_kv_heads: int, head_dim: int, chunk: int = CHUNK_BYTES) -> int:
    need = max_tokens * row_bytes(n_kv_heads, head_dim)
    return (need + chunk - 1) // chunk * chunk


def chunks_for_len(length: int, n_kv_heads: int, head_dim: int, chunk: int = CHUNK_BYTES) -> int:
    """Chunks that must be mapped (per region, K or V) to back `length` token rows."""
    return (length * row_bytes(n_kv_heads, head_dim) + chunk - 1) // chunk


def decode_plan(kv_lens: Sequence[int], n_kv_heads: int,
                slots: int = PLAN_WAVE_SLOTS) -> Tuple[int, List[int], int, int]:
    """Returns (segment length, pieces per request, max pieces, n_units)."""
    total = sum(int(L) for L in kv_lens)
    n_seg = max(1, min(slots // n_kv_heads, (total + 31) // 32))
    seg_len = (total + n_seg - 1) // n_seg
    seg_len = (seg_len + 31) // 32 * 32
    pieces, start = [], 0
    for L in kv_lens:
        L = int(L)
        pieces.append((start + L - 1) // seg_len - start // seg_len + 1)
        start += L
    units = (total + seg_len - 1) // seg_len * n_kv_heads
    return seg_len, pieces, (max(pieces) if pieces else 0), units


def piece_range(kv_lens: Sequence[int], seg_len: int, b: int, piece: int) -> Tuple[int, int]:
    """Token range [begin, end) inside request b of its piece number `piece`."""
    start = sum(int(L) for L in kv_lens[:b])
    L = int(kv_lens[b])
    seg = start // seg_len + piece
    return max(seg * seg_len - start, 0), min((seg + 1) * seg_len - start, L)


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
