"""Integer metadata of virtually contiguous K/V regions and of the decode split plan (CPU oracle).

TEST INFRASTRUCTURE ONLY; shares no code with the library.

Region arithmetic follows the paper's vTensor description ("vTensor" and the
Allocation paragraphs of "vTensor Operation"): a request gets a virtual range sized for
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
                slots: int = PLAN_WAVE_SLOTS, n_q_heads: int = 0) -> Tuple[int, List[int], int, int]:
    """Returns (segment length, pieces per request, max pieces, n_units).  A wavefront carries at most 16 query
    heads of one KV head, so a segment is worked on by n_kv_heads * ceil(group / 16) wavefronts."""
    total = sum(int(L) for L in kv_lens)
    group = max(1, n_q_heads // n_kv_heads) if n_q_heads else 1
    n_kv_heads = n_kv_heads * ((group + 15) // 16)
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


# ---- prefix-prefill work decomposition (this library's own rule, spelled out from its definition) -------------

PREFILL_TILE = 64          # keys per tile
PREFILL_ROWS = 256         # query rows per workgroup
PREFILL_COST_ITEM, PREFILL_COST_FAST, PREFILL_COST_MASKED = 8, 2, 3
PREFILL_MIN_COST_PER_GROUP = 64


def prefill_item_tiles(P: int, N: int, t: int, tb: int, split: bool) -> List[bool]:
    """The key tiles item (token tile t of tb tokens, request with P cached and N new rows) sweeps, in sweep
    order; True = fast.  The item's tokens sit at new-row positions tok0 .. tok0+ntok-1 and see the cached rows and
    the new rows up to their own.  When cached and new rows come from two buffers (split) each buffer is tiled from
    its own row 0; otherwise they are one run of rows.  A tile is fast when all its 64 rows exist and even the
    first token of the item sees its last row.  Fast tiles are swept first."""
    tok0 = t * tb
    ntok = min(tb, N - tok0)
    assert ntok >= 1
    vis = tok0 + ntok
    # each segment: list of absolute key positions
    segs = [list(range(P)), [P + r for r in range(vis)]] if split else [list(range(P + vis))]
    first_tok_pos = P + tok0
    fast, other = [], []
    for seg in segs:
        for k0 in range(0, len(seg), PREFILL_TILE):
            rows = seg[k0:k0 + PREFILL_TILE]
            is_fast = len(rows) == PREFILL_TILE and rows[-1] <= first_tok_pos
            (fast if is_fast else other).append(is_fast)
    return fast + other


def prefill_plan(cu_seqlens: Sequence[int], prefix_lens: Sequence[int], n_q_heads: int, n_kv_heads: int,
                 head_dim: int, split: bool, n_cus: int = 256):
    """Returns (total_cost, n_tiles, n_items, n_groups, workspace_bytes, pieces) with pieces a list of
    (group, request, kv_head, token_tile, tile_begin, tile_end) in execution order.

    Items are laid end to end by request, kv head, token tile; an item costs 8 units, then 2 per fast tile and 3 per
    other tile in sweep order; group w of n owns units [total*w//n, total*(w+1)//n); a tile belongs to the group
    that owns its first unit; consecutive tiles of an item with the same owner form a piece."""
    tb = PREFILL_ROWS // (n_q_heads // n_kv_heads)
    items = []
    for b in range(len(prefix_lens)):
        N = int(cu_seqlens[b + 1]) - int(cu_seqlens[b])
        for g in range(n_kv_heads):
            for t in range((N + tb - 1) // tb):
                items.append((b, g, t, prefill_item_tiles(int(prefix_lens[b]), N, t, tb, split)))
    cost = lambda tiles: PREFILL_COST_ITEM + sum(PREFILL_COST_FAST if f else PREFILL_COST_MASKED for f in tiles)
    total = sum(cost(it[3]) for it in items)
    n_tiles = sum(len(it[3]) for it in items)
    if total == 0:
        return 0, 0, 0, 0, 0, []
    n_groups = max(1, min(n_cus, total // PREFILL_MIN_COST_PER_GROUP))
    bounds = [total * w // n_groups for w in range(n_groups + 1)]
    import bisect
    owner = lambda unit: bisect.bisect_right(bounds, unit) - 1
    pieces = []
    begin = 0
    for b, g, t, tiles in items:
        unit = begin + PREFILL_COST_ITEM
        run = None
        for s, f in enumerate(tiles):
            w = owner(unit)   # the item's 8 fixed units come before its first tile
            if run is not None and run[0] == w:
                run[5] = s + 1
            else:
                if run is not None:
                    pieces.append(tuple(run))
                run = [w, b, g, t, s, s + 1]
            unit += PREFILL_COST_FAST if f else PREFILL_COST_MASKED
        if run is not None:
            pieces.append(tuple(run))
        begin += cost(tiles)
    piece_floats = 512 + 256 * head_dim
    ws = 2 * n_groups * piece_floats * 4
    # pieces are executed group by group; within a group in item order (which is the order built above)
    pieces.sort(key=lambda p: p[0])
    return total, n_tiles, len(items), n_groups, ws, pieces
