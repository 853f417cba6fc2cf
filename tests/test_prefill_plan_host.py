"""Host logic of the prefix-prefill work decomposition (vt_plan_prefill, no GPU): the library's pieces against the
rule written out from its definition in oracle/meta.py, and that rule against what must hold of any such
decomposition - every (token, key) pair a new token sees is covered by exactly one tile, fast tiles are wholly
visible, every tile of every item is computed exactly once, the groups' shares are even."""

import numpy as np
import pytest

import paper_2407_15309_amd as vt
import workloads
from oracle import meta
from workloads import CONFIGS


@pytest.fixture(scope="module")
def ctx():
    c = vt.vt_init_host(0, 0)
    yield c
    vt.vt_destroy(c)


def lens_of(cfg_id):
    cfg = CONFIGS[cfg_id]
    seed = workloads.gen.base_seed(cfg_id)
    P = workloads.gen.draw_lengths(seed, workloads.gen.T_KV_LEN, cfg.batch, *cfg.kv_len)
    N = workloads.gen.draw_lengths(seed, workloads.gen.T_NEW_LEN, cfg.batch, *cfg.new_len)
    return np.concatenate([[0], np.cumsum(N)]).astype(np.int32), P.astype(np.int32)


CASES = [
    ("edges", [0, 0, 1, 63, 64, 65, 127, 500, 0, 300, 129], [1, 130, 1, 64, 65, 63, 1, 1, 64, 257, 128], 32, 8, 128),
    ("empty-request", [50, 70, 10], [5, 0, 9], 32, 8, 128),
    ("mha", [299, 104, 24], [274, 46, 46], 8, 8, 128),
    ("g7", [125, 166, 59], [35, 53, 131], 56, 8, 128),
    ("mqa-d64", [1000, 3], [300, 700], 32, 1, 64),
    ("one-long-item", [10153], [84], 32, 8, 128),
]


@pytest.mark.parametrize("split", [True, False])
@pytest.mark.parametrize("name,plens,nlens,hq,hkv,d", CASES)
def test_library_plan_equals_the_rule(ctx, name, plens, nlens, hq, hkv, d, split):
    cu = np.concatenate([[0], np.cumsum(nlens)]).astype(np.int32)
    check_against_rule(ctx, cu, np.array(plens, np.int32), hq, hkv, d, split)


@pytest.mark.parametrize("cfg_id", [3, 4])
def test_library_plan_equals_the_rule_on_the_workloads(ctx, cfg_id):
    cu, P = lens_of(cfg_id)
    cfg = CONFIGS[cfg_id]
    plan = check_against_rule(ctx, cu, P, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, True)
    assert plan.n_groups == 256      # both fill the chip, also config 4 with its 200 items
    check_against_rule(ctx, cu, P, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, False)


def check_against_rule(ctx, cu, P, hq, hkv, d, split):
    plan, pieces = vt.vt_plan_prefill(ctx, cu, P, hq, hkv, d, new_rows_in_cache=not split, want_pieces=True)
    ref = meta.prefill_plan(cu, P, hq, hkv, d, split)
    assert (plan.total_cost, plan.n_tiles, plan.n_items, plan.n_groups, plan.workspace_bytes) == ref[:5]
    got = [(p.group, p.request, p.kv_head, p.token_tile, p.tile_begin, p.tile_end) for p in pieces]
    assert got == ref[5]
    # per-item tile counts as reported with each piece
    tb = 256 // (hq // hkv)
    for p in pieces:
        tiles = meta.prefill_item_tiles(int(P[p.request]), int(cu[p.request + 1] - cu[p.request]), p.token_tile, tb, split)
        assert (p.n_tiles, p.n_fast) == (len(tiles), sum(tiles))
    return plan


@pytest.mark.parametrize("split", [True, False])
def test_tiles_cover_every_visible_pair_once_and_fast_tiles_need_no_mask(split):
    """Brute force on small lengths: rebuild the tiles of an item as sets of key positions (same tiling as the
    rule: segments from their own row 0) and check them against the visibility definition."""
    tb = 64
    for P in (0, 1, 63, 64, 65, 130, 200):
        for N in (1, 63, 64, 65, 129, 200):
            for t in range((N + tb - 1) // tb):
                tok0 = t * tb
                ntok = min(tb, N - tok0)
                vis = tok0 + ntok
                segs = [list(range(P)), [P + r for r in range(vis)]] if split else [list(range(P + vis))]
                tiles = [seg[k:k + 64] for seg in segs for k in range(0, len(seg), 64)]
                flags = meta.prefill_item_tiles(P, N, t, tb, split)
                assert len(flags) == len(tiles)
                assert flags == sorted(flags, reverse=True)           # fast tiles are swept first
                # the multiset of keys over all tiles is exactly the keys the last token sees, each once
                keys = sorted(k for tile in tiles for k in tile)
                assert keys == list(range(P + vis))
                # number of fast tiles = number of full tiles wholly visible to the first token
                n_fast = sum(1 for tile in tiles if len(tile) == 64 and all(k <= P + tok0 for k in tile))
                assert sum(flags) == n_fast
                # every token of the item sees every key of a fast tile (no mask needed there)
                assert all(k <= P + tok0 + i for tile in tiles if len(tile) == 64 and tile[-1] <= P + tok0
                           for k in tile for i in range(ntok))


def check_decomposition(pieces, total_cost, n_tiles, n_items, n_groups, P, N_of, tb, split):
    """What must hold of any such decomposition, whoever computed it.  pieces: (group, request, kv_head,
    token_tile, tile_begin, tile_end) in execution order.  The tile counts per item come from the tile enumeration
    of the rule (itself pinned by brute force above)."""
    shape = {}
    def tiles_of(r, t):
        if (r, t) not in shape:
            shape[(r, t)] = meta.prefill_item_tiles(int(P[r]), int(N_of(r)), t, tb, split)
        return shape[(r, t)]
    # coverage: per item the pieces tile [0, n_tiles) without gap or overlap, in increasing groups
    by_item = {}
    for pc in pieces:
        by_item.setdefault(pc[1:4], []).append(pc)
    assert len(by_item) == n_items
    for (r, g, t), ps in by_item.items():
        nt = len(tiles_of(r, t))
        assert ps[0][4] == 0 and ps[-1][5] == nt
        for a, b in zip(ps, ps[1:]):
            assert a[5] == b[4] and a[0] < b[0]
        assert all(pc[5] > pc[4] for pc in ps)
    assert sum(pc[5] - pc[4] for pc in pieces) == n_tiles
    # a group continues at most one item (first) and leaves at most one unfinished (last)
    groups = {}
    for pc in pieces:
        groups.setdefault(pc[0], []).append(pc)
    assert all(0 <= w < n_groups for w in groups)
    for w, ps in groups.items():
        assert all(pc[4] == 0 for pc in ps[1:])
        assert all(pc[5] == len(tiles_of(pc[1], pc[3])) for pc in ps[:-1])
    # even shares: a group's cost (per fast tile, per other tile, per started item) stays within one tile and one
    # item start of the ideal share
    cf, cm, ci = meta.PREFILL_COST_FAST, meta.PREFILL_COST_MASKED, meta.PREFILL_COST_ITEM
    ideal = total_cost / n_groups
    for w, ps in groups.items():
        c = 0
        for pc in ps:
            flags = tiles_of(pc[1], pc[3])[pc[4]:pc[5]]
            c += sum(cf if f else cm for f in flags) + (ci if pc[4] == 0 else 0)
        assert abs(c - ideal) <= cm + ci + 1, (w, c, ideal)


@pytest.mark.parametrize("cfg_id,split", [(3, True), (4, True), (3, False)])
def test_every_tile_is_computed_once_and_shares_are_even(ctx, cfg_id, split):
    """The properties are asserted on the rule's own output (oracle/meta.py, so that the rule is pinned by what any
    decomposition must satisfy and not only by agreeing with the library) and on the library's output."""
    cu, P = lens_of(cfg_id)
    cfg = CONFIGS[cfg_id]
    tb = 256 // (cfg.n_q_heads // cfg.n_kv_heads)
    N_of = lambda r: cu[r + 1] - cu[r]
    total, n_tiles, n_items, n_groups, ws, ref_pieces = meta.prefill_plan(cu, P, cfg.n_q_heads, cfg.n_kv_heads,
                                                                          cfg.head_dim, split)
    check_decomposition(ref_pieces, total, n_tiles, n_items, n_groups, P, N_of, tb, split)
    plan, pieces = vt.vt_plan_prefill(ctx, cu, P, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                                      new_rows_in_cache=not split, want_pieces=True)
    got = [(p.group, p.request, p.kv_head, p.token_tile, p.tile_begin, p.tile_end) for p in pieces]
    check_decomposition(got, plan.total_cost, plan.n_tiles, plan.n_items, plan.n_groups, P, N_of, tb, split)
    # workspace: two piece slots per group
    assert plan.workspace_bytes == plan.n_groups * 2 * (512 + 256 * cfg.head_dim) * 4


@pytest.mark.parametrize("name,plens,nlens,hq,hkv,d", CASES)
def test_rule_properties_on_small_cases(name, plens, nlens, hq, hkv, d):
    cu = np.concatenate([[0], np.cumsum(nlens)]).astype(np.int32)
    P = np.array(plens, np.int32)
    for split in (True, False):
        for n_cus in (256, 7):
            total, n_tiles, n_items, n_groups, ws, pieces = meta.prefill_plan(cu, P, hq, hkv, d, split, n_cus=n_cus)
            check_decomposition(pieces, total, n_tiles, n_items, n_groups, P, lambda r: cu[r + 1] - cu[r],
                                256 // (hq // hkv), split)


def test_bad_arguments(ctx):
    cu = np.array([0, 5], np.int32)
    P = np.array([10], np.int32)
    with pytest.raises(vt.VtError):
        vt.vt_plan_prefill(ctx, cu, P, 32, 5, 128)            # heads do not divide
    with pytest.raises(vt.VtError):
        vt.vt_plan_prefill(ctx, cu, P, 32, 8, 96)             # unsupported head_dim
    with pytest.raises(vt.VtError):
        vt.vt_plan_prefill(ctx, np.array([0, -1], np.int32), P, 32, 8, 128)
    plan = vt.vt_plan_prefill(ctx, np.array([0, 0], np.int32), P, 32, 8, 128)
    assert (plan.total_cost, plan.n_groups, plan.workspace_bytes) == (0, 0, 0)
