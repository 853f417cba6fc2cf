"""Region bookkeeping of libvt on the host-memory backend (no GPU): reserve / extend / release / share /
trim, error paths and rollback, checked against the oracle's integer model and the paper's statements
about vTensor regions ("vTensor and Management")."""

import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2407_15309_amd as vt
from oracle import meta

CHUNK = 64 * 1024          # small chunks keep the tests light; arithmetic is the same as with 2 MiB
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture
def ctx():
    c = vt.vt_init_host(CHUNK, 0)
    yield c
    vt.vt_destroy(c)


def host_view(ptr, nbytes):
    return np.ctypeslib.as_array((C.c_uint8 * nbytes).from_address(ptr))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "vt.h")).read()
    declared = set(re.findall(r"\b(vt_[a-z_]+)\s*\(", header))
    declared -= {"vt_status", "vt_dtype"}
    assert len(declared) >= 18
    for name in sorted(declared):
        assert hasattr(vt.binding.lib, name), name
    assert set(vt.binding.EXPORTS) == declared


def test_strerror():
    assert vt.vt_strerror(0) == "ok"
    assert "max_tokens" in vt.vt_strerror(vt.VT_E_CAPACITY)


def test_reserve_maps_nothing_and_metadata_matches_closed_forms(ctx):
    kv = vt.vt_reserve(ctx, 8, 128, vt.VT_BF16, 1000)
    info = vt.vt_query(kv)
    assert info.len == 0 and info.chunks_mapped == 0
    assert info.row_bytes == meta.row_bytes(8, 128) == 2048
    assert info.capacity_bytes == meta.capacity_bytes(1000, 8, 128, CHUNK)
    assert info.k_ptr % CHUNK == 0 and info.v_ptr % CHUNK == 0 and info.k_ptr != info.v_ptr
    st = vt.vt_stats(ctx)
    assert st.mapped_bytes == 0 and st.phys_bytes == 0 and st.chunks_created == 0
    assert st.reserved_va_bytes == 2 * info.capacity_bytes and st.live_regions == 1


def test_chunk_count_is_exact_for_every_length(ctx):
    """Exhaustive: chunks_mapped == ceil(len*row_bytes/chunk) for every length up to capacity."""
    hkv, d, mt = 3, 40, 1200         # row = 240 B: rows straddle chunk boundaries
    kv = vt.vt_reserve(ctx, hkv, d, vt.VT_F16, mt)
    base = vt.vt_query(kv)
    for L in range(0, mt + 1):
        vt.vt_extend(kv, L)
        info = vt.vt_query(kv)
        assert info.len == L
        assert info.chunks_mapped == meta.chunks_for_len(L, hkv, d, CHUNK)
        assert info.k_ptr == base.k_ptr and info.v_ptr == base.v_ptr
        assert info.capacity_bytes >= info.chunks_mapped * CHUNK >= L * info.row_bytes
    st = vt.vt_stats(ctx)
    assert st.mapped_bytes == 2 * meta.chunks_for_len(mt, hkv, d, CHUNK) * CHUNK == st.phys_bytes


def test_virtual_range_is_contiguous_over_scattered_chunks(ctx):
    """A byte ramp written through the range reads back contiguous although the chunks come from the pool
    in another order (paper "vTensor": contiguous VA over non-contiguous physical chunks)."""
    a = vt.vt_reserve(ctx, 4, 64, vt.VT_F16, 2048)      # row 512 B, 128 rows per chunk
    vt.vt_extend(a, 128 * 5)
    ka = vt.vt_query(a)
    host_view(ka.k_ptr, 5 * CHUNK)[:] = 7                # dirty the chunks
    vt.vt_release(a)                                     # 10 chunks into the pool (LIFO)
    b = vt.vt_reserve(ctx, 4, 64, vt.VT_F16, 2048)
    vt.vt_extend(b, 128 * 3 + 1)                         # 4 chunks per region, all from the pool
    st = vt.vt_stats(ctx)
    assert st.chunks_created == 10 and st.chunks_reused == 8 and st.chunks_pooled == 2
    kb = vt.vt_query(b)
    n = 4 * CHUNK
    ramp = (np.arange(n, dtype=np.uint64) * 2654435761 >> 7).astype(np.uint8)
    host_view(kb.k_ptr, n)[:] = ramp
    host_view(kb.v_ptr, n)[:] = ramp[::-1]
    np.testing.assert_array_equal(host_view(kb.k_ptr, n), ramp)
    np.testing.assert_array_equal(host_view(kb.v_ptr, n), ramp[::-1])


def test_extend_never_moves_base_or_touches_old_bytes(ctx):
    kv = vt.vt_reserve(ctx, 2, 64, vt.VT_BF16, 4096)     # row 256 B
    vt.vt_extend(kv, 300)
    info0 = vt.vt_query(kv)
    rows = np.random.default_rng(0).integers(0, 255, size=300 * 256, dtype=np.uint8)
    vt.vt_append(kv, rows, rows[::-1].copy(), 300, 0)
    for L in (301, 512, 513, 4096):
        vt.vt_extend(kv, L)
        info = vt.vt_query(kv)
        assert (info.k_ptr, info.v_ptr) == (info0.k_ptr, info0.v_ptr)
        np.testing.assert_array_equal(host_view(info.k_ptr, 300 * 256), rows)
        np.testing.assert_array_equal(host_view(info.v_ptr, 300 * 256), rows[::-1])


def test_pool_is_used_before_new_allocations(ctx):
    a = vt.vt_reserve(ctx, 8, 128, vt.VT_BF16, 512)
    vt.vt_extend(a, 96)                                  # 3 chunks per region -> 6
    vt.vt_release(a)
    created = vt.vt_stats(ctx).chunks_created
    b = vt.vt_reserve(ctx, 8, 128, vt.VT_BF16, 512)
    vt.vt_extend(b, 64)                                  # 2 + 2 chunks, all pooled
    st = vt.vt_stats(ctx)
    assert st.chunks_created == created and st.chunks_reused == 4 and st.chunks_pooled == 2
    vt.vt_extend(b, 128)                                 # 2 more each: 2 pooled + 2 new
    st = vt.vt_stats(ctx)
    assert st.chunks_created == created + 2 and st.chunks_pooled == 0


def test_released_range_is_reused_by_next_reserve_of_same_size(ctx):
    a = vt.vt_reserve(ctx, 8, 128, vt.VT_BF16, 512)
    ia = vt.vt_query(a)
    vt.vt_release(a)
    b = vt.vt_reserve(ctx, 8, 128, vt.VT_BF16, 512)
    ib = vt.vt_query(b)
    assert {ib.k_ptr, ib.v_ptr} == {ia.k_ptr, ia.v_ptr}
    st = vt.vt_stats(ctx)
    assert st.va_reserved_calls == 2 and st.va_reused == 2


def test_physical_memory_only_changes_in_extend_and_trim(ctx):
    phys = lambda: vt.vt_stats(ctx).phys_bytes
    a = vt.vt_reserve(ctx, 8, 128, vt.VT_BF16, 512)
    assert phys() == 0
    vt.vt_extend(a, 40)
    p1 = phys()
    assert p1 == 2 * meta.chunks_for_len(40, 8, 128, CHUNK) * CHUNK
    vt.vt_query(a)
    vt.vt_release(a)
    assert phys() == p1                                   # lazy deallocation keeps the chunks
    vt.vt_trim(ctx, 1)
    assert phys() == CHUNK and vt.vt_stats(ctx).chunks_pooled == 1
    vt.vt_trim(ctx, 0)
    st = vt.vt_stats(ctx)
    assert st.phys_bytes == 0 and st.reserved_va_bytes == 0


def test_error_paths_leave_state_unchanged(ctx):
    kv = vt.vt_reserve(ctx, 8, 128, vt.VT_BF16, 100)
    vt.vt_extend(kv, 50)
    before = (vt.vt_query(kv).len, vt.vt_query(kv).chunks_mapped, vt.vt_stats(ctx).asdict())
    for new_len, status in ((49, vt.VT_E_INVALID), (101, vt.VT_E_CAPACITY)):
        with pytest.raises(vt.VtError) as e:
            vt.vt_extend(kv, new_len)
        assert e.value.status == status
        assert (vt.vt_query(kv).len, vt.vt_query(kv).chunks_mapped, vt.vt_stats(ctx).asdict()) == before
    with pytest.raises(vt.VtError) as e:
        vt.vt_append(kv, np.zeros(2048 * 2, np.uint8), np.zeros(2048 * 2, np.uint8), 2, 49)   # beyond len
    assert e.value.status == vt.VT_E_INVALID
    with pytest.raises(vt.VtError):
        vt.vt_reserve(ctx, 0, 128, vt.VT_BF16, 100)
    with pytest.raises(vt.VtError):
        vt.vt_reserve(ctx, 8, 128, 7, 100)
    vt.vt_release(kv)
    for fn in (lambda: vt.vt_release(kv), lambda: vt.vt_extend(kv, 60), lambda: vt.vt_query(kv)):
        with pytest.raises(vt.VtError) as e:
            fn()
        assert e.value.status == vt.VT_E_INVALID          # double release / use after release


def test_physical_budget_gives_oom_without_partial_state():
    c = vt.vt_init_host(CHUNK, 6 * CHUNK)
    try:
        kv = vt.vt_reserve(c, 8, 128, vt.VT_BF16, 1024)
        vt.vt_extend(kv, 64)                              # 2 + 2 chunks
        with pytest.raises(vt.VtError) as e:
            vt.vt_extend(kv, 128)                         # needs 4 more: over the budget of 6
        assert e.value.status == vt.VT_E_OOM
        info, st = vt.vt_query(kv), vt.vt_stats(c)
        assert info.len == 64 and info.chunks_mapped == 2 and st.phys_bytes == 4 * CHUNK and st.chunks_pooled == 0
        vt.vt_extend(kv, 96)                              # 1 + 1 more fits exactly
        assert vt.vt_stats(c).phys_bytes == 6 * CHUNK
    finally:
        vt.vt_destroy(c)


def test_failing_map_midway_rolls_back(ctx):
    kv = vt.vt_reserve(ctx, 8, 128, vt.VT_BF16, 1024)
    vt.vt_extend(kv, 32)
    vt.vt_host_fail_after(ctx, 2, 3)                      # third map call of the next extend fails
    with pytest.raises(vt.VtError) as e:
        vt.vt_extend(kv, 32 * 4)                          # 3 + 3 new chunks
    assert e.value.status == vt.VT_E_DRIVER
    info, st = vt.vt_query(kv), vt.vt_stats(ctx)
    assert info.len == 32 and info.chunks_mapped == 1
    assert st.mapped_bytes == 2 * CHUNK and st.chunks_pooled == 6 and st.phys_bytes == 8 * CHUNK
    vt.vt_extend(kv, 32 * 4)                              # works afterwards, from the pool
    st = vt.vt_stats(ctx)
    assert st.chunks_pooled == 0 and st.mapped_bytes == 8 * CHUNK and vt.vt_query(kv).chunks_mapped == 4


def test_failing_create_changes_nothing(ctx):
    kv = vt.vt_reserve(ctx, 8, 128, vt.VT_BF16, 1024)
    vt.vt_host_fail_after(ctx, 1, 2)
    before = vt.vt_stats(ctx).asdict()
    with pytest.raises(vt.VtError) as e:
        vt.vt_extend(kv, 64)
    assert e.value.status == vt.VT_E_OOM
    after = vt.vt_stats(ctx).asdict()
    before.pop("driver_ns"), after.pop("driver_ns")
    assert before == after and vt.vt_query(kv).len == 0


def test_extend_batch_and_stop_at_first_failure(ctx):
    kvs = [vt.vt_reserve(ctx, 8, 128, vt.VT_BF16, 100) for _ in range(3)]
    vt.vt_extend_batch(kvs, [10, 20, 30])
    assert [vt.vt_query(k).len for k in kvs] == [10, 20, 30]
    with pytest.raises(vt.VtError) as e:
        vt.vt_extend_batch(kvs, [11, 101, 31])
    assert e.value.status == vt.VT_E_CAPACITY
    assert [vt.vt_query(k).len for k in kvs] == [11, 20, 30]


def test_prefix_sharing_aliases_the_same_physical_chunks(ctx):
    """Prefix match maps the SAME chunks into a second range: no new memory, writes through one alias are
    visible through the other, chunks return to the pool only when the last mapping goes (paper "vTensor Scheduler",
    Prefix Record and Match; "vTensor Pool", pSet reference counts)."""
    src = vt.vt_reserve(ctx, 8, 128, vt.VT_BF16, 256)    # 32 rows per chunk
    vt.vt_extend(src, 80)
    s = vt.vt_query(src)
    host_view(s.k_ptr, 64 * 2048)[:] = np.arange(64 * 2048, dtype=np.uint32).astype(np.uint8)
    phys = vt.vt_stats(ctx).phys_bytes
    with pytest.raises(vt.VtError):
        vt.vt_share_prefix(src, 70, 256)                 # not chunk aligned
    dst = vt.vt_share_prefix(src, 64, 256)
    d = vt.vt_query(dst)
    assert d.len == 64 and d.chunks_mapped == 2 and d.shared_chunks == 2 and d.k_ptr != s.k_ptr
    assert vt.vt_stats(ctx).phys_bytes == phys            # nothing allocated
    np.testing.assert_array_equal(host_view(d.k_ptr, 64 * 2048), host_view(s.k_ptr, 64 * 2048))
    host_view(s.k_ptr, 8)[:] = 99
    assert host_view(d.k_ptr, 8).tolist() == [99] * 8     # same memory
    vt.vt_extend(dst, 100)                                # private chunks after the shared ones
    assert vt.vt_query(dst).chunks_mapped == 4
    host_view(d.k_ptr + 2 * CHUNK, 8)[:] = 55
    assert host_view(s.k_ptr + 2 * CHUNK, 8).tolist() != [55] * 8
    vt.vt_release(src)
    st = vt.vt_stats(ctx)
    assert st.chunks_pooled == 2                          # only src's unshared third chunks (K and V)
    assert host_view(d.k_ptr, 8).tolist() == [99] * 8     # still mapped through dst
    vt.vt_release(dst)
    assert vt.vt_stats(ctx).chunks_pooled == 10 and vt.vt_stats(ctx).mapped_bytes == 0


def test_plan_decode_matches_the_documented_rule(ctx):
    rng = np.random.default_rng(5)
    for hkv, lo, hi, B in ((32, 512, 4096, 64), (8, 1024, 8192, 256), (8, 16, 256, 4), (1, 1, 1, 1), (4, 1, 70000, 9)):
        lens = rng.integers(lo, hi + 1, size=B).astype(np.int32)
        plan, ns = vt.vt_plan_decode(ctx, lens, hkv, hkv * 2, 128)
        span, n_splits, mx, units = meta.decode_plan(lens, hkv)
        assert (plan.span_tokens, plan.max_splits, plan.n_units) == (span, mx, units)
        assert ns.tolist() == n_splits
        assert plan.workspace_bytes >= B * mx * hkv * 2 * 130 * 4        # room for every (m, l, acc) partial
    # groups of more than 16 query heads take ceil(G / 16) wavefronts per (segment, kv head)
    for hq, hkv in ((32, 1), (40, 1), (64, 2), (34, 2), (32, 2)):
        lens = rng.integers(100, 5000, size=7).astype(np.int32)
        plan, ns = vt.vt_plan_decode(ctx, lens, hkv, hq, 128)
        span, n_splits, mx, units = meta.decode_plan(lens, hkv, n_q_heads=hq)
        assert (plan.span_tokens, plan.max_splits, plan.n_units, ns.tolist()) == (span, mx, units, n_splits)
    assert vt.vt_plan_decode(ctx, np.array([64000], np.int32), 1, 32, 128)[0].n_units == 2 * 1000   # 1024 slots -> 1000 x 64
    with pytest.raises(vt.VtError):
        vt.vt_plan_decode(ctx, np.array([5, 0], np.int32), 8, 8, 128)     # empty KV is invalid in decode
    for slots in (8, 64, 100000):
        vt.vt_set_plan_target(ctx, slots)
        lens = np.array([1000, 3000, 17], np.int32)
        plan, ns = vt.vt_plan_decode(ctx, lens, 8, 8, 128)
        want = meta.decode_plan(lens, 8, slots)
        assert (plan.span_tokens, ns.tolist(), plan.max_splits, plan.n_units) == want


def test_attention_on_a_host_context_is_refused(ctx):
    a = vt.make_decode_args(vt.VT_BF16, 1, 8, 8, 128, 0.1, 1, 1, 1, 1, 1, np.array([4], np.int32))
    with pytest.raises(vt.VtError) as e:
        vt.vt_attn_decode(ctx, a)
    assert e.value.status == vt.VT_E_UNSUPPORTED


def test_asynchronous_extension_runs_in_order_and_reports_status(ctx):
    """vt_extend_batch_async / vt_extend_wait on the host backend: same end state as the synchronous call, tickets
    finish in order, a failing request reports its own status and later ones still run."""
    kvs = [vt.vt_reserve(ctx, 8, 128, vt.VT_BF16, 4096) for _ in range(3)]
    t1 = vt.vt_extend_batch_async(kvs, [100, 1025, 0])
    t2 = vt.vt_extend_batch_async(kvs, [2049, 1025, 7])
    assert t2 == t1 + 1
    vt.vt_extend_wait(ctx, t2)                      # waits for t1 as well
    vt.vt_extend_wait(ctx, t1)
    assert [vt.vt_query(k).len for k in kvs] == [2049, 1025, 7]
    assert [vt.vt_query(k).chunks_mapped for k in kvs] == [meta.chunks_for_len(n, 8, 128, CHUNK) for n in (2049, 1025, 7)]
    bad = vt.vt_extend_batch_async(kvs[:1], [5000])  # beyond the reserved range
    ok = vt.vt_extend_batch_async(kvs[1:2], [1100])
    with pytest.raises(vt.VtError):
        vt.vt_extend_wait(ctx, bad)
    vt.vt_extend_wait(ctx, ok)
    assert vt.vt_query(kvs[0]).len == 2049 and vt.vt_query(kvs[1]).len == 1100
    with pytest.raises(vt.VtError):
        vt.vt_extend_wait(ctx, ok + 10)              # never issued
    for k in kvs:
        vt.vt_release(k)


def test_destroy_runs_queued_extensions():
    c = vt.vt_init_host(0, 0)
    kv = vt.vt_reserve(c, 8, 128, vt.VT_BF16, 4096)
    for n in range(1, 200):
        vt.vt_extend_batch_async([kv], [n * 20])
    vt.vt_destroy(c)                                 # no hang, no crash: the worker drains its queue and leaves
