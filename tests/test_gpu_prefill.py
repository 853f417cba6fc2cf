"""GPU parity of vt_attn_prefix_prefill (through the C ABI) against the fp64 oracle, and the multi-turn
scenario: prefix-prefill, then extend + append the new turn, then one decode step over the grown cache."""

import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2407_15309_amd as vt
import workloads
from oracle import meta
from workloads import CONFIGS

pytestmark = pytest.mark.gpu

from gpu_util import TOL, Regions, dev_bits, run_decode, run_prefill, stream  # noqa: E402


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def ctx():
    c = vt.vt_init(0, 0, 0)
    yield c
    torch.cuda.synchronize()
    vt.vt_destroy(c)


def oracle_prefill(cfg, d, scale=None):
    w = lambda x: oracle.widen(x, cfg.dtype)
    return oracle.prefix_prefill(w(d["q_new"]), w(d["k_new"]), w(d["v_new"]), d["cu_seqlens"],
                                 [w(x) for x in d["k"]], [w(x) for x in d["v"]], cfg.scale if scale is None else scale)


def check_prefill(ctx, cfg, d, tag, new_in_cache=False, scale=None):
    say("prefill case", tag, "dtype", cfg.dtype, "B", cfg.batch, "Hq/Hkv", cfg.n_q_heads, cfg.n_kv_heads, "D",
        cfg.head_dim, "P", d["prefix_lens"][:8].tolist(), "N", d["new_lens"][:8].tolist(), "seed", d["seed"],
        "new_in_cache", new_in_cache)
    if new_in_cache:
        cu = d["cu_seqlens"]
        k = [np.concatenate([d["k"][b], d["k_new"][cu[b]:cu[b + 1]]]) for b in range(cfg.batch)]
        v = [np.concatenate([d["v"][b], d["v_new"][cu[b]:cu[b + 1]]]) for b in range(cfg.batch)]
    else:
        k, v = d["k"], d["v"]
    reg = Regions(ctx, k, v, cfg.dtype, headroom=1)
    try:
        got = run_prefill(ctx, cfg.dtype, d, reg.k_ptrs, reg.v_ptrs, cfg.n_kv_heads,
                          cfg.scale if scale is None else scale, new_in_cache)
    finally:
        reg.release()
    ref = oracle_prefill(cfg, d, scale)
    gv = oracle.widen(got, cfg.dtype)
    assert np.isfinite(gv).all()
    err = np.abs(gv - ref)
    say("  max abs err", float(err.max()), "tolerance", TOL[cfg.dtype])
    assert err.max() <= TOL[cfg.dtype]
    return got


def with_lens(cfg, plens, nlens, seed=21):
    cfg = cfg.replace(batch=len(plens))
    d = workloads.prefill_inputs(cfg.replace(kv_len=(1, 2), new_len=(1, 2)), seed=seed)
    g = workloads.gen
    d["prefix_lens"] = np.array(plens, np.int32)
    d["new_lens"] = np.array(nlens, np.int32)
    d["cu_seqlens"] = np.concatenate([[0], np.cumsum(nlens)]).astype(np.int32)
    kv = lambda t, b, n: workloads.normal_bits(seed, t, b, (n, cfg.n_kv_heads, cfg.head_dim), cfg.dtype)
    d["k"] = [kv(g.T_K, b, p) for b, p in enumerate(plens)]
    d["v"] = [kv(g.T_V, b, p) for b, p in enumerate(plens)]
    d["k_new"] = np.concatenate([kv(g.T_KNEW, b, n) for b, n in enumerate(nlens)])
    d["v_new"] = np.concatenate([kv(g.T_VNEW, b, n) for b, n in enumerate(nlens)])
    d["q_new"] = np.concatenate([workloads.normal_bits(seed, g.T_QNEW, b, (n, cfg.n_q_heads, cfg.head_dim), cfg.dtype)
                                 for b, n in enumerate(nlens)])
    return cfg, d


def test_small_gqa_bf16(ctx):
    cfg = CONFIGS[3].replace(batch=3, kv_len=(100, 700), new_len=(1, 200))
    check_prefill(ctx, cfg, workloads.prefill_inputs(cfg, seed=31), "small")


def test_config3_full(ctx):
    cfg = CONFIGS[3]
    d = workloads.prefill_inputs(cfg)
    assert meta.prefill_flops(d["prefix_lens"], d["new_lens"], 32, 128) > 1e11
    check_prefill(ctx, cfg, d, "config3")


@pytest.mark.parametrize("dtype,hq,hkv,d", [
    ("bf16", 8, 8, 128), ("bf16", 16, 2, 128), ("bf16", 56, 8, 128), ("f16", 32, 8, 128), ("f16", 8, 2, 64),
    ("bf16", 32, 1, 128), ("bf16", 12, 4, 64), ("f16", 3, 3, 128),
])
def test_head_group_shapes(ctx, dtype, hq, hkv, d):
    cfg = CONFIGS[3].replace(dtype=dtype, batch=3, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, kv_len=(0, 300),
                             new_len=(1, 300))
    check_prefill(ctx, cfg, workloads.prefill_inputs(cfg, seed=500 + hq * 3 + hkv), "shapes")


@pytest.mark.parametrize("seed", range(10))
def test_seeded_random_shapes_and_lengths(ctx, seed):
    """Seeded draws of head shapes, batch and (prefix, new) lengths, biased towards the 64-key tile edges."""
    from test_gpu_decode import edge_biased_length, random_shape
    rng = np.random.default_rng(9100 + seed)
    dtype, hq, hkv, d = random_shape(rng)
    nb = int(rng.integers(1, 5))
    plens = [int(rng.integers(2)) * edge_biased_length(rng, 64, 700) for _ in range(nb)]
    nlens = [edge_biased_length(rng, 64, 300) for _ in range(nb)]
    cfg, data = with_lens(CONFIGS[3].replace(dtype=dtype, n_q_heads=hq, n_kv_heads=hkv, head_dim=d), plens, nlens,
                          seed=800 + seed)
    check_prefill(ctx, cfg, data, "random", new_in_cache=bool(seed % 3 == 2))


def test_edge_lengths(ctx):
    """No prefix (plain causal attention), single new token (= decode), lengths around the tile sizes."""
    plens = [0, 0, 1, 63, 64, 65, 127, 500, 0, 300, 129]
    nlens = [1, 130, 1, 64, 65, 63, 1, 1, 64, 257, 128]
    cfg, d = with_lens(CONFIGS[3], plens, nlens)
    check_prefill(ctx, cfg, d, "edges")
    cfg, d = with_lens(CONFIGS[3].replace(dtype="f16", n_q_heads=4, n_kv_heads=4, head_dim=64), plens, nlens, seed=22)
    check_prefill(ctx, cfg, d, "edges-mha-f16-d64")


def test_paper_sweep_point_16k_context_ratio_half(ctx):
    """One full point of the paper-shaped sweeps: context 16384, prefix ratio 0.5 (8192 cached + 8192 new tokens),
    batch 1, the paper's default 32 query / 4 KV heads; every output row against the oracle."""
    cfg, d = with_lens(CONFIGS[3].replace(n_q_heads=32, n_kv_heads=4), [8192], [8192], seed=1607)
    check_prefill(ctx, cfg, d, "sweep p1 point")


def test_four_wavefront_kernel_at_head_dim_128():
    """head_dim 128 runs as eight wavefronts of 32 rows; a context created under VT_PREFILL_WIDE=1 runs the
    four-wavefront kernel (the one head_dim 64 always uses) on the same inputs: edge lengths, a shared item, a
    dominant late key (the fallback to the classic softmax) and workload 3, each against the oracle."""
    import os
    os.environ["VT_PREFILL_WIDE"] = "1"
    try:
        wide = vt.vt_init(0, 0, 0)
    finally:
        del os.environ["VT_PREFILL_WIDE"]
    try:
        plens = [0, 0, 1, 63, 64, 65, 127, 500, 0, 300, 129]
        nlens = [1, 130, 1, 64, 65, 63, 1, 1, 64, 257, 128]
        cfg, d = with_lens(CONFIGS[3], plens, nlens)
        check_prefill(wide, cfg, d, "wide edges")
        cfg, d = with_lens(CONFIGS[3].replace(dtype="f16", n_q_heads=8, n_kv_heads=8), [5000], [40], seed=77)
        check_prefill(wide, cfg, d, "wide shared item")
        cfg, d = with_lens(CONFIGS[3], [300, 200], [70, 130], seed=77)
        q = oracle.widen(d["q_new"], cfg.dtype) + 0.5
        d["q_new"] = workloads.gen._round_bits(q.astype(np.float32), cfg.dtype)
        d["k"][0][250] = workloads.gen._round_bits(np.full((cfg.n_kv_heads, cfg.head_dim), 40.0, np.float32), cfg.dtype)
        check_prefill(wide, cfg, d, "wide dominant late key")
        check_prefill(wide, CONFIGS[3], workloads.prefill_inputs(CONFIGS[3]), "wide config3")
    finally:
        torch.cuda.synchronize()
        vt.vt_destroy(wide)


def test_one_item_shared_by_many_workgroups(ctx):
    """A single (request, kv head, token tile) with a long prefix: its key tiles are spread over several workgroups
    and the merge kernel combines more than two pieces."""
    cfg, d = with_lens(CONFIGS[3].replace(n_q_heads=4, n_kv_heads=1), [20000], [64], seed=29)
    plan, pieces = vt.vt_plan_prefill(ctx, d["cu_seqlens"], d["prefix_lens"], 4, 1, 128, want_pieces=True)
    assert plan.n_items == 1 and len(pieces) == plan.n_groups >= 8
    check_prefill(ctx, cfg, d, "one-item-many-groups")
    cfg, d = with_lens(CONFIGS[3].replace(dtype="f16", n_q_heads=2, n_kv_heads=2, head_dim=64), [9000, 5000], [300, 1], seed=30)
    check_prefill(ctx, cfg, d, "few-items-many-groups-f16-d64")


def test_empty_request_in_batch(ctx):
    cfg, d = with_lens(CONFIGS[3], [50, 70, 10], [5, 0, 9])
    check_prefill(ctx, cfg, d, "empty-request")


def test_new_rows_already_in_cache_agrees_with_split_sources(ctx):
    """The new tokens' K/V either come from k_new / v_new or are already appended to the regions.  The two calls
    tile the keys differently (cached and new rows are tiled separately when they come from two buffers), so the
    results agree to rounding, not bit for bit; each is checked against the oracle as well."""
    cfg = CONFIGS[3].replace(batch=3, kv_len=(100, 700), new_len=(30, 200))
    d = workloads.prefill_inputs(cfg, seed=41)
    a = check_prefill(ctx, cfg, d, "split-sources", new_in_cache=False)
    b = check_prefill(ctx, cfg, d, "in-cache", new_in_cache=True)
    diff = np.abs(oracle.widen(a, cfg.dtype) - oracle.widen(b, cfg.dtype)).max()
    say("  max abs difference between the two calls", float(diff))
    assert diff <= TOL[cfg.dtype] / 2


def test_causality_on_gpu(ctx):
    """Dropping the last new token changes no earlier output row (bitwise)."""
    cfg, d = with_lens(CONFIGS[3], [200], [90], seed=23)
    full = check_prefill(ctx, cfg, d, "causal-full")
    cfg2, d2 = with_lens(CONFIGS[3], [200], [89], seed=23)
    np.testing.assert_array_equal(d2["q_new"], d["q_new"][:89])
    part = check_prefill(ctx, cfg2, d2, "causal-part")
    np.testing.assert_array_equal(full[:89], part)


def sampled_rows_check(cfg, d, got, rows_per_request=3):
    """Oracle on sampled new tokens: row i equals decode with q_i over the first P+i+1 keys."""
    w = lambda x: oracle.widen(x, cfg.dtype)
    cu = d["cu_seqlens"]
    worst = 0.0
    for b in range(cfg.batch):
        n, P = int(d["new_lens"][b]), int(d["prefix_lens"][b])
        kc = np.concatenate([w(d["k"][b]), w(d["k_new"][cu[b]:cu[b + 1]])])
        vc = np.concatenate([w(d["v"][b]), w(d["v_new"][cu[b]:cu[b + 1]])])
        for i in sorted({0, n // 2, n - 1})[:rows_per_request]:
            ref = oracle.decode(w(d["q_new"][cu[b] + i])[None], [kc[: P + i + 1]], [vc[: P + i + 1]], cfg.scale)[0]
            worst = max(worst, float(np.abs(w(got[cu[b] + i]) - ref).max()))
    return worst


def test_config4_multiturn_full_size_then_extend_and_decode(ctx):
    """Config 4 at full size: prefix-prefill over 8K-32K token histories (every output row against the oracle),
    then vt_extend grows each request by its new turn, the rows are appended, and one decode step runs over
    the extended cache (checked on every output)."""
    cfg = CONFIGS[4]
    d = workloads.prefill_inputs(cfg, threads=16)
    say("config4: P", d["prefix_lens"].tolist(), "N", d["new_lens"].tolist())
    reg = Regions(ctx, d["k"], d["v"], cfg.dtype, max_tokens=cfg.kv_len[1] + cfg.new_len[1] + 1)
    try:
        base = reg.k_ptrs.clone()
        got = run_prefill(ctx, cfg.dtype, d, reg.k_ptrs, reg.v_ptrs, cfg.n_kv_heads, cfg.scale)
        assert np.isfinite(oracle.widen(got, cfg.dtype)).all()
        say("  oracle over all", int(d["cu_seqlens"][-1]), "new tokens ...")
        ref_all = oracle_prefill(cfg, d)
        err = float(np.abs(oracle.widen(got, cfg.dtype) - ref_all).max())
        say("  prefill max abs err over every output row", err)
        assert err <= TOL[cfg.dtype]
        # (the same rows once more by the other route: row i = decode with q_i over its visible keys)
        assert sampled_rows_check(cfg, d, got) <= TOL[cfg.dtype]
        # grow every request by its new turn and write the rows
        cu = d["cu_seqlens"]
        new_total = (d["prefix_lens"] + d["new_lens"]).astype(np.int64)
        vt.vt_extend_batch(reg.kvs, new_total.tolist())
        for b, kv in enumerate(reg.kvs):
            vt.vt_append(kv, dev_bits(d["k_new"][cu[b]:cu[b + 1]]), dev_bits(d["v_new"][cu[b]:cu[b + 1]]),
                         int(d["new_lens"][b]), int(d["prefix_lens"][b]), stream())
            info = vt.vt_query(kv)
            assert info.len == new_total[b]
            assert info.chunks_mapped == meta.chunks_for_len(int(new_total[b]), cfg.n_kv_heads, cfg.head_dim)
        torch.cuda.synchronize()
        reg.refresh()
        assert torch.equal(reg.k_ptrs, base)
        # one decode step over the extended cache
        q = np.stack([workloads.normal_bits(d["seed"], workloads.gen.T_STEP_Q, b, (cfg.n_q_heads, cfg.head_dim),
                                            cfg.dtype) for b in range(cfg.batch)])
        out = run_decode(ctx, cfg.dtype, q, reg.k_ptrs, reg.v_ptrs, reg.lens, cfg.n_kv_heads, cfg.scale)
        w = lambda x: oracle.widen(x, cfg.dtype)
        kc = [np.concatenate([w(d["k"][b]), w(d["k_new"][cu[b]:cu[b + 1]])]) for b in range(cfg.batch)]
        vc = [np.concatenate([w(d["v"][b]), w(d["v_new"][cu[b]:cu[b + 1]])]) for b in range(cfg.batch)]
        ref = oracle.decode(w(q), kc, vc, cfg.scale)
        derr = float(np.abs(w(out) - ref).max())
        say("  decode after extend max abs err", derr)
        assert derr <= TOL[cfg.dtype]
        # the prefill in "rows already in cache" mode now sees the same keys (tiled differently: agreement to
        # rounding, and the same sampled rows against the oracle)
        again = run_prefill(ctx, cfg.dtype, d, reg.k_ptrs, reg.v_ptrs, cfg.n_kv_heads, cfg.scale, new_in_cache=True)
        assert np.isfinite(w(again)).all()
        err2 = float(np.abs(w(again) - ref_all).max())
        diff = float(np.abs(w(again) - w(got)).max())
        say("  in-cache prefill max abs err over every row", err2, "max abs difference to the first call", diff)
        assert err2 <= TOL[cfg.dtype] and diff <= TOL[cfg.dtype] / 2
    finally:
        reg.release()


@pytest.mark.parametrize("dtype,boost,where", [("bf16", 40.0, 250), ("f16", 6.0, 250), ("bf16", 40.0, 0),
                                               ("f16", 6.0, 3), ("bf16", 40.0, 299)])
def test_scores_far_above_the_first_keys(ctx, dtype, boost, where):
    """One cached key whose score exceeds everything seen before it by hundreds of units: the kernel's fast
    path works with reference maxima fixed after the first keys and must notice that its weights overflow
    (key late in the prefix) or simply underflow the rest (key among the first ones); either way the result is
    the oracle's, which is dominated by that key's value row."""
    cfg, d = with_lens(CONFIGS[3].replace(dtype=dtype), [300, 200], [70, 130], seed=77)
    one = np.array([1.0], np.float32)
    bits = lambda x: workloads.gen._round_bits(np.full((cfg.n_kv_heads, cfg.head_dim), x, np.float32), dtype)
    half = oracle.widen(bits(0.5), dtype)[0, 0]
    assert half == 0.5
    # queries get a +0.5 offset in every coordinate, key `where` of request 0 is boost in every coordinate
    q = oracle.widen(d["q_new"], dtype) + 0.5
    d["q_new"] = workloads.gen._round_bits(q.astype(np.float32), dtype)
    d["k"][0][where] = bits(boost)
    got = check_prefill(ctx, cfg, d, "dominant-key-%d" % where)
    want = oracle.widen(d["v"][0][where], dtype)                      # [Hkv, D]
    rows = oracle.widen(got[: 70], dtype)                             # request 0, all heads
    G = cfg.n_q_heads // cfg.n_kv_heads
    assert np.abs(rows - np.repeat(want, G, axis=0)[None]).max() <= TOL[dtype]


@pytest.mark.parametrize("scale", [-0.2, 0.0, 1.5])
def test_any_finite_scale(ctx, scale):
    """Negative (the smallest score weighs most), zero (plain mean of the visible value rows) and large scales follow
    the same definition."""
    cfg = CONFIGS[3].replace(batch=3, kv_len=(0, 500), new_len=(1, 200))
    check_prefill(ctx, cfg, workloads.prefill_inputs(cfg, seed=52), "scale %g" % scale, scale=scale)
    cfg = cfg.replace(dtype="f16", head_dim=64, n_q_heads=6, n_kv_heads=2)
    check_prefill(ctx, cfg, workloads.prefill_inputs(cfg, seed=53), "scale %g f16" % scale, new_in_cache=True, scale=scale)


@pytest.mark.parametrize("gap,where", [(15.0, 0), (18.0, 17), (21.5, 31), (21.5, 3), (24.0, 9), (30.0, 30)])
def test_fp16_outlier_among_the_first_keys_of_a_long_prefix(ctx, gap, where):
    """fp16 weights have a short exponent range.  One of the first 32 cached keys scores `gap` log2 units above all
    the others, which all score 0, and there are 20000 of them with value rows of ones against the outlier's zeros:
    the output is w / (1 + w) in every coordinate with w = 20000 * 2^-gap, and a kernel that fixes its reference
    maximum on the first keys must not flush the small weights to zero (w = 0.007 at gap 21.5 is above the tolerance)."""
    P, N, dtype = 20000, 70, "f16"
    cfg, d = with_lens(CONFIGS[3].replace(dtype=dtype, n_q_heads=4, n_kv_heads=1), [P], [N], seed=88)
    f16 = lambda x: np.asarray(x, np.float16).view(np.uint16)
    d["q_new"][:] = f16(0.5)
    d["k"][0][:] = f16(0.0)
    d["k_new"][:] = f16(0.0)
    d["v"][0][:] = f16(1.0)
    d["v_new"][:] = f16(1.0)
    c = gap / (1.4426950408889634 * 64.0 * cfg.scale)             # score = c * sum(q) * scale, in log2 units: gap
    d["k"][0][where] = f16(c)
    d["v"][0][where] = f16(0.0)
    got = check_prefill(ctx, cfg, d, "fp16-outlier gap %g at %d" % (gap, where))
    c_exact = float(np.float16(c))
    i = np.arange(N)
    w = (P + i) * np.exp(-c_exact * 64.0 * cfg.scale)       # P + i keys of score 0 beside the outlier (score 64 c scale)
    want = (w / (1.0 + w))[:, None, None]
    err = float(np.abs(oracle.widen(got, dtype) - want).max())
    say("  max abs err against the closed form", err)
    assert err <= TOL[dtype]


def test_bad_arguments_are_refused(ctx):
    t = torch.zeros(4, 8, 128, dtype=torch.int16).cuda()
    cu, pl = np.array([0, 4], np.int32), np.array([3], np.int32)
    ok = dict(dtype=vt.VT_BF16, batch=1, n_q_heads=8, n_kv_heads=8, head_dim=128, scale=0.1, total_new_tokens=4,
              q_new=t, out=t, k_new=t, v_new=t, k_ptrs=t, v_ptrs=t, cu_seqlens=t, prefix_lens=t, cu_seqlens_host=cu,
              prefix_lens_host=pl)
    for change, status in ((dict(v_new=None), vt.VT_E_INVALID), (dict(head_dim=80), vt.VT_E_UNSUPPORTED),
                           (dict(total_new_tokens=5), vt.VT_E_INVALID), (dict(n_kv_heads=5), vt.VT_E_INVALID),
                           (dict(prefix_lens_host=np.array([-1], np.int32)), vt.VT_E_INVALID),
                           (dict(out=None), vt.VT_E_INVALID), (dict(scale=float("nan")), vt.VT_E_INVALID),
                           (dict(scale=float("-inf")), vt.VT_E_INVALID)):
        with pytest.raises(vt.VtError) as e:
            vt.vt_attn_prefix_prefill(ctx, vt.make_prefill_args(**dict(ok, **change)), stream())
        assert e.value.status == status, change
