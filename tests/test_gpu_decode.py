"""GPU parity of vt_attn_decode (through the C ABI) against the fp64 oracle, plus region behaviour on the
device: contiguity over scattered chunks, base-pointer stability, bit-identity with plain device memory."""

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

from gpu_util import TOL, Regions, dev_bits, host_bits, read_device, run_decode, stream  # noqa: E402


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def ctx():
    c = vt.vt_init(0, 0, 0)
    yield c
    torch.cuda.synchronize()
    vt.vt_destroy(c)


def oracle_decode(cfg, data, scale=None):
    q = oracle.widen(data["q"], cfg.dtype)
    k = [oracle.widen(x, cfg.dtype) for x in data["k"]]
    v = [oracle.widen(x, cfg.dtype) for x in data["v"]]
    return oracle.decode(q, k, v, cfg.scale if scale is None else scale)


def check_decode(ctx, cfg, data, tag, scale=None):
    say("decode case", tag, "dtype", cfg.dtype, "B", cfg.batch, "Hq/Hkv", cfg.n_q_heads, cfg.n_kv_heads, "D",
        cfg.head_dim, "lens", data["kv_lens"][:8].tolist(), "seed", data["seed"])
    reg = Regions(ctx, data["k"], data["v"], cfg.dtype)
    try:
        got = run_decode(ctx, cfg.dtype, data["q"], reg.k_ptrs, reg.v_ptrs, reg.lens, cfg.n_kv_heads,
                         cfg.scale if scale is None else scale)
    finally:
        reg.release()
    ref = oracle_decode(cfg, data, scale)
    err = np.abs(oracle.widen(got, cfg.dtype) - ref)
    say("  max abs err", float(err.max()), "tolerance", TOL[cfg.dtype])
    assert np.isfinite(oracle.widen(got, cfg.dtype)).all()
    assert err.max() <= TOL[cfg.dtype]
    return got


def with_lens(cfg, lens, seed=11):
    """Decode inputs of `cfg`'s shape with the given per-request lengths."""
    cfg = cfg.replace(batch=len(lens))
    d = workloads.decode_inputs(cfg, seed=seed)
    for b, L in enumerate(lens):
        shp = (L, cfg.n_kv_heads, cfg.head_dim)
        d["k"][b] = workloads.normal_bits(seed, workloads.gen.T_K, b, shp, cfg.dtype)
        d["v"][b] = workloads.normal_bits(seed, workloads.gen.T_V, b, shp, cfg.dtype)
    d["kv_lens"] = np.array(lens, dtype=np.int32)
    return cfg, d


def test_config1_fp16_small(ctx):
    cfg = CONFIGS[1]
    check_decode(ctx, cfg, workloads.decode_inputs(cfg), "config1")


def test_config2_bf16_mha_full(ctx):
    cfg = CONFIGS[2]
    data = workloads.decode_inputs(cfg)
    assert meta.decode_kv_bytes(data["kv_lens"], 32, 128) > 1.5e9
    check_decode(ctx, cfg, data, "config2")


@pytest.mark.parametrize("dtype,hq,hkv,d", [
    ("bf16", 32, 8, 128), ("bf16", 64, 8, 128), ("bf16", 32, 2, 128), ("bf16", 32, 4, 128), ("f16", 32, 8, 128),
    ("bf16", 16, 8, 64), ("f16", 24, 3, 64), ("bf16", 5, 1, 128), ("f16", 6, 6, 128), ("bf16", 14, 7, 64),
    # groups of more than 16 query heads (multi-query attention with 32 heads, 40 = 16 + 16 + 8, 17 = 16 + 1)
    ("bf16", 32, 1, 128), ("f16", 40, 1, 64), ("bf16", 64, 2, 128), ("bf16", 34, 2, 128),
])
def test_head_group_shapes(ctx, dtype, hq, hkv, d):
    cfg = CONFIGS[2].replace(dtype=dtype, batch=5, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, kv_len=(1, 700))
    check_decode(ctx, cfg, workloads.decode_inputs(cfg, seed=1000 + hq * 7 + hkv), "shapes")


def random_shape(rng):
    """A seeded draw of (dtype, Hq, Hkv, D): every group size the kernels special-case turns up over the seeds."""
    dtype = ("bf16", "f16")[int(rng.integers(2))]
    d = (64, 128)[int(rng.integers(2))]
    hkv = int(rng.choice([1, 2, 3, 4, 8]))
    g = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 17, 24]))
    return dtype, hkv * g, hkv, d


def edge_biased_length(rng, unit, hi):
    """A length in [1, hi]: half the draws sit within 2 of a multiple of `unit` (tile and span edges)."""
    if rng.integers(2):
        return int(np.clip(unit * rng.integers(1, max(2, hi // unit + 1)) + rng.integers(-2, 3), 1, hi))
    return int(rng.integers(1, hi + 1))


@pytest.mark.parametrize("seed", range(10))
def test_seeded_random_shapes_and_lengths(ctx, seed):
    rng = np.random.default_rng(9000 + seed)
    dtype, hq, hkv, d = random_shape(rng)
    lens = [edge_biased_length(rng, 128, 1500) for _ in range(int(rng.integers(1, 7)))]
    cfg, data = with_lens(CONFIGS[1].replace(dtype=dtype, n_q_heads=hq, n_kv_heads=hkv, head_dim=d), lens,
                          seed=700 + seed)
    check_decode(ctx, cfg, data, "random")


def test_edge_lengths_around_tiles_and_spans(ctx):
    lens = [1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 1023, 1024, 1025]
    cfg, d = with_lens(CONFIGS[2].replace(n_q_heads=8, n_kv_heads=4), lens)
    check_decode(ctx, cfg, d, "edges")
    cfg, d = with_lens(CONFIGS[1], lens[:12], seed=12)
    check_decode(ctx, cfg, d, "edges-f16-d64")


def test_plans_with_few_and_many_segments(ctx):
    """The result does not depend on how the tape is cut: few long segments (pieces span several requests) and
    many short ones (a request is cut into dozens of pieces) both match the oracle."""
    cfg, d = with_lens(CONFIGS[2].replace(n_q_heads=16, n_kv_heads=4), [3000, 517, 9000, 33, 1])
    try:
        for slots in (4, 8, 64, 100000):
            vt.vt_set_plan_target(ctx, slots)
            plan, ns = vt.vt_plan_decode(ctx, d["kv_lens"], 4, 16, 128)
            want = meta.decode_plan(d["kv_lens"], 4, slots)
            assert (plan.span_tokens, ns.tolist(), plan.max_splits, plan.n_units) == want
            say("slots", slots, "segment", plan.span_tokens, "pieces", ns.tolist())
            check_decode(ctx, cfg, d, "tape-split")
    finally:
        vt.vt_set_plan_target(ctx, 0)


def plain_memory_case(cfg, lens, seed):
    """Decode inputs whose K/V rows live in ONE plain device allocation (to the kernel a pointer is a pointer):
    request b's rows start at slot b * max(lens).  Returns (data, k_ptrs, v_ptrs, keep-alive tensors)."""
    B, hkv, d = len(lens), cfg.n_kv_heads, cfg.head_dim
    Lmax = int(max(lens))
    k_all = workloads.normal_bits(seed, workloads.gen.T_K, 0, (B, Lmax, hkv, d), cfg.dtype)
    v_all = workloads.normal_bits(seed, workloads.gen.T_V, 0, (B, Lmax, hkv, d), cfg.dtype)
    q = workloads.normal_bits(seed, workloads.gen.T_Q, 0, (B, cfg.n_q_heads, d), cfg.dtype)
    kd, vd = dev_bits(k_all), dev_bits(v_all)
    stride = Lmax * hkv * d * 2
    kp = torch.tensor([kd.data_ptr() + b * stride for b in range(B)], dtype=torch.int64).cuda()
    vp = torch.tensor([vd.data_ptr() + b * stride for b in range(B)], dtype=torch.int64).cuda()
    data = {"q": q, "k": [k_all[b, :L] for b, L in enumerate(lens)], "v": [v_all[b, :L] for b, L in enumerate(lens)],
            "kv_lens": np.array(lens, np.int32), "seed": seed}
    return data, kp, vp, (kd, vd)


def test_largest_admitted_batch(ctx):
    """Batch 4096, the most requests one launch takes (the table of tape positions has 4097 entries, the last one the
    tape's total), with tiny lengths; one more request is refused."""
    cfg = CONFIGS[1].replace(n_q_heads=4, n_kv_heads=2)
    rng = np.random.default_rng(4096)
    for B in (4096, 4095, 257, 256, 255):
        lens = rng.integers(1, 6, size=B).tolist()
        data, kp, vp, keep = plain_memory_case(cfg, lens, seed=4000 + B)
        say("decode case largest-batch B", B, "sum(L)", sum(lens))
        got = run_decode(ctx, cfg.dtype, data["q"], kp, vp, data["kv_lens"], cfg.n_kv_heads, cfg.scale)
        ref = oracle_decode(cfg.replace(batch=B), data)
        err = np.abs(oracle.widen(got, cfg.dtype) - ref)
        say("  max abs err", float(err.max()))
        assert err.max() <= TOL[cfg.dtype]
        plan, ns = vt.vt_plan_decode(ctx, data["kv_lens"], 2, 4, 64)
        assert (plan.span_tokens, ns.tolist(), plan.max_splits, plan.n_units) == meta.decode_plan(lens, 2, n_q_heads=4)
    lens = [1] * 4097
    data, kp, vp, keep = plain_memory_case(cfg, lens, seed=1)
    with pytest.raises(vt.VtError) as e:
        run_decode(ctx, cfg.dtype, data["q"], kp, vp, data["kv_lens"], cfg.n_kv_heads, cfg.scale)
    assert e.value.status == vt.VT_E_UNSUPPORTED


@pytest.mark.parametrize("scale", [-0.3, 0.0, 2.5])
def test_any_finite_scale(ctx, scale):
    """The scale is an argument of the problem statement: negative (the smallest score weighs most), zero (plain mean
    of the value rows) and large ones follow the same definition; a non-finite one is refused."""
    cfg = CONFIGS[1].replace(batch=3, kv_len=(1, 300))
    check_decode(ctx, cfg, workloads.decode_inputs(cfg, seed=77), "scale %g" % scale, scale=scale)
    d = workloads.decode_inputs(cfg, seed=77)
    for bad in (float("nan"), float("inf")):
        with pytest.raises(vt.VtError) as e:
            reg = Regions(ctx, d["k"], d["v"], cfg.dtype)
            try:
                run_decode(ctx, cfg.dtype, d["q"], reg.k_ptrs, reg.v_ptrs, reg.lens, cfg.n_kv_heads, bad)
            finally:
                reg.release()
        assert e.value.status == vt.VT_E_INVALID


def test_paper_sweep_point_16k_batch16_gqa_32_4(ctx):
    """One full point of the paper-shaped sweeps (KV length 16384, batch 16, the paper's default 32 query / 4 KV
    heads), every output against the oracle; and batch 1 at the same length, where the request is cut into hundreds
    of pieces and the merge kernel's many-wavefront path runs."""
    cfg = CONFIGS[2].replace(batch=16, n_q_heads=32, n_kv_heads=4, kv_len=(16384, 16384))
    check_decode(ctx, cfg, workloads.decode_inputs(cfg, seed=1604, threads=16), "sweep d1/d2 point")
    cfg1 = cfg.replace(batch=1)
    d1 = workloads.decode_inputs(cfg1, seed=1605)
    plan, ns = vt.vt_plan_decode(ctx, d1["kv_lens"], 4, 32, 128)
    assert ns.max() > 16                       # more pieces than the four-wavefront merge takes
    check_decode(ctx, cfg1, d1, "sweep d1 batch 1")
    cfg2 = cfg.replace(batch=3, dtype="f16", head_dim=64, n_q_heads=8, n_kv_heads=8, kv_len=(5000, 9000))
    check_decode(ctx, cfg2, workloads.decode_inputs(cfg2, seed=1606), "many pieces f16 d64")


def test_vmm_region_equals_plain_device_memory_bit_for_bit(ctx):
    """To a kernel a region is an ordinary pointer (paper "vTensor"): same bytes, same result bits."""
    cfg = CONFIGS[2].replace(batch=6, n_q_heads=32, n_kv_heads=8, kv_len=(300, 3000))
    data = workloads.decode_inputs(cfg, seed=77)
    reg = Regions(ctx, data["k"], data["v"], cfg.dtype)
    try:
        a = run_decode(ctx, cfg.dtype, data["q"], reg.k_ptrs, reg.v_ptrs, reg.lens, cfg.n_kv_heads, cfg.scale)
    finally:
        reg.release()
    kt = [dev_bits(x) for x in data["k"]]
    vt_ = [dev_bits(x) for x in data["v"]]
    kp = torch.tensor([t.data_ptr() for t in kt], dtype=torch.int64).cuda()
    vp = torch.tensor([t.data_ptr() for t in vt_], dtype=torch.int64).cuda()
    b = run_decode(ctx, cfg.dtype, data["q"], kp, vp, data["kv_lens"], cfg.n_kv_heads, cfg.scale)
    np.testing.assert_array_equal(a, b)


def test_region_is_contiguous_over_scattered_chunks_on_device(ctx):
    hkv, d = 8, 128                                      # 2 KiB rows, 1024 rows per 2 MiB chunk
    a = vt.vt_reserve(ctx, hkv, d, vt.VT_BF16, 8192)
    vt.vt_extend(a, 5 * 1024)
    vt.vt_release(a)                                     # 10 chunks into the pool
    b = vt.vt_reserve(ctx, hkv, d, vt.VT_BF16, 8192)
    L = 3 * 1024 + 7
    vt.vt_extend(b, L)                                   # 4 + 4 chunks, pool first
    info = vt.vt_query(b)
    assert info.chunks_mapped == meta.chunks_for_len(L, hkv, d) == 4
    assert info.k_ptr % (2 << 20) == 0 and info.capacity_bytes == meta.capacity_bytes(8192, hkv, d)
    rng = np.random.default_rng(3)
    rows = rng.integers(0, 65535, size=(L, hkv, d), dtype=np.uint16)
    rows_v = rng.integers(0, 65535, size=(L, hkv, d), dtype=np.uint16)
    vt.vt_append(b, dev_bits(rows), dev_bits(rows_v), L, 0, stream())
    np.testing.assert_array_equal(read_device(info.k_ptr, L * 2048).view(np.uint16).reshape(L, hkv, d), rows)
    np.testing.assert_array_equal(read_device(info.v_ptr, L * 2048).view(np.uint16).reshape(L, hkv, d), rows_v)
    vt.vt_release(b)


def test_extend_changes_no_prior_output_and_never_moves_the_base(ctx):
    """Appending via vt_extend leaves decode over the old length bit-identical, also when the extension is
    issued while a decode kernel over the old rows is still in flight (paper "vTensor Scheduler", Extend)."""
    cfg = CONFIGS[2].replace(batch=4, n_q_heads=32, n_kv_heads=8, kv_len=(900, 1100))
    data = workloads.decode_inputs(cfg, seed=5)
    reg = Regions(ctx, data["k"], data["v"], cfg.dtype, max_tokens=4096)
    try:
        old = reg.lens.copy()
        k0, v0 = reg.k_ptrs.clone(), reg.v_ptrs.clone()
        before = run_decode(ctx, cfg.dtype, data["q"], reg.k_ptrs, reg.v_ptrs, old, cfg.n_kv_heads, cfg.scale)
        # launch again and extend across a chunk boundary while it runs
        q = dev_bits(data["q"])
        out = torch.zeros_like(q)
        lens_dev = torch.from_numpy(old).cuda()
        args = vt.make_decode_args(vt.VT_BF16, cfg.batch, 32, 8, 128, cfg.scale, q, out, reg.k_ptrs, reg.v_ptrs,
                                   lens_dev, old)
        vt.vt_attn_decode(ctx, args, stream())
        vt.vt_extend_batch(reg.kvs, [int(x) + 1500 for x in old])
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host_bits(out), before)
        reg.refresh()
        assert torch.equal(reg.k_ptrs, k0) and torch.equal(reg.v_ptrs, v0)
        for kv, L in zip(reg.kvs, old):
            info = vt.vt_query(kv)
            assert info.len == L + 1500 and info.chunks_mapped == meta.chunks_for_len(int(L) + 1500, 8, 128)
        after = run_decode(ctx, cfg.dtype, data["q"], reg.k_ptrs, reg.v_ptrs, old, cfg.n_kv_heads, cfg.scale)
        np.testing.assert_array_equal(after, before)
    finally:
        reg.release()


def test_decode_invariants_on_gpu(ctx):
    """Key permutation leaves the output unchanged within tolerance; identical V rows return that row."""
    cfg = CONFIGS[2].replace(batch=2, n_q_heads=8, n_kv_heads=2, kv_len=(200, 400))
    data = workloads.decode_inputs(cfg, seed=9)
    a = check_decode(ctx, cfg, data, "perm-base")
    rng = np.random.default_rng(1)
    perm = [rng.permutation(len(x)) for x in data["k"]]
    data2 = dict(data, k=[x[p] for x, p in zip(data["k"], perm)], v=[x[p] for x, p in zip(data["v"], perm)])
    b = check_decode(ctx, cfg, data2, "perm-shuffled")
    assert np.abs(oracle.widen(a, "bf16") - oracle.widen(b, "bf16")).max() <= TOL["bf16"]
    row = workloads.normal_bits(3, 4, 0, (1, 2, 128), "bf16")
    data3 = dict(data, v=[np.broadcast_to(row, x.shape).copy() for x in data["v"]])
    c = check_decode(ctx, cfg, data3, "same-v-rows")
    want = np.repeat(oracle.widen(row[0], "bf16"), 4, axis=0)
    assert np.abs(oracle.widen(c, "bf16") - want[None]).max() <= 2.0 ** -7 * np.abs(want).max()


def test_bad_arguments_are_refused(ctx):
    q = torch.zeros(1, 8, 128, dtype=torch.int16).cuda()
    lens = np.array([4], np.int32)
    ok = dict(dtype=vt.VT_BF16, batch=1, n_q_heads=8, n_kv_heads=8, head_dim=128, scale=0.1, q=q, out=q, k_ptrs=q,
              v_ptrs=q, kv_lens=q, kv_lens_host=lens)
    for change, status in ((dict(n_kv_heads=3), vt.VT_E_INVALID), (dict(head_dim=96), vt.VT_E_UNSUPPORTED),
                           (dict(q=None), vt.VT_E_INVALID), (dict(dtype=9), vt.VT_E_INVALID),
                           (dict(n_q_heads=8 * 257, n_kv_heads=8), vt.VT_E_UNSUPPORTED),
                           (dict(kv_lens_host=np.array([0], np.int32)), vt.VT_E_INVALID)):
        with pytest.raises(vt.VtError) as e:
            vt.vt_attn_decode(ctx, vt.make_decode_args(**dict(ok, **change)), stream())
        assert e.value.status == status, change


def test_steady_state_decode_steps_with_extend_and_append(ctx):
    """Config-5-shaped loop at reduced batch: each step extends every request by one token, appends the new
    K/V rows with one launch, then decodes over the extended cache; metadata is checked every step."""
    cfg = CONFIGS[5].replace(batch=6, kv_len=(1000, 1030), steps=40)
    data = workloads.decode_inputs(cfg)
    k = [oracle.widen(x, cfg.dtype) for x in data["k"]]
    v = [oracle.widen(x, cfg.dtype) for x in data["v"]]
    reg = Regions(ctx, data["k"], data["v"], cfg.dtype, max_tokens=8192 + cfg.steps)
    try:
        k0 = reg.k_ptrs.clone()
        lens = reg.lens.copy()
        for step in range(cfg.steps):
            si = workloads.step_inputs(cfg, step)
            lens = lens + 1
            vt.vt_extend_batch(reg.kvs, lens.tolist())
            lens_dev = torch.from_numpy(lens).cuda()
            vt.vt_append_batch(ctx, reg.k_ptrs, reg.v_ptrs, lens_dev, dev_bits(si["k_row"]), dev_bits(si["v_row"]),
                               cfg.batch, cfg.n_kv_heads, cfg.head_dim, stream())
            got = run_decode(ctx, cfg.dtype, si["q"], reg.k_ptrs, reg.v_ptrs, lens, cfg.n_kv_heads, cfg.scale,
                             lens_dev)
            for b in range(cfg.batch):
                k[b] = np.concatenate([k[b], oracle.widen(si["k_row"][b], cfg.dtype)[None]])
                v[b] = np.concatenate([v[b], oracle.widen(si["v_row"][b], cfg.dtype)[None]])
                info = vt.vt_query(reg.kvs[b])
                assert info.len == lens[b] and info.chunks_mapped == meta.chunks_for_len(int(lens[b]), 8, 128)
            ref = oracle.decode(oracle.widen(si["q"], cfg.dtype), k, v, cfg.scale)
            err = np.abs(oracle.widen(got, cfg.dtype) - ref).max()
            assert err <= TOL[cfg.dtype], (step, err)
        assert torch.equal(reg.k_ptrs, k0)
        say("steady-state", cfg.steps, "steps ok; chunk crossings:",
            sum(int(meta.chunks_for_len(int(L), 8, 128) > meta.chunks_for_len(int(L) - cfg.steps, 8, 128)) for L in lens))
    finally:
        reg.release()


def test_config5_full_size_all_32_steps(ctx):
    """Config 5 at full size (batch 256, 64/8 heads, lengths 1024..8192): all 32 decode steps, each extending every
    request by one token and appending its K/V row; every output of every step is compared with the oracle, the
    split plan with its rule, and the region metadata with its closed forms."""
    cfg = CONFIGS[5]
    data = workloads.decode_inputs(cfg, threads=16)
    say("config5: sum(L)", int(data["kv_lens"].sum()), "bytes/step", meta.decode_kv_bytes(data["kv_lens"], 8, 128))
    reg = Regions(ctx, data["k"], data["v"], cfg.dtype, max_tokens=cfg.kv_len[1] + cfg.steps)
    try:
        lens = reg.lens.copy()
        # fp64 copies of the caches with room for the rows of all steps, appended in place
        def grown(x):
            a = np.empty((x.shape[0] + cfg.steps,) + x.shape[1:], np.float64)
            a[: x.shape[0]] = oracle.widen(x, cfg.dtype)
            return a
        k = [grown(x) for x in data["k"]]
        v = [grown(x) for x in data["v"]]
        crossings, worst = 0, 0.0
        for step in range(cfg.steps):
            si = workloads.step_inputs(cfg, step)
            lens = lens + 1
            vt.vt_extend_batch(reg.kvs, lens.tolist())
            lens_dev = torch.from_numpy(lens).cuda()
            vt.vt_append_batch(ctx, reg.k_ptrs, reg.v_ptrs, lens_dev, dev_bits(si["k_row"]), dev_bits(si["v_row"]),
                               cfg.batch, cfg.n_kv_heads, cfg.head_dim, stream())
            got = run_decode(ctx, cfg.dtype, si["q"], reg.k_ptrs, reg.v_ptrs, lens, cfg.n_kv_heads, cfg.scale, lens_dev)
            plan, pieces = vt.vt_plan_decode(ctx, lens, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim)
            assert (plan.span_tokens, pieces.tolist(), plan.max_splits, plan.n_units) == meta.decode_plan(lens, 8)
            kr, vr = oracle.widen(si["k_row"], cfg.dtype), oracle.widen(si["v_row"], cfg.dtype)
            for b in range(cfg.batch):
                k[b][lens[b] - 1] = kr[b]
                v[b][lens[b] - 1] = vr[b]
                info = vt.vt_query(reg.kvs[b])
                assert info.len == lens[b] and info.chunks_mapped == meta.chunks_for_len(int(lens[b]), 8, 128)
                crossings += int(meta.chunks_for_len(int(lens[b]), 8, 128) > meta.chunks_for_len(int(lens[b]) - 1, 8, 128))
            ref = oracle.decode(oracle.widen(si["q"], cfg.dtype), [k[b][: lens[b]] for b in range(cfg.batch)],
                                [v[b][: lens[b]] for b in range(cfg.batch)], cfg.scale)
            err = float(np.abs(oracle.widen(got, cfg.dtype) - ref).max())
            worst = max(worst, err)
            say("  step", step, "max abs err", err)
            assert err <= TOL[cfg.dtype]
        say("config5: 32 steps ok, worst err", worst, "chunk boundaries crossed", crossings)
    finally:
        reg.release()


def test_prefix_sharing_maps_the_same_chunks_into_a_second_region(ctx):
    """Prefix match by aliasing (paper "vTensor Scheduler", Prefix Record and Match): the second request's region starts with the SAME physical
    chunks as the first one's - no copy, no new memory - then grows privately; decode over the shared prefix gives
    identical bits through either region."""
    cfg = CONFIGS[5].replace(batch=1, kv_len=(2048, 2048))      # 2 chunks of 1024 rows per region
    data = workloads.decode_inputs(cfg, seed=91)
    reg = Regions(ctx, data["k"], data["v"], cfg.dtype, max_tokens=4096)
    dst = None
    try:
        phys = vt.vt_stats(ctx).phys_bytes
        try:
            dst = vt.vt_share_prefix(reg.kvs[0], 2048, 4096)
        except vt.VtError as e:
            if e.status == vt.VT_E_DRIVER:
                pytest.skip("the driver refused to map a chunk at a second address")
            raise
        assert vt.vt_stats(ctx).phys_bytes == phys               # nothing allocated
        info = vt.vt_query(dst)
        assert info.len == 2048 and info.shared_chunks == 2 and info.k_ptr != vt.vt_query(reg.kvs[0]).k_ptr
        lens = np.array([2048], np.int32)
        a = run_decode(ctx, cfg.dtype, data["q"], reg.k_ptrs, reg.v_ptrs, lens, cfg.n_kv_heads, cfg.scale)
        kp = torch.tensor([info.k_ptr], dtype=torch.int64).cuda()
        vp = torch.tensor([info.v_ptr], dtype=torch.int64).cuda()
        b = run_decode(ctx, cfg.dtype, data["q"], kp, vp, lens, cfg.n_kv_heads, cfg.scale)
        np.testing.assert_array_equal(a, b)
        # the sharer grows on private chunks and decodes over prefix + its own rows
        extra = workloads.normal_bits(92, 3, 0, (100, 8, 128), cfg.dtype)
        extra_v = workloads.normal_bits(92, 4, 0, (100, 8, 128), cfg.dtype)
        before = vt.vt_stats(ctx)
        vt.vt_extend(dst, 2148)
        vt.vt_append(dst, dev_bits(extra), dev_bits(extra_v), 100, 2048, stream())
        after = vt.vt_stats(ctx)
        # one private chunk each for K and V, new or taken from the pool of released chunks
        assert (after.chunks_created + after.chunks_reused) - (before.chunks_created + before.chunks_reused) == 2
        assert after.mapped_bytes - before.mapped_bytes == 2 * (2 << 20)
        lens2 = np.array([2148], np.int32)
        got = run_decode(ctx, cfg.dtype, data["q"], kp, vp, lens2, cfg.n_kv_heads, cfg.scale)
        w = lambda x: oracle.widen(x, cfg.dtype)
        ref = oracle.decode(w(data["q"]), [np.concatenate([w(data["k"][0]), w(extra)])],
                            [np.concatenate([w(data["v"][0]), w(extra_v)])], cfg.scale)
        assert np.abs(w(got) - ref).max() <= TOL[cfg.dtype]
        # the owner is untouched
        c = run_decode(ctx, cfg.dtype, data["q"], reg.k_ptrs, reg.v_ptrs, lens, cfg.n_kv_heads, cfg.scale)
        np.testing.assert_array_equal(a, c)
    finally:
        torch.cuda.synchronize()
        if dst is not None:
            vt.vt_release(dst)
        reg.release()


def test_extension_overlaps_the_decode_steps(ctx):
    """Paper "vTensor Scheduler" (Extend) and "FlexInfer Scheduler": memory for coming tokens is extended while the current step computes.  A decode loop
    on a stream that does not synchronise with the default stream, (a) on regions extended beforehand, (b) with
    vt_extend_batch inside every step, (c) with the extension queued two steps ahead on the context's worker
    thread: the three produce identical bits, and the loops that extend take about as long as the one that does
    not (the mapping calls then run beside the kernels instead of draining the queue first; the times are printed,
    the benchmark reports them).  The last step of every mode is compared with the oracle."""
    import time
    cfg = CONFIGS[2].replace(batch=32, kv_len=(1500, 2560))
    data = workloads.decode_inputs(cfg, seed=123)
    steps, ahead = 40, 2
    B, hq, hkv, d = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    lens0 = data["kv_lens"].astype(np.int64)
    rows = [workloads.step_inputs(cfg, s) for s in range(steps)]
    results, times, maps = {}, {}, {}
    side = torch.cuda.Stream()
    for mode in ("pre", "sync", "async"):
        with torch.cuda.stream(side):
            reg = Regions(ctx, data["k"], data["v"], cfg.dtype, max_tokens=cfg.kv_len[1] + steps + ahead + 1)
            st = stream()
            q = dev_bits(data["q"])
            out = torch.zeros_like(q)
            outs = []
            k_rows = [dev_bits(r["k_row"]) for r in rows]
            v_rows = [dev_bits(r["v_row"]) for r in rows]
            lens_host = [np.ascontiguousarray((lens0 + s + 1).astype(np.int32)) for s in range(steps + ahead)]
            lens_dev = [torch.from_numpy(x).cuda() for x in lens_host]
            args = [vt.make_decode_args(vt.DTYPES[cfg.dtype], B, hq, hkv, d, cfg.scale, q, out, reg.k_ptrs, reg.v_ptrs,
                                        lens_dev[s], lens_host[s]) for s in range(steps)]
            plan, _ = vt.vt_plan_decode(ctx, lens_host[steps - 1], hkv, hq, d)
            vt.vt_workspace_reserve(ctx, plan.workspace_bytes)
            m0 = vt.vt_stats(ctx).map_calls
            tickets = {}
            if mode == "pre":
                vt.vt_extend_batch(reg.kvs, lens_host[steps - 1].tolist())
            if mode == "async":
                for s in range(ahead):
                    tickets[s] = vt.vt_extend_batch_async(reg.kvs, lens_host[s].tolist())
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for s in range(steps):
                if mode == "sync":
                    vt.vt_extend_batch(reg.kvs, lens_host[s].tolist())
                elif mode == "async":
                    vt.vt_extend_wait(ctx, tickets.pop(s))
                vt.vt_append_batch(ctx, reg.k_ptrs, reg.v_ptrs, lens_dev[s], k_rows[s], v_rows[s], B, hkv, d, st)
                vt.vt_attn_decode(ctx, args[s], st)
                if mode == "async" and s + ahead < steps:
                    tickets[s + ahead] = vt.vt_extend_batch_async(reg.kvs, lens_host[s + ahead].tolist())
                if s % 13 == 0 or s == steps - 1:
                    outs.append(out.clone())
            torch.cuda.synchronize()
            times[mode] = (time.perf_counter() - t0) / steps
            maps[mode] = vt.vt_stats(ctx).map_calls - m0
            results[mode] = [host_bits(o) for o in outs]
            reg.release()
    say("  per step: pre-extended %.1f us, extend in step %.1f us, extend ahead %.1f us; chunks mapped in the loops %s"
        % (times["pre"] * 1e6, times["sync"] * 1e6, times["async"] * 1e6, maps))
    assert maps["sync"] == maps["async"] and maps["sync"] >= 10      # the loops really map new chunks
    for a, b, c in zip(results["pre"], results["sync"], results["async"]):
        np.testing.assert_array_equal(a, b)
        np.testing.assert_array_equal(a, c)
    # the last step of every mode against the oracle: the caches as they are after all appended rows
    w = lambda x: oracle.widen(x, cfg.dtype)
    kf = [np.concatenate([w(data["k"][b])] + [w(r["k_row"][b])[None] for r in rows]) for b in range(B)]
    vf = [np.concatenate([w(data["v"][b])] + [w(r["v_row"][b])[None] for r in rows]) for b in range(B)]
    ref = oracle.decode(w(data["q"]), kf, vf, cfg.scale)
    for mode in ("pre", "sync", "async"):
        err = float(np.abs(w(results[mode][-1]) - ref).max())
        say("  last step of mode", mode, "max abs err", err)
        assert err <= TOL[cfg.dtype]


def test_lazy_release_and_trim_on_the_device(ctx):
    """Lazy deallocation and explicit emptying (paper, vTensor Operation: Deallocation; vTensor Scheduler: Release) on
    the HIP backend, on a context of its own: release keeps the physical chunks pooled and the ranges free-listed;
    vt_trim(k) really frees chunks beyond k and all idle ranges; after vt_trim(0) nothing is held and the next request
    creates again."""
    c = vt.vt_init(0, 0, 0)
    try:
        hkv, d, chunk = 8, 128, 2 << 20
        st0 = vt.vt_stats(c)
        assert (st0.phys_bytes, st0.reserved_va_bytes, st0.mapped_bytes, st0.chunks_pooled) == (0, 0, 0, 0)
        kvs = [vt.vt_reserve(c, hkv, d, vt.VT_BF16, 8192) for _ in range(3)]
        for kv, L in zip(kvs, (1024, 3000, 5000)):          # 1, 3 and 5 chunks per region
            vt.vt_extend(kv, L)
        n_chunks = 2 * sum(meta.chunks_for_len(L, hkv, d) for L in (1024, 3000, 5000))
        cap = meta.capacity_bytes(8192, hkv, d)
        st = vt.vt_stats(c)
        assert st.phys_bytes == st.mapped_bytes == n_chunks * chunk and st.chunks_created == n_chunks == 18
        assert st.reserved_va_bytes == 3 * 2 * cap and st.live_regions == 3
        # the rows are really there
        rows = workloads.normal_bits(5, 1, 0, (5000, hkv, d), "bf16")
        vt.vt_append(kvs[2], dev_bits(rows), dev_bits(rows), 5000, 0, stream())
        info = vt.vt_query(kvs[2])
        np.testing.assert_array_equal(read_device(info.v_ptr, 5000 * 2048).view(np.uint16).reshape(5000, hkv, d), rows)
        for kv in kvs:
            vt.vt_release(kv)
        st = vt.vt_stats(c)                                   # lazy: nothing given back yet
        assert st.phys_bytes == n_chunks * chunk and st.mapped_bytes == 0 and st.chunks_pooled == n_chunks
        assert st.reserved_va_bytes == 3 * 2 * cap and st.live_regions == 0 and st.release_calls == 0
        vt.vt_trim(c, 4)
        st = vt.vt_stats(c)
        assert st.chunks_pooled == 4 and st.phys_bytes == 4 * chunk and st.release_calls == n_chunks - 4
        assert st.reserved_va_bytes == 0 and st.va_free_calls == 6
        # a new request takes the 4 pooled chunks first and creates the rest, on newly reserved ranges
        kv = vt.vt_reserve(c, hkv, d, vt.VT_BF16, 8192)
        vt.vt_extend(kv, 3000)
        st2 = vt.vt_stats(c)
        assert st2.chunks_reused - st.chunks_reused == 4 and st2.chunks_created - st.chunks_created == 2
        assert st2.va_reserved_calls - st.va_reserved_calls == 2 and st2.phys_bytes == 6 * chunk
        vt.vt_append(kv, dev_bits(rows[:3000]), dev_bits(rows[:3000]), 3000, 0, stream())
        info = vt.vt_query(kv)
        np.testing.assert_array_equal(read_device(info.k_ptr, 3000 * 2048).view(np.uint16).reshape(3000, hkv, d),
                                      rows[:3000])
        vt.vt_release(kv)
        vt.vt_trim(c, 0)
        st3 = vt.vt_stats(c)
        assert (st3.phys_bytes, st3.reserved_va_bytes, st3.mapped_bytes, st3.chunks_pooled) == (0, 0, 0, 0)
        before = vt.vt_stats(c)
        kv = vt.vt_reserve(c, hkv, d, vt.VT_BF16, 8192)
        vt.vt_extend(kv, 1)
        after = vt.vt_stats(c)
        assert after.chunks_created - before.chunks_created == 2 and after.create_calls - before.create_calls == 2
        assert after.chunks_reused == before.chunks_reused and after.phys_bytes == 2 * chunk
        vt.vt_release(kv)
    finally:
        torch.cuda.synchronize()
        vt.vt_destroy(c)
