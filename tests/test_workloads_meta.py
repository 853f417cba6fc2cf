"""Seeded input generators and the oracle's integer metadata / accounting."""

import os

import numpy as np
import pytest

import oracle
import workloads
from oracle import meta
from workloads import CONFIGS

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")


def golden():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = float(v)
    return out


def test_generators_are_deterministic_and_order_independent():
    a = workloads.normal_bits(7, workloads.gen.T_K, 3, (5, 2, 8), "bf16")
    _ = workloads.normal_bits(7, workloads.gen.T_K, 2, (50, 2, 8), "bf16")
    b = workloads.normal_bits(7, workloads.gen.T_K, 3, (5, 2, 8), "bf16")
    np.testing.assert_array_equal(a, b)
    c = workloads.normal_bits(7, workloads.gen.T_V, 3, (5, 2, 8), "bf16")
    assert not np.array_equal(a, c)
    d = workloads.normal_bits(8, workloads.gen.T_K, 3, (5, 2, 8), "bf16")
    assert not np.array_equal(a, d)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_values_look_standard_normal(dtype):
    x = oracle.widen(workloads.normal_bits(1, 2, 0, (200000,), dtype), dtype)
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1.0) < 0.01
    assert np.isfinite(x).all()


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20], dtype=np.float32)
    bits = workloads.gen._round_bits(x, "bf16")
    np.testing.assert_array_equal(oracle.widen(bits, "bf16"), [1.0, 1.0, 1.0 + 2 ** -7, 1.0 + 2 ** -6, 1.0 + 2 ** -7])


def test_config_shapes_and_length_ranges():
    cfg = CONFIGS[1]
    d = workloads.decode_inputs(cfg)
    assert d["kv_lens"].dtype == np.int32 and d["kv_lens"].shape == (4,)
    assert all(16 <= L <= 256 for L in d["kv_lens"])
    assert d["q"].shape == (4, 8, 64) and d["q"].dtype == np.uint16
    for b in range(4):
        assert d["k"][b].shape == (d["kv_lens"][b], 8, 64) == d["v"][b].shape
    small3 = CONFIGS[3].replace(batch=3, kv_len=(10, 40), new_len=(2, 9))
    p = workloads.prefill_inputs(small3)
    assert p["cu_seqlens"][0] == 0 and p["cu_seqlens"][-1] == p["new_lens"].sum() == p["q_new"].shape[0]
    assert p["q_new"].shape[1:] == (32, 128) and p["k_new"].shape[1:] == (8, 128)
    assert all(10 <= x <= 40 for x in p["prefix_lens"]) and all(2 <= x <= 9 for x in p["new_lens"])
    # the five named configs carry the shapes the benchmark definition states
    assert (CONFIGS[2].batch, CONFIGS[2].n_q_heads, CONFIGS[2].n_kv_heads, CONFIGS[2].head_dim) == (64, 32, 32, 128)
    assert (CONFIGS[5].batch, CONFIGS[5].n_q_heads, CONFIGS[5].n_kv_heads, CONFIGS[5].steps) == (256, 64, 8, 32)


def test_lengths_cover_the_inclusive_range():
    lens = workloads.draw_lengths(3, 0, 20000, 16, 19)
    assert set(np.unique(lens)) == {16, 17, 18, 19}


def test_region_arithmetic_matches_the_papers_example():
    """A 2 MB chunk of a 32-head, 128-dim fp16 K region holds 256 token rows, the initial allocation the
    paper gives as its example next to a 4096-token virtual range ("vTensor Pool", vSet)."""
    g = golden()
    chunk = int(g["chunk_megabytes"]) * 1024 * 1024
    assert chunk == meta.CHUNK_BYTES
    assert meta.row_bytes(32, 128) == 8192
    assert chunk // meta.row_bytes(32, 128) == int(g["example_initial_tokens"])
    assert meta.chunks_for_len(int(g["example_initial_tokens"]), 32, 128) == 1
    assert meta.chunks_for_len(int(g["example_initial_tokens"]) + 1, 32, 128) == 2
    assert meta.capacity_bytes(int(g["example_max_tokens"]), 32, 128) == 16 * chunk
    assert meta.chunks_for_len(0, 8, 128) == 0
    # capacity is a whole number of chunks and never less than the rows asked for
    for mt in (1, 1023, 1024, 1025, 8224):
        cap = meta.capacity_bytes(mt, 8, 128)
        assert cap % chunk == 0 and 0 <= cap - mt * 2048 < chunk


def test_chunks_for_len_is_monotone_and_tight():
    for (h, d) in ((8, 128), (3, 40), (32, 128)):
        rb = meta.row_bytes(h, d)
        prev = 0
        for L in range(0, 4000, 7):
            c = meta.chunks_for_len(L, h, d, chunk=65536)
            assert c >= prev and c * 65536 >= L * rb and (c == 0 or (c - 1) * 65536 < L * rb)
            prev = c


def test_mha_decode_arithmetic_intensity_matches_the_papers_roofline():
    """flops / bytes of MHA decode is ~1 (the paper's roofline figure puts MHA at 0.99)."""
    g = golden()
    lens = workloads.draw_lengths(1, 0, 64, 512, 4096)
    ai = meta.decode_flops(lens, 32, 128) / meta.decode_kv_bytes(lens, 32, 128)
    assert abs(ai - g["mha_decode_arithmetic_intensity"]) < 0.02
    # grouped heads raise it by the group size (paper: intensity grows from MHA to GQA to MQA)
    ai_gqa = meta.decode_flops(lens, 32, 128) / meta.decode_kv_bytes(lens, int(g["kernel_eval_kv_heads"]), 128)
    assert abs(ai_gqa / ai - 8.0) < 1e-12


def test_prefill_flops_counts_unmasked_pairs_only():
    # one request, P=2, N=3: pairs = 3*2 + (1+2+3) = 12
    assert meta.prefill_flops([2], [3], 1, 1) == 4 * 12
    # brute count
    P, N = 5, 4
    pairs = sum(1 for i in range(N) for j in range(P + N) if j <= P + i)
    assert meta.prefill_flops([P], [N], 2, 8) == 4 * 2 * 8 * pairs


def test_decode_plan_rule():
    """Tape split: equal segments over the concatenated tokens; pieces tile every request exactly."""
    lens = [1, 128, 129, 4096]
    seg, pieces, mx, units = meta.decode_plan(lens, 4, slots=64)       # 16 segments over 4354 tokens
    assert seg == 288 and seg % 32 == 0 and 16 * seg >= sum(lens) > 15 * seg - 32 * 16
    assert pieces == [1, 1, 1, 16] and mx == 16 and units == 16 * 4
    for b, (L, n) in enumerate(zip(lens, pieces)):
        got = [meta.piece_range(lens, seg, b, i) for i in range(n)]
        assert got[0][0] == 0 and got[-1][1] == L
        assert all(x[1] == y[0] for x, y in zip(got, got[1:])) and all(e > s for s, e in got)
        assert all(e - s <= seg for s, e in got)
    # brute force: mark the segment of every tape position, count distinct segments per request
    owner = [i // seg for i in range(sum(lens))]
    start = 0
    for L, n in zip(lens, pieces):
        assert len(set(owner[start:start + L])) == n
        start += L
    # never more segments than wavefront slots per head, never fewer than one, at least a tile each
    lens = workloads.draw_lengths(2, 0, 64, 512, 4096)
    seg, pieces, mx, units = meta.decode_plan(lens, 32)
    assert units // 32 <= meta.PLAN_WAVE_SLOTS // 32 and (units // 32) * seg >= lens.sum() > (units // 32 - 1) * seg
    assert meta.decode_plan([5], 8) == (32, [1], 1, 8)
    assert meta.decode_plan([40], 8)[0:2] == (32, [2])
    assert meta.decode_plan([7, 9], 4096)[0] == 32            # more heads than slots: one segment per head


def test_traffic_summary_has_a_line_for_every_bench_leg():
    """bench.py takes the `traffic` field of its roofline objects from profiles/hbm_traffic_per_kernel.md: every
    workload's line must be there and parse (a measured ratio near 1 for the memory-bound kernel, measured bytes at
    or above the algorithmic ones for the other)."""
    import importlib.util
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    for cfg_id in (1, 2, 4, 5):
        ratio = bench.traffic_entry("traffic_ratio", "decode_kernel", CONFIGS[cfg_id].name)
        assert ratio is not None and 1.0 <= ratio < 1.3, (cfg_id, ratio)
    for cfg_id in (3, 4):
        nbytes = bench.traffic_entry("traffic_bytes", "prefill_kernel", CONFIGS[cfg_id].name)
        lo, hi = CONFIGS[cfg_id].kv_len
        assert nbytes is not None and nbytes > CONFIGS[cfg_id].batch * lo * 2 * CONFIGS[cfg_id].n_kv_heads * 128 * 2
