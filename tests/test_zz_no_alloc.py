"""The decode entry point that allocates nothing (vt_attn_decode_static) against vt_attn_decode, through the C ABI:
same kernels and plan, so the output bits must be identical; two calls in a row on the one fixed buffer, the second
with a smaller input; a plan that does not fit the buffer is refused without launching anything."""

import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2407_15309_amd as vt
import workloads
from workloads import CONFIGS

pytestmark = pytest.mark.gpu

from gpu_util import TOL, Regions, dev_bits, host_bits, stream  # noqa: E402


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def both_ways(ctx, cfg, data, reg):
    B, hq, d = data["q"].shape
    q = dev_bits(data["q"])
    outs = []
    for fn in (vt.vt_attn_decode, vt.vt_attn_decode_static):
        out = torch.zeros_like(q)
        args = vt.make_decode_args(vt.DTYPES[cfg.dtype], B, hq, cfg.n_kv_heads, d, cfg.scale, q, out, reg.k_ptrs,
                                   reg.v_ptrs, reg.lens_dev, reg.lens)
        fn(ctx, args, stream())
        torch.cuda.synchronize()
        outs.append(host_bits(out))
    return outs


def test_static_scratch_decode_matches_the_allocating_entry_point():
    ctx = vt.vt_init(0, 0, 0)
    try:
        assert vt.vt_static_scratch_bytes() == 32 << 20
        # first call: requests cut into several pieces (the merge reads the fixed buffer); second call: smaller
        # batch, other head shape and dtype, on the same buffer with the first call's contents still in it
        cases = [(CONFIGS[2].replace(batch=24, n_q_heads=32, n_kv_heads=8, kv_len=(300, 5000)), 301),
                 (CONFIGS[1].replace(batch=3, kv_len=(1, 900)), 302)]
        for cfg, seed in cases:
            data = workloads.decode_inputs(cfg, seed=seed)
            reg = Regions(ctx, data["k"], data["v"], cfg.dtype)
            try:
                plan, pieces = vt.vt_plan_decode(ctx, reg.lens, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim)
                say("static-scratch case", cfg.dtype, "B", cfg.batch, "pieces", pieces.tolist()[:8], "workspace bytes",
                    plan.workspace_bytes)
                assert plan.workspace_bytes <= vt.vt_static_scratch_bytes()
                assert pieces.max() > 1 or cfg.batch < 24
                a, b = both_ways(ctx, cfg, data, reg)
            finally:
                reg.release()
            np.testing.assert_array_equal(a, b)
            w = lambda x: oracle.widen(x, cfg.dtype)
            ref = oracle.decode(w(data["q"]), [w(x) for x in data["k"]], [w(x) for x in data["v"]], cfg.scale)
            err = float(np.abs(w(b) - ref).max())
            say("  identical bits; max abs err against the oracle", err)
            assert err <= TOL[cfg.dtype]
        # a plan that needs more than the buffer: refused on the host, nothing is launched
        B = 4096
        lens = np.full(B, 2, np.int32)
        q = torch.zeros(B, 64, 128, dtype=torch.int16).cuda()
        lens_dev = torch.from_numpy(lens).cuda()
        plan, _ = vt.vt_plan_decode(ctx, lens, 8, 64, 128)
        assert plan.workspace_bytes > vt.vt_static_scratch_bytes()
        args = vt.make_decode_args(vt.VT_BF16, B, 64, 8, 128, 0.1, q, q, q, q, lens_dev, lens)
        with pytest.raises(vt.VtError) as e:
            vt.vt_attn_decode_static(ctx, args, stream())
        assert e.value.status == vt.VT_E_WORKSPACE
    finally:
        torch.cuda.synchronize()
        vt.vt_destroy(ctx)
