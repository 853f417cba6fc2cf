#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

Headline line (one JSON object on stdout): decode attention over VMM-backed, virtually contiguous KV
regions on the Llama-2-7B-shaped MHA workload (batch 64, 32/32 heads, head_dim 128, KV lengths uniform
in [512, 4096], bf16, 2 MiB chunks).  One step = extend every request by one token (vt_extend_batch),
write the new K/V rows (vt_append_batch), decode over the extended cache (vt_attn_decode: split pass +
combine).  `value` is the algorithmic K/V bytes of the timed steps divided by their wall time, inputs
resident in HBM.  The same line carries the roofline of the dominant kernel (live HIP-event timing),
the prefix-prefill kernel's figures on the Llama-3-8B-shaped GQA workload, and the fp64 CPU oracle timed
on a bounded sample of the same workload.

Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--no-prefill]
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published
# Measured HBM bytes per decode_kernel launch divided by its algorithmic bytes: rocprofv3 FETCH_SIZE + WRITE_SIZE,
# each scaled by what the same counter reads for a plain 1 GiB copy (FETCH_SIZE x 2.000, WRITE_SIZE x 1.000), over
# 22 dispatches of this workload.
DECODE_TRAFFIC_RATIO = 1.001


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def decode_kv_bytes(lens, hkv, d):
    """K and V bytes one decode step must read: every cached row once per KV head, 2-byte elements."""
    return int(np.sum(lens, dtype=np.int64)) * 2 * hkv * d * 2


def prefill_flops(plens, nlens, hq, d):
    """2 x multiply-adds of both products over the unmasked (query, key) pairs only."""
    p, n = np.asarray(plens, np.int64), np.asarray(nlens, np.int64)
    return int(4 * hq * d * np.sum(n * p + n * (n + 1) // 2))


def upload_regions(vt, torch, ctx, cfg, k, v, max_tokens):
    kvs = []
    st = torch.cuda.current_stream().cuda_stream
    for b in range(len(k)):
        L = k[b].shape[0]
        kv = vt.vt_reserve(ctx, cfg.n_kv_heads, cfg.head_dim, vt.DTYPES[cfg.dtype], max_tokens)
        vt.vt_extend(kv, L)
        kd = torch.from_numpy(k[b].view(np.int16)).cuda()
        vd = torch.from_numpy(v[b].view(np.int16)).cuda()
        vt.vt_append(kv, kd, vd, L, 0, st)
        torch.cuda.synchronize()
        kvs.append(kv)
    infos = [vt.vt_query(x) for x in kvs]
    k_ptrs = torch.tensor([i.k_ptr for i in infos], dtype=torch.int64).cuda()
    v_ptrs = torch.tensor([i.v_ptr for i in infos], dtype=torch.int64).cuda()
    return kvs, k_ptrs, v_ptrs


def bench_decode(vt, torch, ctx, args):
    import workloads
    cfg = workloads.CONFIGS[2]
    t0 = time.time()
    data = workloads.decode_inputs(cfg, threads=16)
    lens0 = data["kv_lens"].astype(np.int64)
    log("decode workload: %s seed %#x  sum(L)=%d min=%d max=%d  checksum(q)=%#x  gen %.1fs" % (
        cfg.name, data["seed"], lens0.sum(), lens0.min(), lens0.max(), workloads.checksum64(data["q"]),
        time.time() - t0))
    n_iter = args.steps + args.warmup
    kvs, k_ptrs, v_ptrs = upload_regions(vt, torch, ctx, cfg, data["k"], data["v"], cfg.kv_len[1] + n_iter + 1)
    B, hq, hkv, d = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    stream = torch.cuda.current_stream().cuda_stream
    q = torch.from_numpy(data["q"].view(np.int16)).cuda()
    out = torch.zeros_like(q)
    # one new K/V row per request and step, resident on the device before timing starts
    rows = [workloads.step_inputs(cfg, s) for s in range(n_iter)]
    k_rows = [torch.from_numpy(r["k_row"].view(np.int16)).cuda() for r in rows]
    v_rows = [torch.from_numpy(r["v_row"].view(np.int16)).cuda() for r in rows]
    lens_host = [np.ascontiguousarray((lens0 + s + 1).astype(np.int32)) for s in range(n_iter)]
    lens_dev = [torch.from_numpy(x).cuda() for x in lens_host]
    step_args = [vt.make_decode_args(vt.DTYPES[cfg.dtype], B, hq, hkv, d, cfg.scale, q, out, k_ptrs, v_ptrs,
                                     lens_dev[s], lens_host[s]) for s in range(n_iter)]
    new_lens = [x.tolist() for x in lens_host]
    plan, _ = vt.vt_plan_decode(ctx, lens_host[-1], hkv, hq, d)
    vt.vt_workspace_reserve(ctx, plan.workspace_bytes)

    def step(s):
        vt.vt_extend_batch(kvs, new_lens[s])
        vt.vt_append_batch(ctx, k_ptrs, v_ptrs, lens_dev[s], k_rows[s], v_rows[s], B, hkv, d, stream)
        vt.vt_attn_decode(ctx, step_args[s], stream)

    for s in range(args.warmup):
        step(s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.warmup, n_iter):
        step(s)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    # Roofline leg: the main decode kernel alone, bracketed by HIP events on the launch stream, on the same
    # regions at their final lengths (the event records would add stream gaps to the loop timed above).
    vt.vt_profile_enable(ctx, True)
    for _ in range(args.steps):
        vt.vt_attn_decode(ctx, step_args[-1], stream)
    torch.cuda.synchronize()
    vt.vt_profile_enable(ctx, False)
    kern_ms, launches = vt.vt_profile_collect(ctx, 0)
    kern_bytes = float(decode_kv_bytes(lens_host[-1], hkv, d))
    step_bytes = [decode_kv_bytes(lens_host[s], hkv, d) for s in range(args.warmup, n_iter)]
    total_bytes = float(sum(step_bytes))
    res = {
        "cfg": cfg, "data": data, "wall_s": wall, "total_bytes": total_bytes,
        "gbps": total_bytes / wall / 1e9, "ms_per_step": wall / args.steps * 1e3,
        "kernel_ms": kern_ms / max(launches, 1), "launches": launches,
        "kernel_gbps": kern_bytes / (kern_ms / max(launches, 1) * 1e-3) / 1e9 if launches else None,
        "kernel_bytes": kern_bytes,
        "tokens_per_s": B * args.steps / wall, "span": plan.span_tokens, "units": plan.n_units,
        "out_bits": out.cpu().numpy().view(np.uint16), "last_lens": lens_host[-1], "rows": rows,
    }
    torch.cuda.synchronize()
    for kv in kvs:
        vt.vt_release(kv)
    return res


def bench_prefill(vt, torch, ctx, args):
    import workloads
    cfg = workloads.CONFIGS[3]
    data = workloads.prefill_inputs(cfg, threads=16)
    kvs, k_ptrs, v_ptrs = upload_regions(vt, torch, ctx, cfg, data["k"], data["v"], cfg.kv_len[1] + cfg.new_len[1])
    stream = torch.cuda.current_stream().cuda_stream
    qn = torch.from_numpy(data["q_new"].view(np.int16)).cuda()
    kn = torch.from_numpy(data["k_new"].view(np.int16)).cuda()
    vn = torch.from_numpy(data["v_new"].view(np.int16)).cuda()
    out = torch.zeros_like(qn)
    cu = np.ascontiguousarray(data["cu_seqlens"], np.int32)
    pl = np.ascontiguousarray(data["prefix_lens"], np.int32)
    a = vt.make_prefill_args(vt.DTYPES[cfg.dtype], cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.scale,
                             int(cu[-1]), qn, out, kn, vn, k_ptrs, v_ptrs, torch.from_numpy(cu).cuda(),
                             torch.from_numpy(pl).cuda(), cu, pl)
    plan = vt.vt_plan_prefill(ctx, cu, pl, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim)
    vt.vt_workspace_reserve(ctx, plan.workspace_bytes)
    try:
        for _ in range(3):
            vt.vt_attn_prefix_prefill(ctx, a, stream)
    except vt.VtError as e:
        for kv in kvs:
            vt.vt_release(kv)
        return {"error": str(e)}
    torch.cuda.synchronize()
    reps = 20
    vt.vt_profile_enable(ctx, True)
    t0 = time.perf_counter()
    for _ in range(reps):
        vt.vt_attn_prefix_prefill(ctx, a, stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    vt.vt_profile_enable(ctx, False)
    kern_ms, launches = vt.vt_profile_collect(ctx, 1)
    flops = prefill_flops(pl, data["new_lens"], cfg.n_q_heads, cfg.head_dim)
    kms = kern_ms / max(launches, 1)
    for kv in kvs:
        vt.vt_release(kv)
    return {"workload": cfg.name, "flops": flops, "ms_per_call": wall / reps * 1e3, "kernel_ms": kms,
            "tflops": flops / (wall / reps) / 1e12, "kernel_tflops": flops / (kms * 1e-3) / 1e12 if launches else None,
            "frac_of_bf16_peak": flops / (kms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS if launches else None,
            "tokens_per_s": int(cu[-1]) / (wall / reps), "new_tokens": int(cu[-1]),
            "kernels": "prefill_kernel + prefill_combine_kernel (the events bracket both)",
            "work_groups": int(plan.n_groups), "key_tiles": int(plan.n_tiles), "items": int(plan.n_items)}


def cpu_baseline(dec):
    """The fp64 oracle, as it stands, on a bounded sample of the decode workload (first requests of the
    batch), timed on the host cores."""
    import oracle
    cfg, data = dec["cfg"], dec["data"]
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    q = oracle.widen(data["q"], cfg.dtype)
    t0 = time.perf_counter()
    reps, nbytes = 0, 0
    while True:
        k = [oracle.widen(x, cfg.dtype) for x in data["k"]]
        v = [oracle.widen(x, cfg.dtype) for x in data["v"]]
        oracle.decode(q, k, v, cfg.scale)
        reps += 1
        nbytes += decode_kv_bytes(data["kv_lens"], cfg.n_kv_heads, cfg.head_dim)
        dt = time.perf_counter() - t0
        if dt >= 10.0 or reps >= 50:
            break
    return {"value": round(nbytes / dt / 1e9, 3), "unit": "GB/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d decode steps over the whole batch of %d requests (initial lengths), %.1f s including the "
                      "widening of K/V to fp64" % (reps, cfg.batch, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prefill", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run plain 1 GiB device copies (reference for the rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1. "
                 "Sharding by KV head or by request would need no exchange inside attention.")
    import torch
    import paper_2407_15309_amd as vt
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(3)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": 1 << 30, "copies": 5}), flush=True)
        return
    ctx = vt.vt_init(0, 0, 0)
    # Everything runs on a stream of its own (torch's side streams do not synchronise with the default stream):
    # the driver's mapping call inside vt_extend waits for the default stream and every stream that synchronises
    # with it, so on the default stream each newly mapped chunk would drain the GPU queue first.
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        dec = bench_decode(vt, torch, ctx, args)
        pre = None if args.no_prefill else bench_prefill(vt, torch, ctx, args)
    torch.cuda.synchronize()
    vt.vt_destroy(ctx)
    cfg = dec["cfg"]
    line = {
        "metric": "decode_attn_hbm_GBps", "value": round(dec["gbps"], 1), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(dec["ms_per_step"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name, "batch": cfg.batch, "n_q_heads": cfg.n_q_heads, "n_kv_heads": cfg.n_kv_heads,
                   "head_dim": cfg.head_dim, "kv_len": "uniform[%d,%d]" % cfg.kv_len, "chunk_bytes": 2 << 20,
                   "step": "vt_extend_batch(+1) + vt_append_batch + vt_attn_decode", "span_tokens": dec["span"],
                   "work_units": dec["units"]},
        "pct_of_hbm_peak": round(100 * dec["gbps"] / HBM_PEAK_GBPS, 2),
        "decode_tokens_per_s": round(dec["tokens_per_s"], 1),
        "roofline": {"bound": "hbm", "kernel": "decode_kernel",
                     "achieved": round(dec["kernel_gbps"], 1) if dec["kernel_gbps"] else None, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(dec["kernel_gbps"] / HBM_PEAK_GBPS, 4) if dec["kernel_gbps"] else None,
                     "avg_launch_ms": round(dec["kernel_ms"], 4), "launches": dec["launches"],
                     "algorithmic_bytes_per_launch": dec["kernel_bytes"],
                     "traffic": round(DECODE_TRAFFIC_RATIO * dec["kernel_bytes"])},
        "prefill": pre,
        "context": "paper (A100, vs vLLM PagedAttention): decode kernel avg 2.78x, peak 3.27x; prefix-prefill vs "
                   "SGLang Triton avg 3.40x, peak 3.92x; no absolute rates published",
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(dec)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
