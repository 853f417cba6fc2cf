#!/usr/bin/env python3
"""Kernel sweeps over the shapes of the paper's kernel evaluation ("Decoding Kernel Evaluation", "Prefix-prefilling
Kernel Evaluation"; default kernel shape of "Evaluation Scenarios": 32 query heads / 4 KV heads), on one MI355X.
A reporting tool like bench.py, not part of the library.

    python sweep.py [--quick] [--only d1,d2,d3,p1,p2,e1,m1]

  d1  decode, KV length 16K, batch 1..64           (batch-size sweep; at 32/4 heads and at 32/32 heads)
  d2  decode, batch 16, KV length 512..32K         (sequence-length sweep; both head shapes)
  d3  decode, batch 16, KV length 16K, 32 query heads, 32..1 KV heads   (KV-head sweep; the arithmetic-intensity
      sweep of the paper's attention roofline)
  p1  prefix-prefill, context 16K, prefix ratio 0.5, batch 1..16        (batch-size sweep; 32/4 and 32/8 heads)
  p2  prefix-prefill, context 16K, batch 4, prefix ratio 0.1..0.9       (prefix-ratio sweep)
  e1  prefix-prefill on N(0,1) data against all-zero data, the first launches on an idle device against the
      settled speed, the kernel of eight 32-row wavefronts against the one of four 64-row wavefronts, with the
      shader clock read from rocm-smi while the kernel loops: how much of the kernel's time is the chip's power
      management (the clock drops under random operands) rather than the instruction schedule
  m1  memory accounting against the running batch size ("Memory Flexibility"): physical memory mapped by the
      regions while the batch grows to 64 requests and shrinks again, against the virtual range reserved and
      against a static preallocation for the largest batch at the maximum length.  Runs on the host backend
      (same bookkeeping, no GPU needed): python sweep.py --only m1

Q/K/V are N(0,1) bf16 from the seeded generator of workloads/ (normal_bits; a pool of 8 distinct requests per point,
reused in turn when the batch is larger), written into VMM-backed regions; the tables give the kernel time (HIP
events inside the library, average over the repetitions; prefix-prefill after 60 ms of untimed launches, since that
kernel's speed settles only under load), the time of a whole call, and the fraction of the HBM (8 TB/s) or dense bf16
MFMA (2.5 PFLOP/s) roofline.  The paper's comparison kernels are not part of this library,
so there is no speed-up column.
"""

from __future__ import annotations

import argparse
import sys

import os

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

SEED = 0x240715309 + 100
POOL = 8   # distinct requests generated per sweep point


def _bits(torch, tensor, request, shape):
    """Seeded N(0,1) bf16 bit patterns on the device."""
    import workloads
    return torch.from_numpy(workloads.normal_bits(SEED, tensor, request, shape, "bf16").view(np.int16)).cuda()


def _regions(vt, torch, ctx, lens, hkv, d, extra=0):
    import workloads
    g = workloads.gen
    kvs = []
    st = torch.cuda.current_stream().cuda_stream
    pool = {}
    for b, L in enumerate(lens):
        kv = vt.vt_reserve(ctx, hkv, d, vt.VT_BF16, int(L) + extra)
        vt.vt_extend(kv, int(L))
        if L:
            key = (b % POOL, int(L))
            if key not in pool:
                pool[key] = (_bits(torch, g.T_K, b % POOL, (int(L), hkv, d)), _bits(torch, g.T_V, b % POOL, (int(L), hkv, d)))
            k, v = pool[key]
            vt.vt_append(kv, k, v, int(L), 0, st)
            torch.cuda.synchronize()
        kvs.append(kv)
    infos = [vt.vt_query(x) for x in kvs]
    kp = torch.tensor([i.k_ptr for i in infos], dtype=torch.int64).cuda()
    vp = torch.tensor([i.v_ptr for i in infos], dtype=torch.int64).cuda()
    return kvs, kp, vp


def decode_case(vt, torch, ctx, batch, L, hq, hkv, d=128, reps=20):
    lens = np.full(batch, L, np.int32)
    kvs, kp, vp = _regions(vt, torch, ctx, lens, hkv, d)
    st = torch.cuda.current_stream().cuda_stream
    import workloads
    q = _bits(torch, workloads.gen.T_Q, 0, (batch, hq, d))
    out = torch.zeros_like(q)
    a = vt.make_decode_args(vt.VT_BF16, batch, hq, hkv, d, d ** -0.5, q, out, kp, vp, torch.from_numpy(lens).cuda(), lens)
    for _ in range(3):
        vt.vt_attn_decode(ctx, a, st)
    torch.cuda.synchronize()
    vt.vt_profile_enable(ctx, True)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        vt.vt_attn_decode(ctx, a, st)
    e1.record()
    torch.cuda.synchronize()
    vt.vt_profile_enable(ctx, False)
    ms, n = vt.vt_profile_collect(ctx, 0)
    call_us = e0.elapsed_time(e1) / reps * 1e3
    for kv in kvs:
        vt.vt_release(kv)
    nbytes = float(batch) * L * 2 * hkv * d * 2
    flops = 4.0 * hq * d * batch * L
    us = ms / n * 1e3
    return {"kernel_us": us, "call_us": call_us, "gbps": nbytes / us / 1e3, "tflops": flops / us / 1e6,
            "ai": flops / nbytes}


def _settled_us(vt, torch, ctx, launch, reps):
    """(us per launch over the first ten launches on an idle device, us per launch once the speed has settled).
    The prefix-prefill kernel speeds up over its first 30 ms of load: 60 ms of launches go untimed, then at least
    30 ms of them are timed."""
    import time

    def run(count, profile):
        if profile:
            vt.vt_profile_enable(ctx, True)
        t0 = time.perf_counter()
        for _ in range(count):
            launch()
        torch.cuda.synchronize()
        w = (time.perf_counter() - t0) / count
        if not profile:
            return w
        vt.vt_profile_enable(ctx, False)
        ms, cnt = vt.vt_profile_collect(ctx, 1)
        return ms / cnt * 1e3
    torch.cuda.synchronize()
    time.sleep(0.2)
    first = run(10, True)
    run(int(np.ceil(0.06 / (first * 1e-6))), False)
    return first, run(max(reps, int(np.ceil(0.03 / (first * 1e-6)))), True)


def prefill_case(vt, torch, ctx, batch, context, ratio, hq=32, hkv=8, d=128, reps=5):
    P = int(round(context * ratio))
    N = context - P
    plens = np.full(batch, P, np.int32)
    kvs, kp, vp = _regions(vt, torch, ctx, plens, hkv, d)
    st = torch.cuda.current_stream().cuda_stream
    T = batch * N
    import workloads
    g = workloads.gen
    rep = lambda t, h: torch.cat([_bits(torch, t, b % POOL, (N, h, d)) for b in range(min(batch, POOL))] *
                                 ((batch + POOL - 1) // POOL))[:T]
    qn, kn, vn = rep(g.T_QNEW, hq), rep(g.T_KNEW, hkv), rep(g.T_VNEW, hkv)
    out = torch.zeros_like(qn)
    cu = (np.arange(batch + 1) * N).astype(np.int32)
    a = vt.make_prefill_args(vt.VT_BF16, batch, hq, hkv, d, d ** -0.5, T, qn, out, kn, vn, kp, vp,
                             torch.from_numpy(cu).cuda(), torch.from_numpy(plens).cuda(), cu, plens)
    us = _settled_us(vt, torch, ctx, lambda: vt.vt_attn_prefix_prefill(ctx, a, st), reps)[1]
    for kv in kvs:
        vt.vt_release(kv)
    flops = 4.0 * hq * d * batch * (N * P + N * (N + 1) / 2)
    return {"us": us, "tflops": flops / us / 1e6, "P": P, "N": N}


def _sclk():
    import subprocess
    try:
        r = subprocess.run(["/opt/rocm/bin/rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=20)
        for line in r.stdout.splitlines():
            if "sclk" in line and "(" in line:
                return line.split("(")[-1].split(")")[0]
    except Exception:
        pass
    return "n/a"


def clock_experiment(vt, torch, ctx, say):
    """Prefix-prefill kernel time against the operand data and the launch pattern."""
    import threading
    import time
    import workloads
    c3 = workloads.CONFIGS[3]
    cases = [("workload 3 (B16, P 1K-4K, N 128-512)", c3, 20),
             ("context 16K, prefix ratio 0.5, batch 4", c3.replace(batch=4, kv_len=(8192, 8192), new_len=(8192, 8192)), 5)]
    say("\n### e1: prefill_kernel, 32/8 heads, bf16: operand data, launch pattern and kernel shape\n")
    say("| shape | kernel | data | first 10 launches on an idle device, us | settled (after 60 ms of launches), us | TFLOP/s | of 2.5 PFLOP/s | sclk after 1 s of launches |")
    say("|---|---|---|---|---|---|---|---|")
    # the four-wavefront kernel is what a context created under VT_PREFILL_WIDE=1 runs at head_dim 128
    os.environ["VT_PREFILL_WIDE"] = "1"
    try:
        wide = vt.vt_init(0, 0, 0)
    finally:
        del os.environ["VT_PREFILL_WIDE"]
    for name, cfg, reps in cases:
        d0 = workloads.prefill_inputs(cfg, threads=16)
        for data in ("N(0,1)", "zeros"):
            d = dict(d0)
            if data == "zeros":
                for key in ("q_new", "k_new", "v_new"):
                    d[key] = np.zeros_like(d0[key])
                d["k"] = [np.zeros_like(x) for x in d0["k"]]
                d["v"] = [np.zeros_like(x) for x in d0["v"]]
            for kernel, c in (("8 wavefronts x 32 rows", ctx), ("4 wavefronts x 64 rows", wide)):
                st = torch.cuda.current_stream().cuda_stream
                kvs = []
                for b in range(cfg.batch):
                    kv = vt.vt_reserve(c, cfg.n_kv_heads, cfg.head_dim, vt.VT_BF16, int(d["prefix_lens"][b]) + 1)
                    vt.vt_extend(kv, int(d["prefix_lens"][b]))
                    kd = torch.from_numpy(d["k"][b].view(np.int16)).cuda()
                    vd = torch.from_numpy(d["v"][b].view(np.int16)).cuda()
                    vt.vt_append(kv, kd, vd, int(d["prefix_lens"][b]), 0, st)
                    torch.cuda.synchronize()
                    kvs.append(kv)
                infos = [vt.vt_query(x) for x in kvs]
                kp = torch.tensor([i.k_ptr for i in infos], dtype=torch.int64).cuda()
                vp = torch.tensor([i.v_ptr for i in infos], dtype=torch.int64).cuda()
                dev = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()
                qn, kn, vn = dev(d["q_new"]), dev(d["k_new"]), dev(d["v_new"])
                out = torch.zeros_like(qn)
                cu = np.ascontiguousarray(d["cu_seqlens"], np.int32)
                pl = np.ascontiguousarray(d["prefix_lens"], np.int32)
                a = vt.make_prefill_args(vt.VT_BF16, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.scale,
                                         int(cu[-1]), qn, out, kn, vn, kp, vp, torch.from_numpy(cu).cuda(),
                                         torch.from_numpy(pl).cuda(), cu, pl)
                n, p = d["new_lens"].astype(np.int64), pl.astype(np.int64)
                flops = float(4 * cfg.n_q_heads * cfg.head_dim * np.sum(n * p + n * (n + 1) // 2))
                launch = lambda: vt.vt_attn_prefix_prefill(c, a, st)
                first, busy = _settled_us(vt, torch, c, launch, reps)
                stop = [False]

                def spin():
                    while not stop[0]:
                        for _ in range(50 if reps > 5 else 5):
                            vt.vt_attn_prefix_prefill(c, a, st)
                        torch.cuda.synchronize()
                t = threading.Thread(target=spin)
                t.start()
                time.sleep(1.0)
                clk = _sclk()
                stop[0] = True
                t.join()
                say("| %s | %s | %s | %.1f | %.1f | %.0f | %.3f | %s |" % (name, kernel, data, first, busy,
                                                                      flops / busy / 1e6, flops / busy / 1e6 / 2500, clk))
                torch.cuda.synchronize()
                for kv in kvs:
                    vt.vt_release(kv)
    torch.cuda.synchronize()
    vt.vt_destroy(wide)


def memory_accounting(vt, say):
    """Llama-2-7B-shaped K/V of one layer (32 KV heads x 128, bf16), lengths uniform in [512, 4096] as in the
    decode workload, maximum length 4096: requests arrive one by one up to 64, then leave one by one."""
    hkv, d, max_len, chunk = 32, 128, 4096, 2 << 20
    rng = np.random.default_rng(2407)
    lens = rng.integers(512, 4097, size=64)
    ctx = vt.vt_init_host(chunk, 0)
    row = hkv * d * 2
    static = 64 * 2 * max_len * row
    say("\n### m1: one layer of K/V, 32 KV heads x 128 x bf16, max length 4096, chunk 2 MiB, lengths uniform[512,4096]\n")
    say("| running batch | tokens | exact bytes | mapped (physical) | reserved (virtual) | static preallocation for 64 x 4096 | mapped / static |")
    say("|---|---|---|---|---|---|---|")
    kvs = []
    def row_of(tag):
        st = vt.vt_stats(ctx)
        tok = int(sum(lens[: len(kvs)]))
        say("| %s | %d | %.1f MiB | %.1f MiB | %.1f MiB | %.1f MiB | %.3f |" % (
            tag, tok, tok * 2 * row / 2 ** 20, st.mapped_bytes / 2 ** 20, st.reserved_va_bytes / 2 ** 20,
            static / 2 ** 20, st.mapped_bytes / static))
    for b in range(64):
        kv = vt.vt_reserve(ctx, hkv, d, vt.VT_BF16, max_len)
        vt.vt_extend(kv, int(lens[b]))
        kvs.append(kv)
        if b + 1 in (1, 2, 4, 8, 16, 32, 64):
            row_of(str(b + 1))
    while kvs:
        vt.vt_release(kvs.pop())
        if len(kvs) in (32, 8, 0):
            st = vt.vt_stats(ctx)
            say("| %d (after releases; %d chunks idle in the pool, %.1f MiB still allocated) | | | %.1f MiB | %.1f MiB | | |" % (
                len(kvs), st.chunks_pooled, st.phys_bytes / 2 ** 20, st.mapped_bytes / 2 ** 20, st.reserved_va_bytes / 2 ** 20))
    vt.vt_trim(ctx, 0)
    st = vt.vt_stats(ctx)
    say("| 0 (after vt_trim) | | | %.1f MiB mapped, %.1f MiB allocated | | | |" % (st.mapped_bytes / 2 ** 20, st.phys_bytes / 2 ** 20))
    vt.vt_destroy(ctx)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--quick", action="store_true", help="fewer points")
    ap.add_argument("--only", default="d1,d2,d3,p1,p2,e1,m1")
    args = ap.parse_args()
    import paper_2407_15309_amd as vt
    only = set(args.only.split(","))
    say = lambda *a: print(*a, flush=True)
    if only == {"m1"}:
        memory_accounting(vt, say)
        return
    import torch
    if not torch.cuda.is_available():
        sys.exit("sweep: no GPU visible; the HIP path has no CPU fallback")
    ctx = vt.vt_init(0, 0, 0)
    with torch.cuda.stream(torch.cuda.Stream()):
        shapes = [(32, 4), (32, 32)]
        if "d1" in only:
            for hq, hkv in shapes:
                say("\n### d1: decode, %d/%d heads, head_dim 128, bf16, KV length 16384, batch sweep\n" % (hq, hkv))
                say("| batch | kernel us | call us (with merge) | GB/s (kernel) | of 8 TB/s | GB/s (call) |\n|---|---|---|---|---|---|")
                for b in ([1, 8, 64] if args.quick else [1, 2, 4, 8, 16, 32, 64]):
                    r = decode_case(vt, torch, ctx, b, 16384, hq, hkv)
                    say("| %d | %.1f | %.1f | %.0f | %.3f | %.0f |" % (b, r["kernel_us"], r["call_us"], r["gbps"], r["gbps"] / 8000,
                                                                   r["gbps"] * r["kernel_us"] / r["call_us"]))
        if "d2" in only:
            for hq, hkv in shapes:
                say("\n### d2: decode, %d/%d heads, batch 16, KV length sweep\n" % (hq, hkv))
                say("| KV length | kernel us | call us (with merge) | GB/s (kernel) | of 8 TB/s | GB/s (call) |\n|---|---|---|---|---|---|")
                for L in ([1024, 16384] if args.quick else [512, 1024, 2048, 4096, 8192, 16384, 32768]):
                    r = decode_case(vt, torch, ctx, 16, L, hq, hkv)
                    say("| %d | %.1f | %.1f | %.0f | %.3f | %.0f |" % (L, r["kernel_us"], r["call_us"], r["gbps"], r["gbps"] / 8000,
                                                                   r["gbps"] * r["kernel_us"] / r["call_us"]))
        if "d3" in only:
            say("\n### d3: decode, 32 query heads, batch 16, KV length 16384, KV-head sweep (MHA ... MQA)\n")
            say("| KV heads | flop per K/V byte | kernel us | call us | GB/s (kernel) | of 8 TB/s | TFLOP/s |\n|---|---|---|---|---|---|---|")
            for hkv in ([32, 4, 1] if args.quick else [32, 16, 8, 4, 2, 1]):
                r = decode_case(vt, torch, ctx, 16, 16384, 32, hkv)
                say("| %d | %.2f | %.1f | %.1f | %.0f | %.3f | %.1f |" % (hkv, r["ai"], r["kernel_us"], r["call_us"], r["gbps"],
                                                                      r["gbps"] / 8000, r["tflops"]))
        if "e1" in only:
            clock_experiment(vt, torch, ctx, say)
        if "p1" in only:
            for hq, hkv in [(32, 4), (32, 8)]:
                say("\n### p1: prefix-prefill, %d/%d heads, head_dim 128, bf16, context 16384, prefix ratio 0.5, batch sweep\n" % (hq, hkv))
                say("| batch | prefix | new | us | TFLOP/s | of 2.5 PFLOP/s |\n|---|---|---|---|---|---|")
                for b in ([1, 4] if args.quick else [1, 2, 4, 8, 16]):
                    r = prefill_case(vt, torch, ctx, b, 16384, 0.5, hq, hkv)
                    say("| %d | %d | %d | %.0f | %.0f | %.3f |" % (b, r["P"], r["N"], r["us"], r["tflops"], r["tflops"] / 2500))
        if "p2" in only:
            for hq, hkv in [(32, 4), (32, 8)]:
                say("\n### p2: prefix-prefill, %d/%d heads, context 16384, batch 4, prefix-ratio sweep\n" % (hq, hkv))
                say("| prefix ratio | prefix | new | us | TFLOP/s | of 2.5 PFLOP/s |\n|---|---|---|---|---|---|")
                for ratio in ([0.25, 0.75] if args.quick else [0.1, 0.25, 0.5, 0.75, 0.9]):
                    r = prefill_case(vt, torch, ctx, 4, 16384, ratio, hq, hkv)
                    say("| %.2f | %d | %d | %.0f | %.0f | %.3f |" % (ratio, r["P"], r["N"], r["us"], r["tflops"], r["tflops"] / 2500))
    torch.cuda.synchronize()
    vt.vt_destroy(ctx)
    if "m1" in only:
        memory_accounting(vt, say)


if __name__ == "__main__":
    main()
