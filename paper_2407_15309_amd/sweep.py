"""Kernel sweeps over the shapes of the paper's kernel evaluation (Section 6.2), on one MI355X.

    python -m paper_2407_15309_amd.sweep [--quick] [--only d1,d2,d3,p1,p2]

  d1  decode, KV length 16K, batch 1..64           (Section 6.2.1, batch-size sweep; 32 query / 32 KV heads)
  d2  decode, batch 16, KV length 512..32K         (Section 6.2.1, sequence-length sweep)
  d3  decode, batch 16, KV length 16K, 32 query heads, 32..1 KV heads   (Section 6.2.1, KV-head sweep; the
      arithmetic-intensity sweep of Section 3.2)
  p1  prefix-prefill, context 16K, prefix ratio 0.5, batch 1..16        (Section 6.2.2, batch-size sweep)
  p2  prefix-prefill, context 16K, batch 4, prefix ratio 0.1..0.9       (Section 6.2.2, prefix-ratio sweep)
  m1  memory accounting against the running batch size (Section 6.4 / Section 3.1): physical memory mapped by the
      regions while the batch grows to 64 requests and shrinks again, against the virtual range reserved and
      against a static preallocation for the largest batch at the maximum length.  Runs on the host backend
      (same bookkeeping, no GPU needed): python -m paper_2407_15309_amd.sweep --only m1

K/V values are random bf16 written into VMM-backed regions; the tables give the kernel time (HIP events inside
the library, average over the repetitions) and the fraction of the HBM (8 TB/s) or dense bf16 MFMA (2.5 PFLOP/s)
roofline.  The paper's comparison kernels are not part of this library, so there is no speed-up column.
"""

from __future__ import annotations

import argparse
import sys

import numpy as np


def _regions(vt, torch, ctx, lens, hkv, d, extra=0):
    kvs = []
    st = torch.cuda.current_stream().cuda_stream
    for L in lens:
        kv = vt.vt_reserve(ctx, hkv, d, vt.VT_BF16, int(L) + extra)
        vt.vt_extend(kv, int(L))
        if L:
            k = torch.randn(int(L), hkv, d, device="cuda", dtype=torch.bfloat16).view(torch.int16)
            v = torch.randn(int(L), hkv, d, device="cuda", dtype=torch.bfloat16).view(torch.int16)
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
    q = torch.randn(batch, hq, d, device="cuda", dtype=torch.bfloat16).view(torch.int16)
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


def prefill_case(vt, torch, ctx, batch, context, ratio, hq=32, hkv=8, d=128, reps=5):
    P = int(round(context * ratio))
    N = context - P
    plens = np.full(batch, P, np.int32)
    kvs, kp, vp = _regions(vt, torch, ctx, plens, hkv, d)
    st = torch.cuda.current_stream().cuda_stream
    T = batch * N
    qn = torch.randn(T, hq, d, device="cuda", dtype=torch.bfloat16).view(torch.int16)
    kn = torch.randn(T, hkv, d, device="cuda", dtype=torch.bfloat16).view(torch.int16)
    vn = torch.randn(T, hkv, d, device="cuda", dtype=torch.bfloat16).view(torch.int16)
    out = torch.zeros_like(qn)
    cu = (np.arange(batch + 1) * N).astype(np.int32)
    a = vt.make_prefill_args(vt.VT_BF16, batch, hq, hkv, d, d ** -0.5, T, qn, out, kn, vn, kp, vp,
                             torch.from_numpy(cu).cuda(), torch.from_numpy(plens).cuda(), cu, plens)
    for _ in range(2):
        vt.vt_attn_prefix_prefill(ctx, a, st)
    torch.cuda.synchronize()
    vt.vt_profile_enable(ctx, True)
    for _ in range(reps):
        vt.vt_attn_prefix_prefill(ctx, a, st)
    torch.cuda.synchronize()
    vt.vt_profile_enable(ctx, False)
    ms, n = vt.vt_profile_collect(ctx, 1)
    for kv in kvs:
        vt.vt_release(kv)
    us = ms / n * 1e3
    flops = 4.0 * hq * d * batch * (N * P + N * (N + 1) / 2)
    return {"us": us, "tflops": flops / us / 1e6, "P": P, "N": N}


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
    ap.add_argument("--only", default="d1,d2,d3,p1,p2,m1")
    args = ap.parse_args()
    import paper_2407_15309_amd as vt
    only = set(args.only.split(","))
    say = lambda *a: print(*a, flush=True)
    if "m1" in only:
        memory_accounting(vt, say)
        only.discard("m1")
    if not only:
        return
    import torch
    if not torch.cuda.is_available():
        sys.exit("sweep: no GPU visible; the HIP path has no CPU fallback")
    ctx = vt.vt_init(0, 0, 0)
    with torch.cuda.stream(torch.cuda.Stream()):
        if "d1" in only:
            say("\n### d1: decode, 32/32 heads, head_dim 128, bf16, KV length 16384, batch sweep\n")
            say("| batch | kernel us | call us (with combine) | GB/s | of 8 TB/s |\n|---|---|---|---|---|")
            for b in ([1, 8, 64] if args.quick else [1, 2, 4, 8, 16, 32, 64]):
                r = decode_case(vt, torch, ctx, b, 16384, 32, 32)
                say("| %d | %.1f | %.1f | %.0f | %.3f |" % (b, r["kernel_us"], r["call_us"], r["gbps"], r["gbps"] / 8000))
        if "d2" in only:
            say("\n### d2: decode, 32/32 heads, batch 16, KV length sweep\n")
            say("| KV length | kernel us | call us (with combine) | GB/s | of 8 TB/s |\n|---|---|---|---|---|")
            for L in ([1024, 16384] if args.quick else [512, 1024, 2048, 4096, 8192, 16384, 32768]):
                r = decode_case(vt, torch, ctx, 16, L, 32, 32)
                say("| %d | %.1f | %.1f | %.0f | %.3f |" % (L, r["kernel_us"], r["call_us"], r["gbps"], r["gbps"] / 8000))
        if "d3" in only:
            say("\n### d3: decode, 32 query heads, batch 16, KV length 16384, KV-head sweep (MHA ... MQA)\n")
            say("| KV heads | flop per K/V byte | kernel us | GB/s | of 8 TB/s | TFLOP/s |\n|---|---|---|---|---|---|")
            for hkv in ([32, 8, 1] if args.quick else [32, 16, 8, 4, 2, 1]):
                r = decode_case(vt, torch, ctx, 16, 16384, 32, hkv)
                say("| %d | %.2f | %.1f | %.0f | %.3f | %.1f |" % (hkv, r["ai"], r["kernel_us"], r["gbps"], r["gbps"] / 8000, r["tflops"]))
        if "p1" in only:
            say("\n### p1: prefix-prefill, 32/8 heads, head_dim 128, bf16, context 16384, prefix ratio 0.5, batch sweep\n")
            say("| batch | prefix | new | us | TFLOP/s | of 2.5 PFLOP/s |\n|---|---|---|---|---|---|")
            for b in ([1, 4] if args.quick else [1, 2, 4, 8, 16]):
                r = prefill_case(vt, torch, ctx, b, 16384, 0.5)
                say("| %d | %d | %d | %.0f | %.0f | %.3f |" % (b, r["P"], r["N"], r["us"], r["tflops"], r["tflops"] / 2500))
        if "p2" in only:
            say("\n### p2: prefix-prefill, 32/8 heads, context 16384, batch 4, prefix-ratio sweep\n")
            say("| prefix ratio | prefix | new | us | TFLOP/s | of 2.5 PFLOP/s |\n|---|---|---|---|---|---|")
            for ratio in ([0.25, 0.75] if args.quick else [0.1, 0.25, 0.5, 0.75, 0.9]):
                r = prefill_case(vt, torch, ctx, 4, 16384, ratio)
                say("| %.2f | %d | %d | %.0f | %.0f | %.3f |" % (ratio, r["P"], r["N"], r["us"], r["tflops"], r["tflops"] / 2500))
    torch.cuda.synchronize()
    vt.vt_destroy(ctx)


if __name__ == "__main__":
    main()
