"""Helpers for the GPU tests: place seeded workloads into VMM regions, call the library, read results back.

Only marshalling lives here; expected values always come from oracle/.
"""

from __future__ import annotations

import ctypes as C
from typing import List, Sequence

import numpy as np
import torch

import paper_2407_15309_amd as vt

TOL = {"bf16": 2e-2, "f16": 5e-3}     # max-abs tolerance against the fp64 oracle

_hip = None


def hip():
    global _hip
    if _hip is None:
        _hip = C.CDLL("libamdhip64.so")
        _hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
        _hip.hipMemcpy.restype = C.c_int
    return _hip


def dev_bits(a: np.ndarray) -> torch.Tensor:
    """uint16 bit patterns -> device int16 tensor holding the same bits."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()


def host_bits(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint16)


def read_device(ptr: int, nbytes: int) -> np.ndarray:
    """Copies raw device bytes at `ptr` to the host."""
    torch.cuda.synchronize()
    out = np.empty(nbytes, dtype=np.uint8)
    rc = hip().hipMemcpy(out.ctypes.data, ptr, nbytes, 2)   # device to host
    assert rc == 0, rc
    return out


def stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class Regions:
    """One VMM-backed K/V region pair per request, filled from host bit arrays."""

    def __init__(self, ctx: int, k: Sequence[np.ndarray], v: Sequence[np.ndarray], dtype: str, max_tokens=None,
                 headroom: int = 0):
        self.ctx = ctx
        self.kvs: List[int] = []
        self.lens = np.array([x.shape[0] for x in k], dtype=np.int32)
        hkv, d = k[0].shape[1], k[0].shape[2]
        self.hkv, self.d = hkv, d
        for b in range(len(k)):
            L = int(self.lens[b])
            mt = max_tokens if max_tokens is not None else max(L + headroom, 1)
            kv = vt.vt_reserve(ctx, hkv, d, vt.DTYPES[dtype], mt)
            vt.vt_extend(kv, L)
            if L:
                kd, vd = dev_bits(k[b]), dev_bits(v[b])
                vt.vt_append(kv, kd, vd, L, 0, stream())
                torch.cuda.synchronize()
            self.kvs.append(kv)
        self.refresh()

    def refresh(self):
        infos = [vt.vt_query(kv) for kv in self.kvs]
        self.k_ptrs = torch.tensor([i.k_ptr for i in infos], dtype=torch.int64).cuda()
        self.v_ptrs = torch.tensor([i.v_ptr for i in infos], dtype=torch.int64).cuda()
        self.lens = np.array([i.len for i in infos], dtype=np.int32)
        self.lens_dev = torch.from_numpy(self.lens).cuda()

    def release(self):
        torch.cuda.synchronize()
        for kv in self.kvs:
            vt.vt_release(kv)
        self.kvs = []


def run_decode(ctx: int, dtype: str, q_bits: np.ndarray, k_ptrs: torch.Tensor, v_ptrs: torch.Tensor,
               lens: np.ndarray, hkv: int, scale: float, lens_dev=None) -> np.ndarray:
    """Calls vt_attn_decode through the C ABI; returns the output bit patterns [B, Hq, D] (uint16)."""
    B, hq, d = q_bits.shape
    q = dev_bits(q_bits)
    out = torch.zeros_like(q)
    lens = np.ascontiguousarray(lens, dtype=np.int32)
    lens_dev = torch.from_numpy(lens).cuda() if lens_dev is None else lens_dev
    args = vt.make_decode_args(vt.DTYPES[dtype], B, hq, hkv, d, scale, q, out, k_ptrs, v_ptrs, lens_dev, lens)
    vt.vt_attn_decode(ctx, args, stream())
    torch.cuda.synchronize()
    return host_bits(out)


def run_prefill(ctx: int, dtype: str, data: dict, k_ptrs: torch.Tensor, v_ptrs: torch.Tensor, hkv: int, scale: float,
                new_in_cache: bool = False) -> np.ndarray:
    """Calls vt_attn_prefix_prefill; returns output bits [T, Hq, D]."""
    qn = dev_bits(data["q_new"])
    T, hq, d = data["q_new"].shape
    out = torch.zeros_like(qn)
    kn = None if new_in_cache else dev_bits(data["k_new"])
    vn = None if new_in_cache else dev_bits(data["v_new"])
    cu = np.ascontiguousarray(data["cu_seqlens"], dtype=np.int32)
    pl = np.ascontiguousarray(data["prefix_lens"], dtype=np.int32)
    cu_d, pl_d = torch.from_numpy(cu).cuda(), torch.from_numpy(pl).cuda()
    args = vt.make_prefill_args(vt.DTYPES[dtype], len(pl), hq, hkv, d, scale, T, qn, out, kn, vn, k_ptrs, v_ptrs,
                                cu_d, pl_d, cu, pl)
    vt.vt_attn_prefix_prefill(ctx, args, stream())
    torch.cuda.synchronize()
    return host_bits(out)
