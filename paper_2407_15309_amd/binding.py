"""ctypes binding of libvt: the same entry points as include/vt.h, argument marshalling only.

Every step of the path runs inside the library's kernels; nothing here computes.  The shared library
must have been built (python -m paper_2407_15309_amd.build); importing this module fails loudly if it
is missing - there is no fallback implementation.
"""

from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvt.so")

VT_F16, VT_BF16 = 1, 2
VT_OK, VT_E_INVALID, VT_E_CAPACITY, VT_E_OOM, VT_E_DRIVER, VT_E_UNSUPPORTED, VT_E_WORKSPACE = 0, -1, -2, -3, -4, -5, -6
DTYPES = {"f16": VT_F16, "bf16": VT_BF16}

if not os.path.exists(LIB_PATH):
    raise ImportError("libvt.so is not built: run `python -m paper_2407_15309_amd.build` (needs hipcc); "
                      "there is no fallback path")
lib = C.CDLL(LIB_PATH)


class VtError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, lib.vt_strerror(status).decode(), status))


class KvInfo(C.Structure):
    _fields_ = [("k_ptr", C.c_void_p), ("v_ptr", C.c_void_p), ("len", C.c_uint64), ("max_tokens", C.c_uint64),
                ("row_bytes", C.c_uint64), ("chunk_bytes", C.c_uint64), ("chunks_mapped", C.c_uint64),
                ("capacity_bytes", C.c_uint64), ("n_kv_heads", C.c_uint32), ("head_dim", C.c_uint32),
                ("dtype", C.c_int32), ("shared_chunks", C.c_int32)]


class Stats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in (
        "reserved_va_bytes", "mapped_bytes", "phys_bytes", "chunks_created", "chunks_reused", "chunks_pooled",
        "va_reserved_calls", "va_reused", "create_calls", "map_calls", "unmap_calls", "release_calls",
        "va_free_calls", "driver_ns", "live_regions")]

    def asdict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class Plan(C.Structure):
    _fields_ = [("span_tokens", C.c_uint32), ("max_splits", C.c_uint32), ("n_units", C.c_uint64),
                ("workspace_bytes", C.c_uint64)]


class PrefillPlan(C.Structure):
    _fields_ = [("total_cost", C.c_uint64), ("n_tiles", C.c_uint64), ("n_items", C.c_uint32),
                ("n_groups", C.c_uint32), ("workspace_bytes", C.c_uint64)]


class PrefillPiece(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("group", "request", "kv_head", "token_tile", "tile_begin", "tile_end",
                                           "n_tiles", "n_fast")]


class DecodeArgs(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("batch", C.c_uint32), ("n_q_heads", C.c_uint32), ("n_kv_heads", C.c_uint32),
                ("head_dim", C.c_uint32), ("scale", C.c_float), ("q", C.c_void_p), ("out", C.c_void_p),
                ("k_ptrs", C.c_void_p), ("v_ptrs", C.c_void_p), ("kv_lens", C.c_void_p),
                ("kv_lens_host", C.c_void_p)]


class PrefillArgs(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("batch", C.c_uint32), ("n_q_heads", C.c_uint32), ("n_kv_heads", C.c_uint32),
                ("head_dim", C.c_uint32), ("scale", C.c_float), ("total_new_tokens", C.c_uint32),
                ("q_new", C.c_void_p), ("out", C.c_void_p), ("k_new", C.c_void_p), ("v_new", C.c_void_p),
                ("k_ptrs", C.c_void_p), ("v_ptrs", C.c_void_p), ("cu_seqlens", C.c_void_p),
                ("prefix_lens", C.c_void_p), ("cu_seqlens_host", C.c_void_p), ("prefix_lens_host", C.c_void_p)]


_vp, _u64, _u32, _i32 = C.c_void_p, C.c_uint64, C.c_uint32, C.c_int
_SIGS = {
    "vt_init": [C.POINTER(_vp), _i32, _u64, _u64],
    "vt_init_host": [C.POINTER(_vp), _u64, _u64],
    "vt_destroy": [_vp],
    "vt_reserve": [_vp, _u32, _u32, _i32, _u64, C.POINTER(_vp)],
    "vt_extend": [_vp, _u64],
    "vt_extend_batch": [C.POINTER(_vp), C.POINTER(_u64), _u32],
    "vt_share_prefix": [_vp, _u64, _u64, C.POINTER(_vp)],
    "vt_release": [_vp],
    "vt_trim": [_vp, _u64],
    "vt_query": [_vp, C.POINTER(KvInfo)],
    "vt_stats": [_vp, C.POINTER(Stats)],
    "vt_append": [_vp, _vp, _vp, _u64, _u64, _vp],
    "vt_append_batch": [_vp, _vp, _vp, _vp, _vp, _vp, _u32, _u32, _u32, _vp],
    "vt_extend_batch_async": [_vp, _vp, _u32, _vp],
    "vt_extend_wait": [_vp, _u64],
    "vt_plan_decode": [_vp, _vp, _u32, _u32, _u32, _u32, C.POINTER(Plan), _vp],
    "vt_plan_prefill": [_vp, _vp, _vp, _u32, _u32, _u32, _u32, C.c_int, C.POINTER(PrefillPlan), _vp, C.c_uint64, _vp],
    "vt_attn_decode": [_vp, C.POINTER(DecodeArgs), _vp],
    "vt_attn_decode_static": [_vp, C.POINTER(DecodeArgs), _vp],
    "vt_attn_prefix_prefill": [_vp, C.POINTER(PrefillArgs), _vp],
    "vt_workspace_reserve": [_vp, _u64],
    "vt_set_plan_target": [_vp, _u64],
    "vt_host_fail_after": [_vp, _i32, _i32],
    "vt_profile_enable": [_vp, _i32],
    "vt_profile_collect": [_vp, _i32, C.POINTER(C.c_double), C.POINTER(_u64)],
}
EXPORTS = sorted(list(_SIGS) + ["vt_strerror", "vt_static_scratch_bytes"])
for _n, _a in _SIGS.items():
    getattr(lib, _n).argtypes = _a
    getattr(lib, _n).restype = C.c_int
lib.vt_static_scratch_bytes.argtypes = []
lib.vt_static_scratch_bytes.restype = C.c_uint64
lib.vt_strerror.argtypes = [C.c_int]
lib.vt_strerror.restype = C.c_char_p


def _ptr(x) -> Optional[int]:
    """Address of a torch tensor / numpy array / ctypes array, an int as is, None as NULL."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if hasattr(x, "ctypes"):
        return x.ctypes.data
    return C.addressof(x)


def _check(rc: int, where: str) -> int:
    if rc != VT_OK:
        raise VtError(rc, where)
    return rc


def vt_strerror(status: int) -> str:
    return lib.vt_strerror(status).decode()


def vt_init(device: int = 0, chunk_bytes: int = 0, max_phys_bytes: int = 0) -> int:
    h = _vp()
    _check(lib.vt_init(C.byref(h), device, chunk_bytes, max_phys_bytes), "vt_init")
    return h.value


def vt_init_host(chunk_bytes: int = 0, max_phys_bytes: int = 0) -> int:
    h = _vp()
    _check(lib.vt_init_host(C.byref(h), chunk_bytes, max_phys_bytes), "vt_init_host")
    return h.value


def vt_destroy(ctx: int) -> None:
    _check(lib.vt_destroy(ctx), "vt_destroy")


def vt_reserve(ctx: int, n_kv_heads: int, head_dim: int, dtype: int, max_tokens: int) -> int:
    h = _vp()
    _check(lib.vt_reserve(ctx, n_kv_heads, head_dim, dtype, max_tokens, C.byref(h)), "vt_reserve")
    return h.value


def vt_extend(kv: int, new_len_tokens: int) -> None:
    _check(lib.vt_extend(kv, new_len_tokens), "vt_extend")


def vt_extend_batch(kvs: Sequence[int], new_lens: Sequence[int]) -> None:
    n = len(kvs)
    a = (_vp * n)(*kvs)
    l = (_u64 * n)(*[int(x) for x in new_lens])
    _check(lib.vt_extend_batch(a, l, n), "vt_extend_batch")


def vt_extend_batch_async(kvs: Sequence[int], new_lens: Sequence[int]) -> int:
    """Queues the extension for the context's worker thread; returns the ticket for vt_extend_wait."""
    n = len(kvs)
    a = (_vp * n)(*kvs)
    l = (_u64 * n)(*[int(x) for x in new_lens])
    t = C.c_uint64(0)
    _check(lib.vt_extend_batch_async(a, l, n, C.addressof(t)), "vt_extend_batch_async")
    return t.value


def vt_extend_wait(ctx: int, ticket: int) -> None:
    _check(lib.vt_extend_wait(ctx, ticket), "vt_extend_wait")


def vt_share_prefix(src: int, n_tokens: int, max_tokens: int) -> int:
    h = _vp()
    _check(lib.vt_share_prefix(src, n_tokens, max_tokens, C.byref(h)), "vt_share_prefix")
    return h.value


def vt_release(kv: int) -> None:
    _check(lib.vt_release(kv), "vt_release")


def vt_trim(ctx: int, keep_pooled_chunks: int = 0) -> None:
    _check(lib.vt_trim(ctx, keep_pooled_chunks), "vt_trim")


def vt_query(kv: int) -> KvInfo:
    info = KvInfo()
    _check(lib.vt_query(kv, C.byref(info)), "vt_query")
    return info


def vt_stats(ctx: int) -> Stats:
    st = Stats()
    _check(lib.vt_stats(ctx, C.byref(st)), "vt_stats")
    return st


def vt_append(kv: int, k_rows, v_rows, n_tokens: int, at_token: int, stream: int = 0) -> None:
    _check(lib.vt_append(kv, _ptr(k_rows), _ptr(v_rows), n_tokens, at_token, stream), "vt_append")


def vt_append_batch(ctx: int, k_ptrs, v_ptrs, kv_lens, k_rows, v_rows, batch: int, n_kv_heads: int, head_dim: int,
                    stream: int = 0) -> None:
    _check(lib.vt_append_batch(ctx, _ptr(k_ptrs), _ptr(v_ptrs), _ptr(kv_lens), _ptr(k_rows), _ptr(v_rows), batch,
                               n_kv_heads, head_dim, stream), "vt_append_batch")


def vt_plan_decode(ctx: int, kv_lens_host, n_kv_heads: int, n_q_heads: int, head_dim: int):
    """kv_lens_host: contiguous int32 numpy array.  Returns (Plan, n_splits int32 numpy array)."""
    import numpy as np
    lens = np.ascontiguousarray(kv_lens_host, dtype=np.int32)
    ns = np.zeros(len(lens), dtype=np.int32)
    plan = Plan()
    _check(lib.vt_plan_decode(ctx, lens.ctypes.data, len(lens), n_kv_heads, n_q_heads, head_dim, C.byref(plan),
                              ns.ctypes.data), "vt_plan_decode")
    return plan, ns


def vt_plan_prefill(ctx: int, cu_seqlens_host, prefix_lens_host, n_q_heads: int, n_kv_heads: int, head_dim: int,
                    new_rows_in_cache: bool = False, want_pieces: bool = False):
    """Host arrays as in make_prefill_args.  Returns PrefillPlan, or (PrefillPlan, [PrefillPiece, ...])."""
    import numpy as np
    cu = np.ascontiguousarray(cu_seqlens_host, dtype=np.int32)
    pl = np.ascontiguousarray(prefix_lens_host, dtype=np.int32)
    plan = PrefillPlan()
    n = C.c_uint64(0)
    _check(lib.vt_plan_prefill(ctx, cu.ctypes.data, pl.ctypes.data, len(pl), n_q_heads, n_kv_heads, head_dim,
                               int(new_rows_in_cache), C.byref(plan), None, 0, C.addressof(n)), "vt_plan_prefill")
    if not want_pieces:
        return plan
    arr = (PrefillPiece * max(1, n.value))()
    _check(lib.vt_plan_prefill(ctx, cu.ctypes.data, pl.ctypes.data, len(pl), n_q_heads, n_kv_heads, head_dim,
                               int(new_rows_in_cache), C.byref(plan), C.addressof(arr), n.value, C.addressof(n)),
           "vt_plan_prefill")
    return plan, list(arr)[: n.value]


def make_decode_args(dtype: int, batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int, scale: float, q, out,
                     k_ptrs, v_ptrs, kv_lens, kv_lens_host) -> DecodeArgs:
    return DecodeArgs(dtype, batch, n_q_heads, n_kv_heads, head_dim, scale, _ptr(q), _ptr(out), _ptr(k_ptrs),
                      _ptr(v_ptrs), _ptr(kv_lens), _ptr(kv_lens_host))


def vt_attn_decode(ctx: int, args: DecodeArgs, stream: int = 0) -> None:
    _check(lib.vt_attn_decode(ctx, C.byref(args), stream), "vt_attn_decode")


def vt_attn_decode_static(ctx: int, args: DecodeArgs, stream: int = 0) -> None:
    _check(lib.vt_attn_decode_static(ctx, C.byref(args), stream), "vt_attn_decode_static")


def vt_static_scratch_bytes() -> int:
    return int(lib.vt_static_scratch_bytes())


def make_prefill_args(dtype: int, batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int, scale: float,
                      total_new_tokens: int, q_new, out, k_new, v_new, k_ptrs, v_ptrs, cu_seqlens, prefix_lens,
                      cu_seqlens_host, prefix_lens_host) -> PrefillArgs:
    return PrefillArgs(dtype, batch, n_q_heads, n_kv_heads, head_dim, scale, total_new_tokens, _ptr(q_new), _ptr(out),
                       _ptr(k_new), _ptr(v_new), _ptr(k_ptrs), _ptr(v_ptrs), _ptr(cu_seqlens), _ptr(prefix_lens),
                       _ptr(cu_seqlens_host), _ptr(prefix_lens_host))


def vt_attn_prefix_prefill(ctx: int, args: PrefillArgs, stream: int = 0) -> None:
    _check(lib.vt_attn_prefix_prefill(ctx, C.byref(args), stream), "vt_attn_prefix_prefill")


def vt_workspace_reserve(ctx: int, nbytes: int) -> None:
    _check(lib.vt_workspace_reserve(ctx, nbytes), "vt_workspace_reserve")


def vt_set_plan_target(ctx: int, target_units: int) -> None:
    _check(lib.vt_set_plan_target(ctx, target_units), "vt_set_plan_target")


def vt_host_fail_after(ctx: int, op: int, countdown: int) -> None:
    _check(lib.vt_host_fail_after(ctx, op, countdown), "vt_host_fail_after")


def vt_profile_enable(ctx: int, on: bool) -> None:
    _check(lib.vt_profile_enable(ctx, 1 if on else 0), "vt_profile_enable")


def vt_profile_collect(ctx: int, which: int):
    """Returns (total_ms, launches) of the kernels of kind `which` recorded since the last collect."""
    ms, n = C.c_double(), _u64()
    _check(lib.vt_profile_collect(ctx, which, C.byref(ms), C.byref(n)), "vt_profile_collect")
    return ms.value, int(n.value)
