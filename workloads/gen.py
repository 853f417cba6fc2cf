"""Seeded generators for the five synthetic workloads.

Every workload is synthetic: request lengths are uniform integers on an
inclusive range and all Q/K/V entries are i.i.d. N(0,1) drawn in fp32 and
rounded to nearest-even into the 16-bit storage type.  The shapes follow the
paper's kernel sweeps (decode over batch / KV length / KV heads, prefix-prefill
over batch and prefix ratio, Evaluation section) and its multi-turn chat
scenario; they stand in for the datasets the paper samples, which are not
needed for kernel-level work.

Generation is counter based: the stream for (seed, tensor, request, step) is a
Philox generator keyed by those four integers, so arrays can be produced in any
order and on any number of threads and always hold the same bits.

Arrays are returned as uint16 bit patterns.  Consumers reinterpret them in their
own code (the oracle widens them to fp64, the HIP kernels read them natively).
"""

from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple

import numpy as np

# tensor ids used to key the random streams
T_KV_LEN, T_NEW_LEN, T_Q, T_K, T_V, T_QNEW, T_KNEW, T_VNEW, T_STEP_Q, T_STEP_K, T_STEP_V = range(11)


@dataclass(frozen=True)
class Config:
    cfg_id: int
    name: str
    kind: str                      # "decode" | "prefill" | "chat" | "steady"
    dtype: str                     # "f16" | "bf16"
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    kv_len: Tuple[int, int]        # cached length (decode) or prefix length (prefill), inclusive
    new_len: Optional[Tuple[int, int]] = None   # new tokens per request (prefill kinds)
    steps: int = 1                 # decode steps (steady kind)

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.head_dim))

    @property
    def row_elems(self) -> int:
        return self.n_kv_heads * self.head_dim

    def replace(self, **kw) -> "Config":
        return dataclasses.replace(self, **kw)


CONFIGS: Dict[int, Config] = {
    1: Config(1, "decode_fp16_small", "decode", "f16", 4, 8, 8, 64, (16, 256)),
    2: Config(2, "decode_bf16_llama2_7b_mha", "decode", "bf16", 64, 32, 32, 128, (512, 4096)),
    3: Config(3, "prefix_prefill_bf16_llama3_8b_gqa", "prefill", "bf16", 16, 32, 8, 128,
              (1024, 4096), (128, 512)),
    4: Config(4, "multiturn_chat_prefill_then_decode_bf16", "chat", "bf16", 8, 32, 8, 128,
              (8192, 32768), (64, 256)),
    5: Config(5, "steady_decode_bf16_70b_gqa", "steady", "bf16", 256, 64, 8, 128,
              (1024, 8192), None, 32),
}


def base_seed(cfg_id: int) -> int:
    return 0x240715309 + int(cfg_id)


def _gen(seed: int, tensor: int, request: int, step: int = 0) -> np.random.Generator:
    return np.random.Generator(
        np.random.Philox(key=[seed & (2**64 - 1), tensor], counter=[request, step, 0, 0]))


def draw_lengths(seed: int, tensor: int, batch: int, lo: int, hi: int) -> np.ndarray:
    """`batch` integers uniform on [lo, hi], as int32."""
    g = _gen(seed, tensor, 0)
    return g.integers(lo, hi + 1, size=batch, dtype=np.int64).astype(np.int32)


def _round_bits(x32: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 -> 16-bit storage bits, round to nearest even."""
    if dtype == "f16":
        return x32.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        u = x32.view(np.uint32)
        return ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)
    raise ValueError(dtype)


def normal_bits(seed: int, tensor: int, request: int, shape, dtype: str, step: int = 0) -> np.ndarray:
    """N(0,1) samples of `shape` as 16-bit storage bit patterns."""
    n = int(np.prod(shape))
    x = _gen(seed, tensor, request, step).standard_normal(n, dtype=np.float32)
    return _round_bits(x, dtype).reshape(shape)


def _per_request(fn, batch: int, threads: int) -> List[np.ndarray]:
    if threads <= 1 or batch <= 1:
        return [fn(b) for b in range(batch)]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(fn, range(batch)))


def decode_inputs(cfg: Config, seed: Optional[int] = None, threads: int = 8) -> dict:
    """Inputs of one decode step: kv_lens[B], q[B,Hq,D], per-request K_b,V_b [L_b,Hkv,D]."""
    seed = base_seed(cfg.cfg_id) if seed is None else seed
    lens = draw_lengths(seed, T_KV_LEN, cfg.batch, *cfg.kv_len)
    q = np.stack([normal_bits(seed, T_Q, b, (cfg.n_q_heads, cfg.head_dim), cfg.dtype)
                  for b in range(cfg.batch)])
    shp = lambda b: (int(lens[b]), cfg.n_kv_heads, cfg.head_dim)
    k = _per_request(lambda b: normal_bits(seed, T_K, b, shp(b), cfg.dtype), cfg.batch, threads)
    v = _per_request(lambda b: normal_bits(seed, T_V, b, shp(b), cfg.dtype), cfg.batch, threads)
    return {"seed": seed, "kv_lens": lens, "q": q, "k": k, "v": v}


def prefill_inputs(cfg: Config, seed: Optional[int] = None, threads: int = 8) -> dict:
    """Inputs of one prefix-prefill call.

    prefix_lens[B], new_lens[B], cu_seqlens[B+1]; cached K_b,V_b [P_b,Hkv,D];
    q_new [T,Hq,D], k_new/v_new [T,Hkv,D] with T = sum(new_lens), requests packed
    back to back.
    """
    seed = base_seed(cfg.cfg_id) if seed is None else seed
    plens = draw_lengths(seed, T_KV_LEN, cfg.batch, *cfg.kv_len)
    nlens = draw_lengths(seed, T_NEW_LEN, cfg.batch, *cfg.new_len)
    cu = np.zeros(cfg.batch + 1, dtype=np.int32)
    cu[1:] = np.cumsum(nlens)
    pshp = lambda b: (int(plens[b]), cfg.n_kv_heads, cfg.head_dim)
    k = _per_request(lambda b: normal_bits(seed, T_K, b, pshp(b), cfg.dtype), cfg.batch, threads)
    v = _per_request(lambda b: normal_bits(seed, T_V, b, pshp(b), cfg.dtype), cfg.batch, threads)
    qn = np.concatenate([normal_bits(seed, T_QNEW, b, (int(nlens[b]), cfg.n_q_heads, cfg.head_dim), cfg.dtype)
                         for b in range(cfg.batch)])
    kn = np.concatenate([normal_bits(seed, T_KNEW, b, (int(nlens[b]), cfg.n_kv_heads, cfg.head_dim), cfg.dtype)
                         for b in range(cfg.batch)])
    vn = np.concatenate([normal_bits(seed, T_VNEW, b, (int(nlens[b]), cfg.n_kv_heads, cfg.head_dim), cfg.dtype)
                         for b in range(cfg.batch)])
    return {"seed": seed, "prefix_lens": plens, "new_lens": nlens, "cu_seqlens": cu,
            "k": k, "v": v, "q_new": qn, "k_new": kn, "v_new": vn}


def step_inputs(cfg: Config, step: int, seed: Optional[int] = None) -> dict:
    """The query and the new K/V row of every request for decode step `step`."""
    seed = base_seed(cfg.cfg_id) if seed is None else seed
    q = np.stack([normal_bits(seed, T_STEP_Q, b, (cfg.n_q_heads, cfg.head_dim), cfg.dtype, step)
                  for b in range(cfg.batch)])
    k = np.stack([normal_bits(seed, T_STEP_K, b, (cfg.n_kv_heads, cfg.head_dim), cfg.dtype, step)
                  for b in range(cfg.batch)])
    v = np.stack([normal_bits(seed, T_STEP_V, b, (cfg.n_kv_heads, cfg.head_dim), cfg.dtype, step)
                  for b in range(cfg.batch)])
    return {"q": q, "k_row": k, "v_row": v}


def checksum64(*arrays) -> int:
    """Order-dependent 64-bit checksum of the given arrays' bytes (reporting only)."""
    h = np.uint64(0xCBF29CE484222325)
    with np.errstate(over="ignore"):
        for a in arrays:
            items = a if isinstance(a, (list, tuple)) else [a]
            for x in items:
                b = np.ascontiguousarray(x).view(np.uint8).ravel()
                pad = (-b.size) % 8
                if pad:
                    b = np.concatenate([b, np.zeros(pad, np.uint8)])
                w = b.view(np.uint64)
                h = (h ^ np.bitwise_xor.reduce(w * np.uint64(0x9E3779B97F4A7C15) + np.arange(w.size, dtype=np.uint64))) \
                    * np.uint64(0x100000001B3)
    return int(h)
