"""fp64 softmax attention over per-request contiguous K/V arrays (CPU oracle).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's CPU-baseline leg, never by the product package, and it shares no
code with the HIP kernels.

What is computed is the plain definition, written out head by head in fp64:

* Attention weights the value rows by the similarity of the query with the key
  rows (paper, Background, "LLM Inference").  The paper never prints the
  formula; the reading taken is the standard one,
  softmax_j(scale * <q, k_j>) applied to the rows v_j.
* Decode uses the last token's query against the whole KV cache of its request
  (Background, "LLM Inference", decode stage).
* With a cached prefix, the new tokens of a request reuse the cached K/V rows of
  the prefix and add their own (Background, "Prefix Cache"); the new tokens are
  causal among themselves and see the whole prefix.
* In grouped-query attention the query heads are divided into groups and each
  group shares one key head and one value head (Background, "KV Cache
  Optimization: GQA and MQA").  The paper does not say which heads form a group;
  the reading taken is contiguous blocks, kv_head = q_head // (Hq // Hkv).

Inputs arrive as the 16-bit storage patterns the GPU receives and are widened
exactly to fp64 by `widen`.  Pins: see tests/test_oracle_pins.py (brute force in
extended precision with no max shift, closed forms, invariants, the float64
scaled_dot_product_attention of a library).
"""

from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np


def widen(bits: np.ndarray, dtype: str) -> np.ndarray:
    """16-bit storage patterns (uint16) -> exact fp64 values."""
    bits = np.asarray(bits)
    if bits.dtype != np.uint16:
        raise TypeError("expected uint16 bit patterns")
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float64)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def softmax_rows(s: np.ndarray) -> np.ndarray:
    """Softmax along the last axis, p_j = exp(s_j - max s) / sum_j exp(s_j - max s)."""
    e = np.exp(s - np.max(s, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def _attend(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float,
            visible: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """One KV head.  q [R, D], k [L, D], v [L, D]; visible[r] = number of leading
    keys row r may see (None = all L).  Returns (out [R, D], p [R, L])."""
    s = scale * (q @ k.T)                                   # [R, L]
    if visible is not None:
        j = np.arange(k.shape[0])[None, :]
        s = np.where(j < visible[:, None], s, -np.inf)
    p = softmax_rows(s)
    return p @ v, p


def decode(q: np.ndarray, k: Sequence[np.ndarray], v: Sequence[np.ndarray], scale: float,
           return_p: bool = False):
    """Batched decode attention.

    q    [B, Hq, D]      fp64, one query token per request
    k[b] [L_b, Hkv, D]   fp64, the request's cached keys (L_b >= 1)
    v[b] [L_b, Hkv, D]   fp64
    Returns out [B, Hq, D] fp64 (and, if return_p, a list of p[b] [Hq, L_b]).
    """
    B, Hq, D = q.shape
    out = np.empty((B, Hq, D), dtype=np.float64)
    ps: List[np.ndarray] = []
    for b in range(B):
        L, Hkv, Dk = k[b].shape
        if L < 1 or Dk != D or v[b].shape != k[b].shape or Hq % Hkv:
            raise ValueError("bad shapes for request %d" % b)
        G = Hq // Hkv
        pb = np.empty((Hq, L), dtype=np.float64) if return_p else None
        for g in range(Hkv):
            hs = slice(g * G, (g + 1) * G)                 # the query heads that share kv head g
            o, p = _attend(q[b, hs, :], k[b][:, g, :], v[b][:, g, :], scale)
            out[b, hs, :] = o
            if return_p:
                pb[hs, :] = p
        if return_p:
            ps.append(pb)
    return (out, ps) if return_p else out


def prefix_prefill(q_new: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, cu_seqlens: np.ndarray,
                   k_prefix: Sequence[np.ndarray], v_prefix: Sequence[np.ndarray], scale: float,
                   return_p: bool = False):
    """Prefix-prefill attention.

    q_new [T, Hq, D], k_new/v_new [T, Hkv, D]: the new tokens of all requests packed
    back to back; request b owns rows cu_seqlens[b] .. cu_seqlens[b+1]-1.
    k_prefix[b], v_prefix[b] [P_b, Hkv, D]: the request's cached prefix (P_b >= 0).
    New token i of request b sits at absolute position P_b + i and sees keys
    0 .. P_b + i of concat(prefix, new).
    Returns out [T, Hq, D] fp64 (and, if return_p, a list over b of p [Hq, N_b, P_b+N_b]).
    """
    T, Hq, D = q_new.shape
    Hkv = k_new.shape[1]
    G = Hq // Hkv
    out = np.empty((T, Hq, D), dtype=np.float64)
    ps = []
    for b in range(len(cu_seqlens) - 1):
        lo, hi = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        N, P = hi - lo, k_prefix[b].shape[0]
        if N == 0:
            if return_p:
                ps.append(np.empty((Hq, 0, P)))
            continue
        kcat = np.concatenate([k_prefix[b], k_new[lo:hi]], axis=0)     # [P+N, Hkv, D]
        vcat = np.concatenate([v_prefix[b], v_new[lo:hi]], axis=0)
        visible = P + np.arange(N) + 1                                 # keys 0..P+i inclusive
        pb = np.empty((Hq, N, P + N)) if return_p else None
        for h in range(Hq):
            g = h // G
            o, p = _attend(q_new[lo:hi, h, :], kcat[:, g, :], vcat[:, g, :], scale, visible)
            out[lo:hi, h, :] = o
            if return_p:
                pb[h] = p
        if return_p:
            ps.append(pb)
    return (out, ps) if return_p else out
