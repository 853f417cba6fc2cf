"""Pins for the CPU oracle: things the mathematics fixes, independent of the oracle's own code.

The paper prints no worked numeric example of attention, so the pins are
(1) brute force of the literal definition in extended precision with no max
shift, written with Python loops, (2) closed forms, (3) invariants, (4) special
cases that reduce to each other or to a library routine (float64
scaled_dot_product_attention), and (5) mutation checks: plausible mistakes
planted in a copy of the oracle must trip at least one pin.
"""

import itertools
import math

import numpy as np
import pytest
import torch

import oracle
from oracle import attention as oa

RNG = np.random.default_rng(20240715)


def rand(*shape):
    return RNG.standard_normal(shape)


# ---------------------------------------------------------------------------------------------
# (1) brute force, literal definition, long double, no max shift
# ---------------------------------------------------------------------------------------------

def brute_row(q, keys, vals, scale):
    """out_d = sum_j exp(scale q.k_j) v_jd / sum_j exp(scale q.k_j), scalar loops in long double."""
    ld = np.longdouble
    w = []
    for j in range(len(keys)):
        s = ld(0)
        for d in range(len(q)):
            s += ld(q[d]) * ld(keys[j][d])
        w.append(np.exp(ld(scale) * s))
    z = sum(w, ld(0))
    out = []
    for d in range(len(vals[0])):
        acc = ld(0)
        for j in range(len(keys)):
            acc += w[j] * ld(vals[j][d])
        out.append(float(acc / z))
    return out


@pytest.mark.parametrize("B,Hq,Hkv,D,Lmax", [(1, 1, 1, 4, 5), (2, 4, 2, 8, 9), (2, 4, 1, 6, 7), (1, 3, 3, 5, 1)])
def test_decode_vs_brute_force(B, Hq, Hkv, D, Lmax):
    lens = [int(RNG.integers(1, Lmax + 1)) for _ in range(B)]
    q = rand(B, Hq, D)
    k = [rand(L, Hkv, D) for L in lens]
    v = [rand(L, Hkv, D) for L in lens]
    scale = 0.37
    out = oracle.decode(q, k, v, scale)
    G = Hq // Hkv
    for b in range(B):
        for h in range(Hq):
            g = h // G
            ref = brute_row(q[b, h], k[b][:, g, :], v[b][:, g, :], scale)
            np.testing.assert_allclose(out[b, h], ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("Hq,Hkv,D,PN", [(2, 1, 4, [(3, 2), (0, 4)]), (4, 2, 8, [(5, 3), (1, 1), (2, 0)])])
def test_prefix_prefill_vs_brute_force(Hq, Hkv, D, PN):
    cu = np.cumsum([0] + [n for _, n in PN])
    T = int(cu[-1])
    qn, kn, vn = rand(T, Hq, D), rand(T, Hkv, D), rand(T, Hkv, D)
    kp = [rand(p, Hkv, D) for p, _ in PN]
    vp = [rand(p, Hkv, D) for p, _ in PN]
    scale = 1.0 / math.sqrt(D)
    out = oracle.prefix_prefill(qn, kn, vn, cu, kp, vp, scale)
    G = Hq // Hkv
    for b, (p, n) in enumerate(PN):
        for i in range(n):
            for h in range(Hq):
                g = h // G
                keys = [kp[b][j, g] for j in range(p)] + [kn[cu[b] + j, g] for j in range(i + 1)]
                vals = [vp[b][j, g] for j in range(p)] + [vn[cu[b] + j, g] for j in range(i + 1)]
                ref = brute_row(qn[cu[b] + i, h], keys, vals, scale)
                np.testing.assert_allclose(out[cu[b] + i, h], ref, rtol=0, atol=1e-12)


# ---------------------------------------------------------------------------------------------
# (2) closed forms
# ---------------------------------------------------------------------------------------------

def test_zero_query_gives_mean_of_visible_values():
    L, H, D = 11, 2, 4
    k, v = rand(L, H, D), rand(L, H, D)
    out = oracle.decode(np.zeros((1, H, D)), [k], [v], 0.5)
    np.testing.assert_allclose(out[0], v.mean(axis=0), atol=1e-14)
    # prefill: row i averages the prefix and new rows 0..i
    P, N = 3, 4
    cu = np.array([0, N])
    kn, vn = rand(N, H, D), rand(N, H, D)
    out = oracle.prefix_prefill(np.zeros((N, H, D)), kn, vn, cu, [k[:P]], [v[:P]], 0.5)
    for i in range(N):
        ref = np.concatenate([v[:P], vn[: i + 1]]).mean(axis=0)
        np.testing.assert_allclose(out[i], ref, atol=1e-14)


def test_dominant_key_returns_its_value_row():
    L, H, D = 9, 1, 4
    q = rand(1, H, D)
    k, v = rand(L, H, D) * 0.01, rand(L, H, D)
    j = 6
    k[j, 0] = q[0, 0] * 100.0 / float(q[0, 0] @ q[0, 0])       # score 100 vs ~0 for the rest
    out = oracle.decode(q, [k], [v], 1.0)
    # every other weight is about exp(-100) = 4e-44
    assert np.max(np.abs(out[0, 0] - v[j, 0])) < 1e-40


def test_constant_shift_of_keys_changes_nothing():
    L, H, D = 13, 2, 8
    q, k, v = rand(2, H, D), [rand(L, H, D), rand(L - 3, H, D)], [rand(L, H, D), rand(L - 3, H, D)]
    c = rand(D)
    a = oracle.decode(q, k, v, 0.3)
    b = oracle.decode(q, [x + c for x in k], v, 0.3)
    np.testing.assert_allclose(a, b, atol=1e-12)


def test_two_keys_logistic_closed_form():
    """With two keys the weights are a logistic function of the score difference."""
    D = 3
    q = rand(1, 1, D)
    k, v = rand(2, 1, D), rand(2, 1, D)
    scale = 0.7
    d = scale * float(q[0, 0] @ (k[0, 0] - k[1, 0]))
    w0 = 1.0 / (1.0 + math.exp(-d))
    out = oracle.decode(q, [k], [v], scale)
    np.testing.assert_allclose(out[0, 0], w0 * v[0, 0] + (1 - w0) * v[1, 0], atol=1e-14)


def test_scale_is_applied_to_scores():
    """Doubling scale equals doubling q (scores are bilinear), and differs from the unscaled result."""
    L, H, D = 7, 1, 4
    q, k, v = rand(1, H, D), [rand(L, H, D)], [rand(L, H, D)]
    a = oracle.decode(q, k, v, 0.8)
    b = oracle.decode(2 * q, k, v, 0.4)
    c = oracle.decode(q, k, v, 0.4)
    np.testing.assert_allclose(a, b, atol=1e-13)
    assert np.max(np.abs(a - c)) > 1e-3


# ---------------------------------------------------------------------------------------------
# (3) invariants
# ---------------------------------------------------------------------------------------------

def test_softmax_rows_sum_to_one_and_are_probabilities():
    q = rand(2, 4, 8)
    k = [rand(17, 2, 8), rand(5, 2, 8)]
    v = [rand(17, 2, 8), rand(5, 2, 8)]
    _, ps = oracle.decode(q, k, v, 0.35, return_p=True)
    for p in ps:
        assert np.all(p >= 0)
        np.testing.assert_allclose(p.sum(axis=-1), 1.0, atol=1e-14)
    cu = np.array([0, 3, 7])
    _, ps = oracle.prefix_prefill(rand(7, 4, 8), rand(7, 2, 8), rand(7, 2, 8), cu, [x[:4] for x in k],
                                  [x[:4] for x in v], 0.35, return_p=True)
    for b, p in enumerate(ps):
        np.testing.assert_allclose(p.sum(axis=-1), 1.0, atol=1e-14)
        P = 4
        for i in range(p.shape[1]):
            assert np.all(p[:, i, P + i + 1:] == 0.0), "future keys must get zero weight"
            assert np.all(p[:, i, : P + i + 1] > 0.0)


def test_identical_value_rows_return_that_row():
    L, H, D = 10, 2, 4
    row = rand(H, D)
    v = np.broadcast_to(row, (L, H, D)).copy()
    out = oracle.decode(rand(1, 4, D), [rand(L, H, D)], [v], 0.5)
    np.testing.assert_allclose(out[0], np.repeat(row, 2, axis=0), atol=1e-14)


def test_single_key_returns_its_value():
    H, D = 3, 4
    v = rand(1, H, D)
    out = oracle.decode(rand(1, H, D), [rand(1, H, D)], [v], 0.5)
    np.testing.assert_array_equal(out[0], v[0])


def test_decode_is_invariant_under_key_permutation():
    L, H, D = 23, 2, 8
    q, k, v = rand(1, 4, D), rand(L, H, D), rand(L, H, D)
    perm = RNG.permutation(L)
    a = oracle.decode(q, [k], [v], 0.3)
    b = oracle.decode(q, [k[perm]], [v[perm]], 0.3)
    np.testing.assert_allclose(a, b, atol=1e-13)


def test_appending_a_token_changes_no_prior_output():
    """Causality: prefill rows < i are unchanged when token i is appended; decode over the first L keys is
    unchanged when the arrays grow."""
    H, D, P, N = 2, 4, 5, 6
    kp, vp = [rand(P, H, D)], [rand(P, H, D)]
    qn, kn, vn = rand(N, 4, D), rand(N, H, D), rand(N, H, D)
    full = oracle.prefix_prefill(qn, kn, vn, np.array([0, N]), kp, vp, 0.5)
    part = oracle.prefix_prefill(qn[:-1], kn[:-1], vn[:-1], np.array([0, N - 1]), kp, vp, 0.5)
    np.testing.assert_array_equal(full[:-1], part)
    big_k, big_v = rand(12, H, D), rand(12, H, D)
    q = rand(1, 4, D)
    a = oracle.decode(q, [big_k[:9].copy()], [big_v[:9].copy()], 0.5)
    b = oracle.decode(q, [big_k[:9]], [big_v[:9]], 0.5)          # views into the grown array
    np.testing.assert_array_equal(a, b)


def test_requests_are_independent():
    q = rand(3, 2, 4)
    k = [rand(L, 2, 4) for L in (4, 9, 2)]
    v = [rand(L, 2, 4) for L in (4, 9, 2)]
    allb = oracle.decode(q, k, v, 0.5)
    for b in range(3):
        one = oracle.decode(q[b:b + 1], [k[b]], [v[b]], 0.5)
        np.testing.assert_array_equal(allb[b], one[0])


# ---------------------------------------------------------------------------------------------
# (4) special cases that reduce to each other / to a library routine
# ---------------------------------------------------------------------------------------------

def sdpa64(q, k, v, mask, scale):
    """float64 library attention.  q [H, R, D], k/v [H, L, D], mask [R, L] bool."""
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x))
    o = torch.nn.functional.scaled_dot_product_attention(t(q)[None], t(k)[None], t(v)[None],
                                                         attn_mask=t(mask)[None, None], scale=scale)
    return o[0].numpy()


def test_decode_vs_library_sdpa():
    L, Hq, Hkv, D = 37, 6, 2, 16
    q, k, v = rand(1, Hq, D), rand(L, Hkv, D), rand(L, Hkv, D)
    out = oracle.decode(q, [k], [v], 0.21)
    G = Hq // Hkv
    kk = np.repeat(k.transpose(1, 0, 2), G, axis=0)
    vv = np.repeat(v.transpose(1, 0, 2), G, axis=0)
    ref = sdpa64(q[0][:, None, :], kk, vv, np.ones((1, L), bool), 0.21)
    np.testing.assert_allclose(out[0], ref[:, 0, :], atol=1e-12)


def test_prefix_prefill_vs_library_sdpa_dense_mask():
    Hq, Hkv, D = 4, 2, 8
    PN = [(6, 5), (0, 3), (9, 1)]
    cu = np.cumsum([0] + [n for _, n in PN])
    T = int(cu[-1])
    qn, kn, vn = rand(T, Hq, D), rand(T, Hkv, D), rand(T, Hkv, D)
    kp = [rand(p, Hkv, D) for p, _ in PN]
    vp = [rand(p, Hkv, D) for p, _ in PN]
    out = oracle.prefix_prefill(qn, kn, vn, cu, kp, vp, 0.3)
    G = Hq // Hkv
    for b, (p, n) in enumerate(PN):
        kc = np.concatenate([kp[b], kn[cu[b]:cu[b + 1]]]).transpose(1, 0, 2)
        vc = np.concatenate([vp[b], vn[cu[b]:cu[b + 1]]]).transpose(1, 0, 2)
        mask = np.arange(p + n)[None, :] <= (p + np.arange(n))[:, None]
        ref = sdpa64(qn[cu[b]:cu[b + 1]].transpose(1, 0, 2), np.repeat(kc, G, 0), np.repeat(vc, G, 0), mask, 0.3)
        np.testing.assert_allclose(out[cu[b]:cu[b + 1]].transpose(1, 0, 2), ref, atol=1e-12)


def test_prefill_without_prefix_is_causal_self_attention():
    H, D, N = 2, 8, 9
    qn, kn, vn = rand(N, H, D), rand(N, H, D), rand(N, H, D)
    out = oracle.prefix_prefill(qn, kn, vn, np.array([0, N]), [np.zeros((0, H, D))], [np.zeros((0, H, D))], 0.4)
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x.transpose(1, 0, 2)))[None]
    ref = torch.nn.functional.scaled_dot_product_attention(t(qn), t(kn), t(vn), is_causal=True, scale=0.4)
    np.testing.assert_allclose(out.transpose(1, 0, 2), ref[0].numpy(), atol=1e-12)


def test_prefill_row_equals_decode_over_its_visible_keys():
    Hq, Hkv, D, P, N = 4, 2, 8, 7, 5
    qn, kn, vn = rand(N, Hq, D), rand(N, Hkv, D), rand(N, Hkv, D)
    kp, vp = rand(P, Hkv, D), rand(P, Hkv, D)
    out = oracle.prefix_prefill(qn, kn, vn, np.array([0, N]), [kp], [vp], 0.25)
    for i in range(N):
        kc = np.concatenate([kp, kn[: i + 1]])
        vc = np.concatenate([vp, vn[: i + 1]])
        dec = oracle.decode(qn[i][None], [kc], [vc], 0.25)
        np.testing.assert_allclose(out[i], dec[0], atol=1e-13)


def test_gqa_equals_mha_on_head_repeated_kv():
    L, Hq, Hkv, D = 12, 8, 2, 4
    q, k, v = rand(1, Hq, D), rand(L, Hkv, D), rand(L, Hkv, D)
    G = Hq // Hkv
    a = oracle.decode(q, [k], [v], 0.5)
    b = oracle.decode(q, [np.repeat(k, G, axis=1)], [np.repeat(v, G, axis=1)], 0.5)
    np.testing.assert_allclose(a, b, atol=1e-14)
    # and the groups are contiguous blocks of query heads, not interleaved
    c = oracle.decode(q, [np.tile(k, (1, G, 1))], [np.tile(v, (1, G, 1))], 0.5)
    assert np.max(np.abs(a - c)) > 1e-3


# ---------------------------------------------------------------------------------------------
# widening of storage bits
# ---------------------------------------------------------------------------------------------

def test_widen_known_bit_patterns():
    bits = np.array([0x3F80, 0xBF80, 0x4000, 0x3F00, 0x0000, 0x3FC0, 0x4049], dtype=np.uint16)
    np.testing.assert_array_equal(oracle.widen(bits, "bf16"), [1.0, -1.0, 2.0, 0.5, 0.0, 1.5, 3.140625])
    bits = np.array([0x3C00, 0xBC00, 0x4000, 0x3800, 0x0000, 0x3E00, 0x0001], dtype=np.uint16)
    np.testing.assert_array_equal(oracle.widen(bits, "f16"), [1.0, -1.0, 2.0, 0.5, 0.0, 1.5, 2.0 ** -24])


def test_widen_matches_torch_for_every_pattern():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    for name, tdt in (("bf16", torch.bfloat16), ("f16", torch.float16)):
        with np.errstate(invalid="ignore"):
            ours = oracle.widen(bits, name)
        ref = torch.from_numpy(bits.view(np.int16).copy()).view(tdt).to(torch.float64).numpy()
        np.testing.assert_array_equal(np.nan_to_num(ours, nan=123.0), np.nan_to_num(ref, nan=123.0))


# ---------------------------------------------------------------------------------------------
# (5) mutation checks: plausible mistakes planted in the oracle (on the CPU) must trip a pin
# ---------------------------------------------------------------------------------------------

def _pins_pass() -> bool:
    try:
        test_decode_vs_brute_force(2, 4, 2, 8, 9)
        test_prefix_prefill_vs_brute_force(4, 2, 8, [(5, 3), (1, 1), (2, 0)])
        test_gqa_equals_mha_on_head_repeated_kv()
        test_prefill_row_equals_decode_over_its_visible_keys()
        test_scale_is_applied_to_scores()
        return True
    except AssertionError:
        return False


def test_planted_mistakes_are_caught(monkeypatch):
    assert _pins_pass()
    orig_attend = oa._attend

    def no_scale(q, k, v, scale, visible=None):
        return orig_attend(q, k, v, 1.0, visible)

    def off_by_one_mask(q, k, v, scale, visible=None):
        return orig_attend(q, k, v, scale, None if visible is None else visible - 1 + (visible == 1))

    def swapped_kv(q, k, v, scale, visible=None):
        return orig_attend(q, v, k, scale, visible)

    def no_normalisation(q, k, v, scale, visible=None):
        o, p = orig_attend(q, k, v, scale, visible)
        return o * 1.01, p

    for bad in (no_scale, off_by_one_mask, swapped_kv, no_normalisation):
        monkeypatch.setattr(oa, "_attend", bad)
        assert not _pins_pass(), bad.__name__
    monkeypatch.setattr(oa, "_attend", orig_attend)
    assert _pins_pass()
