"""Pins for the oracle's decode-step attention (one generated token attending to the compact prompt held in the
contiguous KV cache: the per-token work inside the decoding cost C_dec of Eq. 2 / Eq. 7).  No HIP code is involved."""
import numpy as np
import pytest
import torch

import oracle


def caches(rng, b, hkv, s_max, d, n_ctx, poison=True):
    kc = rng.standard_normal((b, hkv, s_max, d)).astype(np.float32)
    vc = rng.standard_normal((b, hkv, s_max, d)).astype(np.float32)
    if poison:                                   # rows the call must never read
        kc[:, :, n_ctx:] = np.nan
        vc[:, :, n_ctx:] = np.nan
    return kc, vc


@pytest.mark.parametrize("shape", [(1, 4, 2, 64, 117, 117), (3, 8, 2, 128, 200, 77), (2, 6, 6, 72, 40, 40), (1, 2, 1, 16, 9, 1)])
def test_decode_matches_library_sdpa(shape):
    """Independent implementation: the library's scaled-dot-product attention in float64 on the first n_ctx rows."""
    b, hq, hkv, d, s_max, n = shape
    rng = np.random.default_rng(hq * d + n)
    q = rng.standard_normal((b, hq, d)).astype(np.float32)
    kc, vc = caches(rng, b, hkv, s_max, d, n)
    o = oracle.decode_attention(q, kc, vc, n)
    rep = hq // hkv
    tk = torch.from_numpy(kc[:, :, :n]).double().repeat_interleave(rep, dim=1)
    tv = torch.from_numpy(vc[:, :, :n]).double().repeat_interleave(rep, dim=1)
    tq = torch.from_numpy(q).double()[:, :, None, :]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[:, :, 0].numpy()
    assert np.isfinite(o).all() and np.abs(o - ref).max() < 1e-12
    o2 = oracle.decode_attention(q, kc, vc, n, scale=0.37)
    ref2 = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=0.37)[:, :, 0].numpy()
    assert np.abs(o2 - ref2).max() < 1e-12


def test_decode_is_the_last_row_of_causal_prefill():
    """The decode step for token n-1 is row n-1 of causal prefill attention over the same K and V (the cache holds
    the prompt's K/V head-major, the prefill oracle takes them token-major)."""
    rng = np.random.default_rng(5)
    b, s, hq, hkv, d = 2, 53, 8, 4, 32
    q = rng.standard_normal((b, s, hq, d)).astype(np.float32)
    k = rng.standard_normal((b, s, hkv, d)).astype(np.float32)
    v = rng.standard_normal((b, s, hkv, d)).astype(np.float32)
    full = oracle.attention(q, k, v, True)
    kc = np.zeros((b, hkv, s + 4, d), dtype=np.float32)
    vc = np.zeros_like(kc)
    oracle.kv_write(k, v, kc, vc, 0)
    for n in (1, 2, 31, s):
        o = oracle.decode_attention(q[:, n - 1], kc, vc, n)
        assert np.abs(o - full[:, n - 1]).max() < 1e-13


def test_decode_closed_forms():
    rng = np.random.default_rng(9)
    b, hq, hkv, d, s_max = 2, 4, 2, 24, 30
    q = rng.standard_normal((b, hq, d)).astype(np.float32)
    kc, vc = caches(rng, b, hkv, s_max, d, s_max, poison=False)
    # one row in the cache: the output is that V row, whatever q and K are
    o = oracle.decode_attention(q, kc, vc, 1)
    assert np.array_equal(o, np.repeat(vc[:, :, 0].astype(np.float64), 2, axis=1))
    # equal keys: uniform weights, the mean of the first n V rows
    k_eq = np.broadcast_to(kc[:, :, :1], kc.shape).copy()
    for n in (2, 17, 30):
        o = oracle.decode_attention(q, k_eq, vc, n)
        assert np.abs(o - np.repeat(vc[:, :, :n].astype(np.float64).mean(axis=2), 2, axis=1)).max() < 1e-14
    # constant V: that constant; a zero query: the mean as well
    v_c = np.broadcast_to(vc[:, :, :1], vc.shape).copy()
    assert np.abs(oracle.decode_attention(q, kc, v_c, 21) - np.repeat(v_c[:, :, 0].astype(np.float64), 2, axis=1)).max() < 1e-14
    o = oracle.decode_attention(np.zeros_like(q), kc, vc, 13)
    assert np.abs(o - np.repeat(vc[:, :, :13].astype(np.float64).mean(axis=2), 2, axis=1)).max() < 1e-14
    # one key far above the rest: the softmax saturates on it (and does not overflow)
    k_big = kc.copy()
    k_big[:, :, 7] = 0.0
    qq = np.ones_like(q)
    k_big[:, :, 7, :] = 400.0
    o = oracle.decode_attention(qq, k_big, vc, 20)
    assert np.isfinite(o).all() and np.abs(o - np.repeat(vc[:, :, 7].astype(np.float64), 2, axis=1)).max() < 1e-12
    # query heads of one group with equal queries give equal outputs; heads of different groups use different caches
    q_same = q.copy()
    q_same[:, 1] = q_same[:, 0]
    o = oracle.decode_attention(q_same, kc, vc, 30)
    assert np.array_equal(o[:, 0], o[:, 1])


def test_decode_brute_force_and_shift_invariance():
    rng = np.random.default_rng(21)
    b, hq, hkv, d, n = 1, 3, 3, 8, 11
    q = rng.standard_normal((b, hq, d)).astype(np.float32)
    kc, vc = caches(rng, b, hkv, n, d, n, poison=False)
    o = oracle.decode_attention(q, kc, vc, n, scale=0.5)
    for h in range(hq):
        z = 0.5 * (kc[0, h].astype(np.float64) @ q[0, h].astype(np.float64))
        p = np.exp(z - z.max())
        p /= p.sum()
        assert np.abs(o[0, h] - p @ vc[0, h].astype(np.float64)).max() < 1e-14
    # adding one vector to every key shifts all logits of a head by the same amount: the weights do not move
    shift = rng.standard_normal(d).astype(np.float32) * 0.25
    kc2 = (kc.astype(np.float64) + shift).astype(np.float32)
    # (exact only in real arithmetic: the shifted keys are rounded to fp32 again, so compare loosely)
    assert np.abs(oracle.decode_attention(q, kc2, vc, n, scale=0.5) - o).max() < 1e-5
