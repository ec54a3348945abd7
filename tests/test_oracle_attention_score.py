"""Pins for the oracle's attention (the prefill-attention term of Eq. 2 / Eq. 7, softmax form of
Eq. 9) and anchor-logit score (Eq. 8).  No HIP code is involved."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_28115_amd import workloads as wl


def sdpa_library(q, k, v, causal, scale=None):
    """Independent third implementation: the library's scaled-dot-product attention in float64."""
    tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(a)).double().permute(0, 2, 1, 3) for a in (q, k, v))
    rep = tq.shape[1] // tk.shape[1]
    tk, tv = tk.repeat_interleave(rep, dim=1), tv.repeat_interleave(rep, dim=1)
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=causal, scale=scale)
    return o.permute(0, 2, 1, 3).numpy()


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("shape", [(1, 117, 4, 2, 64), (2, 70, 6, 6, 72), (1, 33, 8, 2, 128), (3, 1, 2, 1, 16)])
def test_attention_matches_library_sdpa(shape, causal):
    b, s, hq, hkv, d = shape
    rng = np.random.default_rng(s * d + hq)
    q = rng.standard_normal((b, s, hq, d)).astype(np.float32)
    k = rng.standard_normal((b, s, hkv, d)).astype(np.float32)
    v = rng.standard_normal((b, s, hkv, d)).astype(np.float32)
    o = oracle.attention(q, k, v, causal)
    assert np.abs(o - sdpa_library(q, k, v, causal)).max() < 1e-12
    o2 = oracle.attention(q, k, v, causal, scale=0.3)
    assert np.abs(o2 - sdpa_library(q, k, v, causal, scale=0.3)).max() < 1e-12


def test_attention_brute_force_definition_on_tiny():
    w = wl.WORKLOADS["tiny"]
    (q, _), (k, _), (v, _) = wl.qkv(w, 0)
    o = oracle.attention(q, k, v, True)
    b, s, hq, d = q.shape
    grp = hq // k.shape[2]
    for h in range(hq):
        z = (q[0, :, h].astype(np.float64) @ k[0, :, h // grp].astype(np.float64).T) / np.sqrt(d)
        z[np.triu_indices(s, 1)] = -np.inf
        p = np.exp(z - z.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        assert np.abs(o[0, :, h] - p @ v[0, :, h // grp].astype(np.float64)).max() < 1e-12


def test_attention_closed_forms():
    rng = np.random.default_rng(11)
    b, s, hq, hkv, d = 2, 40, 4, 2, 32
    q = rng.standard_normal((b, s, hq, d)).astype(np.float32)
    k = rng.standard_normal((b, s, hkv, d)).astype(np.float32)
    v = rng.standard_normal((b, s, hkv, d)).astype(np.float32)
    o = oracle.attention(q, k, v, True)
    # causal row 0 sees only key 0
    assert np.allclose(o[:, 0], np.repeat(v[:, 0], 2, axis=1), atol=1e-14)
    # all keys equal -> uniform weights -> running mean of V (causal) / mean of V (full)
    k_eq = np.broadcast_to(k[:, :1], k.shape).copy()
    o = oracle.attention(q, k_eq, v, True)
    run_mean = np.cumsum(v.astype(np.float64), axis=1) / np.arange(1, s + 1)[None, :, None, None]
    assert np.abs(o - np.repeat(run_mean, 2, axis=2)).max() < 1e-12
    o = oracle.attention(q, k_eq, v, False)
    assert np.abs(o - np.repeat(v.astype(np.float64).mean(axis=1, keepdims=True), 2, axis=2)).max() < 1e-12
    # constant V comes back unchanged
    v_c = np.broadcast_to(v[:, :1], v.shape).copy()
    o = oracle.attention(q, k, v_c, False)
    assert np.abs(o - np.repeat(v_c.astype(np.float64), 2, axis=2)).max() < 1e-12
    # q heads of one group with equal queries give equal outputs; heads of different groups do not
    q2 = q.copy()
    q2[:, :, 1] = q2[:, :, 0]
    q2[:, :, 2] = q2[:, :, 0]
    o = oracle.attention(q2, k, v, True)
    assert np.array_equal(o[:, :, 0], o[:, :, 1]) and not np.allclose(o[:, :, 0], o[:, :, 2])
    # one dominant key: softmax saturates on it
    k_big = k.copy()
    k_big[:, 5] = 0
    q_one = np.zeros_like(q)
    q_one[..., 0] = 50.0
    k_big[:, :, :, 0] = -50.0
    k_big[:, 5, :, 0] = 50.0
    o = oracle.attention(q_one, k_big, v, False)
    assert np.abs(o - np.repeat(v[:, 5:6].astype(np.float64), 2, axis=2)).max() < 1e-12


def test_attention_strided_views_and_row_sampling():
    rng = np.random.default_rng(12)
    hid = rng.standard_normal((2, 30, 4 * 16)).astype(np.float32)
    q = hid.reshape(2, 30, 4, 16)
    kv = hid[:, :, :32].reshape(2, 30, 2, 16)             # K = V = first columns of the same rows
    o = oracle.attention(q, kv, kv, True)
    ref = sdpa_library(q, np.ascontiguousarray(kv), np.ascontiguousarray(kv), True)
    assert np.abs(o - ref).max() < 1e-12
    part = oracle.attention(q, kv, kv, True, row_step=7)
    assert np.array_equal(part[:, ::7], o[:, ::7]) and np.isnan(part[:, 1]).all()


def test_score_is_the_pearson_correlation_with_the_anchor():
    rng = np.random.default_rng(13)
    dim = 96
    a = (rng.standard_normal(dim) * 3 + 1).astype(np.float32)
    x = (rng.standard_normal((50, dim)) * rng.uniform(0.1, 10, (50, 1)) + rng.uniform(-5, 5, (50, 1))).astype(np.float32)
    q = oracle.anchor_normalize(a)
    assert abs(q.sum()) < 1e-12 and abs((q * q).sum() - 1) < 1e-12
    tau = 0.25
    s = oracle.score(x, q.astype(np.float32), 1 / tau)
    corr = np.asarray([np.corrcoef(a.astype(np.float64), r.astype(np.float64))[0, 1] for r in x])
    assert np.abs(s * tau - corr).max() < 2e-7            # fp32 rounding of q and of the result
    # eps of the layer norm rescales LN(a) only, Norm removes it again
    assert np.abs(oracle.anchor_normalize(a, eps=1e-6) - oracle.anchor_normalize(a, eps=0.5)).max() < 1e-12


def test_score_special_rows_and_invariances():
    rng = np.random.default_rng(14)
    dim = 64
    a = rng.standard_normal(dim).astype(np.float32)
    q = oracle.anchor_normalize(a).astype(np.float32)
    x = rng.standard_normal((8, dim)).astype(np.float32)
    x[0] = 2.5                                            # constant row
    x[1] = a                                              # the anchor itself
    x[2] = -3 * a + 4                                     # anti-aligned, shifted
    s = oracle.score(x, q, 2.0)
    assert s[0] == 0.0 and abs(s[1] - 2.0) < 1e-6 and abs(s[2] + 2.0) < 1e-6
    assert np.all(np.abs(s) <= 2.0 + 1e-6)
    s_aff = oracle.score(4 * x - 8, q, 2.0)               # exact in fp32: invariant to x -> alpha x + beta
    assert np.abs(s_aff - s).max() < 1e-6
    assert np.abs(oracle.score(x, q, 1.0) * 2 - s).max() < 1e-6
    # matches the definition written with library routines: <Norm(LN(a)), Norm(LN(x))>
    t = torch.from_numpy(x).double()
    ln = torch.nn.functional.layer_norm(t, (dim,), eps=1e-6)
    k0 = torch.nn.functional.normalize(ln, dim=-1)
    ref = (k0 @ torch.from_numpy(q).double()).numpy() * 2.0
    assert np.abs(s[1:] - ref[1:]).max() < 1e-5           # eps = 1e-6 perturbs the library form slightly


def test_bf16_bits_round_to_nearest_even_like_the_library():
    rng = np.random.default_rng(15)
    x = np.concatenate([rng.standard_normal(4096).astype(np.float32) * 100,
                        np.asarray([1.00390625, 1.01171875, -1.00390625, 0.0, -0.0, 65504.0, 1e-30], dtype=np.float32)])
    bits = wl.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), ref.view(torch.int16).numpy())
    assert np.array_equal(wl.bf16_bits_to_f32(bits), ref.float().numpy())
