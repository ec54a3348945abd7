"""Pins for the oracle's encoder-side functions: the soft anchor aggregation of Eq. 8 and the KV-compressed visual
attention of Eq. 9.  No HIP code is involved."""
import numpy as np
import pytest
import torch

import oracle


def test_aggregate_matches_library_composition():
    """layer_norm -> normalize -> softmax over tokens -> matmul, from the library, in float64."""
    rng = np.random.default_rng(0)
    b, t, m, d = 2, 37, 9, 24
    x = (rng.standard_normal((b, t, d)) * 2 + 0.5).astype(np.float32)
    a = rng.standard_normal((m, d)).astype(np.float32)
    for inv_tau in (1.0, 14.0):
        z, cs = oracle.anchor_aggregate(x, a, inv_tau, want_col_sum=True)
        tx, ta = torch.from_numpy(x).double(), torch.from_numpy(a).double()
        k0 = torch.nn.functional.normalize(torch.nn.functional.layer_norm(tx, (d,), eps=1e-6), dim=-1)
        qa = torch.nn.functional.normalize(torch.nn.functional.layer_norm(ta, (d,), eps=1e-6), dim=-1)
        w = torch.softmax(qa @ k0.transpose(1, 2) * inv_tau, dim=-1)             # [b, m, t], softmax over the dense tokens
        assert np.abs(z - (w @ tx).numpy()).max() < 1e-12
        assert np.abs(cs - w.sum(dim=1).numpy()).max() < 1e-12


def test_aggregate_logits_are_the_single_anchor_scores():
    """Row a of the logits is what oracle_score gives for anchor a: W_A[a, :] = softmax of the scores."""
    rng = np.random.default_rng(1)
    t, m, d = 50, 4, 32
    x = rng.standard_normal((1, t, d)).astype(np.float32)
    a = (rng.standard_normal((m, d)) + 0.25).astype(np.float32)
    z = oracle.anchor_aggregate(x, a, 3.0, eps=0.0)
    for i in range(m):
        q = oracle.anchor_normalize(a[i], eps=0.0).astype(np.float32)
        s = oracle.score(x[0], q, 3.0).astype(np.float64)
        w = np.exp(s - s.max())
        w /= w.sum()
        assert np.abs(z[0, i] - w @ x[0].astype(np.float64)).max() < 1e-5       # (scores and q pass through fp32)


def test_aggregate_closed_forms():
    rng = np.random.default_rng(2)
    b, t, m, d = 1, 20, 5, 16
    x = rng.standard_normal((b, t, d)).astype(np.float32)
    a = rng.standard_normal((m, d)).astype(np.float32)
    # infinite temperature: uniform weights, every anchor returns the mean token
    z, cs = oracle.anchor_aggregate(x, a, 0.0, want_col_sum=True)
    assert np.abs(z - x.astype(np.float64).mean(axis=1, keepdims=True)).max() < 1e-13
    assert np.abs(cs - m / t).max() < 1e-13
    # the weights of an anchor sum to one: a constant column of X_0 comes through unchanged, outputs stay inside
    # the range of the tokens, and the total weight handed out is the number of anchors
    x2 = x.copy()
    x2[..., 3] = 7.5
    z, cs = oracle.anchor_aggregate(x2, a, 5.0, want_col_sum=True)
    assert np.abs(z[..., 3] - 7.5).max() < 1e-12 and abs(cs.sum() - m) < 1e-12
    x64 = x2.astype(np.float64)
    assert (z <= x64.max(axis=1, keepdims=True) + 1e-12).all() and (z >= x64.min(axis=1, keepdims=True) - 1e-12).all()
    # a cold softmax on an anchor that is one of the tokens picks that token
    a3 = x[0, [4, 11]].copy()
    z = oracle.anchor_aggregate(x, a3, 2000.0)
    assert np.abs(z[0] - x[0, [4, 11]].astype(np.float64)).max() < 1e-9
    # the aggregation does not care how tokens are ordered
    perm = rng.permutation(t)
    assert np.abs(oracle.anchor_aggregate(x[:, perm], a, 4.0) - oracle.anchor_aggregate(x, a, 4.0)).max() < 1e-13


def test_kv_compress_and_cross_attention():
    rng = np.random.default_rng(3)
    b, m, h, d, s = 2, 30, 4, 16, 7
    q = rng.standard_normal((b, m, h, d)).astype(np.float32)
    k = rng.standard_normal((b, m, h, d)).astype(np.float32)
    v = rng.standard_normal((b, m, h, d)).astype(np.float32)
    r = rng.random((m, s)).astype(np.float32)
    kc = oracle.kv_compress(k.reshape(b, m, h * d), r)
    rbar = r.astype(np.float64) / r.astype(np.float64).sum(axis=0, keepdims=True)
    assert np.abs(rbar.sum(axis=0) - 1).max() < 1e-14
    assert np.abs(kc - np.einsum("ms,bmw->bsw", rbar, k.reshape(b, m, h * d).astype(np.float64))).max() < 1e-13
    # library attention over the compressed keys and values
    vc = oracle.kv_compress(v.reshape(b, m, h * d), r)
    kc4, vc4 = kc.reshape(b, s, h, d).astype(np.float32), vc.reshape(b, s, h, d).astype(np.float32)
    o = oracle.cross_attention(q, kc4, vc4)
    ref = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q).double().permute(0, 2, 1, 3),
                                                           torch.from_numpy(kc4).double().permute(0, 2, 1, 3),
                                                           torch.from_numpy(vc4).double().permute(0, 2, 1, 3))
    assert np.abs(o - ref.permute(0, 2, 1, 3).numpy()).max() < 1e-12
    # R = identity: nothing is compressed, the result is plain bidirectional attention
    eye = np.eye(m, dtype=np.float32)
    assert np.array_equal(oracle.kv_compress(k.reshape(b, m, h * d), eye), k.reshape(b, m, h * d).astype(np.float64))
    assert np.abs(oracle.cross_attention(q, k, v) - oracle.attention(q, k, v, False)).max() < 1e-13
    # a permutation matrix reorders the memory slots, which attention does not see
    pm = eye[:, rng.permutation(m)]
    kp = oracle.kv_compress(k.reshape(b, m, h * d), pm).reshape(b, m, h, d).astype(np.float32)
    vp = oracle.kv_compress(v.reshape(b, m, h * d), pm).reshape(b, m, h, d).astype(np.float32)
    assert np.abs(oracle.cross_attention(q, kp, vp) - oracle.attention(q, k, v, False)).max() < 1e-13
    # one memory slot fed by every row: K_c is the mean key, V_c the mean value, every query returns the mean value
    ones = np.ones((m, 1), dtype=np.float32)
    v1 = oracle.kv_compress(v.reshape(b, m, h * d), ones)
    assert np.abs(v1[:, 0] - v.reshape(b, m, h * d).astype(np.float64).mean(axis=1)).max() < 1e-14
    o1 = oracle.cross_attention(q, oracle.kv_compress(k.reshape(b, m, h * d), ones).reshape(b, 1, h, d).astype(np.float32),
                                v1.reshape(b, 1, h, d).astype(np.float32))
    assert np.abs(o1 - v1.reshape(b, 1, h, d).astype(np.float32).astype(np.float64)).max() < 1e-14
    # scaling a column of R changes nothing (columns are normalised); an all-zero column gives a zero row
    r2 = r.copy()
    r2[:, 2] *= 9.0
    assert np.abs(oracle.kv_compress(k.reshape(b, m, h * d), r2) - kc).max() < 1e-6
    r2[:, 2] = 0.0
    assert not oracle.kv_compress(k.reshape(b, m, h * d), r2)[:, 2].any()
    # grouped heads: query heads of one group share the compressed keys of their KV head
    k2, v2 = k[:, :s, :2], v[:, :s, :2]
    og = oracle.cross_attention(q, k2, v2)
    rep = lambda a: np.repeat(a, 2, axis=2)
    assert np.abs(og - oracle.cross_attention(q, rep(k2), rep(v2))).max() < 1e-14


def test_ragged_items_are_compressed_and_attended_one_by_one():
    """Items of different sizes packed back to back (images of different grids in one batch, Eq. 9)."""
    rng = np.random.default_rng(5)
    sizes, h, d, s = [9, 30, 1, 17], 2, 8, 5
    off = np.concatenate([[0], np.cumsum(sizes)])
    total = int(off[-1])
    q = rng.standard_normal((total, h, d)).astype(np.float32)
    k = rng.standard_normal((total, h * d)).astype(np.float32)
    v = rng.standard_normal((total, h * d)).astype(np.float32)
    r = rng.random((total, s)).astype(np.float32)
    kc, vc = oracle.kv_compress_ragged(k, r, off), oracle.kv_compress_ragged(v, r, off)
    assert kc.shape == (4, s, h * d)
    # every item against the definition written out with numpy, on its own rows only
    for i, (a, b) in enumerate(zip(off[:-1], off[1:])):
        rb = r[a:b].astype(np.float64)
        rb = rb / rb.sum(axis=0, keepdims=True)
        assert np.abs(kc[i] - rb.T @ k[a:b].astype(np.float64)).max() < 1e-13
    # an item does not see the others: changing item 1 leaves items 0, 2, 3 as they were
    k2 = k.copy()
    k2[off[1]:off[2]] += 3.0
    kc2 = oracle.kv_compress_ragged(k2, r, off)
    assert np.array_equal(kc2[[0, 2, 3]], kc[[0, 2, 3]]) and not np.array_equal(kc2[1], kc[1])
    # attention of the packed queries over their own item's compressed keys: library attention item by item
    k4, v4 = kc.reshape(4, s, h, d).astype(np.float32), vc.reshape(4, s, h, d).astype(np.float32)
    o = oracle.cross_attention_ragged(q, k4, v4, off)
    for i, (a, b) in enumerate(zip(off[:-1], off[1:])):
        t = lambda x: torch.from_numpy(x).double().permute(1, 0, 2)[None]
        ref = torch.nn.functional.scaled_dot_product_attention(t(q[a:b]), t(k4[i]), t(v4[i]))[0].permute(1, 0, 2).numpy()
        assert np.abs(o[a:b] - ref).max() < 1e-12
    # equal sizes: the packed form is the rectangular one
    m = 6
    off_eq = np.arange(0, 4 * m + 1, m)
    xe = rng.standard_normal((4, m, h * d)).astype(np.float32)
    re = rng.random((m, s)).astype(np.float32)
    assert np.array_equal(oracle.kv_compress_ragged(xe.reshape(4 * m, -1), np.tile(re, (4, 1)), off_eq), oracle.kv_compress(xe, re))
    qe = rng.standard_normal((4, m, h, d)).astype(np.float32)
    assert np.array_equal(oracle.cross_attention_ragged(qe.reshape(4 * m, h, d), k4, v4, off_eq), oracle.cross_attention(qe, k4, v4).reshape(4 * m, h, d))
