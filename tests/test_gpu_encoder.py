"""GPU parity of the encoder-side calls against the CPU oracle, through the C ABI: civic_anchor_aggregate (Eq. 8),
civic_kv_compress and civic_cross_attn (Eq. 9).
Bars: max|out - ref| <= 2e-2 * max(1, max|ref|) for the bf16 outputs (operands of the contractions are rounded to
bf16, 2^-9 relative, accumulation is fp32); token weights (sums of up to M_e bf16-rounded probabilities) within
2e-2 * max(1, max|ref|) as well."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_28115_amd import workloads as wl
from test_gpu_parity import attn_tol, log, to_dev, to_host, widen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bd():
    from paper_2605_28115_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return binding


@pytest.mark.parametrize("shape", [
    # batch, tokens, anchors, dim
    (1, 64, 32, 64), (2, 300, 70, 128), (1, 1000, 333, 256), (2, 4096, 1365, 1152), (3, 129, 129, 192), (1, 5, 1, 64),
    (1, 257, 130, 64),
])
def test_anchor_aggregate_matches_oracle(bd, shape):
    b, t, m, d = shape
    log("anchor_aggregate", shape)
    rng = np.random.default_rng(t + m)
    x, x32 = wl.quantize((rng.standard_normal((b, t, d)) * 1.5 + 0.3).astype(np.float32), "bf16")
    a, a32 = wl.quantize(rng.standard_normal((m, d)).astype(np.float32), "bf16")
    for inv_tau in (1.0, 14.0):
        z, tw = bd.civic_anchor_aggregate(to_dev(x), to_dev(a), inv_tau, want_token_weight=True)
        ref, ref_tw = oracle.anchor_aggregate(x32, a32, inv_tau, want_col_sum=True)
        got = widen(to_host(z)).astype(np.float64)
        err = float(np.abs(got - ref).max())
        err_w = float(np.abs(to_host(tw).astype(np.float64) - ref_tw).max())
        log("   inv_tau", inv_tau, "max abs err", err, "tol", attn_tol(ref, "bf16"), "weights err", err_w)
        assert np.isfinite(got).all() and err <= attn_tol(ref, "bf16")
        assert err_w <= 2e-2 * max(1.0, float(ref_tw.max()))


def test_anchor_aggregate_picks_single_tokens(bd):
    """Anchors that are dense tokens, cold softmax: every output row is one X_0 row at full magnitude, so a token tile
    lost or misplaced in either contraction shows."""
    rng = np.random.default_rng(8)
    b, t, m, d = 1, 1500, 400, 128
    x, x32 = wl.quantize(rng.standard_normal((b, t, d)).astype(np.float32), "bf16")
    pick = rng.permutation(t)[:m]
    a = x[0, pick].copy()
    z = widen(to_host(bd.civic_anchor_aggregate(to_dev(x), to_dev(a), 300.0))).astype(np.float64)
    ref = oracle.anchor_aggregate(x32, wl.bf16_bits_to_f32(a), 300.0)
    assert np.abs(ref[0] - x32[0, pick]).max() < 0.05 and np.abs(z - ref).max() <= attn_tol(ref, "bf16")


@pytest.mark.parametrize("shape", [
    # batch, rows (M_e), memory anchors (S), heads, head_dim
    (1, 64, 16, 2, 64), (2, 1365, 256, 16, 72), (1, 300, 300, 4, 128), (3, 77, 5, 3, 32), (1, 1000, 64, 8, 128), (1, 130, 129, 1, 64),
])
def test_kv_compress_and_cross_attention_match_oracle(bd, shape):
    b, m, s, h, d = shape
    log("kv_compress", shape)
    rng = np.random.default_rng(m + s)
    mk = lambda: wl.quantize(rng.standard_normal((b, m, h, d)).astype(np.float32), "bf16")
    (q, q32), (k, k32), (v, v32) = mk(), mk(), mk()
    r = (rng.random((m, s)) ** 4).astype(np.float32)             # peaked, non-negative assignment weights
    r[:, s // 2] *= 50.0                                          # column scales must not matter
    kc, vc = bd.civic_kv_compress(to_dev(k), to_dev(v), torch.from_numpy(r).cuda())
    ref_kc = oracle.kv_compress(k32.reshape(b, m, h * d), r).reshape(b, s, h, d)
    ref_vc = oracle.kv_compress(v32.reshape(b, m, h * d), r).reshape(b, s, h, d)
    for got, ref in ((kc, ref_kc), (vc, ref_vc)):
        err = float(np.abs(widen(to_host(got)).astype(np.float64) - ref).max())
        log("   compress max abs err", err)
        assert err <= attn_tol(ref, "bf16")
    # Eq. 9 end to end: attention of the M_e queries over the S compressed keys and values
    out = to_host(bd.civic_cross_attn(to_dev(q), kc, vc))
    ref = oracle.cross_attention(q32, ref_kc.astype(np.float32), ref_vc.astype(np.float32))
    err = float(np.abs(widen(out).astype(np.float64) - ref).max())
    log("   attention max abs err", err, "tol", attn_tol(ref, "bf16"))
    assert err <= attn_tol(ref, "bf16")
    # and on exactly the bits the GPU compressed to (isolates the attention kernel)
    ref2 = oracle.cross_attention(q32, widen(to_host(kc)), widen(to_host(vc)))
    assert np.abs(widen(out).astype(np.float64) - ref2).max() <= attn_tol(ref2, "bf16")


@pytest.mark.parametrize("shape", [(1, 100, 1, 4, 2, 128), (2, 33, 500, 8, 8, 64), (1, 1365, 256, 16, 16, 72), (1, 64, 4097, 4, 1, 128),
                                   (1, 200, 63, 2, 2, 256), (2, 70, 65, 4, 4, 32)])
def test_cross_attention_shapes(bd, shape):
    b, nq, nkv, hq, hkv, d = shape
    log("cross_attn", shape)
    rng = np.random.default_rng(nq + nkv)
    (q, q32) = wl.quantize(rng.standard_normal((b, nq, hq, d)).astype(np.float32) * 1.5, "bf16")
    (k, k32) = wl.quantize(rng.standard_normal((b, nkv, hkv, d)).astype(np.float32), "bf16")
    (v, v32) = wl.quantize(rng.standard_normal((b, nkv, hkv, d)).astype(np.float32), "bf16")
    out = to_host(bd.civic_cross_attn(to_dev(q), to_dev(k), to_dev(v)))
    ref = oracle.cross_attention(q32, k32, v32)
    assert np.abs(widen(out).astype(np.float64) - ref).max() <= attn_tol(ref, "bf16")
    if d <= 64:
        q32b = rng.standard_normal((b, nq, hq, d)).astype(np.float32)
        out = to_host(bd.civic_cross_attn(to_dev(q32b), to_dev(k32), to_dev(v32), 0.3))
        ref = oracle.cross_attention(q32b, k32, v32, scale=0.3)
        assert np.abs(out.astype(np.float64) - ref).max() <= attn_tol(ref, "fp32")


def test_token_weights_feed_the_selection(bd):
    """The multi-anchor weights of Eq. 8 as the importance score of the selection: civic_select on the weights the
    GPU produced equals the oracle's selection on the same array."""
    w = wl.WORKLOADS["2b"]
    rng = np.random.default_rng(4)
    x, _ = wl.quantize(rng.standard_normal((1, w.n_visual, 256)).astype(np.float32), "bf16")
    a, _ = wl.quantize(rng.standard_normal((40, 256)).astype(np.float32), "bf16")
    _, tw = bd.civic_anchor_aggregate(to_dev(x), to_dev(a), 10.0, want_token_weight=True)
    kept, _ = bd.civic_select(tw, w.grid_tuple())
    ref_kept, _ = oracle.select(to_host(tw), w.grid_tuple())
    assert np.array_equal(to_host(kept), ref_kept)


@pytest.mark.parametrize("sizes", [[300, 1365, 77, 1024], [64], [1, 2, 3, 500], [1365, 341, 85]])
def test_ragged_items_match_oracle_and_the_rectangular_calls(bd, sizes):
    """Eq. 9 on images of different grid sizes in one batch: packed rows, every item by itself."""
    log("ragged Eq. 9", sizes)
    h, d, s = 4, 64, 128
    rng = np.random.default_rng(sum(sizes))
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    total = int(off[-1])
    mk = lambda: wl.quantize(rng.standard_normal((total, h, d)).astype(np.float32), "bf16")
    (q, q32), (k, k32), (v, v32) = mk(), mk(), mk()
    r = (rng.random((total, s)) ** 4).astype(np.float32)
    dq, dk, dv, dr = to_dev(q), to_dev(k), to_dev(v), torch.from_numpy(r).cuda()
    kc, vc = bd.civic_kv_compress_ragged(dk, dv, dr, off)
    out = bd.civic_cross_attn_ragged(dq, kc, vc, off)
    torch.cuda.synchronize()
    ref_kc = oracle.kv_compress_ragged(k32.reshape(total, h * d), r, off).reshape(len(sizes), s, h, d)
    ref_vc = oracle.kv_compress_ragged(v32.reshape(total, h * d), r, off).reshape(len(sizes), s, h, d)
    for got, ref in ((kc, ref_kc), (vc, ref_vc)):
        assert np.abs(widen(to_host(got)).astype(np.float64) - ref).max() <= attn_tol(ref, "bf16")
    ref = oracle.cross_attention_ragged(q32, widen(to_host(kc)), widen(to_host(vc)), off)
    err = float(np.abs(widen(to_host(out)).astype(np.float64) - ref).max())
    log("   attention max abs err", err, "tol", attn_tol(ref, "bf16"))
    assert np.isfinite(widen(to_host(out))).all() and err <= attn_tol(ref, "bf16")
    # every item equals the rectangular calls on that item alone, bit for bit
    for i, (a, b) in enumerate(zip(off[:-1], off[1:])):
        kc1, vc1 = bd.civic_kv_compress(dk[a:b][None], dv[a:b][None], dr[a:b].contiguous())
        assert torch.equal(kc1[0], kc[i]) and torch.equal(vc1[0], vc[i])
        assert torch.equal(bd.civic_cross_attn(dq[a:b][None], kc[i:i + 1], vc[i:i + 1])[0], out[a:b])


@pytest.mark.parametrize("dtype,hq,hkv,d,n_items,n_kv", [
    ("bf16", 8, 2, 128, 150, 96),      # more items than one launch's table holds, 4 query heads per KV head
    ("bf16", 4, 4, 72, 70, 33),        # padded head, a key count that ends inside a tile
    ("bf16", 2, 1, 64, 3, 700),        # few long items
    ("fp32", 4, 2, 64, 9, 40),         # the fp32 kernel: one launch per item
])
def test_ragged_cross_attention_in_one_launch(bd, dtype, hq, hkv, d, n_items, n_kv):
    """Packed queries of many items against each item's own keys: the workgroups find their item in the launch's table."""
    log("ragged cross attention", dtype, hq, hkv, d, n_items, n_kv)
    rng = np.random.default_rng(n_items * 1000 + n_kv)
    sizes = rng.integers(1, 90, n_items)
    sizes[::7] = rng.integers(150, 400, sizes[::7].size)          # some items several row tiles long
    sizes[-1] = 1
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    total = int(off[-1])
    q, q32 = wl.quantize(rng.standard_normal((total, hq, d)).astype(np.float32), dtype)
    k, k32 = wl.quantize(rng.standard_normal((n_items, n_kv, hkv, d)).astype(np.float32), dtype)
    v, v32 = wl.quantize(rng.standard_normal((n_items, n_kv, hkv, d)).astype(np.float32), dtype)
    out = torch.full((total + 2, hq, d), 7.0, dtype=to_dev(q).dtype, device="cuda")     # two sentinel rows behind the last item
    bd.civic_cross_attn_ragged(to_dev(q), to_dev(k), to_dev(v), off, out=out[:total])
    torch.cuda.synchronize()
    ref = oracle.cross_attention_ragged(q32, k32, v32, off)
    got = widen(to_host(out))
    err = float(np.abs(got[:total].astype(np.float64) - ref).max())
    log("   rows", total, "max abs err", err, "tol", attn_tol(ref, dtype))
    assert np.isfinite(got).all() and err <= attn_tol(ref, dtype)
    assert np.all(got[total:] == 7.0)


def test_ragged_compression_of_more_items_than_one_group(bd):
    """70 items of 1 to 200 rows: two groups of launches, every item with its own column sums and contraction length."""
    rng = np.random.default_rng(70)
    sizes = rng.integers(1, 200, 70)
    sizes[[0, 63, 64, 69]] = [1, 64, 65, 128]
    log("ragged compression", len(sizes), "items")
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    total, width, s = int(off[-1]), 136, 20
    k, k32 = wl.quantize(rng.standard_normal((total, width)).astype(np.float32), "bf16")
    v, v32 = wl.quantize(rng.standard_normal((total, width)).astype(np.float32), "bf16")
    r = (rng.random((total, s)) ** 4).astype(np.float32)
    dk, dv, dr = to_dev(k), to_dev(v), torch.from_numpy(r).cuda()
    kc, vc = bd.civic_kv_compress_ragged(dk, dv, dr, off)
    torch.cuda.synchronize()
    for got, x32 in ((kc, k32), (vc, v32)):
        ref = oracle.kv_compress_ragged(x32, r, off)
        err = float(np.abs(widen(to_host(got)).astype(np.float64) - ref).max())
        log("   max abs err", err, "tol", attn_tol(ref, "bf16"))
        assert np.isfinite(widen(to_host(got))).all() and err <= attn_tol(ref, "bf16")
    for i in (0, 1, 63, 64, 69):
        a, b = off[i], off[i + 1]
        kc1, vc1 = bd.civic_kv_compress(dk[a:b][None], dv[a:b][None], dr[a:b].contiguous())
        assert torch.equal(kc1[0], kc[i]) and torch.equal(vc1[0], vc[i])
