"""GPU parity of the rotary-embedding calls (civic_mrope_table, civic_mrope_apply, civic_kv_write_rope,
civic_prefill_attn_rope) against the CPU oracle, through the C ABI.
Bars: table entries within 2.5e-7 (the angle is formed and reduced in double precision, the result rounded to fp32);
rotated bf16 rows within 2^-8 * max(1, max|ref|) (fp32 arithmetic, one rounding to bf16), fp32 rows within 2e-6 * max(1,
max|ref|); V rows and untouched cache rows bit-exact; attention within the attention bar (2e-2 / 1e-4 * max(1, max|ref|))."""
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


def tables(d, theta=1.0e6, interleaved=False):
    n = d // 2
    inv = (theta ** (-np.arange(n, dtype=np.float64) * 2.0 / d)).astype(np.float32)
    if interleaved:
        axis = (np.arange(n) % 3).astype(np.int32)
    else:
        a, b = n // 4, (n - n // 4) // 2
        axis = np.repeat(np.arange(3), (a, b, n - a - b)).astype(np.int32)
    return axis, inv


def rope_tol(ref, dtype):
    return (2.0 ** -8 if dtype == "bf16" else 2e-6) * max(1.0, float(np.abs(ref).max()))


@pytest.mark.parametrize("name", list(wl.WORKLOADS))
def test_table_matches_oracle_on_compact_ids(bd, name):
    """The ids are the ones civic_compact carries (pos_c of the workload's selection)."""
    w = wl.WORKLOADS[name]
    log("mrope table", name)
    kept, _ = oracle.select(wl.scores(w, 0), w.grid_tuple())
    hid, _ = wl.hidden(w, 0)
    pos = wl.position_ids(w)
    _, pos_c, _ = bd.civic_compact(to_dev(hid), torch.from_numpy(pos.copy()).cuda(), w.grid_tuple(), wl.frame_starts(w),
                                   torch.from_numpy(kept).cuda())
    _, ref_pos_c, _ = oracle.compact(hid, pos, w.grid_tuple(), wl.frame_starts(w), kept)
    assert np.array_equal(to_host(pos_c), ref_pos_c)
    for inter in (False, True):
        axis, inv = tables(w.head_dim, interleaved=inter)
        cs = to_host(bd.civic_mrope_table(pos_c, axis, inv))
        ref = oracle.mrope_table(ref_pos_c, axis, inv)
        assert cs.shape == ref.shape and np.abs(cs - ref).max() <= 2.5e-7


def test_table_large_ids_and_odd_sizes(bd):
    rng = np.random.default_rng(3)
    for b, s, n in ((1, 1, 4), (2, 37, 36), (3, 1000, 64), (1, 5, 128)):
        pos = rng.integers(0, 2_000_000_000, (3, b, s)).astype(np.int32)     # far beyond what fp32 holds exactly
        pos[:, :, 0] = 0
        axis = rng.integers(0, 3, n).astype(np.int32)
        inv = (10000.0 ** (-np.arange(n) / n)).astype(np.float32)
        cs = to_host(bd.civic_mrope_table(torch.from_numpy(pos).cuda(), axis, inv))
        ref = oracle.mrope_table(pos, axis, inv)
        log("mrope table large ids", (b, s, n), float(np.abs(cs - ref).max()))
        assert np.abs(cs - ref).max() <= 2.5e-7 and np.array_equal(cs[:, 0, :, 0], np.ones((b, n), dtype=np.float32))


@pytest.mark.parametrize("shape,dtype", [((4, 938, 32, 128), "bf16"), ((1, 117, 4, 64), "fp32"), ((2, 33, 3, 96), "bf16"),
                                         ((1, 7, 1, 16), "bf16"), ((3, 50, 5, 8), "fp32"), ((1, 300, 2, 256), "bf16")])
def test_apply_matches_oracle(bd, shape, dtype):
    b, s, h, d = shape
    log("mrope apply", shape, dtype)
    rng = np.random.default_rng(d + s)
    st, x32 = wl.quantize(rng.standard_normal((b, s, h, d)).astype(np.float32) * 2, dtype)
    pos = rng.integers(0, 20000, (3, b, s)).astype(np.int32)
    axis, inv = tables(d)
    cs = bd.civic_mrope_table(torch.from_numpy(pos).cuda(), axis, inv)
    ref = oracle.mrope_apply(x32, oracle.mrope_table(pos, axis, inv))
    dx = to_dev(st)
    got = widen(to_host(bd.civic_mrope_apply(dx, cs))).astype(np.float64)
    assert np.abs(got - ref).max() <= rope_tol(ref, dtype)
    # strided input (head rows embedded in wider rows) and in place
    wide = torch.zeros((b, s, h, d + 16), dtype=dx.dtype, device="cuda")
    wide[..., :d] = dx
    view = wide[..., :d]
    bd.civic_mrope_apply(view, cs, out=view)
    assert np.array_equal(to_host(view), to_host(bd.civic_mrope_apply(dx, cs))) and not wide[..., d:].any()


@pytest.mark.parametrize("name", ["tiny", "2b", "8b", "video"])
def test_kv_write_rope_matches_oracle(bd, name):
    w = wl.WORKLOADS[name]
    log("kv_write_rope", name)
    _, (k, k32), (v, _) = wl.qkv(w, 2)
    b, s = k.shape[0], k.shape[1]
    rng = np.random.default_rng(w.index)
    pos = np.sort(rng.integers(0, 3 * s, (3, b, s)).astype(np.int32), axis=2)
    axis, inv = tables(w.head_dim, interleaved=True)
    cs = bd.civic_mrope_table(torch.from_numpy(pos).cuda(), axis, inv)
    ref_k = oracle.mrope_apply(k32, oracle.mrope_table(pos, axis, inv)).transpose(0, 2, 1, 3)     # [b, h, s, d]
    s_max, pos0 = s + 9, 4
    fill = 0x7B7B if k.dtype == np.uint16 else 123.0
    kc = np.full((b, w.n_kv_heads, s_max, w.head_dim), fill, dtype=k.dtype)
    dk, dv = to_dev(kc), to_dev(kc.copy())
    bd.civic_kv_write_rope(to_dev(k), to_dev(v), cs, dk, dv, pos0)
    hk, hv = to_host(dk), to_host(dv)
    ref_v = kc.copy()
    oracle.kv_write(v, v, ref_v, ref_v.copy(), pos0)
    assert np.array_equal(hv, ref_v)                                                   # V and its untouched rows: bit for bit
    assert np.array_equal(hk[:, :, :pos0], kc[:, :, :pos0]) and np.array_equal(hk[:, :, pos0 + s:], kc[:, :, pos0 + s:])
    got = widen(hk[:, :, pos0:pos0 + s]).astype(np.float64)
    assert np.abs(got - ref_k).max() <= rope_tol(ref_k, w.dtype)


@pytest.mark.parametrize("shape,causal,dtype", [((4, 938, 32, 8, 128), True, "bf16"), ((1, 469, 16, 8, 128), True, "bf16"),
                                                ((2, 200, 8, 8, 64), False, "bf16"), ((1, 150, 6, 2, 96), True, "bf16"),
                                                ((1, 117, 4, 2, 64), True, "fp32"), ((2, 70, 4, 4, 96), False, "bf16"),
                                                ((1, 90, 4, 2, 32), True, "bf16"), ((1, 60, 2, 1, 256), True, "bf16")])
def test_prefill_attn_rope_on_the_rotated_cache(bd, shape, causal, dtype):
    """The layer as it runs: K rotated into the cache by civic_kv_write_rope, attention reads K and V from the cache
    (head-major rows through the stride arguments) and rotates Q on the fly.  Oracle: attention(rope(q), rope(k), v) in
    fp64 on the unrounded rotations."""
    b, s, hq, hkv, d = shape
    log("attn_rope", shape, causal, dtype)
    rng = np.random.default_rng(s + d)
    mk = lambda h: wl.quantize(rng.standard_normal((b, s, h, d)).astype(np.float32), dtype)
    (q, q32), (k, k32), (v, v32) = mk(hq), mk(hkv), mk(hkv)
    pos = np.sort(rng.integers(0, 2 * s + 5, (3, b, s)).astype(np.int32), axis=2)
    axis, inv = tables(d)
    cs = bd.civic_mrope_table(torch.from_numpy(pos).cuda(), axis, inv)
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    s_max = s + 3
    kc = torch.zeros((b, hkv, s_max, d), dtype=dq.dtype, device="cuda")
    vc = torch.zeros_like(kc)
    bd.civic_kv_write_rope(dk, dv, cs, kc, vc, 0)
    k_view, v_view = kc[:, :, :s].permute(0, 2, 1, 3), vc[:, :, :s].permute(0, 2, 1, 3)   # [b, s, h_kv, d] views of the caches
    out = to_host(bd.civic_prefill_attn_rope(dq, k_view, v_view, cs, causal))
    ref_cs = oracle.mrope_table(pos, axis, inv)
    rq = oracle.mrope_apply(q32, ref_cs).astype(np.float32)
    rk = oracle.mrope_apply(k32, ref_cs).astype(np.float32)
    ref = oracle.attention(rq, rk, v32, causal)
    err = float(np.abs(widen(out).astype(np.float64) - ref).max())
    log("   max abs err", err, "tol", attn_tol(ref, dtype))
    assert err <= attn_tol(ref, dtype)
    # the same through the unfused calls: rotate Q with civic_mrope_apply, then plain attention on the cache views
    out2 = to_host(bd.civic_prefill_attn(bd.civic_mrope_apply(dq, cs), k_view, v_view, causal))
    if dtype == "bf16" and d in (64, 96, 128):
        assert np.array_equal(out, out2)                      # same kernel, same rounding of the rotated query
    else:                                                     # the fp32 kernel keeps the rotated query unrounded
        assert np.abs(widen(out2).astype(np.float64) - ref).max() <= attn_tol(ref, dtype)
