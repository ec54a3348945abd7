"""GPU parity of the path for samples of different length and grid packed along the token axis (images of different grid
sizes in one batch): civic_compact_prefill_ragged and civic_prefill_attn_ragged through the C ABI against the oracle's
per-sample definitions, and against the rectangular calls on every sample alone (bit for bit).
Bars as in test_gpu_parity.py: indices, ids, rows and caches bit-exact; scores within 2e-5 * inv_tau; attention within
2e-2 (bf16) / 1e-4 (fp32) times max(1, max|ref|)."""
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


def layout(rng, grids, max_gap):
    starts, lens = [], []
    for g in grids:
        frames, hw = g[0], g[1] * g[2]
        gaps = rng.integers(0, max_gap + 1, frames + 1) if max_gap >= 0 else np.full(frames + 1, -max_gap)   # (negative: that gap everywhere)
        s, p = [], int(gaps[0])
        for f in range(frames):
            s.append(p)
            p += hw + int(gaps[f + 1])
        starts.append(np.asarray(s, dtype=np.int64)); lens.append(p)
    return starts, lens


MIXES = {
    # grids of the tabulated workloads side by side, and small ragged ones (odd cells, frame floors, nothing kept)
    "workload grids": ([(1, 16, 16, 4, 4, 2, 0, 85), (2, 32, 32, 4, 4, 1, 0, 682), (1, 32, 32, 4, 4, 1, 0, 341), (4, 24, 24, 4, 4, 1, 16, 768)], 96),
    # runs of samples of one shape (same grid, length and frame starts), which go through the kernels as one batch each
    "repeated shapes": ([(1, 16, 16, 4, 4, 2, 0, 85)] * 3 + [(2, 8, 8, 4, 4, 1, 0, 40)] + [(1, 32, 32, 4, 4, 1, 0, 341)] * 2 + [(1, 16, 16, 4, 4, 2, 0, 85)], -5),
    "small grids": ([(1, 3, 5, 2, 2, 1, 0, 4), (3, 2, 2, 2, 2, 0, 1, 5), (1, 1, 1, 1, 1, 0, 0, 0), (2, 7, 9, 3, 4, 2, 3, 40), (1, 8, 8, 8, 8, 0, 0, 64)], 7),
    # more frames than the merge's table holds per sample (those go out by themselves), and more samples than one launch takes
    "many frames, many samples": ([(9, 2, 3, 1, 1, 0, 1, 20), (1, 4, 4, 2, 2, 1, 0, 5), (16, 4, 4, 4, 4, 1, 2, 90), (16, 4, 4, 4, 4, 1, 2, 90)] +
                                  [(1 + i % 3, 3 + i % 4, 2 + i % 5, 2, 2, i % 2, i % 3, (1 + i % 3) * (3 + i % 4) * (2 + i % 5) // 3) for i in range(40)], 4),
}


@pytest.mark.parametrize("mix", list(MIXES))
@pytest.mark.parametrize("dtype,dim", [("bf16", 256), ("fp32", 64)])
def test_ragged_front_matches_oracle_and_the_rectangular_calls(bd, mix, dtype, dim):
    grids, max_gap = MIXES[mix]
    log("ragged front", mix, dtype, dim)
    rng = np.random.default_rng(len(grids) + dim)
    starts, lens = layout(rng, grids, max_gap)
    seq, vis, koff, comp = oracle.ragged_offsets(lens, grids)
    total = int(seq[-1])
    hid, hid32 = wl.quantize(rng.standard_normal((total, dim)).astype(np.float32), dtype)
    pos = rng.integers(0, 5000, (3, total)).astype(np.int32)
    anchor = rng.standard_normal(dim).astype(np.float32) + 0.25
    q_anchor = bd.civic_anchor_normalize(anchor)
    inv_tau = 3.0
    d_hid, d_pos, d_q = to_dev(hid), torch.from_numpy(pos).cuda(), torch.from_numpy(q_anchor).cuda()
    scores, kept, hc, pc, si = bd.civic_compact_prefill_ragged(d_hid, d_pos, lens, grids, starts, d_q, inv_tau)
    torch.cuda.synchronize()
    scores_h, kept_h = to_host(scores), to_host(kept)
    # scores of every sample's visual rows, in the order the selection reads them
    for b, g in enumerate(grids):
        hw = g[1] * g[2]
        rows = np.concatenate([np.arange(s, s + hw) for s in starts[b]]) + seq[b]
        ref = oracle.score(hid32[rows], q_anchor, inv_tau)
        assert np.abs(scores_h[vis[b]:vis[b + 1]] - ref).max() <= 2e-5 * inv_tau
    # the selection on the scores the GPU produced, then the merge on the GPU's kept list: both bit-exact
    assert np.array_equal(kept_h, oracle.select_ragged(scores_h, grids))
    ref_hc, ref_pc, ref_si = oracle.compact_ragged(hid, pos, lens, grids, starts, kept_h)
    assert np.array_equal(to_host(si), ref_si) and np.array_equal(to_host(pc), ref_pc) and np.array_equal(to_host(hc), ref_hc)
    # every sample equals the rectangular front call on that sample alone
    for b, g in enumerate(grids):
        a, e = int(seq[b]), int(seq[b + 1])
        s1, k1, h1, p1, i1 = bd.civic_compact_prefill(d_hid[a:e][None], d_pos[:, a:e][:, None].contiguous(), g, starts[b], d_q, inv_tau)
        assert torch.equal(s1[0], scores[vis[b]:vis[b + 1]]) and torch.equal(k1[0], kept[koff[b]:koff[b + 1]])
        assert torch.equal(h1[0], hc[comp[b]:comp[b + 1]]) and torch.equal(p1[:, 0], pc[:, comp[b]:comp[b + 1]])
        assert torch.equal(i1[0], si[comp[b]:comp[b + 1]])


@pytest.mark.parametrize("case", [
    # dtype, H_q, H_kv, d, sample lengths
    ("bf16", 32, 8, 128, [117, 938, 469, 64, 65, 1]),
    ("bf16", 8, 8, 72, [300, 2, 1365]),
    ("bf16", 4, 2, 64, list(range(1, 71))),                 # 70 samples: two groups of launches
    ("bf16", 2, 2, 96, [129]),
    ("fp32", 4, 2, 64, [117, 5, 40]),                        # the fp32 kernel: one launch per sample
    ("bf16", 4, 4, 256, [33, 70]),                           # head_dim > 128 takes it too
])
@pytest.mark.parametrize("causal", [True, False])
def test_ragged_attention_and_cache_match_oracle_and_the_rectangular_calls(bd, case, causal):
    dtype, hq, hkv, d, sizes = case
    log("ragged attention", case[:4], len(sizes), "samples, causal", causal)
    rng = np.random.default_rng(sum(sizes) + d)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    total, n = int(off[-1]), len(sizes)
    q, q32 = wl.quantize(rng.standard_normal((total, hq, d)).astype(np.float32), dtype)
    k, k32 = wl.quantize(rng.standard_normal((total, hkv, d)).astype(np.float32), dtype)
    v, v32 = wl.quantize(rng.standard_normal((total, hkv, d)).astype(np.float32), dtype)
    s_max, pos0 = max(sizes) + 5, 3
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    sentinel = 0x7FC1 if dtype == "bf16" else np.float32(-77.0)
    kc0 = np.full((n, hkv, s_max, d), sentinel, dtype=k.dtype)
    kc, vc = to_dev(kc0), to_dev(kc0)
    out = bd.civic_prefill_attn_ragged(dq, dk, dv, off, causal, 0.0, kc, vc, pos0)
    plain = bd.civic_prefill_attn_ragged(dq, dk, dv, off, causal)
    torch.cuda.synchronize()
    ref = oracle.attention_ragged(q32, k32, v32, off, causal)
    got = widen(to_host(out)).astype(np.float64)
    err = float(np.abs(got - ref).max())
    log("   rows", total, "max abs err", err, "tol", attn_tol(ref, dtype))
    assert np.isfinite(got).all() and err <= attn_tol(ref, dtype)
    assert torch.equal(out, plain)                            # with and without the caches: the same attention
    ref_kc, ref_vc = kc0.copy(), kc0.copy()
    oracle.kv_write_ragged(k, v, off, ref_kc, ref_vc, pos0)
    assert np.array_equal(to_host(kc).view(ref_kc.dtype), ref_kc) and np.array_equal(to_host(vc).view(ref_vc.dtype), ref_vc)
    # every sample equals the rectangular call on that sample alone (a few of them when there are many)
    for i in sorted({0, min(1, n - 1), n // 2, n - 1}):
        a, b = int(off[i]), int(off[i + 1])
        one = bd.civic_prefill_attn(dq[a:b][None], dk[a:b][None], dv[a:b][None], causal)
        assert torch.equal(one[0], out[a:b])


def test_ragged_path_chained(bd):
    """Front and attention of a ragged batch back to back: the compact rows are Q, their leading columns K and V (strided views),
    against the oracle fed with the GPU's own compact rows."""
    grids, max_gap = MIXES["workload grids"]
    rng = np.random.default_rng(17)
    starts, lens = layout(rng, grids, max_gap)
    seq, vis, koff, comp = oracle.ragged_offsets(lens, grids)
    dim, hq, hkv, d = 512, 4, 2, 128
    hid, _ = wl.quantize(rng.standard_normal((int(seq[-1]), dim)).astype(np.float32), "bf16")
    pos = rng.integers(0, 5000, (3, int(seq[-1]))).astype(np.int32)
    d_q = torch.from_numpy(bd.civic_anchor_normalize(rng.standard_normal(dim).astype(np.float32))).cuda()
    _, _, hc, _, _ = bd.civic_compact_prefill_ragged(to_dev(hid), torch.from_numpy(pos).cuda(), lens, grids, starts, d_q)
    qv = hc.view(-1, hq, d)                                   # [total_c, 4, 128]
    kv = hc[:, :hkv * d].view(-1, hkv, d)                     # leading columns, token stride = dim
    s_max = int(max(np.diff(comp)))
    kc = torch.zeros((len(grids), hkv, s_max, d), dtype=hc.dtype, device="cuda"); vc = torch.zeros_like(kc)
    out = bd.civic_prefill_attn_ragged(qv, kv, kv, comp, True, 0.0, kc, vc, 0)
    torch.cuda.synchronize()
    h32 = widen(to_host(hc))
    ref = oracle.attention_ragged(np.ascontiguousarray(h32.reshape(-1, hq, d)), np.ascontiguousarray(h32[:, :hkv * d].reshape(-1, hkv, d)),
                                  np.ascontiguousarray(h32[:, :hkv * d].reshape(-1, hkv, d)), comp, True)
    assert np.abs(widen(to_host(out)).astype(np.float64) - ref).max() <= attn_tol(ref, "bf16")
    for i in range(len(grids)):
        a, b = int(comp[i]), int(comp[i + 1])
        assert torch.equal(kc[i, :, :b - a], kv[a:b].permute(1, 0, 2)) and torch.equal(kc[i, :, b - a:], torch.zeros_like(kc[i, :, b - a:]))


@pytest.mark.parametrize("case", [
    # dtype, H_q, H_kv, d, context lengths
    ("bf16", 32, 8, 128, [117, 938, 469, 64, 65, 1]),
    ("bf16", 8, 8, 72, [300, 2, 1365]),
    ("bf16", 4, 2, 64, list(range(1, 301))),                 # 300 samples: two groups of launches
    ("fp32", 4, 2, 64, [117, 5, 40, 4000]),
    ("bf16", 16, 2, 128, [3000, 1, 1, 1]),                    # one long context next to empty-handed splits
])
def test_ragged_decode_matches_oracle_and_the_rectangular_call(bd, case):
    dtype, hq, hkv, d, sizes = case
    log("ragged decode", case[:4], len(sizes), "samples")
    rng = np.random.default_rng(sum(sizes) + d)
    n, s_max = len(sizes), max(sizes) + 3
    q, q32 = wl.quantize(rng.standard_normal((n, hq, d)).astype(np.float32), dtype)
    kc, kc32 = wl.quantize(rng.standard_normal((n, hkv, s_max, d)).astype(np.float32), dtype)     # rows past a sample's length hold data too
    vc, vc32 = wl.quantize(rng.standard_normal((n, hkv, s_max, d)).astype(np.float32), dtype)
    dq, dkc, dvc = to_dev(q), to_dev(kc), to_dev(vc)
    out = bd.civic_decode_attn_ragged(dq, dkc, dvc, sizes)
    torch.cuda.synchronize()
    ref = oracle.decode_attention_ragged(q32, kc32, vc32, sizes)
    got = widen(to_host(out)).astype(np.float64)
    err = float(np.abs(got - ref).max())
    log("   max abs err", err, "tol", attn_tol(ref, dtype))
    assert np.isfinite(got).all() and err <= attn_tol(ref, dtype)
    # a sample alone through the rectangular call: the same rows, possibly another split of them
    for i in sorted({0, n // 2, n - 1}):
        one = bd.civic_decode_attn(dq[i:i + 1], dkc[i:i + 1], dvc[i:i + 1], int(sizes[i]))
        assert np.abs(widen(to_host(one)).astype(np.float64) - got[i:i + 1]).max() <= attn_tol(ref, dtype)
