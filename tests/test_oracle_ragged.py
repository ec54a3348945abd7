"""Pins of the oracle's ragged forms (samples of different length and grid packed along the token axis): every sample
against definitions that are not the oracle's own - the best feasible set by enumeration, numpy indexing, the library's
fp64 attention - and the properties that make a batch ragged: a sample never sees another one, the causal mask counts
from the sample's first row, equal sizes reproduce the rectangular functions, and the packed offsets follow Eq. 13."""
import numpy as np
import torch

import oracle

from test_oracle_properties import best_feasible_set

GRIDS = [(1, 3, 4, 2, 2, 1, 0, 4), (2, 2, 3, 1, 3, 0, 2, 5), (1, 1, 5, 1, 2, 1, 1, 0), (3, 2, 2, 2, 2, 0, 0, 7)]


def layout(rng, grids):
    """Per sample: frame starts with random text gaps, the sample's length."""
    starts, lens = [], []
    for g in grids:
        frames, hw = g[0], g[1] * g[2]
        gaps = rng.integers(0, 4, frames + 1)
        s, p = [], int(gaps[0])
        for f in range(frames):
            s.append(p)
            p += hw + int(gaps[f + 1])
        starts.append(np.asarray(s, dtype=np.int64)); lens.append(p)
    return starts, lens


def test_offsets_follow_the_compact_length_of_every_sample():
    rng = np.random.default_rng(0)
    starts, lens = layout(rng, GRIDS)
    seq, vis, kept, comp = oracle.ragged_offsets(lens, GRIDS)
    for b, g in enumerate(GRIDS):
        nv = g[0] * g[1] * g[2]
        cells = sum(min(g[5], (min(g[3], g[1] - r) * min(g[4], g[2] - c))) for r in range(0, g[1], g[3]) for c in range(0, g[2], g[4]))
        per_frame = cells + min(g[6], g[1] * g[2] - cells)
        k = max(g[7], g[0] * per_frame)
        assert seq[b + 1] - seq[b] == lens[b] and vis[b + 1] - vis[b] == nv and kept[b + 1] - kept[b] == k
        assert comp[b + 1] - comp[b] == lens[b] - nv + k


def test_selection_of_every_sample_is_its_own_best_feasible_set():
    rng = np.random.default_rng(1)
    for trial in range(20):
        scores = [np.round(rng.standard_normal(g[0] * g[1] * g[2]) * 2).astype(np.float32) / 2 for g in GRIDS]   # with ties
        packed = np.concatenate(scores)
        kept = oracle.select_ragged(packed, GRIDS)
        _, _, koff, _ = oracle.ragged_offsets([g[0] * g[1] * g[2] for g in GRIDS], GRIDS)
        for b, g in enumerate(GRIDS):
            assert kept[koff[b]:koff[b + 1]].tolist() == best_feasible_set(scores[b], g)
        # a sample does not see the others
        other = packed.copy()
        other[:scores[0].size] = rng.standard_normal(scores[0].size).astype(np.float32)
        assert np.array_equal(oracle.select_ragged(other, GRIDS)[koff[1]:], kept[koff[1]:])


def test_merge_of_every_sample_equals_numpy_indexing():
    rng = np.random.default_rng(2)
    starts, lens = layout(rng, GRIDS)
    seq, vis, koff, comp = oracle.ragged_offsets(lens, GRIDS)
    hidden = rng.integers(0, 2 ** 16, (int(seq[-1]), 6)).astype(np.uint16)
    pos = rng.integers(0, 1000, (3, int(seq[-1]))).astype(np.int32)
    kept = oracle.select_ragged(rng.standard_normal(int(vis[-1])).astype(np.float32), GRIDS)
    hc, pc, si = oracle.compact_ragged(hidden, pos, lens, GRIDS, starts, kept)
    assert hc.shape == (comp[-1], 6) and pc.shape == (3, comp[-1]) and si.shape == (comp[-1],)
    for b, g in enumerate(GRIDS):
        hw = g[1] * g[2]
        dense_of_visual = np.concatenate([np.arange(s, s + hw) for s in starts[b]])
        keep = np.ones(lens[b], dtype=bool)
        keep[dense_of_visual] = False
        keep[dense_of_visual[kept[koff[b]:koff[b + 1]]]] = True
        src = np.flatnonzero(keep)                             # sample-local dense indices, ascending
        assert np.array_equal(si[comp[b]:comp[b + 1]], src)
        assert np.array_equal(hc[comp[b]:comp[b + 1]], hidden[seq[b] + src])
        assert np.array_equal(pc[:, comp[b]:comp[b + 1]], pos[:, seq[b] + src])


def test_equal_samples_reproduce_the_rectangular_functions():
    rng = np.random.default_rng(3)
    g = (2, 3, 3, 2, 2, 1, 1, 8)
    grids = [g, g, g]
    fs = np.asarray([2, 14], dtype=np.int64)
    s_len, nv = 25, 18
    scores = rng.standard_normal((3, nv)).astype(np.float32)
    kept_rect, _ = oracle.select(scores, g)
    kept = oracle.select_ragged(scores.reshape(-1), grids)
    assert np.array_equal(kept, kept_rect.reshape(-1))
    hidden = rng.integers(0, 255, (3, s_len, 4)).astype(np.uint8)
    pos = rng.integers(0, 99, (3, 3, s_len)).astype(np.int32)
    hc_r, pc_r, si_r = oracle.compact(hidden, pos, g, fs, kept_rect)
    hc, pc, si = oracle.compact_ragged(hidden.reshape(-1, 4), pos.reshape(3, -1), [s_len] * 3, grids, [fs] * 3, kept)
    assert np.array_equal(hc, hc_r.reshape(-1, 4)) and np.array_equal(pc, pc_r.reshape(3, -1)) and np.array_equal(si, si_r.reshape(-1))
    q = rng.standard_normal((3, 7, 4, 8)).astype(np.float32)
    k = rng.standard_normal((3, 7, 2, 8)).astype(np.float32)
    v = rng.standard_normal((3, 7, 2, 8)).astype(np.float32)
    off = [0, 7, 14, 21]
    for causal in (True, False):
        rag = oracle.attention_ragged(q.reshape(-1, 4, 8), k.reshape(-1, 2, 8), v.reshape(-1, 2, 8), off, causal)
        assert np.array_equal(rag, oracle.attention(q, k, v, causal).reshape(-1, 4, 8))


def test_attention_of_every_sample_equals_library_attention_on_its_rows():
    rng = np.random.default_rng(4)
    sizes = [1, 5, 17, 2]
    off = np.concatenate([[0], np.cumsum(sizes)])
    hq, hkv, d = 4, 2, 8
    q = rng.standard_normal((off[-1], hq, d)).astype(np.float32)
    k = rng.standard_normal((off[-1], hkv, d)).astype(np.float32)
    v = rng.standard_normal((off[-1], hkv, d)).astype(np.float32)
    t = lambda x, rep: torch.from_numpy(x).double().permute(1, 0, 2).repeat_interleave(rep, dim=0)[None]
    for causal in (True, False):
        out = oracle.attention_ragged(q, k, v, off, causal)
        for a, b in zip(off[:-1], off[1:]):
            ref = torch.nn.functional.scaled_dot_product_attention(t(q[a:b], 1), t(k[a:b], hq // hkv), t(v[a:b], hq // hkv),
                                                                   is_causal=causal)[0].permute(1, 0, 2).numpy()
            assert np.abs(out[a:b] - ref).max() < 1e-12
        # the first row of a causal sample sees its own key only, whatever precedes it in the packed tensor
        if causal:
            for a in off[:-1]:
                assert np.abs(out[a] - np.repeat(v[a], hq // hkv, axis=0)).max() < 1e-12
        # another sample's keys and values do not matter
        k2, v2 = k.copy(), v.copy()
        k2[off[2]:off[3]] += 3.0; v2[off[2]:off[3]] -= 2.0
        out2 = oracle.attention_ragged(q, k2, v2, off, causal)
        assert np.array_equal(out2[:off[2]], out[:off[2]]) and np.array_equal(out2[off[3]:], out[off[3]:])


def test_every_sample_is_cached_at_its_own_rows():
    rng = np.random.default_rng(5)
    sizes = [3, 1, 6]
    off = np.concatenate([[0], np.cumsum(sizes)])
    hkv, d, s_max, pos0 = 2, 4, 9, 2
    k = rng.integers(0, 2 ** 16, (off[-1], hkv, d)).astype(np.uint16)
    v = rng.integers(0, 2 ** 16, (off[-1], hkv, d)).astype(np.uint16)
    kc = np.full((3, hkv, s_max, d), 0xBEEF, dtype=np.uint16)
    vc = np.full((3, hkv, s_max, d), 0xBEEF, dtype=np.uint16)
    nbytes = oracle.kv_write_ragged(k, v, off, kc, vc, pos0)
    assert nbytes == 2 * off[-1] * hkv * d * 2
    for i, (a, b) in enumerate(zip(off[:-1], off[1:])):
        assert np.array_equal(kc[i, :, pos0:pos0 + (b - a)], k[a:b].transpose(1, 0, 2))
        assert np.array_equal(vc[i, :, pos0:pos0 + (b - a)], v[a:b].transpose(1, 0, 2))
        assert np.all(kc[i, :, :pos0] == 0xBEEF) and np.all(kc[i, :, pos0 + (b - a):] == 0xBEEF)
        assert np.all(vc[i, :, :pos0] == 0xBEEF) and np.all(vc[i, :, pos0 + (b - a):] == 0xBEEF)


def test_decode_step_reads_every_sample_up_to_its_own_length():
    rng = np.random.default_rng(6)
    sizes = [1, 9, 4, 17]
    off = np.concatenate([[0], np.cumsum(sizes)])
    hq, hkv, d, s_max = 4, 2, 8, 20
    q = rng.standard_normal((off[-1], hq, d)).astype(np.float32)
    k = rng.standard_normal((off[-1], hkv, d)).astype(np.float32)
    v = rng.standard_normal((off[-1], hkv, d)).astype(np.float32)
    kc = rng.standard_normal((len(sizes), hkv, s_max, d)).astype(np.float32) * 50.0      # rows past a sample's length: loud garbage
    vc = rng.standard_normal((len(sizes), hkv, s_max, d)).astype(np.float32) * 50.0
    oracle.kv_write_ragged(k, v, off, kc, vc, 0)
    last_q = np.stack([q[b - 1] for b in off[1:]])                                           # every sample's last query
    dec = oracle.decode_attention_ragged(last_q, kc, vc, sizes)
    full = oracle.attention_ragged(q, k, v, off, True)
    assert np.abs(dec - np.stack([full[b - 1] for b in off[1:]])).max() < 1e-12
    # and against library attention over exactly the rows the sample owns
    for i, n in enumerate(sizes):
        t = lambda x: torch.from_numpy(x).double()
        ref = torch.nn.functional.scaled_dot_product_attention(t(last_q[i])[None, :, None, :], t(kc[i, :, :n]).repeat_interleave(hq // hkv, 0)[None],
                                                               t(vc[i, :, :n]).repeat_interleave(hq // hkv, 0)[None])[0, :, 0].numpy()
        assert np.abs(dec[i] - ref).max() < 1e-12
