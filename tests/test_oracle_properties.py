"""Property-based pins of the oracle (hypothesis draws the cases; derandomised, so every run sees the same ones).

Selection: for any scores, ties included, the kept set is the best feasible set under the strict order "higher
score first, equal scores to the lower index" - found here by enumerating every subset of the right size that meets
the cell and frame lower bounds, with weights 2^(rank) so that no two subsets tie.  Compact merge: equals plain numpy
indexing on any layout of frames and text.  Attention and its decode step: equal the library's fp64 attention on
any small shape.
"""
import itertools

import numpy as np
import pytest
import torch
from hypothesis import given, settings, strategies as st

import oracle

from test_oracle_select import cells_of, floor_sum, order

SETTINGS = dict(deadline=None, derandomize=True)


@st.composite
def grids_and_scores(draw):
    frames = draw(st.integers(1, 3))
    h = draw(st.integers(1, 4))
    w = draw(st.integers(1, 4))
    while frames * h * w > 12:                                # keeps the enumeration below small
        if frames > 1:
            frames -= 1
        elif h > 1:
            h -= 1
        else:
            w -= 1
    nv = frames * h * w
    grid = (frames, h, w, draw(st.integers(1, h)), draw(st.integers(1, w)), draw(st.integers(0, 2)),
            draw(st.integers(0, 3)), draw(st.integers(0, nv)))
    pool = draw(st.sampled_from([[0.0, 1.0], [-1.5, 0.0, 0.25, 2.0], [-0.0, 0.0, 1.0], None]))
    if pool is None:
        scores = draw(st.lists(st.floats(-4, 4, allow_nan=False, width=32), min_size=nv, max_size=nv))
    else:
        scores = draw(st.lists(st.sampled_from(pool), min_size=nv, max_size=nv))
    return grid, np.asarray(scores, dtype=np.float32)


def best_feasible_set(scores, grid):
    frames, H, W, ch, cw, cf, ff, budget = grid
    nv = frames * H * W
    K = max(budget, floor_sum(grid))
    cells = cells_of(grid)
    cell_of = np.zeros(nv, dtype=np.int64)
    for ci, cell in enumerate(cells):
        cell_of[cell] = ci
    cell_lb = np.asarray([min(cf, len(c)) for c in cells])
    frame_lb = floor_sum((1, H, W, ch, cw, cf, ff, 0))
    o = order(scores)                                         # strict order, best first
    weight = np.zeros(nv, dtype=np.float64)
    weight[o] = 2.0 ** np.arange(nv - 1, -1, -1)              # exact, and every subset has its own sum
    best, best_sum = None, -1.0
    for sub in itertools.combinations(range(nv), K):
        a = np.asarray(sub, dtype=np.int64)
        if K and np.any(np.bincount(cell_of[a], minlength=len(cells)) < cell_lb):
            continue
        if K and np.any(np.bincount(a // (H * W), minlength=frames) < frame_lb):
            continue
        t = weight[a].sum()
        if t > best_sum:
            best, best_sum = list(sub), t
    return best


@settings(max_examples=150, **SETTINGS)
@given(grids_and_scores())
def test_selection_is_the_best_feasible_set_under_the_strict_order(case):
    grid, scores = case
    idx, flags = oracle.select(scores[None], grid)
    assert idx[0].tolist() == best_feasible_set(scores, grid)
    assert flags[0].sum() == idx.shape[1] and np.all(flags[0][idx[0]] == 1)


@st.composite
def layouts(draw):
    frames = draw(st.integers(1, 4))
    hw = draw(st.integers(1, 6))
    gaps = draw(st.lists(st.integers(0, 5), min_size=frames + 1, max_size=frames + 1))
    starts, p = [], gaps[0]
    for f in range(frames):
        starts.append(p)
        p += hw + gaps[f + 1]
    seq = p
    nv = frames * hw
    n_kept = draw(st.integers(0, nv))
    kept = sorted(draw(st.permutations(range(nv)))[:n_kept])
    batch = draw(st.integers(1, 2))
    dim = draw(st.sampled_from([1, 3, 8]))
    return frames, hw, np.asarray(starts, dtype=np.int64), seq, np.asarray(kept, dtype=np.int32), batch, dim


@settings(max_examples=150, **SETTINGS)
@given(layouts(), st.integers(0, 2 ** 31 - 1))
def test_compact_equals_numpy_indexing_on_any_layout(layout, seed):
    frames, hw, starts, seq, kept, batch, dim = layout
    rng = np.random.default_rng(seed)
    grid = (frames, 1, hw, 1, 1, 0, 0, len(kept))
    hidden = rng.integers(0, 2 ** 16, (batch, seq, dim)).astype(np.uint16)
    pos = rng.integers(0, 1000, (3, batch, seq)).astype(np.int32)
    kept_b = np.stack([kept] * batch)
    hc, pc, si = oracle.compact(hidden, pos, grid, starts, kept_b)
    is_visual = np.zeros(seq, dtype=bool)
    dense_of_visual = np.concatenate([np.arange(s, s + hw) for s in starts])
    is_visual[dense_of_visual] = True
    keep = ~is_visual
    keep[dense_of_visual[kept]] = True
    src = np.flatnonzero(keep)
    assert np.array_equal(si, np.stack([src] * batch))
    assert np.array_equal(hc, hidden[:, src]) and np.array_equal(pc, pos[:, :, src])


@settings(max_examples=60, **SETTINGS)
@given(st.integers(1, 2), st.integers(1, 40), st.sampled_from([(1, 1), (2, 1), (4, 2), (3, 3)]), st.sampled_from([8, 24, 40]),
       st.booleans(), st.integers(0, 2 ** 31 - 1))
def test_attention_and_decode_equal_library_attention(batch, seq, heads, d, causal, seed):
    hq, hkv = heads
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((batch, seq, hq, d)).astype(np.float32)
    k = rng.standard_normal((batch, seq, hkv, d)).astype(np.float32)
    v = rng.standard_normal((batch, seq, hkv, d)).astype(np.float32)
    t = lambda x, rep: torch.from_numpy(x).double().permute(0, 2, 1, 3).repeat_interleave(rep, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(t(q, 1), t(k, hq // hkv), t(v, hq // hkv), is_causal=causal)
    ref = ref.permute(0, 2, 1, 3).numpy()
    out = oracle.attention(q, k, v, causal)
    assert np.abs(out - ref).max() < 1e-12
    # the decode step: the last query against the caches holding all keys
    kc = np.ascontiguousarray(k.transpose(0, 2, 1, 3))
    vc = np.ascontiguousarray(v.transpose(0, 2, 1, 3))
    dec = oracle.decode_attention(q[:, -1], kc, vc, seq)
    last = ref[:, -1] if causal else oracle.attention(q, k, v, True)[:, -1]
    assert np.abs(dec - last).max() < 1e-12
