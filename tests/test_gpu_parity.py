"""GPU parity: every stage of the HIP path, called through the C ABI, against the CPU oracle on the
same seeded inputs.  Integer, byte and index results are bit-exact; attention is within
2e-2 * max(1, max|ref|) for bf16 and 1e-4 * max(1, max|ref|) for fp32; scores within 2e-5 / tau."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_28115_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bd():
    from paper_2605_28115_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return binding


def to_dev(storage: np.ndarray) -> torch.Tensor:
    if storage.dtype == np.uint16:
        return torch.from_numpy(storage.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(storage).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def widen(storage: np.ndarray) -> np.ndarray:
    return wl.bf16_bits_to_f32(storage) if storage.dtype == np.uint16 else storage.astype(np.float32)


def log(*a):
    print(*a, flush=True)


# ----------------------------------------------------------------------------------------- score
@pytest.mark.parametrize("name", list(wl.WORKLOADS))
def test_score_matches_oracle(bd, name):
    w = wl.WORKLOADS[name]
    log("score", name)
    rows = min(w.batch * w.seq_len, 3000)
    for trial in range(5):
        hid, hid32 = wl.hidden(w, trial)
        hid = hid.reshape(-1, w.dim)[:rows]
        hid32 = hid32.reshape(-1, w.dim)[:rows]
        q = bd.civic_anchor_normalize(wl.anchor(w, trial))
        assert np.abs(q - oracle.anchor_normalize(wl.anchor(w, trial))).max() < 1e-7
        for inv_tau in (1.0, 14.0):
            s = to_host(bd.civic_score(to_dev(hid), torch.from_numpy(q).cuda(), inv_tau))
            ref = oracle.score(hid32, q, inv_tau)
            assert s.shape == ref.shape and np.abs(s - ref).max() <= 2e-5 * inv_tau


def test_score_edge_rows_and_strides(bd):
    rng = np.random.default_rng(0)
    for dim, dtype in ((8, "bf16"), (520, "bf16"), (1152, "bf16"), (8192, "bf16"), (4, "fp32"), (260, "fp32"), (4096, "fp32")):
        log("score edge", dim, dtype)
        x = rng.standard_normal((37, dim)).astype(np.float32) * 3 + 40          # large mean: needs the centred pass
        x[0] = 1.25                                                              # constant row -> 0
        st, x32 = wl.quantize(x, dtype)
        q = bd.civic_anchor_normalize(rng.standard_normal(dim).astype(np.float32))
        s = to_host(bd.civic_score(to_dev(st), torch.from_numpy(q).cuda(), 2.0))
        ref = oracle.score(x32, q, 2.0)
        assert s[0] == 0.0 and np.abs(s - ref).max() <= 2e-5 * 2.0
    # offsets on both sides of |mean| = standard deviation, where the bf16 kernel changes from its one-pass
    # sums to the centred two passes; magnitudes far from 1; all-zero and constant rows in between
    for dim in (256, 4096):
        ratios = np.array([0.0, 0.3, 0.7, 0.9, 0.97, 1.0, 1.03, 1.1, 1.5, 3.0, -0.95, -1.05, 30.0])
        mags = np.array([1.0, 1e-12, 1e-17, 1e12, 1e15, 37.0])      # squares stay inside fp32
        x = rng.standard_normal((len(mags), len(ratios), dim)).astype(np.float32)
        x = (x + ratios[None, :, None]) * mags[:, None, None]
        x = x.reshape(-1, dim).astype(np.float32)
        x[5] = 0.0
        x[17] = -3.5
        log("score offsets", dim)
        st, x32 = wl.quantize(x, "bf16")
        q = bd.civic_anchor_normalize(rng.standard_normal(dim).astype(np.float32) + 0.25)
        s = to_host(bd.civic_score(to_dev(st), torch.from_numpy(q).cuda(), 1.0))
        ref = oracle.score(x32, q, 1.0)
        assert s[5] == 0.0 and s[17] == 0.0 and np.abs(s - ref).max() <= 2e-5
    # rows embedded in a wider buffer (row stride > dim)
    x = rng.standard_normal((50, 256)).astype(np.float32)
    st, x32 = wl.quantize(x, "bf16")
    q = bd.civic_anchor_normalize(rng.standard_normal(64).astype(np.float32))
    s = to_host(bd.civic_score(to_dev(st)[:, 64:128], torch.from_numpy(q).cuda(), 1.0))
    assert np.abs(s - oracle.score(np.ascontiguousarray(x32[:, 64:128]), q, 1.0)).max() <= 2e-5


@pytest.mark.parametrize("name", list(wl.WORKLOADS))
def test_score_visual_scores_the_frame_spans_in_place(bd, name):
    """civic_score_visual on the dense sequence against the oracle on the gathered visual rows, and bit for bit
    against civic_score on the same rows gathered by hand (same kernel, same order of summation)."""
    w = wl.WORKLOADS[name]
    fs, grid, hw = wl.frame_starts(w), w.grid_tuple(), w.height * w.width
    for trial in (0, 3):
        log("score_visual", name, trial)
        hid, hid32 = wl.hidden(w, trial)
        d_hid = to_dev(hid)
        q = bd.civic_anchor_normalize(wl.anchor(w, trial))
        dq = torch.from_numpy(q).cuda()
        s = bd.civic_score_visual(d_hid, grid, fs, dq, 2.0)
        vis = torch.cat([d_hid[:, f:f + hw] for f in fs], dim=1).contiguous()
        assert torch.equal(s, bd.civic_score(vis, dq, 2.0))
        vis32 = np.concatenate([hid32[:, f:f + hw] for f in fs], axis=1).reshape(-1, w.dim)
        ref = oracle.score(vis32, q, 2.0).reshape(w.batch, -1)
        assert s.shape == ref.shape and np.abs(to_host(s) - ref).max() <= 2e-5 * 2.0


def test_score_visual_scattered_frames(bd):
    # frames separated by text of every length, a frame at row 0 and one ending at the last row; more (batch, frame)
    # slices than blocks fit; rows that take the centred two-pass branch
    rng = np.random.default_rng(12)
    for frames, h, wd, dim, batch, dtype in ((5, 3, 4, 64, 3, "bf16"), (128, 2, 2, 8, 2, "bf16"), (7, 9, 5, 260, 2, "fp32"),
                                             (3, 40, 40, 1152, 40, "bf16")):
        hw = h * wd
        gaps = rng.integers(0, 9, frames + 1)
        gaps[0] = 0
        gaps[-1] = 0
        fs, t = [], 0
        for f in range(frames):
            t += int(gaps[f])
            fs.append(t)
            t += hw
        seq = t
        log("score_visual scattered", frames, h, wd, dim, batch, dtype, "seq", seq)
        x = rng.standard_normal((batch, seq, dim)).astype(np.float32)
        x[:, ::5] += 4.0
        st, x32 = wl.quantize(x, dtype)
        q = bd.civic_anchor_normalize(rng.standard_normal(dim).astype(np.float32))
        grid = (frames, h, wd, 2, 2, 0, 0, 0)
        s = to_host(bd.civic_score_visual(to_dev(st), grid, fs, torch.from_numpy(q).cuda(), 1.0))
        vis32 = np.concatenate([x32[:, f:f + hw] for f in fs], axis=1).reshape(-1, dim)
        ref = oracle.score(vis32, q, 1.0).reshape(batch, -1)
        assert s.shape == ref.shape and np.abs(s - ref).max() <= 2e-5


def test_score_many_rows_per_wavefront(bd):
    # Far more rows than resident wavefronts (4096): every wavefront walks a dozen rows, refilling its registers
    # with the next row while it reduces the current one; a third of the rows take the centred two-pass branch.
    rng = np.random.default_rng(3)
    for dtype, dim, rows in (("bf16", 1024, 50001), ("bf16", 72, 70000), ("fp32", 512, 30011)):
        log("score many rows", dtype, dim, rows)
        x = rng.standard_normal((rows, dim)).astype(np.float32)
        x[::3] += 5.0
        x[7] = 0.0
        st, x32 = wl.quantize(x, dtype)
        q = bd.civic_anchor_normalize(rng.standard_normal(dim).astype(np.float32))
        s = to_host(bd.civic_score(to_dev(st), torch.from_numpy(q).cuda(), 3.0))
        ref = oracle.score(x32, q, 3.0)
        assert s[7] == 0.0 and np.isfinite(s).all() and np.abs(s - ref).max() <= 2e-5 * 3.0


# ---------------------------------------------------------------------------------------- select
def check_select(bd, scores: np.ndarray, grid):
    idx, flags = bd.civic_select(torch.from_numpy(scores).cuda(), grid, want_flags=True)
    ref_idx, ref_flags = oracle.select(scores, grid)
    assert np.array_equal(to_host(idx), ref_idx), grid
    assert np.array_equal(to_host(flags), ref_flags), grid


@pytest.mark.parametrize("name", list(wl.WORKLOADS))
def test_select_matches_oracle_on_workloads(bd, name):
    w = wl.WORKLOADS[name]
    for trial in range(5):
        log("select", name, trial)
        check_select(bd, wl.scores(w, trial), w.grid_tuple())


@pytest.mark.parametrize("grid", wl.small_grid_cases())
def test_select_matches_oracle_on_degenerate_grids(bd, grid):
    log("select grid", grid)
    nv = grid[0] * grid[1] * grid[2]
    rng = np.random.default_rng(nv)
    s = np.stack([
        rng.standard_normal(nv),
        np.round(rng.standard_normal(nv) * 2) / 2,               # heavy ties
        np.zeros(nv),
        rng.integers(0, 2, nv) * 1.0,
        np.where(rng.random(nv) < 0.5, 0.0, -0.0),               # signed zeros tie
        np.where(rng.random(nv) < 0.1, np.inf, np.where(rng.random(nv) < 0.1, -np.inf, rng.integers(-1, 2, nv))),
        -np.arange(nv, dtype=np.float64), np.arange(nv, dtype=np.float64),
    ]).astype(np.float32)
    check_select(bd, s, grid)


def test_select_budget_sweep_and_ties_at_the_threshold(bd):
    w = wl.WORKLOADS["8b"]
    s = np.round(wl.scores(w, 3) * 8) / 8                        # many equal keys at any threshold
    g = list(w.grid_tuple())
    for budget in (0, 1, 127, 128, 129, 682, 1500, 2047, 2048):
        log("select budget", budget)
        g[7] = budget
        check_select(bd, s.astype(np.float32), g)
    g = list(wl.WORKLOADS["video"].grid_tuple())
    sv = np.round(wl.scores(wl.WORKLOADS["video"], 1) * 4) / 4
    for ff in (0, 1, 16, 540, 576):
        log("select frame floor", ff)
        g[6] = ff
        check_select(bd, sv.astype(np.float32), g)


def test_select_at_the_size_limit(bd):
    grid = (8, 64, 64, 4, 4, 1, 50, 32768 // 3)                   # N_v = 32768, the documented maximum
    rng = np.random.default_rng(1)
    log("select limit")
    check_select(bd, rng.standard_normal((2, 32768)).astype(np.float32), grid)
    check_select(bd, np.zeros((1, 32768), dtype=np.float32), grid)


def test_select_with_nan_scores_keeps_its_shape(bd):
    # NaN scores are a caller error and the oracle rejects them, so there is no expected kept set; what the kernel
    # promises is a well-formed answer: exactly K distinct in-range indices in ascending order, flags that agree
    # with them, and every cell and frame still holding its floor.
    rng = np.random.default_rng(8)
    for grid in ((2, 32, 32, 4, 4, 1, 0, 682), (3, 10, 7, 3, 2, 2, 5, 70), (16, 24, 24, 4, 4, 1, 16, 3072), (1, 64, 64, 8, 8, 1, 0, 1365)):
        frames, h, w, ch, cw, cell_floor, frame_floor, _ = grid
        nv = frames * h * w
        for frac, sign in ((0.01, 1.0), (0.3, -1.0), (1.0, 1.0)):
            s = rng.standard_normal((2, nv)).astype(np.float32)
            s[rng.random((2, nv)) < frac] = np.float32(np.nan) * sign
            log("select with NaN", grid, frac)
            idx, flags = bd.civic_select(torch.from_numpy(s).cuda(), grid, want_flags=True)
            idx, flags = to_host(idx), to_host(flags)
            k = bd.civic_kept_count(grid)
            assert idx.shape == (2, k)
            for b in range(2):
                assert (np.diff(idx[b]) > 0).all() and idx[b, 0] >= 0 and idx[b, -1] < nv
                mask = np.zeros(nv, dtype=np.uint8)
                mask[idx[b]] = 1
                assert np.array_equal(mask, flags[b])
                m = mask.reshape(frames, h, w)
                for f in range(frames):
                    cells = 0
                    for r0 in range(0, h, ch):
                        for c0 in range(0, w, cw):
                            cell = m[f, r0:r0 + ch, c0:c0 + cw]
                            assert cell.sum() >= min(cell_floor, cell.size), (grid, f, r0, c0)
                            cells += min(cell_floor, cell.size)
                    assert m[f].sum() >= min(cells + frame_floor, h * w), (grid, f)


# --------------------------------------------------------------------------------------- compact
def check_compact(bd, hid, pos, grid, fs, kept):
    hc, pc, si = bd.civic_compact(to_dev(hid), torch.from_numpy(pos).cuda(), grid, fs, torch.from_numpy(kept).cuda())
    rhc, rpc, rsi = oracle.compact(hid, pos, grid, fs, kept)
    assert np.array_equal(to_host(si), rsi)
    assert np.array_equal(to_host(pc), rpc)
    assert np.array_equal(to_host(hc), rhc)


@pytest.mark.parametrize("name", list(wl.WORKLOADS))
def test_compact_matches_oracle_on_workloads(bd, name):
    w = wl.WORKLOADS[name]
    for trial in range(5):
        log("compact", name, trial)
        hid, _ = wl.hidden(w, trial)
        kept, _ = oracle.select(wl.scores(w, trial), w.grid_tuple())
        check_compact(bd, hid, wl.position_ids(w), w.grid_tuple(), wl.frame_starts(w), kept)


def test_compact_edge_cases(bd):
    rng = np.random.default_rng(2)
    w = wl.WORKLOADS["tiny"]
    hid, _ = wl.hidden(w, 3)
    pos, fs = wl.position_ids(w), wl.frame_starts(w)
    log("compact keep-all / keep-none")
    check_compact(bd, hid, pos, (1, 16, 16, 4, 4, 0, 0, 256), fs, np.arange(256, dtype=np.int32)[None])
    check_compact(bd, hid, pos, (1, 16, 16, 4, 4, 0, 0, 0), fs, np.zeros((1, 0), dtype=np.int32))
    # frames scattered through the text, some frames with no kept token, odd row sizes (2, 4, 8 byte vectors)
    for dim, dtype in ((7, np.uint16), (6, np.uint16), (3, np.float32), (36, np.uint16), (1152, np.uint16)):
        log("compact odd rows", dim, dtype)
        grid = (5, 3, 4, 2, 2, 0, 0, 0)
        fs = np.asarray([2, 14, 30, 42, 60], dtype=np.int64)
        seq = 75
        hid = rng.integers(0, 60000, (3, seq, dim)).astype(dtype)
        pos = rng.integers(0, 1000, (3, 3, seq)).astype(np.int32)
        kept = np.stack([np.sort(rng.choice(np.r_[0:12, 36:60], 9, replace=False)) for _ in range(3)]).astype(np.int32)
        check_compact(bd, hid, pos, grid, fs, kept)
    # nothing kept and no text: an empty compact sequence (the binding hands over NULL outputs)
    log("compact empty result")
    hid0 = rng.integers(0, 60000, (2, 12, 8)).astype(np.uint16)
    check_compact(bd, hid0, rng.integers(0, 9, (3, 2, 12)).astype(np.int32), (1, 3, 4, 2, 2, 0, 0, 0), np.zeros(1, dtype=np.int64),
                  np.zeros((2, 0), dtype=np.int32))
    # 128 frames (the documented maximum) of 2x2 tokens, no text at all
    log("compact 128 frames")
    grid = (128, 2, 2, 2, 2, 1, 0, 200)
    hid = rng.integers(0, 60000, (2, 512, 64)).astype(np.uint16)
    pos = rng.integers(0, 1000, (3, 2, 512)).astype(np.int32)
    kept, _ = oracle.select(rng.standard_normal((2, 512)).astype(np.float32), grid)
    check_compact(bd, hid, pos, grid, np.arange(128, dtype=np.int64) * 4, kept)


def test_compact_many_rows_per_block(bd):
    # 200 000 compact rows: blocks own the maximum of 64 rows each and walk them in several passes; row sizes that
    # use the 16-, 8- and 2-byte copies.
    rng = np.random.default_rng(33)
    frames, h, w = 8, 64, 64
    hw, batch = h * w, 4
    gaps = [700, 0, 1500, 3, 0, 900, 64, 1, 2500]
    fs, t = [], gaps[0]
    for f in range(frames):
        fs.append(t)
        t += hw + gaps[f + 1]
    seq, fs = t, np.asarray(fs, dtype=np.int64)
    for dim, dtype, k in ((64, np.uint16, frames * hw), (20, np.uint16, 20000), (3, np.uint16, 29000)):
        log("compact many rows", dim, k, "seq", seq)
        kept = np.stack([np.sort(rng.choice(frames * hw, k, replace=False)) for _ in range(batch)]).astype(np.int32)
        hid = rng.integers(0, 60000, (batch, seq, dim)).astype(dtype)
        pos = rng.integers(0, 100000, (3, batch, seq)).astype(np.int32)
        check_compact(bd, hid, pos, (frames, h, w, 1, 1, 0, 0, k), fs, kept)


def test_compact_long_kept_lists(bd):
    # More than 1024 kept tokens per sample: the kernel brackets the frame boundaries with 256 probes (one entry
    # out of P = ceil(K / 256)) and searches between them.  Boundaries on and next to probe positions, frames
    # without a kept token, everything in the first or the last frame, with and without text around the frames.
    frames, h, w = 8, 32, 32
    hw, rng = h * w, np.random.default_rng(21)

    def take(per_frame):                                       # per_frame[f] tokens of frame f, at random positions
        return np.concatenate([f * hw + np.sort(rng.choice(hw, n, replace=False)) for f, n in enumerate(per_frame)]).astype(np.int32)

    lists = {
        "boundary on a probe (P = 10)": take([1024, 256, 0, 1024, 256, 0, 0, 0]),
        "boundary one past a probe": take([1024, 257, 0, 1024, 255, 0, 0, 0]),
        "boundary one before a probe": take([1024, 255, 0, 0, 0, 0, 257, 1024]),
        "whole frames 2, 3 and 5": take([0, 0, 1024, 1024, 0, 1024, 0, 0]),
        "first frame only": take([1024, 1, 0, 0, 0, 0, 0, 0]),
        "last frame only": take([0, 0, 0, 0, 0, 0, 1, 1024]),
        "one token per boundary": take([1018, 1, 1, 1, 1, 1, 1, 1]),
        "every other token": np.arange(0, frames * hw, 2, dtype=np.int32),
        "everything": np.arange(frames * hw, dtype=np.int32),
    }
    for gaps in ([0] * 9, [5, 0, 300, 0, 0, 17, 1, 0, 40], [0, 900, 0, 0, 0, 0, 0, 200, 0]):   # the last: too much text between the frames, full pass
        fs, t = [], gaps[0]
        for f in range(frames):
            fs.append(t)
            t += hw + gaps[f + 1]
        seq, fs = t, np.asarray(fs, dtype=np.int64)
        hid = rng.integers(0, 60000, (1, seq, 64)).astype(np.uint16)
        pos = rng.integers(0, 100000, (3, 1, seq)).astype(np.int32)
        for name, kept in lists.items():
            log("compact long list:", name, "K", kept.size, "text", gaps[:3])
            check_compact(bd, hid, pos, (frames, h, w, 1, 1, 0, 0, int(kept.size)), fs, kept.reshape(1, -1))


# ------------------------------------------------------------------------------------- attention
def attn_tol(ref: np.ndarray, dtype: str) -> float:
    return (2e-2 if dtype == "bf16" else 1e-4) * max(1.0, float(np.nanmax(np.abs(ref))))


def check_attn(bd, q, k, v, causal, dtype, row_step=1, scale=0.0):
    out = to_host(bd.civic_prefill_attn(to_dev(q), to_dev(k), to_dev(v), causal, scale))
    ref = oracle.attention(widen(q), widen(k), widen(v), causal, scale=None if scale == 0.0 else scale, row_step=row_step)
    got = widen(out).astype(np.float64)[:, ::row_step]
    ref = ref[:, ::row_step]
    err = float(np.abs(got - ref).max())
    log("   max abs err", err, "tol", attn_tol(ref, dtype))
    assert np.isfinite(got).all() and err <= attn_tol(ref, dtype)


@pytest.mark.parametrize("name,row_step", [("tiny", 1), ("2b", 1), ("8b", 1), ("vit", 1), ("video", 13)])
def test_attention_matches_oracle_on_workloads(bd, name, row_step):
    """Every output row of every head against the oracle, five seeds; the video workload (105 GFLOP in the
    oracle's scalar loops) on every 13th query row, 276 of 3584, every head."""
    w = wl.WORKLOADS[name]
    for trial in range(5):
        log("attention", name, "trial", trial)
        (q, _), (k, _), (v, _) = wl.qkv(w, trial)
        check_attn(bd, q, k, v, w.causal, w.dtype, row_step)


def peaked_qkv(rng, b, s, hq, hkv, d, causal, sharp=3.0):
    """Q, K, V for which every query attends to ONE key, at a random visible position: K ~ N(0,1), V ~ N(0,1)
    (distinct per key), q_i = sharp * k_j(i).  The matching logit is about sharp * sqrt(d) standard deviations
    above the others, so out_i = V[j(i)] up to a few percent, at full magnitude: a key tile lost, read from the
    wrong ring stage or put into the wrong lane changes the output by O(1), not by the softmax average's O(0.03)."""
    k = rng.standard_normal((b, s, hkv, d)).astype(np.float32)
    v = rng.standard_normal((b, s, hkv, d)).astype(np.float32)
    group = hq // hkv
    q = np.empty((b, s, hq, d), dtype=np.float32)
    rows = np.arange(s)
    for bi in range(b):
        for h in range(hq):
            hi = np.minimum((rng.random(s) * (rows + 1 if causal else s)).astype(np.int64), rows if causal else s - 1)
            q[bi, :, h] = sharp * k[bi, hi, h // group]
    return (wl.quantize(x, "bf16")[0] for x in (q, k, v))


# The first four shapes are the sizes that matter (the 8B-shaped workload, 4096 and 20000 tokens, the encoder's
# head size); the others are causal launches with more workgroups than compute units, where a workgroup walks two
# row tiles (a heavy and a light one): odd and even numbers of row tiles, a full and a ragged last tile, 2 and 4
# heads per workgroup, padded heads, and the KV-cache copy in the same launch.
@pytest.mark.parametrize("shape,row_step", [((4, 938, 32, 8, 128), 1), ((1, 4096, 8, 2, 128), 1), ((1, 1365, 4, 4, 72), 1),
                                            ((1, 20000, 4, 2, 128), 41), ((4, 896, 32, 8, 128), 1), ((5, 961, 32, 8, 128), 1),
                                            ((8, 700, 16, 8, 128), 1), ((16, 1100, 12, 4, 96), 1), ((20, 1000, 8, 8, 64), 1),
                                            ((40, 130, 32, 8, 128), 1), ((3, 2049, 16, 4, 72), 1)])
@pytest.mark.parametrize("causal", [True, False])
def test_attention_one_key_per_query(bd, shape, row_step, causal):
    b, s, hq, hkv, d = shape
    log("attention, one key per query", shape, "causal", causal)
    q, k, v = peaked_qkv(np.random.default_rng(s + d), b, s, hq, hkv, d, causal)
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    kc = torch.zeros((b, hkv, s + 2, d), dtype=dq.dtype, device="cuda")
    vc = torch.zeros_like(kc)
    out = bd.civic_prefill_attn_kv(dq, dk, dv, kc, vc, 1, causal, 0.0)
    assert torch.equal(kc[:, :, 1:s + 1], dk.permute(0, 2, 1, 3)) and torch.equal(vc[:, :, 1:s + 1], dv.permute(0, 2, 1, 3))
    assert not kc[:, :, 0].any() and not kc[:, :, s + 1].any() and not vc[:, :, 0].any() and not vc[:, :, s + 1].any()
    assert torch.equal(out, bd.civic_prefill_attn(dq, dk, dv, causal, 0.0))
    out = to_host(out)
    ref = oracle.attention(widen(q), widen(k), widen(v), causal, row_step=row_step)[:, ::row_step]
    got = widen(out).astype(np.float64)[:, ::row_step]
    err = float(np.abs(got - ref).max())
    log("   max abs err", err, "tol", attn_tol(ref, "bf16"), "mean |ref|", float(np.abs(ref).mean()))
    assert np.abs(ref).mean() > 0.5                          # the outputs really are single V rows, not averages
    assert np.isfinite(got).all() and err <= attn_tol(ref, "bf16")


@pytest.mark.parametrize("shape", [
    (1, 1, 4, 4, 128), (2, 31, 8, 2, 128), (1, 33, 4, 1, 128), (1, 64, 2, 2, 128), (1, 65, 6, 3, 128),
    (2, 200, 8, 8, 64), (1, 257, 12, 4, 64), (1, 130, 16, 16, 72), (1, 77, 3, 3, 96), (1, 90, 4, 2, 32),
    (1, 100, 2, 1, 256), (1, 50, 4, 2, 160),
])
@pytest.mark.parametrize("causal", [True, False])
def test_attention_shapes_tails_and_head_dims(bd, shape, causal):
    b, s, hq, hkv, d = shape
    log("attention shape", shape, causal)
    rng = np.random.default_rng(s * 7 + d)
    mk = lambda h: wl.quantize(rng.standard_normal((b, s, h, d)).astype(np.float32) * 1.5, "bf16")[0]
    check_attn(bd, mk(hq), mk(hkv), mk(hkv), causal, "bf16")
    if d <= 64:
        mk32 = lambda h: rng.standard_normal((b, s, h, d)).astype(np.float32)
        check_attn(bd, mk32(hq), mk32(hkv), mk32(hkv), causal, "fp32", scale=0.2)


def test_attention_large_logits_stay_finite(bd):
    rng = np.random.default_rng(5)
    log("attention large logits")
    q = wl.quantize(rng.standard_normal((1, 150, 4, 128)).astype(np.float32) * 30, "bf16")[0]
    k = wl.quantize(rng.standard_normal((1, 150, 2, 128)).astype(np.float32) * 30, "bf16")[0]
    v = wl.quantize(rng.standard_normal((1, 150, 2, 128)).astype(np.float32), "bf16")[0]
    check_attn(bd, q, k, v, True, "bf16")
    check_attn(bd, q, k, v, False, "bf16")


def test_attention_long_sequence_sampled_rows(bd):
    # 20000 tokens (313 key tiles per workgroup, 20 MB between a head's first and last row): the oracle computes
    # every 613-th query row; the fused call must also have written all 20000 cache rows and nothing before them.
    rng = np.random.default_rng(17)
    b, s, hq, hkv, d = 1, 20000, 4, 2, 128
    log("attention long sequence", (b, s, hq, hkv, d))
    q, k, v = (wl.quantize(rng.standard_normal((b, s, h, d)).astype(np.float32), "bf16")[0] for h in (hq, hkv, hkv))
    qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
    kc = torch.zeros((b, hkv, s + 3, d), dtype=qd.dtype, device="cuda")
    vc = torch.zeros_like(kc)
    for causal in (True, False):
        out = bd.civic_prefill_attn_kv(qd, kd, vd, kc, vc, 3, causal, 0.0)
        ref = oracle.attention(widen(q), widen(k), widen(v), causal, scale=None, row_step=613)[:, ::613]
        got = widen(to_host(out)).astype(np.float64)[:, ::613]
        err = float(np.abs(got - ref).max())
        log("   causal", causal, "max abs err", err, "tol", attn_tol(ref, "bf16"))
        assert np.isfinite(widen(to_host(out))).all() and err <= attn_tol(ref, "bf16")
        assert torch.equal(kc[:, :, 3:], kd.permute(0, 2, 1, 3)) and torch.equal(vc[:, :, 3:], vd.permute(0, 2, 1, 3))
        assert not kc[:, :, :3].any() and not vc[:, :, :3].any()


@pytest.mark.parametrize("causal", [True, False])
def test_attention_logits_growing_along_the_sequence(bd, causal):
    """Keys whose logits grow steadily with the key index: every later tile outgrows the softmax
    offset taken from the first tile by far more than fp32 can absorb, so the running offset has to
    move, again and again, with rescaling of everything accumulated so far."""
    log("attention growing logits", causal)
    rng = np.random.default_rng(11)
    b, s, hq, hkv, d = 1, 700, 8, 2, 128
    q = rng.standard_normal((b, s, hq, d)).astype(np.float32)
    q[..., 0] = 8.0                                          # logit = 8 * k[..., 0] / sqrt(d) + noise
    k = rng.standard_normal((b, s, hkv, d)).astype(np.float32)
    k[..., 0] = np.arange(s, dtype=np.float32)[None, :, None] * 2.0      # about +1.4 per key, +90 per 64-key tile
    v = rng.standard_normal((b, s, hkv, d)).astype(np.float32)
    q, k, v = (wl.quantize(x, "bf16")[0] for x in (q, k, v))
    check_attn(bd, q, k, v, causal, "bf16")
    # and decreasing: the first tile holds the maximum, later terms underflow towards zero
    k2 = widen(k).copy()
    k2[..., 0] = -k2[..., 0]
    check_attn(bd, q, wl.quantize(k2, "bf16")[0], v, causal, "bf16")


# -------------------------------------------------------------------------------------- KV write
@pytest.mark.parametrize("name", ["tiny", "2b", "8b", "video"])
def test_kv_write_matches_oracle(bd, name):
    w = wl.WORKLOADS[name]
    for trial in range(5):
        log("kv_write", name, trial)
        _, (k, _), (v, _) = wl.qkv(w, trial)
        seq = k.shape[1]
        for s_max, pos0 in ((seq, 0), (seq + 37, 21)):
            fill = 0x7B7B if k.dtype == np.uint16 else 123.0
            kc = np.full((w.batch, w.n_kv_heads, s_max, w.head_dim), fill, dtype=k.dtype)
            vc = kc.copy()
            dk, dv = to_dev(kc), to_dev(vc)
            bd.civic_kv_write(to_dev(k), to_dev(v), dk, dv, pos0)
            oracle.kv_write(k, v, kc, vc, pos0)
            assert np.array_equal(to_host(dk), kc) and np.array_equal(to_host(dv), vc)   # includes the untouched rows


@pytest.mark.parametrize("shape,causal,dtype", [
    ((4, 938, 32, 8, 128), True, "bf16"), ((1, 469, 16, 8, 128), True, "bf16"), ((2, 333, 16, 16, 72), False, "bf16"),
    ((1, 257, 12, 4, 64), True, "bf16"), ((1, 130, 8, 8, 128), False, "bf16"), ((1, 200, 3, 1, 96), True, "bf16"),
    ((1, 100, 2, 1, 256), True, "bf16"), ((1, 77, 4, 2, 32), True, "fp32"),
])
def test_fused_attention_kv_write_equals_the_two_calls(bd, shape, causal, dtype):
    """civic_prefill_attn_kv against civic_prefill_attn + civic_kv_write (both already checked against the
    oracle above): same attention output and same caches, bit for bit, including the untouched rows."""
    b, s, hq, hkv, d = shape
    log("fused attention + kv write", shape, causal, dtype)
    rng = np.random.default_rng(s + d)
    mk = lambda h: wl.quantize(rng.standard_normal((b, s, h, d)).astype(np.float32), dtype)[0]
    q, k, v = mk(hq), mk(hkv), mk(hkv)
    s_max, pos0 = s + 19, 7
    fill = 0x7B7B if k.dtype == np.uint16 else 123.0
    cache = np.full((b, hkv, s_max, d), fill, dtype=k.dtype)
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    kc1, vc1, kc2, vc2 = (to_dev(cache.copy()) for _ in range(4))
    out1 = bd.civic_prefill_attn(dq, dk, dv, causal)
    bd.civic_kv_write(dk, dv, kc1, vc1, pos0)
    out2 = bd.civic_prefill_attn_kv(dq, dk, dv, kc2, vc2, pos0, causal)
    assert np.array_equal(to_host(out1), to_host(out2))
    assert np.array_equal(to_host(kc1), to_host(kc2)) and np.array_equal(to_host(vc1), to_host(vc2))
    ref = oracle.attention(widen(q), widen(k), widen(v), causal)                    # the fused call against the oracle itself
    err = float(np.abs(widen(to_host(out2)).astype(np.float64) - ref).max())
    assert err <= attn_tol(ref, dtype), err
    ref_k, ref_v = cache.copy(), cache.copy()
    oracle.kv_write(k, v, ref_k, ref_v, pos0)
    assert np.array_equal(to_host(kc2), ref_k) and np.array_equal(to_host(vc2), ref_v)


@pytest.mark.parametrize("name", ["tiny", "2b", "8b", "vit", "video"])
def test_front_call_equals_the_three_calls_and_the_oracle(bd, name):
    """civic_compact_prefill: one call for score -> select -> compact.  Same kernels, so every output equals the
    three calls' bit for bit; the chain is also checked against the oracle (selection on the GPU's scores)."""
    w = wl.WORKLOADS[name]
    log("front call", name)
    hid, hid32 = wl.hidden(w, 2)
    pos, fs, grid = wl.position_ids(w), wl.frame_starts(w), w.grid_tuple()
    hw = w.height * w.width
    d_hid, d_pos = to_dev(hid), torch.from_numpy(pos.copy()).cuda()
    q_anchor = bd.civic_anchor_normalize(wl.anchor(w, 2))
    d_anchor = torch.from_numpy(q_anchor).cuda()
    scores, kept, hc, pc, si = bd.civic_compact_prefill(d_hid, d_pos, grid, fs, d_anchor, 1.5)
    scores3 = bd.civic_score_visual(d_hid, grid, fs, d_anchor, 1.5)
    kept3, _ = bd.civic_select(scores3, grid)
    hc3, pc3, si3 = bd.civic_compact(d_hid, d_pos, grid, fs, kept3)
    torch.cuda.synchronize()
    assert torch.equal(scores, scores3) and torch.equal(kept, kept3)
    assert torch.equal(si, si3) and torch.equal(pc, pc3) and np.array_equal(to_host(hc), to_host(hc3))
    h_scores = to_host(scores)
    vis32 = np.concatenate([hid32[:, s:s + hw] for s in fs], axis=1).reshape(-1, w.dim)
    assert np.abs(h_scores.reshape(-1) - oracle.score(vis32, q_anchor, 1.5)).max() <= 2e-5 * 1.5
    ref_kept, _ = oracle.select(h_scores, grid)
    assert np.array_equal(to_host(kept), ref_kept)
    rhc, rpc, rsi = oracle.compact(hid, pos, grid, fs, ref_kept)
    assert np.array_equal(to_host(si), rsi) and np.array_equal(to_host(pc), rpc) and np.array_equal(to_host(hc), rhc)


# -------------------------------------------------------------------------------------- the path
@pytest.mark.parametrize("name", ["tiny", "2b", "8b", "vit", "video"])
def test_whole_path_chained(bd, name):
    """score -> select -> compact -> attention -> KV write on device, each stage fed by the previous
    one's device output.  Selection parity is defined on a given score array, so the oracle selects on
    the scores the GPU produced; since H_q * d = D the compact rows serve as Q and their first
    H_kv * d columns as K = V (strided views)."""
    w = wl.WORKLOADS[name]
    log("chain", name)
    hid, hid32 = wl.hidden(w, 4)
    pos, fs, grid = wl.position_ids(w), wl.frame_starts(w), w.grid_tuple()
    hw = w.height * w.width
    d_hid = to_dev(hid)
    q_anchor = bd.civic_anchor_normalize(wl.anchor(w, 4))
    scores = bd.civic_score_visual(d_hid, grid, fs, torch.from_numpy(q_anchor).cuda(), 1.0)   # on the dense sequence, in place
    kept, _ = bd.civic_select(scores, grid)
    hc, pc, si = bd.civic_compact(d_hid, torch.from_numpy(pos).cuda(), grid, fs, kept)
    s_c = hc.shape[1]
    assert s_c == w.seq_compact
    qv = hc.view(w.batch, s_c, w.n_q_heads, w.head_dim)
    kv = hc[:, :, :w.n_kv_heads * w.head_dim].unflatten(2, (w.n_kv_heads, w.head_dim))
    out = bd.civic_prefill_attn(qv, kv, kv, w.causal)
    kc = torch.zeros((w.batch, w.n_kv_heads, s_c, w.head_dim), dtype=hc.dtype, device="cuda")
    vc = torch.zeros_like(kc)
    bd.civic_kv_write(kv, kv, kc, vc, 0)
    torch.cuda.synchronize()

    h_scores = to_host(scores)
    vis32 = np.concatenate([hid32[:, s:s + hw] for s in fs], axis=1).reshape(-1, w.dim)
    assert np.abs(h_scores.reshape(-1) - oracle.score(vis32, q_anchor, 1.0)).max() <= 2e-5
    ref_kept, _ = oracle.select(h_scores, grid)
    assert np.array_equal(to_host(kept), ref_kept)
    rhc, rpc, rsi = oracle.compact(hid, pos, grid, fs, ref_kept)
    assert np.array_equal(to_host(si), rsi) and np.array_equal(to_host(pc), rpc) and np.array_equal(to_host(hc), rhc)
    r32 = widen(rhc)
    rq = r32.reshape(w.batch, s_c, w.n_q_heads, w.head_dim)
    rkv = r32[:, :, :w.n_kv_heads * w.head_dim].reshape(w.batch, s_c, w.n_kv_heads, w.head_dim)
    step = 1 if s_c < 2000 else 29                        # video: 124 of 3584 query rows, every head
    ref = oracle.attention(rq, rkv, rkv, w.causal, row_step=step)[:, ::step]
    got = widen(to_host(out)).astype(np.float64)[:, ::step]
    assert np.abs(got - ref).max() <= attn_tol(ref, w.dtype)
    rkc = np.zeros((w.batch, w.n_kv_heads, s_c, w.head_dim), dtype=rhc.dtype)
    rvc = rkc.copy()
    rkv_bits = rhc[:, :, :w.n_kv_heads * w.head_dim].reshape(w.batch, s_c, w.n_kv_heads, w.head_dim)
    oracle.kv_write(rkv_bits, rkv_bits, rkc, rvc, 0)
    assert np.array_equal(to_host(kc), rkc) and np.array_equal(to_host(vc), rvc)


# ---------------------------------------------------------------------------------- kernel timer
def test_kernel_timer_brackets_one_launch_and_leaves_results_alone(bd):
    w = wl.WORKLOADS["8b"]
    log("kernel timer", w.name)
    hid, _ = wl.hidden(w, 0)
    h = to_dev(hid.reshape(-1, w.dim))
    q = torch.from_numpy(bd.civic_anchor_normalize(wl.anchor(w, 0))).cuda()
    plain = bd.civic_score(h, q, 1.0)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    outer0, outer1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(); b.record()
    torch.cuda.synchronize()
    bd.civic_time_next_kernel(a, b)
    outer0.record()
    timed = bd.civic_score(h, q, 1.0)
    outer1.record()
    torch.cuda.synchronize()
    kernel_ms, outer_ms = a.elapsed_time(b), outer0.elapsed_time(outer1)
    log("  kernel", kernel_ms * 1e3, "us inside", outer_ms * 1e3, "us")
    assert torch.equal(plain, timed)
    assert 1e-3 < kernel_ms <= outer_ms             # 8b scoring reads 32 MB: several microseconds at any clock
    # one-shot: the next launch does not touch the two events
    again = bd.civic_score(h, q, 1.0)
    torch.cuda.synchronize()
    assert a.elapsed_time(b) == kernel_ms and torch.equal(again, plain)
