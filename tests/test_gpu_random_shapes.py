"""GPU parity on randomly drawn shapes: a fixed number of seeded cases per stage, each against the
CPU oracle, to the same bars as test_gpu_parity.py.  The draws favour the sizes where a kernel
changes path (tile and wavefront boundaries, cell widths that are or are not multiples of four,
empty results, offsets around |mean| = standard deviation)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_28115_amd import workloads as wl
from test_gpu_parity import attn_tol, to_dev, to_host, widen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bd():
    from paper_2605_28115_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return binding


def log(*a):
    print(*a, flush=True)


def draw_scores(rng, kind: int, shape) -> np.ndarray:
    if kind == 0:
        s = rng.standard_normal(shape)
    elif kind == 1:
        s = np.exp(rng.standard_normal(shape))
    elif kind == 2:
        s = np.round(rng.standard_normal(shape) * 2) / 2                       # heavy ties
    elif kind == 3:
        s = rng.integers(0, 3, shape) * 1.0
    elif kind == 4:
        s = rng.standard_normal(shape) * 1e-30
    elif kind == 5:
        s = np.where(rng.random(shape) < 0.3, -rng.random(shape), rng.random(shape) * 1e6)
    elif kind == 6:
        s = np.zeros(shape)
    elif kind == 7:
        s = rng.standard_normal(shape).astype(np.float16).astype(np.float64)   # many exact ties
    elif kind == 8:                                                            # two outliers squeeze the rest into one bucket
        s = rng.standard_normal(shape)
        s.flat[rng.integers(0, s.size)] = 1e30
        s.flat[rng.integers(0, s.size)] = -1e30
    elif kind == 9:                                                            # infinities: no finite range
        s = rng.standard_normal(shape)
        s[rng.random(shape) < 0.05] = np.inf
        s[rng.random(shape) < 0.05] = -np.inf
    elif kind == 10:                                                           # a range that overflows fp32
        s = rng.choice([-3e38, 3e38, 1.0, -1.0], shape) * rng.random(shape)
    elif kind == 11:                                                           # 64 distinct values
        s = np.floor(rng.random(shape) * 64) / 64
    else:                                                                      # two clusters far apart
        s = rng.standard_normal(shape) + rng.choice([0.0, 1e4], shape)
    return s.astype(np.float32)


def test_select_random_grids(bd):
    rng = np.random.default_rng(12345)
    done = 0
    while done < 1500:
        frames = int(rng.choice([1, 1, 2, 3, 5, 16]))
        h, w = int(rng.integers(1, 70)), int(rng.integers(1, 70))
        if rng.random() < 0.5:
            w = int(rng.choice([4, 8, 12, 16, 24, 32, 64]))
        nv = frames * h * w
        if nv > 32768:
            continue
        ch = max(1, min(int(rng.choice([1, 2, 3, 4, 4, 4, 7, 8, 16, h])), h))
        cw = max(1, min(int(rng.choice([1, 2, 3, 4, 4, 4, 8, 8, 12, 16, w])), w))
        cell_floor, frame_floor = int(rng.choice([0, 1, 1, 1, 2, 3, 70])), int(rng.choice([0, 0, 0, 1, 16, 100]))
        budget = int(rng.choice([0, nv // 3, nv // 3, nv // 2, nv, int(rng.integers(0, nv + 1))]))
        grid = (frames, h, w, ch, cw, cell_floor, frame_floor, budget)
        batch = int(rng.choice([1, 2, 4]))
        s = draw_scores(rng, int(rng.integers(0, 13)), (batch, nv))
        if done % 100 == 0:
            log("select random", done, grid, batch)
        if rng.random() < 0.2:                                                # a start that is not 16-byte aligned
            sd = torch.from_numpy(np.concatenate([np.zeros(1, np.float32), s.ravel()])).cuda()[1:].view(batch, nv)
        else:
            sd = torch.from_numpy(s).cuda()
        idx, flags = bd.civic_select(sd, grid, want_flags=True)
        ref_idx, ref_flags = oracle.select(s, grid)
        assert np.array_equal(to_host(idx), ref_idx), (grid, batch)
        assert np.array_equal(to_host(flags), ref_flags), (grid, batch)
        done += 1


def test_compact_random_layouts(bd):
    rng = np.random.default_rng(777)
    shapes = [(8, np.uint16), (64, np.uint16), (256, np.float32), (512, np.uint16), (1152, np.uint16), (2048, np.uint16),
              (4096, np.uint16), (36, np.uint16), (7, np.uint16), (1024, np.float32)]
    done = 0
    while done < 400:
        frames = int(rng.choice([1, 1, 2, 3, 5, 16, 40, 128]))
        h, w = int(rng.integers(1, 40)), int(rng.integers(1, 40))
        hw = h * w
        nv = frames * hw
        if nv > (8192 if done % 8 else 32768):                                   # long kept lists take another path in the kernel
            continue
        gaps = rng.integers(0, 40 if rng.random() < 0.8 else 1500, frames + 1)   # text before, between and after the frames
        if rng.random() < 0.3:
            gaps[:] = 0
        fs, t = [], int(gaps[0])
        for f in range(frames):
            fs.append(t)
            t += hw + int(gaps[f + 1])
        seq, batch = t, int(rng.choice([1, 2, 4]))
        dim, dtype = shapes[int(rng.integers(0, len(shapes)))]
        if batch * seq * dim > 3e7:
            continue
        k = int(rng.choice([0, nv // 3, nv // 2, nv, int(rng.integers(0, nv + 1))]))
        kept = np.stack([np.sort(rng.choice(nv, k, replace=False)) for _ in range(batch)]).astype(np.int32).reshape(batch, k)
        grid = (frames, h, w, 1, 1, 0, 0, k)
        hid = rng.integers(0, 60000, (batch, seq, dim)).astype(dtype)
        pos = rng.integers(0, 100000, (3, batch, seq)).astype(np.int32)
        fs = np.asarray(fs, dtype=np.int64)
        if done % 50 == 0:
            log("compact random", done, grid, seq, batch, dim, dtype.__name__)
        hc, pc, si = bd.civic_compact(to_dev(hid), torch.from_numpy(pos).cuda(), grid, fs, torch.from_numpy(kept).cuda())
        rh, rp, rs = oracle.compact(hid, pos, grid, fs, kept)
        assert np.array_equal(to_host(si), rs) and np.array_equal(to_host(pc), rp), (grid, seq, batch, dim)
        assert np.array_equal(to_host(hc), rh), (grid, seq, batch, dim)
        done += 1


def test_attention_random_shapes(bd):
    rng = np.random.default_rng(4242)
    done, worst = 0, 0.0
    while done < 300:
        d = int(rng.choice([32, 64, 72, 96, 128, 128, 128, 160, 256]))
        hkv = int(rng.choice([1, 2, 3, 8]))
        hq = hkv * int(rng.choice([1, 2, 3, 4, 4, 8]))
        b = int(rng.choice([1, 2, 3]))
        s = int(rng.choice([1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 200, 255, 257, 300, 469, 513, int(rng.integers(1, 700))]))
        if b * s * hq * d > 6e6:
            continue
        causal = bool(rng.integers(0, 2))
        dtype = "bf16" if rng.random() < 0.85 else "fp32"
        amp = float(rng.choice([0.5, 1.0, 1.5, 3.0]))
        mk = lambda heads: wl.quantize((rng.standard_normal((b, s, heads, d)) * amp).astype(np.float32), dtype)[0]
        q, k, v = mk(hq), mk(hkv), mk(hkv)
        qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
        fused = rng.random() < 0.5
        if done % 50 == 0:
            log("attention random", done, (b, s, hq, hkv, d), causal, dtype, fused)
        if fused:
            s_max = s + int(rng.integers(0, 5))
            pos0 = int(rng.integers(0, s_max - s + 1))
            kc = torch.zeros((b, hkv, s_max, d), dtype=qd.dtype, device="cuda")
            vc = torch.zeros_like(kc)
            out = bd.civic_prefill_attn_kv(qd, kd, vd, kc, vc, pos0, causal, 0.0)
            assert torch.equal(kc[:, :, pos0:pos0 + s], kd.permute(0, 2, 1, 3)), (b, s, hq, hkv, d)
            assert torch.equal(vc[:, :, pos0:pos0 + s], vd.permute(0, 2, 1, 3)), (b, s, hq, hkv, d)
        else:
            out = bd.civic_prefill_attn(qd, kd, vd, causal, 0.0)
        step = 1
        ref = oracle.attention(widen(q), widen(k), widen(v), causal, scale=None, row_step=step)[:, ::step]
        got = widen(to_host(out)).astype(np.float64)[:, ::step]
        err, tol = float(np.abs(got - ref).max()), attn_tol(ref, dtype)
        worst = max(worst, err / tol)
        assert np.isfinite(got).all() and err <= tol, ((b, s, hq, hkv, d), causal, dtype, fused, err, tol)
        done += 1
    log("   worst error / tolerance", worst)


def test_score_random_rows(bd):
    rng = np.random.default_rng(99)
    done, worst = 0, 0.0
    while done < 600:
        dtype = "bf16" if rng.random() < 0.7 else "fp32"
        mult = 8 if dtype == "bf16" else 4
        dim = int(rng.choice([mult, 2 * mult, 64, 72, 256, 520, 1024, 1152, 2048, 4096, 4096, 6144 if dtype == "bf16" else 2048,
                              8192 if dtype == "bf16" else 4096, mult * int(rng.integers(1, 200))]))
        rows = int(rng.choice([1, 2, 7, 64, 100, 513, 1200]))
        if rows * dim > 4e6:
            rows = max(1, int(4e6 // dim))
        # offsets on both sides of |mean| = standard deviation, magnitudes far from 1, an all-zero and a constant row
        ratio = rng.choice([0.0, 0.5, 0.9, 1.0, 1.1, 2.0, 50.0], size=(rows, 1)) * rng.choice([-1.0, 1.0], size=(rows, 1))
        mag = rng.choice([1.0, 1e-6, 1e6, 37.0, 1e-14, 1e10], size=(rows, 1))
        x = ((rng.standard_normal((rows, dim)) * rng.choice([1.0, 0.01, 5.0]) + ratio) * mag).astype(np.float32)
        if rows > 3:
            x[1], x[2] = 0.0, 2.5
        st, x32 = wl.quantize(x, dtype)
        q = bd.civic_anchor_normalize((rng.standard_normal(dim) + rng.choice([0.0, 0.25, 3.0])).astype(np.float32))
        inv_tau = float(rng.choice([1.0, 14.0, 0.07]))
        if done % 100 == 0:
            log("score random", done, dtype, dim, rows, inv_tau)
        s = to_host(bd.civic_score(to_dev(st), torch.from_numpy(q).cuda(), inv_tau))
        ref = oracle.score(x32, q, inv_tau)
        err, tol = float(np.abs(s - ref).max()), 2e-5 * inv_tau
        worst = max(worst, err / tol)
        assert np.isfinite(s).all() and err <= tol, (dtype, dim, rows, inv_tau, err)
        if rows > 3:
            assert s[1] == 0.0 and s[2] == 0.0
        done += 1
    log("   worst error / tolerance", worst)


def test_ragged_random_batches(bd):
    """Eq. 9 on packed items of random sizes: the grouped compression and the one-launch attention against the oracle
    item by item; item counts around the 64 of one group, lengths around the 64-row contraction tile, head sizes that
    are padded or not, grouped heads."""
    rng = np.random.default_rng(99)
    worst_c, worst_a = 0.0, 0.0
    for case in range(40):
        n_items = int(rng.choice([1, 2, 5, 63, 64, 65, 90])) if case % 4 == 0 else int(rng.integers(1, 12))
        sizes = rng.choice([1, 2, 63, 64, 65, 127, 128, 129, 300], n_items) if case % 3 == 0 else rng.integers(1, 200, n_items)
        off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
        total = int(off[-1])
        hkv = int(rng.choice([1, 2, 4]))
        hq = hkv * int(rng.choice([1, 2, 4]))
        d = int(rng.choice([32, 64, 72, 96, 128]))
        s = 4 * int(rng.integers(1, 40))
        k, k32 = wl.quantize(rng.standard_normal((total, hkv, d)).astype(np.float32), "bf16")
        v, v32 = wl.quantize(rng.standard_normal((total, hkv, d)).astype(np.float32), "bf16")
        q, q32 = wl.quantize((rng.standard_normal((total, hq, d)) * rng.choice([0.5, 1.0, 2.0])).astype(np.float32), "bf16")
        r = (rng.random((total, s)) ** 4).astype(np.float32)
        log("ragged case", case, "items", n_items, "rows", total, "heads", hq, hkv, "d", d, "S", s)
        kc, vc = bd.civic_kv_compress_ragged(to_dev(k), to_dev(v), torch.from_numpy(r).cuda(), off)
        out = bd.civic_cross_attn_ragged(to_dev(q), kc, vc, off)
        torch.cuda.synchronize()
        for got, x32 in ((kc, k32), (vc, v32)):
            ref = oracle.kv_compress_ragged(x32.reshape(total, hkv * d), r, off).reshape(n_items, s, hkv, d)
            err = float(np.abs(widen(to_host(got)).astype(np.float64) - ref).max())
            worst_c = max(worst_c, err / attn_tol(ref, "bf16"))
            assert err <= attn_tol(ref, "bf16")
        ref = oracle.cross_attention_ragged(q32, widen(to_host(kc)), widen(to_host(vc)), off)
        got = widen(to_host(out)).astype(np.float64)
        err = float(np.abs(got - ref).max())
        worst_a = max(worst_a, err / attn_tol(ref, "bf16"))
        assert np.isfinite(got).all() and err <= attn_tol(ref, "bf16")
    log("ragged: worst error / tolerance, compression", worst_c, "attention", worst_a)
