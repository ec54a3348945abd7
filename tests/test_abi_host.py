"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares, the
host-side functions agree with the tabulated grids, and every documented argument error is
rejected before any HIP call (no compute call is made here)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2605_28115_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def bd():
    from paper_2605_28115_amd import binding
    return binding


def test_exports_every_declared_symbol(bd):
    header = open(os.path.join(ROOT, "include", "civic.h")).read()
    declared = set(re.findall(r"\b(civic_[a-z_]+)\s*\(", header))
    assert declared == set(bd.EXPORTS)
    for name in declared:
        assert hasattr(bd.lib, name), name
    assert bd.lib.civic_last_hip_error() == 0


def test_header_limits_match_binding(bd):
    header = open(os.path.join(ROOT, "include", "civic.h")).read()
    lim = dict(re.findall(r"#define (CIVIC_MAX_[A-Z_]+)\s+(\d+)", header))
    assert int(lim["CIVIC_MAX_VISUAL_TOKENS"]) == bd.MAX_VISUAL_TOKENS
    assert int(lim["CIVIC_MAX_FRAMES"]) == bd.MAX_FRAMES
    assert int(lim["CIVIC_MAX_SCORE_DIM"]) == bd.MAX_SCORE_DIM
    assert int(lim["CIVIC_MAX_HEAD_DIM"]) == bd.MAX_HEAD_DIM


@pytest.mark.parametrize("name", list(wl.WORKLOADS))
def test_kept_count_of_tabulated_workloads(bd, name):
    w = wl.WORKLOADS[name]
    assert bd.civic_kept_count(w.grid_tuple()) == w.kept
    assert bd.civic_select_workspace_bytes(w.grid_tuple(), w.batch) == 0
    assert bd.civic_compact_workspace_bytes(w.batch, w.seq_len) == 0


def test_kept_count_closed_form_on_ragged_grids(bd):
    for grid in wl.small_grid_cases():
        frames, H, W, ch, cw, cf, ff, budget = grid
        per_frame = 0
        for r0 in range(0, H, ch):
            for c0 in range(0, W, cw):
                per_frame += min(cf, (min(r0 + ch, H) - r0) * (min(c0 + cw, W) - c0))
        per_frame += min(ff, H * W - per_frame)
        assert bd.civic_kept_count(grid) == max(budget, frames * per_frame), grid


@pytest.mark.parametrize("grid", [
    (0, 4, 4, 2, 2, 1, 0, 1), (1, 0, 4, 2, 2, 1, 0, 1), (1, 4, -1, 2, 2, 1, 0, 1), (1, 4, 4, 0, 2, 1, 0, 1),
    (1, 4, 4, 2, 0, 1, 0, 1), (1, 4, 4, 2, 2, -1, 0, 1), (1, 4, 4, 2, 2, 1, -1, 1), (1, 4, 4, 2, 2, 1, 0, -1),
    (1, 4, 4, 2, 2, 1, 0, 17), (70000, 70000, 2, 2, 2, 1, 0, 1),
])
def test_bad_grids_are_rejected(bd, grid):
    assert bd.lib.civic_kept_count(C.byref(bd.make_grid(grid))) == bd.ERR_INVALID_ARG
    assert bd.lib.civic_kept_count(None) == bd.ERR_INVALID_ARG
    fake = C.c_void_p(0x1000)
    assert bd.lib.civic_select(fake, 1, C.byref(bd.make_grid(grid)), fake, None, None, 0, None) == bd.ERR_INVALID_ARG


def test_anchor_normalize_host(bd):
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(300) * 2 + 5).astype(np.float32)
    q = bd.civic_anchor_normalize(a)
    assert abs(float(q.astype(np.float64).sum())) < 1e-5 and abs(float((q.astype(np.float64) ** 2).sum()) - 1) < 1e-6
    c = a.astype(np.float64) - a.astype(np.float64).mean()
    assert np.abs(q - c / np.linalg.norm(c)).max() < 1e-7
    with pytest.raises(bd.CivicError):
        bd.civic_anchor_normalize(np.full(8, 3.0, dtype=np.float32))
    assert bd.lib.civic_anchor_normalize(None, 8, None) == bd.ERR_INVALID_ARG


def test_argument_errors_precede_any_hip_call(bd):
    L, F, I = bd.lib, C.c_void_p(0x1000), bd.ERR_INVALID_ARG
    odd = C.c_void_p(0x1004)
    st = (C.c_int64 * 3)(1024, 128, 128)
    g = bd.make_grid((1, 4, 4, 2, 2, 1, 0, 5))
    # civic_score: null, bad dtype, dim not a vector multiple, stride < dim, misaligned, too wide
    assert L.civic_score(None, 1, 4, 64, 64, F, 1.0, F, None) == I
    assert L.civic_score(F, 7, 4, 64, 64, F, 1.0, F, None) == I
    assert L.civic_score(F, 1, 4, 64, 60, F, 1.0, F, None) == I
    assert L.civic_score(F, 1, 4, 32, 64, F, 1.0, F, None) == I
    assert L.civic_score(odd, 1, 4, 64, 64, F, 1.0, F, None) == I
    assert L.civic_score(F, 1, -1, 64, 64, F, 1.0, F, None) == I
    assert L.civic_score(F, 1, 4, 16384, 16384, F, 1.0, F, None) == bd.ERR_UNSUPPORTED
    assert L.civic_score(F, 1, 0, 64, 64, F, 1.0, F, None) == bd.CIVIC_OK          # nothing to do
    # civic_score_visual: the same checks plus the frame spans
    def score_vis(fs, seq_len=40, grid=g, hidden=F, dim=64, batch=1, dt=1, scores=F, anchor=F):
        arr = np.asarray(fs, dtype=np.int64)
        return L.civic_score_visual(hidden, dt, batch, seq_len, dim, C.byref(grid), C.c_void_p(arr.ctypes.data), anchor,
                                    C.c_float(1.0), scores, None)
    assert score_vis([30]) == I and score_vis([-1]) == I and score_vis([0], seq_len=15) == I
    assert score_vis([0], hidden=None) == I and score_vis([0], hidden=odd) == I and score_vis([0], dim=60) == I
    assert score_vis([0], dt=5) == I and score_vis([0], scores=None) == I and score_vis([0], anchor=None) == I
    assert score_vis([0], batch=-1) == I and score_vis([0], batch=0, hidden=None, scores=None) == bd.CIVIC_OK
    assert score_vis([0], dim=16384) == bd.ERR_UNSUPPORTED and score_vis([0], batch=70000) == bd.ERR_UNSUPPORTED
    two = bd.make_grid((2, 4, 4, 2, 2, 1, 0, 5))
    assert score_vis([0, 8], grid=two) == I and score_vis([20, 0], grid=two) == I
    assert L.civic_score_visual(F, 1, 1, 40, 64, C.byref(g), None, F, C.c_float(1.0), F, None) == I
    # civic_select: null scores / output, too many tokens
    assert L.civic_select(None, 1, C.byref(g), F, None, None, 0, None) == I
    assert L.civic_select(F, 1, C.byref(g), None, None, None, 0, None) == I
    assert L.civic_select(F, -1, C.byref(g), F, None, None, 0, None) == I
    big = bd.make_grid((1, 256, 256, 4, 4, 1, 0, 100))
    assert L.civic_select(F, 1, C.byref(big), F, None, None, 0, None) == bd.ERR_UNSUPPORTED
    assert L.civic_select(F, 0, C.byref(g), F, None, None, 0, None) == bd.CIVIC_OK
    # civic_compact: frame spans out of range / overlapping / not ascending, seq shorter than N_v
    def compact(fs, seq_len=40, n_kept=5, grid=g, hidden=F, dim=64):
        arr = np.asarray(fs, dtype=np.int64)
        return L.civic_compact(hidden, 1, dim, F, 1, seq_len, C.byref(grid), C.c_void_p(arr.ctypes.data), F, n_kept,
                               F, F, F, None, 0, None)
    assert compact([30]) == I and compact([-1]) == I and compact([0], seq_len=15) == I
    assert compact([0], n_kept=17) == I and compact([0], hidden=None) == I and compact([0], hidden=odd) == I
    g2 = bd.make_grid((2, 4, 4, 2, 2, 1, 0, 5))
    assert compact([0, 8], grid=g2) == I and compact([20, 0], grid=g2) == I
    many = bd.make_grid((200, 1, 1, 1, 1, 0, 0, 5))
    assert compact(list(range(200)), seq_len=400, grid=many) == bd.ERR_UNSUPPORTED
    # civic_compact_prefill: the checks of all three stages, before anything is launched
    def front(fs=(0,), seq_len=40, grid=g, hidden=F, dim=64, batch=1, pos=F, anchor=F, scores=F, kept=F, hc=F, pc=F, si=F):
        arr = np.asarray(fs, dtype=np.int64)
        return L.civic_compact_prefill(hidden, 1, batch, seq_len, dim, pos, C.byref(grid), C.c_void_p(arr.ctypes.data), anchor,
                                       C.c_float(1.0), scores, kept, hc, pc, si, None, 0, None)
    assert front(fs=[30]) == I and front(seq_len=15) == I and front(hidden=None) == I and front(hidden=odd) == I
    assert front(dim=60) == I and front(anchor=None) == I and front(scores=None) == I and front(kept=None) == I
    assert front(pos=None) == I and front(hc=None) == I and front(pc=None) == I and front(si=None) == I
    assert front(kept=C.c_void_p(0x1002)) == I and front(batch=-1) == I
    assert front(grid=big, seq_len=70000) == bd.ERR_UNSUPPORTED and front(dim=16384) == bd.ERR_UNSUPPORTED
    assert front(batch=0, hidden=None, pos=None, scores=None, kept=None, hc=None, pc=None, si=None) == bd.CIVIC_OK
    # civic_prefill_attn: head mismatch, head_dim, alignment, scale
    def attn(**kw):
        a = dict(q=F, k=F, v=F, o=F, dt=1, b=1, s=8, hq=4, hkv=2, d=64, qs=st, ks=st, os=st, causal=1, scale=0.0)
        a.update(kw)
        return L.civic_prefill_attn(a["q"], a["k"], a["v"], a["o"], a["dt"], a["b"], a["s"], a["hq"], a["hkv"], a["d"],
                                    a["qs"], a["ks"], a["os"], a["causal"], C.c_float(a["scale"]), None)
    assert attn(hq=3) == I and attn(d=60) == I and attn(q=odd) == I and attn(k=None) == I and attn(dt=2) == I
    assert attn(scale=-1.0) == I and attn(scale=float("nan")) == I and attn(qs=None) == I
    assert attn(qs=(C.c_int64 * 3)(1024, 100, 68)) == I
    assert attn(d=512) == bd.ERR_UNSUPPORTED and attn(s=0) == bd.CIVIC_OK
    # civic_kv_write: rows past the cache end, negative pos0, head bytes not a vector multiple
    def kvw(**kw):
        a = dict(k=F, v=F, st=st, dt=1, kc=F, vc=F, b=1, s=8, h=2, d=64, smax=16, pos0=0)
        a.update(kw)
        return L.civic_kv_write(a["k"], a["v"], a["st"], a["dt"], a["kc"], a["vc"], a["b"], a["s"], a["h"], a["d"],
                                a["smax"], a["pos0"], None)
    assert kvw(pos0=9) == I and kvw(pos0=-1) == I and kvw(d=4) == I and kvw(kc=None) == I and kvw(v=odd) == I
    assert kvw(st=None) == I and kvw(h=0) == I and kvw(s=0) == bd.CIVIC_OK
    # civic_prefill_attn_kv: the checks of both calls, and the caches are mandatory
    def attn_kv(**kw):
        a = dict(q=F, k=F, v=F, o=F, kc=F, vc=F, dt=1, b=1, s=8, hq=4, hkv=2, d=64, qs=st, ks=st, os=st, smax=16, pos0=0,
                 causal=1, scale=0.0)
        a.update(kw)
        return L.civic_prefill_attn_kv(a["q"], a["k"], a["v"], a["o"], a["kc"], a["vc"], a["dt"], a["b"], a["s"], a["hq"],
                                       a["hkv"], a["d"], a["qs"], a["ks"], a["os"], a["smax"], a["pos0"], a["causal"],
                                       C.c_float(a["scale"]), None)
    assert attn_kv(kc=None) == I and attn_kv(vc=None) == I and attn_kv(vc=odd) == I
    assert attn_kv(pos0=9) == I and attn_kv(pos0=-1) == I and attn_kv(smax=7) == I
    assert attn_kv(hq=3) == I and attn_kv(d=60) == I and attn_kv(scale=-1.0) == I and attn_kv(ks=None) == I
    # civic_decode_attn: context outside the cache, empty context, head mismatch, alignment, workspace
    def dec(**kw):
        a = dict(q=F, kc=F, vc=F, o=F, dt=1, b=2, hq=4, hkv=2, d=64, smax=100, n=50, scale=0.0, ws=F, wsb=1 << 30)
        a.update(kw)
        return L.civic_decode_attn(a["q"], a["kc"], a["vc"], a["o"], a["dt"], a["b"], a["hq"], a["hkv"], a["d"], a["smax"],
                                   a["n"], C.c_float(a["scale"]), a["ws"], a["wsb"], None)
    assert dec(n=101) == I and dec(n=0) == I and dec(n=-1) == I and dec(hq=3) == I and dec(d=60) == I
    assert dec(q=None) == I and dec(kc=odd) == I and dec(o=None) == I and dec(dt=3) == I and dec(scale=-1.0) == I
    assert dec(d=1024) == bd.ERR_UNSUPPORTED and dec(b=0, q=None, kc=None, vc=None, o=None) == bd.CIVIC_OK
    need = bd.civic_decode_attn_workspace_bytes(__import__("torch").bfloat16, 2, 4, 2, 64, 50)
    assert need == 0                                        # 50 rows are one round of one workgroup: nothing to combine
    need = bd.civic_decode_attn_workspace_bytes(__import__("torch").bfloat16, 2, 4, 2, 64, 5000)
    assert need > 0 and need % 4 == 0
    assert dec(smax=6000, n=5000, ws=None, wsb=0) == bd.ERR_WORKSPACE
    assert dec(smax=6000, n=5000, wsb=need - 4) == bd.ERR_WORKSPACE and dec(smax=6000, n=5000, ws=odd) == bd.ERR_WORKSPACE
    # rotary calls: tables, head sizes, alignment, cache bounds
    ax = np.asarray([0, 1, 2, 1], dtype=np.int32); fr = np.asarray([1.0, 0.5, 0.25, 0.1], dtype=np.float32)
    def table(axis=ax, freq=fr, n=4, pos=F, out=F, b=1, s=8):
        return L.civic_mrope_table(pos, b, s, n, C.c_void_p(axis.ctypes.data) if axis is not None else None,
                                   C.c_void_p(freq.ctypes.data) if freq is not None else None, out, None)
    assert table(axis=None) == I and table(freq=None) == I and table(n=0) == I and table(pos=None) == I and table(out=odd) == I
    assert table(axis=np.asarray([0, 3, 0, 0], dtype=np.int32)) == I
    assert table(freq=np.asarray([1.0, np.inf, 0.0, 0.0], dtype=np.float32)) == I
    assert table(n=129, axis=np.zeros(129, dtype=np.int32), freq=np.zeros(129, dtype=np.float32)) == bd.ERR_UNSUPPORTED
    assert table(s=0, pos=None, out=None) == bd.CIVIC_OK
    def apply(**kw):
        a = dict(x=F, o=F, dt=1, b=1, s=8, h=2, d=64, xs=st, os=st, cs=F)
        a.update(kw)
        return L.civic_mrope_apply(a["x"], a["o"], a["dt"], a["b"], a["s"], a["h"], a["d"], a["xs"], a["os"], a["cs"], None)
    assert apply(d=24) == I and apply(d=63) == I and apply(x=None) == I and apply(cs=None) == I and apply(o=odd) == I
    assert apply(xs=None) == I and apply(dt=9) == I and apply(d=512) == bd.ERR_UNSUPPORTED and apply(s=0, x=None, o=None, cs=None) == bd.CIVIC_OK
    def kvr(**kw):
        a = dict(k=F, v=F, st=st, dt=1, cs=F, kc=F, vc=F, b=1, s=8, h=2, d=64, smax=16, pos0=0)
        a.update(kw)
        return L.civic_kv_write_rope(a["k"], a["v"], a["st"], a["dt"], a["cs"], a["kc"], a["vc"], a["b"], a["s"], a["h"], a["d"],
                                     a["smax"], a["pos0"], None)
    assert kvr(pos0=9) == I and kvr(d=24) == I and kvr(cs=None) == I and kvr(kc=None) == I and kvr(cs=odd) == I and kvr(s=0) == bd.CIVIC_OK
    def attn_rope(**kw):
        a = dict(q=F, k=F, v=F, o=F, dt=1, b=1, s=8, hq=4, hkv=2, d=64, qs=st, ks=st, os=st, causal=1, scale=0.0, cs=F)
        a.update(kw)
        return L.civic_prefill_attn_rope(a["q"], a["k"], a["v"], a["o"], a["dt"], a["b"], a["s"], a["hq"], a["hkv"], a["d"],
                                         a["qs"], a["ks"], a["os"], a["causal"], C.c_float(a["scale"]), a["cs"], None)
    assert attn_rope(cs=None) == I and attn_rope(cs=odd) == I and attn_rope(hq=3) == I and attn_rope(s=0, cs=None) == bd.CIVIC_OK
    # encoder-side calls
    def agg(**kw):
        a = dict(x=F, a=F, dt=1, b=1, t=100, m=10, d=64, tau=1.0, z=F, tw=None, ws=F, wsb=1 << 40)
        a.update(kw)
        return L.civic_anchor_aggregate(a["x"], a["a"], a["dt"], a["b"], a["t"], a["m"], a["d"], C.c_float(a["tau"]), a["z"], a["tw"],
                                        a["ws"], a["wsb"], None)
    assert agg(x=None) == I and agg(a=odd) == I and agg(t=0) == I and agg(m=0) == I and agg(tau=-1.0) == I and agg(dt=4) == I
    assert agg(d=72) == bd.ERR_UNSUPPORTED and agg(dt=0) == bd.ERR_UNSUPPORTED
    assert agg(ws=None) == bd.ERR_WORKSPACE and agg(wsb=1000) == bd.ERR_WORKSPACE
    assert bd.lib.civic_anchor_aggregate_workspace_bytes(1, 100, 10, 64) > 0 and bd.lib.civic_anchor_aggregate_workspace_bytes(1, 0, 10, 64) == 0
    assert agg(b=0, x=None, z=None) == bd.CIVIC_OK
    def comp(**kw):
        a = dict(k=F, v=F, dt=1, r=F, b=1, m=100, s=10, w=64, kc=F, vc=F, ws=F, wsb=1 << 40)
        a.update(kw)
        return L.civic_kv_compress(a["k"], a["v"], a["dt"], a["r"], a["b"], a["m"], a["s"], a["w"], a["kc"], a["vc"], a["ws"], a["wsb"], None)
    assert comp(k=None) == I and comp(r=None) == I and comp(m=0) == I and comp(s=0) == I and comp(vc=odd) == I
    assert comp(dt=0) == bd.ERR_UNSUPPORTED and comp(ws=None) == bd.ERR_WORKSPACE and comp(wsb=10) == bd.ERR_WORKSPACE
    def cross(**kw):
        a = dict(q=F, k=F, v=F, o=F, dt=1, b=1, nq=8, nkv=5, hq=4, hkv=2, d=64, qs=st, ks=st, os=st, scale=0.0)
        a.update(kw)
        return L.civic_cross_attn(a["q"], a["k"], a["v"], a["o"], a["dt"], a["b"], a["nq"], a["nkv"], a["hq"], a["hkv"], a["d"],
                                  a["qs"], a["ks"], a["os"], C.c_float(a["scale"]), None)
    assert cross(nkv=0) == I and cross(nkv=-1) == I and cross(hq=3) == I and cross(k=None) == I and cross(nq=0, nkv=0) == bd.CIVIC_OK
    # a tensor without elements needs no pointer: NULL is accepted exactly then
    OK = bd.CIVIC_OK
    assert L.civic_score(None, 1, 0, 64, 64, F, 1.0, None, None) == OK and L.civic_score(F, 1, 0, 64, 64, None, 1.0, F, None) == I
    assert L.civic_select(None, 0, C.byref(g), None, None, None, 0, None) == OK
    none_kept = bd.make_grid((1, 4, 4, 2, 2, 0, 0, 0))
    fs0 = np.zeros(1, dtype=np.int64)
    def compact0(batch, seq_len, n_kept, out):
        return L.civic_compact(F if batch else None, 1, 64, F if batch else None, batch, seq_len, C.byref(none_kept),
                               C.c_void_p(fs0.ctypes.data), None, n_kept, out, out, out, None, 0, None)
    assert compact0(0, 16, 0, None) == OK                # empty batch
    assert compact0(1, 16, 0, None) == OK                # no text, nothing kept: S_c = 0
    assert compact0(1, 17, 0, None) == I                 # one text token: outputs are needed
    assert attn(q=None, k=None, v=None, o=None, s=0) == OK and attn(q=None, k=None, v=None, o=None, b=0) == OK
    assert kvw(k=None, v=None, kc=None, vc=None, s=0) == OK and kvw(k=None, v=None, kc=None, vc=None, b=0) == OK
    assert attn_kv(q=None, k=None, v=None, o=None, kc=None, vc=None, s=0) == OK
    wide = (C.c_int64 * 3)(8192, 1024, 512)
    assert attn_kv(d=512, qs=wide, ks=wide, os=wide) == bd.ERR_UNSUPPORTED and attn_kv(s=0) == bd.CIVIC_OK
    # ragged Eq. 9 calls: offsets (null, not starting at 0, an empty item), row alignment, workspace
    def offs(*v):
        return np.asarray(v, dtype=np.int64)
    def rcomp(off=offs(0, 5, 12), batch=2, k=F, r=F, n_mem=8, width=64, ws=F, wsb=1 << 30, dt=1):
        return L.civic_kv_compress_ragged(k, F, dt, r, batch, C.c_void_p(off.ctypes.data) if off is not None else None, n_mem, width,
                                          F, F, ws, wsb, None)
    assert rcomp(off=None) == I and rcomp(off=offs(1, 5, 12)) == I and rcomp(off=offs(0, 5, 5)) == I and rcomp(off=offs(0, 5, 3)) == I
    assert rcomp(k=None) == I and rcomp(r=None) == I and rcomp(k=odd) == I and rcomp(batch=-1) == I and rcomp(dt=9) == I
    assert rcomp(width=60) == bd.ERR_UNSUPPORTED and rcomp(n_mem=6) == bd.ERR_UNSUPPORTED and rcomp(dt=0) == bd.ERR_UNSUPPORTED
    assert rcomp(ws=None, wsb=0) == bd.ERR_WORKSPACE and rcomp(wsb=16) == bd.ERR_WORKSPACE and rcomp(batch=0, off=None) == OK
    o3 = offs(0, 5, 12)
    need = L.civic_kv_compress_ragged_workspace_bytes(2, C.c_void_p(o3.ctypes.data), 8, 64)
    # per item 32 rows of partial column sums and Rbar^T (S x its rows rounded up to 64, bf16)
    a256 = lambda x: (x + 255) // 256 * 256
    assert need == a256(2 * 8 * 4 * 32) + a256(8 * (64 + 64) * 2)
    def rattn(off=offs(0, 5, 12), batch=2, q=F, k=F, o=F, hq=4, hkv=2, d=64, qs=st, ks=st):
        return L.civic_cross_attn_ragged(q, k, k, o, 1, batch, C.c_void_p(off.ctypes.data) if off is not None else None, 8, hq, hkv, d,
                                         qs, ks, st, C.c_float(0.0), None)
    assert rattn(off=None) == I and rattn(off=offs(2, 5, 12)) == I and rattn(off=offs(0, 5, 5)) == I and rattn(q=None) == I
    assert rattn(hq=3) == I and rattn(d=60) == I and rattn(qs=None) == I and rattn(k=odd) == I and rattn(batch=0, off=None) == OK
    assert bd.lib.civic_last_hip_error() == 0


def test_kernel_timer_argument_checks(bd):
    # only the handles' values are looked at here: nothing is launched, so nothing touches them
    one, two = C.c_void_p(0x1000), C.c_void_p(0x2000)
    f = bd.lib.civic_time_next_kernel
    assert f(one, None) == bd.ERR_INVALID_ARG
    assert f(None, two) == bd.ERR_INVALID_ARG
    assert f(one, one) == bd.ERR_INVALID_ARG
    assert f(one, two) == bd.CIVIC_OK
    assert f(None, None) == bd.CIVIC_OK             # disarmed again: no later launch of this thread sees the handles


def test_ragged_path_offsets_and_argument_errors(bd):
    """civic_ragged_offsets is a host function (checked against the oracle's own count); the two ragged path calls
    reject every documented error before any HIP call."""
    import oracle
    L = bd.lib
    I, OK = bd.ERR_INVALID_ARG, bd.CIVIC_OK
    grids = [(1, 16, 16, 4, 4, 2, 0, 85), (2, 5, 7, 2, 3, 1, 2, 20), (1, 1, 1, 1, 1, 0, 0, 0), (16, 24, 24, 4, 4, 1, 16, 3072)]
    lens = [288, 90, 1, 9728]
    got = bd.civic_ragged_offsets(lens, grids)
    ref = oracle.ragged_offsets(lens, grids)
    for a, b in zip(got, ref):
        assert np.array_equal(a, b)
    gs = (bd.Grid * 2)(bd.make_grid(grids[0]), bd.make_grid(grids[1]))
    off = lambda *v: np.asarray(v, dtype=np.int64)
    out = np.zeros(3, dtype=np.int64)
    P = lambda a: C.c_void_p(a.ctypes.data) if a is not None else None
    ro = lambda o=off(0, 288, 378), g=gs, b=2: L.civic_ragged_offsets(b, P(o), g, P(out), None, None)
    assert ro() == OK and out.tolist() == [0, 256, 326]
    assert ro(o=None) == I and ro(o=off(1, 288, 378)) == I and ro(o=off(0, 255, 378)) == I and ro(g=None) == I and ro(b=-1) == I
    bad = (bd.Grid * 2)(bd.make_grid(grids[0]), bd.Grid(1, 0, 7, 1, 1, 0, 0, 0))
    assert ro(g=bad) == I and ro(b=0, g=None) == OK

    F = C.c_void_p(0x1000)
    fs = off(16, 3, 50)
    def front(hidden=F, dt=1, b=2, o=off(0, 288, 378), dim=64, pos=F, g=gs, f=fs, aq=F, sc=F, kept=F, hc=F, pc=F, si=F):
        return L.civic_compact_prefill_ragged(hidden, dt, b, P(o), dim, pos, g, P(f), aq, C.c_float(1.0), sc, kept, hc, pc, si, None)
    assert front(dt=7) == I and front(dim=0) == I and front(o=None) == I and front(o=off(0, 100, 378)) == I and front(g=None) == I
    assert front(f=None) == I and front(hidden=None) == I and front(aq=None) == I and front(sc=None) == I and front(kept=None) == I
    assert front(hc=None) == I and front(pc=None) == I and front(si=None) == I and front(pos=None) == I
    assert front(f=off(16, 3, 30)) == I                              # second sample: overlapping frames (3 + 35 > 30)
    assert front(f=off(40, 3, 50)) == I                              # first sample: the frame runs past its rows
    assert front(dim=60) == I                                        # rows that are not whole 16-byte pieces
    assert front(b=0, o=off(0), g=None, f=None, hidden=None) == OK

    st = (C.c_int64 * 3)(0, 512, 128)
    def attn(q=F, k=F, o=F, b=2, ro_=off(0, 5, 12), hq=4, hkv=2, d=128, qs=st, ks=st, causal=1, kc=None, vc=None, smax=0, pos0=0, dt=1):
        return L.civic_prefill_attn_ragged(q, k, k, o, dt, b, P(ro_), hq, hkv, d, qs, ks, st, causal, C.c_float(0.0), kc, vc, smax, pos0, None)
    assert attn(ro_=None) == I and attn(ro_=off(1, 5, 12)) == I and attn(ro_=off(0, 5, 5)) == I and attn(q=None) == I and attn(k=None) == I
    assert attn(o=None) == I and attn(hq=3) == I and attn(d=60) == I and attn(qs=None) == I and attn(dt=5) == I and attn(b=-1) == I
    assert attn(kc=F) == I and attn(vc=F) == I                        # one cache without the other
    assert attn(kc=F, vc=F, smax=6) == I                              # the longest sample (7 rows) does not fit
    assert attn(kc=F, vc=F, smax=16, pos0=10) == I and attn(kc=F, vc=F, smax=16, pos0=-1) == I
    assert attn(b=0, ro_=None) == OK and attn(d=512, qs=(C.c_int64 * 3)(0, 2048, 512), ks=(C.c_int64 * 3)(0, 1024, 512)) == bd.ERR_UNSUPPORTED
    assert bd.lib.civic_last_hip_error() == 0


def test_ragged_decode_argument_errors(bd):
    L, F = bd.lib, C.c_void_p(0x1000)
    I, OK = bd.ERR_INVALID_ARG, bd.CIVIC_OK
    ctx = lambda *v: np.asarray(v, dtype=np.int32)
    P = lambda a: C.c_void_p(a.ctypes.data) if a is not None else None
    def dec(q=F, kc=F, vc=F, o=F, dt=1, b=3, n=ctx(5, 938, 17), hq=32, hkv=8, d=128, smax=1000, scale=0.0, ws=F, wsb=1 << 30):
        return L.civic_decode_attn_ragged(q, kc, vc, o, dt, b, P(n), hq, hkv, d, smax, C.c_float(scale), ws, wsb, None)
    assert dec(n=None) == I and dec(n=ctx(5, 0, 17)) == I and dec(n=ctx(5, 1001, 17)) == I and dec(n=ctx(-1, 2, 3)) == I
    assert dec(q=None) == I and dec(kc=None) == I and dec(vc=None) == I and dec(o=None) == I and dec(dt=4) == I and dec(b=-1) == I
    assert dec(hq=30) == I and dec(d=60) == I and dec(scale=-1.0) == I and dec(q=C.c_void_p(0x1004)) == I
    assert dec(d=1024) == bd.ERR_UNSUPPORTED and dec(b=0, n=None, q=None) == OK
    need = L.civic_decode_attn_ragged_workspace_bytes(1, 3, P(ctx(5, 938, 17)), 32, 8, 128)
    assert need == L.civic_decode_attn_workspace_bytes(1, 3, 32, 8, 128, 938) > 0      # laid out for the longest context
    assert dec(ws=None, wsb=0) == bd.ERR_WORKSPACE and dec(wsb=need - 1) == bd.ERR_WORKSPACE
    assert L.civic_decode_attn_ragged_workspace_bytes(1, 3, P(ctx(5, 0, 17)), 32, 8, 128) == 0
    assert bd.lib.civic_last_hip_error() == 0


def test_header_is_plain_c(tmp_path):
    """include/civic.h is a C ABI: it compiles as C99 and as C++ with nothing but the standard headers."""
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text('#include "civic.h"\nint main(void) { return CIVIC_OK; }\n')
    inc = os.path.join(ROOT, "include")
    for cmd in (["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror"], ["g++", "-std=c++17", "-x", "c++", "-Wall", "-Wextra", "-pedantic"]):
        r = subprocess.run(cmd + ["-I", inc, "-fsyntax-only", str(src)], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
