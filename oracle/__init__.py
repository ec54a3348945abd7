"""ctypes front end of the CPU oracle (oracle/civic_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  It shares nothing with the HIP library and the product path never
imports it.  All arrays are host numpy arrays; bf16 inputs are passed as their exact fp32
widening (floating-point steps) or as raw bytes (copy steps).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "civic_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP on the outermost loops)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class Grid(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("frames", "height", "width", "cell_h", "cell_w",
                                         "cell_floor", "frame_floor", "budget")]


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        P = C.c_void_p
        L.oracle_threads.restype = C.c_int
        L.oracle_anchor_normalize.restype = C.c_int
        L.oracle_anchor_normalize.argtypes = [P, C.c_int32, C.c_double, P]
        L.oracle_score.restype = None
        L.oracle_score.argtypes = [P, C.c_int64, C.c_int64, C.c_int32, P, C.c_double, P]
        L.oracle_select_batch.restype = C.c_int64
        L.oracle_select_batch.argtypes = [P, C.c_int32, C.POINTER(Grid), C.c_int, P, C.c_int64, P]
        L.oracle_kept_count.restype = C.c_int64
        L.oracle_kept_count.argtypes = [C.POINTER(Grid), C.c_int]
        L.oracle_compact.restype = C.c_int64
        L.oracle_compact.argtypes = [P, C.c_int64, P, C.c_int32, C.c_int64, C.POINTER(Grid), P, P,
                                     C.c_int64, C.c_int64, P, P, P]
        L.oracle_attention.restype = None
        L.oracle_attention.argtypes = [P, P, P, P, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                       C.c_int32, P, P, C.c_int, C.c_double, C.c_int32]
        L.oracle_kv_write.restype = C.c_int64
        L.oracle_kv_write.argtypes = [P, P, P, P, P, C.c_int32, C.c_int32, C.c_int32, C.c_int64,
                                      C.c_int64, C.c_int64]
        L.oracle_anchor_aggregate.restype = None
        L.oracle_anchor_aggregate.argtypes = [P, P, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_double, C.c_double, P, P]
        L.oracle_kv_compress.restype = None
        L.oracle_kv_compress.argtypes = [P, P, C.c_int32, C.c_int32, C.c_int32, C.c_int32, P]
        L.oracle_cross_attention.restype = None
        L.oracle_cross_attention.argtypes = [P, P, P, P, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                             C.c_double]
        L.oracle_mrope_table.restype = None
        L.oracle_mrope_table.argtypes = [P, C.c_int32, C.c_int64, C.c_int32, P, P, P]
        L.oracle_mrope_apply.restype = None
        L.oracle_mrope_apply.argtypes = [P, P, C.c_int32, C.c_int64, C.c_int32, C.c_int32, P, P]
        L.oracle_decode_attention.restype = None
        L.oracle_decode_attention.argtypes = [P, P, P, P, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int64,
                                              C.c_int64, C.c_double]
        _lib = L
    return _lib


def _ptr(a: np.ndarray) -> C.c_void_p:
    return C.c_void_p(a.ctypes.data)


def _grid(g: Sequence[int]) -> Grid:
    return Grid(*[int(x) for x in g])


def threads() -> int:
    return int(lib().oracle_threads())


def anchor_normalize(a: np.ndarray, eps: float = 1e-6) -> np.ndarray:
    """Q_A = Norm(LN(a)) (Eq. 8) as float64 [dim]."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    q = np.empty(a.shape[0], dtype=np.float64)
    rc = lib().oracle_anchor_normalize(_ptr(a), a.shape[0], float(eps), _ptr(q))
    if rc != 0:
        raise ValueError("anchor has zero variance")
    return q


def score(x: np.ndarray, q: np.ndarray, inv_tau: float = 1.0) -> np.ndarray:
    """Anchor logit of Eq. 8 for every row of x [n_rows, dim] (fp32 widening of the input);
    q is the fp32 pre-normalised anchor the library is given.  Returns fp32 [n_rows]."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    q = np.ascontiguousarray(q, dtype=np.float32)
    assert x.ndim == 2 and q.shape == (x.shape[1],)
    out = np.empty(x.shape[0], dtype=np.float32)
    lib().oracle_score(_ptr(x), x.shape[0], x.shape[1], x.shape[1], _ptr(q), float(inv_tau), _ptr(out))
    return out


def kept_count(grid: Sequence[int], nested: bool = False) -> int:
    k = int(lib().oracle_kept_count(C.byref(_grid(grid)), int(nested)))
    if k < 0:
        raise ValueError(f"bad grid {tuple(grid)}")
    return k


def select(scores: np.ndarray, grid: Sequence[int], nested: bool = False) -> Tuple[np.ndarray, np.ndarray]:
    """scores fp32 [batch, N_v] -> (kept_idx int32 [batch, K] ascending, keep_flags u8 [batch, N_v])."""
    s = np.ascontiguousarray(scores, dtype=np.float32)
    assert s.ndim == 2
    g = _grid(grid)
    k = kept_count(grid, nested)
    idx = np.full((s.shape[0], k), -1, dtype=np.int32)
    flags = np.zeros(s.shape, dtype=np.uint8)
    rc = int(lib().oracle_select_batch(_ptr(s), s.shape[0], C.byref(g), int(nested), _ptr(idx), k, _ptr(flags)))
    if rc == -2:
        raise ValueError("NaN score")
    if rc != k and s.shape[0] > 0:
        raise RuntimeError(f"oracle_select_batch returned {rc}, expected {k}")
    return idx, flags


def compact(hidden: np.ndarray, pos_ids: np.ndarray, grid: Sequence[int], frame_start: np.ndarray,
            kept_idx: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """hidden [batch, S, dim] (any dtype; rows copied as bytes), pos_ids int32 [3, batch, S],
    kept_idx int32 [batch, K] -> (hidden_c [batch, S_c, dim], pos_c [3, batch, S_c], src_idx [batch, S_c])."""
    h = np.ascontiguousarray(hidden)
    p = np.ascontiguousarray(pos_ids, dtype=np.int32)
    fs = np.ascontiguousarray(frame_start, dtype=np.int64)
    ki = np.ascontiguousarray(kept_idx, dtype=np.int32)
    batch, seq, dim = h.shape
    g = _grid(grid)
    nv = g.frames * g.height * g.width
    cap = seq - nv + ki.shape[1]
    hc = np.zeros((batch, cap, dim), dtype=h.dtype)
    pc = np.zeros((3, batch, cap), dtype=np.int32)
    si = np.zeros((batch, cap), dtype=np.int32)
    row_bytes = dim * h.dtype.itemsize
    rc = int(lib().oracle_compact(_ptr(h), row_bytes, _ptr(p), batch, seq, C.byref(g), _ptr(fs), _ptr(ki),
                                  ki.shape[1], cap, _ptr(hc), _ptr(pc), _ptr(si)))
    if rc != cap:
        raise RuntimeError(f"oracle_compact produced length {rc}, expected {cap}")
    return hc, pc, si


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, causal: bool, scale: Optional[float] = None,
              row_step: int = 1) -> np.ndarray:
    """q [batch, seq, H_q, d], k/v [batch, seq, H_kv, d] as fp32 views (strides honoured on the
    first three axes) -> float64 [batch, seq, H_q, d].  With row_step > 1 only rows
    i % row_step == 0 are filled (the rest stay NaN)."""
    for a in (q, k, v):
        assert a.dtype == np.float32 and a.ndim == 4 and a.strides[3] == 4
    batch, seq, hq, d = q.shape
    hkv = k.shape[2]
    assert v.shape == k.shape and k.shape[0] == batch and k.shape[1] == seq and hq % hkv == 0
    assert k.strides == v.strides
    qs = np.asarray([s // 4 for s in q.strides[:3]], dtype=np.int64)
    ks = np.asarray([s // 4 for s in k.strides[:3]], dtype=np.int64)
    out = np.full((batch, seq, hq, d), np.nan, dtype=np.float64)
    sc = (1.0 / np.sqrt(d)) if scale is None else float(scale)
    lib().oracle_attention(_ptr(q), _ptr(k), _ptr(v), _ptr(out), batch, seq, hq, hkv, d, _ptr(qs), _ptr(ks),
                           int(bool(causal)), sc, int(row_step))
    return out


def kv_write(k: np.ndarray, v: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, pos0: int = 0) -> int:
    """k/v [batch, seq, H_kv, d] (any dtype, strided on the first three axes) are copied into
    k_cache/v_cache [batch, H_kv, s_max, d] (C-contiguous, modified in place) at rows
    [pos0, pos0 + seq).  Returns the bytes written."""
    batch, seq, hkv, d = k.shape
    assert v.shape == k.shape and k.strides == v.strides and k.strides[3] == k.dtype.itemsize
    assert k_cache.flags.c_contiguous and v_cache.flags.c_contiguous
    assert k_cache.shape == v_cache.shape and k_cache.shape[0] == batch and k_cache.shape[1] == hkv
    assert k_cache.shape[3] == d and k_cache.dtype == k.dtype
    s_max = k_cache.shape[2]
    assert 0 <= pos0 and pos0 + seq <= s_max
    st = np.asarray(k.strides[:3], dtype=np.int64)
    return int(lib().oracle_kv_write(_ptr(k), _ptr(v), _ptr(st), _ptr(k_cache), _ptr(v_cache), batch, seq, hkv,
                                     d * k.dtype.itemsize, s_max, int(pos0)))


def decode_attention(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, n_ctx: int,
                     scale: Optional[float] = None) -> np.ndarray:
    """q [batch, H_q, d]; k_cache, v_cache [batch, H_kv, s_max, d] (fp32 widening of what the caches hold,
    C-contiguous); attends to cache rows [0, n_ctx) -> float64 [batch, H_q, d]."""
    q = np.ascontiguousarray(q, dtype=np.float32)
    kc = np.ascontiguousarray(k_cache, dtype=np.float32)
    vc = np.ascontiguousarray(v_cache, dtype=np.float32)
    batch, hq, d = q.shape
    assert kc.shape == vc.shape and kc.ndim == 4 and kc.shape[0] == batch and kc.shape[3] == d
    hkv, s_max = kc.shape[1], kc.shape[2]
    assert hq % hkv == 0 and 1 <= n_ctx <= s_max
    out = np.empty((batch, hq, d), dtype=np.float64)
    sc = (1.0 / np.sqrt(d)) if scale is None else float(scale)
    lib().oracle_decode_attention(_ptr(q), _ptr(kc), _ptr(vc), _ptr(out), batch, hq, hkv, d, s_max, int(n_ctx), sc)
    return out


def mrope_table(pos_ids: np.ndarray, axis_of_pair: np.ndarray, inv_freq: np.ndarray) -> np.ndarray:
    """pos_ids int32 [3, batch, seq]; axis_of_pair int32 [n_pairs] in {0,1,2}; inv_freq fp32 [n_pairs]
    -> float64 [batch, seq, n_pairs, 2] holding (cos, sin) of pos[axis[i]] * inv_freq[i]."""
    p = np.ascontiguousarray(pos_ids, dtype=np.int32)
    ax = np.ascontiguousarray(axis_of_pair, dtype=np.int32)
    fr = np.ascontiguousarray(inv_freq, dtype=np.float32)
    assert p.ndim == 3 and p.shape[0] == 3 and ax.shape == fr.shape and ax.ndim == 1
    assert ax.min() >= 0 and ax.max() <= 2
    _, batch, seq = p.shape
    out = np.empty((batch, seq, ax.shape[0], 2), dtype=np.float64)
    lib().oracle_mrope_table(_ptr(p), batch, seq, ax.shape[0], _ptr(ax), _ptr(fr), _ptr(out))
    return out


def mrope_apply(x: np.ndarray, cos_sin: np.ndarray) -> np.ndarray:
    """x fp32 view [batch, seq, heads, d] (strides honoured on the first three axes); cos_sin float64
    [batch, seq, d/2, 2] -> float64 [batch, seq, heads, d], pairs (i, i + d/2) rotated."""
    assert x.dtype == np.float32 and x.ndim == 4 and x.strides[3] == 4
    batch, seq, heads, d = x.shape
    cs = np.ascontiguousarray(cos_sin, dtype=np.float64)
    assert d % 2 == 0 and cs.shape == (batch, seq, d // 2, 2)
    st = np.asarray([s // 4 for s in x.strides[:3]], dtype=np.int64)
    out = np.empty((batch, seq, heads, d), dtype=np.float64)
    lib().oracle_mrope_apply(_ptr(x), _ptr(st), batch, seq, heads, d // 2, _ptr(cs), _ptr(out))
    return out


def anchor_aggregate(x0: np.ndarray, anchors: np.ndarray, inv_tau: float = 1.0, eps: float = 1e-6,
                     want_col_sum: bool = False):
    """Eq. 8: x0 fp32 [batch, T, D], anchors fp32 [M, D] -> z0 float64 [batch, M, D] (and, if asked, the total
    weight every dense token receives, float64 [batch, T])."""
    x = np.ascontiguousarray(x0, dtype=np.float32)
    a = np.ascontiguousarray(anchors, dtype=np.float32)
    batch, t, d = x.shape
    m = a.shape[0]
    assert a.shape == (m, d)
    z = np.empty((batch, m, d), dtype=np.float64)
    cs = np.empty((batch, t), dtype=np.float64) if want_col_sum else None
    lib().oracle_anchor_aggregate(_ptr(x), _ptr(a), batch, t, m, d, float(inv_tau), float(eps), _ptr(z),
                                  _ptr(cs) if cs is not None else None)
    return (z, cs) if want_col_sum else z


def kv_compress(x: np.ndarray, r: np.ndarray) -> np.ndarray:
    """Eq. 9: x fp32 [batch, M, width], r fp32 [M, S] -> Rbar^T x, float64 [batch, S, width] (Rbar = r with every
    column divided by its sum)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    r = np.ascontiguousarray(r, dtype=np.float32)
    batch, m, width = x.shape
    assert r.ndim == 2 and r.shape[0] == m
    out = np.empty((batch, r.shape[1], width), dtype=np.float64)
    lib().oracle_kv_compress(_ptr(x), _ptr(r), batch, m, r.shape[1], width, _ptr(out))
    return out


def cross_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: Optional[float] = None) -> np.ndarray:
    """q fp32 [batch, n_q, H_q, d]; k, v fp32 [batch, n_kv, H_kv, d]; no mask -> float64 [batch, n_q, H_q, d]."""
    q, k, v = (np.ascontiguousarray(a, dtype=np.float32) for a in (q, k, v))
    batch, n_q, hq, d = q.shape
    n_kv, hkv = k.shape[1], k.shape[2]
    assert k.shape == v.shape and k.shape[0] == batch and k.shape[3] == d and hq % hkv == 0
    out = np.empty((batch, n_q, hq, d), dtype=np.float64)
    sc = (1.0 / np.sqrt(d)) if scale is None else float(scale)
    lib().oracle_cross_attention(_ptr(q), _ptr(k), _ptr(v), _ptr(out), batch, n_q, n_kv, hq, hkv, d, sc)
    return out


def _check_offsets(row_offsets, total: int) -> np.ndarray:
    off = np.asarray(row_offsets, dtype=np.int64)
    assert off.ndim == 1 and off.size >= 1 and off[0] == 0 and off[-1] == total and np.all(np.diff(off) >= 1)
    return off


def kv_compress_ragged(x: np.ndarray, r: np.ndarray, row_offsets) -> np.ndarray:
    """Eq. 9 for items of different sizes (images of different grids) packed back to back: item b owns rows
    [row_offsets[b], row_offsets[b+1]) of x fp32 [total, width] and of its own assignment rows r fp32 [total, S];
    every item is compressed by itself -> float64 [batch, S, width]."""
    off = _check_offsets(row_offsets, x.shape[0])
    assert r.shape[0] == x.shape[0]
    return np.stack([kv_compress(x[None, a:b], r[a:b])[0] for a, b in zip(off[:-1], off[1:])])


def cross_attention_ragged(q: np.ndarray, k: np.ndarray, v: np.ndarray, row_offsets, scale: Optional[float] = None) -> np.ndarray:
    """q fp32 [total, H_q, d] packed as above; k, v fp32 [batch, n_kv, H_kv, d]: the queries of item b attend to the
    keys of item b only, no mask -> float64 [total, H_q, d]."""
    off = _check_offsets(row_offsets, q.shape[0])
    assert k.shape[0] == off.size - 1
    return np.concatenate([cross_attention(q[None, a:b], k[i:i + 1], v[i:i + 1], scale)[0]
                           for i, (a, b) in enumerate(zip(off[:-1], off[1:]))])


# ---------------------------------------------------------------------------------------------------------------
# The path for a batch whose samples differ in size and grid (images of different grid sizes in one batch): every
# sample's rows are packed back to back along the token axis, and every sample is scored, selected, merged, attended
# and cached by itself with the functions above (plain loops over the samples; the definitions are per sample).
def ragged_offsets(seq_lens: Sequence[int], grids: Sequence[Sequence[int]]):
    """Row offsets [batch + 1] of the packed tensors: (dense rows, visual tokens, kept tokens, compact rows) per sample,
    where a sample's compact length is its length minus its visual tokens plus K of its grid (Eq. 13)."""
    seq, vis, kept, comp = [0], [0], [0], [0]
    for s, g in zip(seq_lens, grids):
        nv = int(g[0]) * int(g[1]) * int(g[2])
        k = kept_count(g)
        assert s >= nv
        seq.append(seq[-1] + int(s)); vis.append(vis[-1] + nv); kept.append(kept[-1] + k); comp.append(comp[-1] + int(s) - nv + k)
    return tuple(np.asarray(x, dtype=np.int64) for x in (seq, vis, kept, comp))


def select_ragged(scores: np.ndarray, grids: Sequence[Sequence[int]]) -> np.ndarray:
    """scores fp32 [sum of N_v] packed sample by sample -> kept indices int32 [sum of K], each sample's own ascending
    visual-local indices."""
    out, at = [], 0
    for g in grids:
        nv = int(g[0]) * int(g[1]) * int(g[2])
        out.append(select(scores[None, at:at + nv], g)[0][0])
        at += nv
    assert at == scores.shape[0]
    return np.concatenate(out) if out else np.zeros(0, dtype=np.int32)


def compact_ragged(hidden: np.ndarray, pos_ids: np.ndarray, seq_lens: Sequence[int], grids: Sequence[Sequence[int]],
                   frame_starts: Sequence[np.ndarray], kept_idx: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """hidden [total, dim], pos_ids int32 [3, total], kept_idx int32 [sum of K] (sample-local), frame_starts one array
    of sample-local sequence indices per sample -> (hidden_c [sum of S_c, dim], pos_c [3, sum of S_c], src_idx
    [sum of S_c], sample-local dense indices)."""
    seq, _, kept, _ = ragged_offsets(seq_lens, grids)
    assert seq[-1] == hidden.shape[0] == pos_ids.shape[1] and kept[-1] == kept_idx.shape[0]
    hc, pc, si = [], [], []
    for b, g in enumerate(grids):
        a, e = seq[b], seq[b + 1]
        h1, p1, s1 = compact(hidden[None, a:e], pos_ids[:, None, a:e], g, frame_starts[b], kept_idx[None, kept[b]:kept[b + 1]])
        hc.append(h1[0]); pc.append(p1[:, 0]); si.append(s1[0])
    return np.concatenate(hc), np.concatenate(pc, axis=1), np.concatenate(si)


def attention_ragged(q: np.ndarray, k: np.ndarray, v: np.ndarray, row_offsets, causal: bool,
                     scale: Optional[float] = None) -> np.ndarray:
    """q fp32 [total, H_q, d], k, v fp32 [total, H_kv, d], sample b owning rows [row_offsets[b], row_offsets[b+1]):
    every sample attends to its own keys only, the causal mask counts from the sample's first row -> float64
    [total, H_q, d]."""
    off = _check_offsets(row_offsets, q.shape[0])
    assert k.shape[0] == q.shape[0] == v.shape[0]
    return np.concatenate([attention(np.ascontiguousarray(q[None, a:b]), np.ascontiguousarray(k[None, a:b]),
                                     np.ascontiguousarray(v[None, a:b]), causal, scale)[0]
                           for a, b in zip(off[:-1], off[1:])])


def kv_write_ragged(k: np.ndarray, v: np.ndarray, row_offsets, k_cache: np.ndarray, v_cache: np.ndarray, pos0: int = 0) -> int:
    """k, v [total, H_kv, d] packed as above: sample b's rows go to rows [pos0, pos0 + its length) of
    k_cache[b], v_cache[b] ([batch, H_kv, s_max, d], modified in place).  Returns the bytes written."""
    off = _check_offsets(row_offsets, k.shape[0])
    assert k_cache.shape[0] == off.size - 1
    return sum(kv_write(np.ascontiguousarray(k[None, a:b]), np.ascontiguousarray(v[None, a:b]), k_cache[i:i + 1], v_cache[i:i + 1], pos0)
               for i, (a, b) in enumerate(zip(off[:-1], off[1:])))


def decode_attention_ragged(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, n_ctx: Sequence[int],
                            scale: Optional[float] = None) -> np.ndarray:
    """The decode step over caches that hold a different number of rows per sample (what a ragged prefill leaves):
    q [batch, H_q, d]; sample b attends to rows [0, n_ctx[b]) of its own cache -> float64 [batch, H_q, d]."""
    assert len(n_ctx) == q.shape[0] == k_cache.shape[0]
    return np.concatenate([decode_attention(q[b:b + 1], k_cache[b:b + 1], v_cache[b:b + 1], int(n), scale) for b, n in enumerate(n_ctx)])
