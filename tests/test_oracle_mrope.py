"""Pins for the oracle's three-axis rotary position embedding (driven by the position ids the compact merge carries:
sentence after Eq. 14).  The paper prints no rotary formula, so the pins are the mathematics of a rotation: the
complex-multiplication form, norm preservation, additivity in the position, and the relative-position property of
the attention logit that is the reason rotary embeddings exist.  No HIP code is involved."""
import numpy as np
import pytest

import oracle
from paper_2605_28115_amd import workloads as wl


def tables(d, theta=10000.0, sections=None, interleaved=False):
    n = d // 2
    inv = (theta ** (-np.arange(n, dtype=np.float64) * 2.0 / d)).astype(np.float32)
    if sections is None:
        sections = (n // 4, (n - n // 4) // 2, n - n // 4 - (n - n // 4) // 2)
    if interleaved:
        axis = (np.arange(n) % 3).astype(np.int32)
    else:
        axis = np.repeat(np.arange(3), sections).astype(np.int32)
    assert axis.shape[0] == n
    return axis, inv


def test_zero_ids_are_the_identity_and_norms_are_kept():
    rng = np.random.default_rng(0)
    b, s, h, d = 2, 9, 3, 16
    x = rng.standard_normal((b, s, h, d)).astype(np.float32)
    axis, inv = tables(d)
    cs = oracle.mrope_table(np.zeros((3, b, s), dtype=np.int32), axis, inv)
    assert np.array_equal(cs[..., 0], np.ones_like(cs[..., 0])) and np.array_equal(cs[..., 1], np.zeros_like(cs[..., 1]))
    assert np.array_equal(oracle.mrope_apply(x, cs), x.astype(np.float64))
    pos = rng.integers(0, 5000, (3, b, s)).astype(np.int32)
    y = oracle.mrope_apply(x, oracle.mrope_table(pos, axis, inv))
    n = d // 2
    # every pair keeps its length, hence every row its norm
    assert np.abs(y[..., :n] ** 2 + y[..., n:] ** 2 - (x[..., :n].astype(np.float64) ** 2 + x[..., n:].astype(np.float64) ** 2)).max() < 1e-12


def test_equals_complex_multiplication():
    """Pair i as the complex number x[i] + 1j * x[i + d/2], multiplied by exp(1j * pos[axis_i] * inv_freq_i)."""
    rng = np.random.default_rng(1)
    b, s, h, d = 1, 20, 2, 32
    x = rng.standard_normal((b, s, h, d)).astype(np.float32)
    pos = rng.integers(0, 3000, (3, b, s)).astype(np.int32)
    for inter in (False, True):
        axis, inv = tables(d, interleaved=inter)
        y = oracle.mrope_apply(x, oracle.mrope_table(pos, axis, inv))
        n = d // 2
        z = x[..., :n].astype(np.float64) + 1j * x[..., n:].astype(np.float64)
        ang = pos[axis].astype(np.float64).transpose(1, 2, 0) * inv.astype(np.float64)          # [b, s, n]
        w = z * np.exp(1j * ang)[:, :, None, :]
        assert np.abs(y[..., :n] - w.real).max() < 1e-12 and np.abs(y[..., n:] - w.imag).max() < 1e-12


def test_text_tokens_reduce_to_one_axis_and_rotations_add():
    rng = np.random.default_rng(2)
    b, s, h, d = 1, 12, 2, 24
    x = rng.standard_normal((b, s, h, d)).astype(np.float32)
    p = rng.integers(0, 900, (b, s)).astype(np.int32)
    pos = np.stack([p, p, p])                               # text: the three ids are equal
    axis, inv = tables(d)
    y = oracle.mrope_apply(x, oracle.mrope_table(pos, axis, inv))
    for other in (np.zeros(d // 2, dtype=np.int32), np.full(d // 2, 2, dtype=np.int32), tables(d, interleaved=True)[0]):
        assert np.array_equal(y, oracle.mrope_apply(x, oracle.mrope_table(pos, other, inv)))
    # rotating by ids a and then by ids b is rotating by a + b (angles add); checked with frequencies 2^-k, for which
    # the fp32 products are exact
    inv2 = (2.0 ** -np.arange(d // 2)).astype(np.float32)
    pa = rng.integers(0, 400, (3, b, s)).astype(np.int32)
    pb = rng.integers(0, 400, (3, b, s)).astype(np.int32)
    ya = oracle.mrope_apply(x, oracle.mrope_table(pa, axis, inv2))
    yab = oracle.mrope_apply(ya.astype(np.float32), oracle.mrope_table(pb, axis, inv2))
    direct = oracle.mrope_apply(x, oracle.mrope_table(pa + pb, axis, inv2))
    assert np.abs(yab - direct).max() < 1e-5               # (ya passes through fp32 between the two rotations)


def test_logits_depend_on_relative_position_only():
    """<rope(q, m), rope(k, n)> is a function of m - n per axis: shifting every id of queries and keys by the same
    offsets leaves all attention logits unchanged."""
    rng = np.random.default_rng(3)
    b, s, h, d = 1, 15, 2, 32
    q = rng.standard_normal((b, s, h, d)).astype(np.float32)
    k = rng.standard_normal((b, s, h, d)).astype(np.float32)
    inv = (2.0 ** -np.arange(d // 2)).astype(np.float32)    # exact products
    axis = tables(d)[0]
    pos = rng.integers(0, 300, (3, b, s)).astype(np.int32)
    shift = np.asarray([17, 400, 3], dtype=np.int32)[:, None, None]
    def logits(p):
        cs = oracle.mrope_table(p, axis, inv)
        rq, rk = oracle.mrope_apply(q, cs), oracle.mrope_apply(k, cs)
        return np.einsum("bihd,bjhd->bhij", rq, rk)
    assert np.abs(logits(pos) - logits(pos + shift)).max() < 1e-9
    # and a shift of the keys alone does change them
    cs, cs2 = oracle.mrope_table(pos, axis, inv), oracle.mrope_table(pos + shift, axis, inv)
    moved = np.einsum("bihd,bjhd->bhij", oracle.mrope_apply(q, cs), oracle.mrope_apply(k, cs2))
    assert np.abs(moved - logits(pos)).max() > 1e-3


def test_strided_rows_and_workload_ids():
    w = wl.WORKLOADS["tiny"]
    pos = wl.position_ids(w)
    axis, inv = tables(w.head_dim)
    cs = oracle.mrope_table(pos, axis, inv)
    assert cs.shape == (w.batch, w.seq_len, w.head_dim // 2, 2)
    rng = np.random.default_rng(4)
    wide = rng.standard_normal((w.batch, w.seq_len, 3, w.head_dim + 8)).astype(np.float32)
    view = wide[..., :w.head_dim]                          # rows embedded in wider rows
    assert np.array_equal(oracle.mrope_apply(view, cs), oracle.mrope_apply(np.ascontiguousarray(view), cs))
    # a visual token's three ids differ: its height pairs turn by its row id, not by its temporal id
    t = int(wl.frame_starts(w)[0]) + 5 * w.width + 3
    assert pos[1, 0, t] != pos[2, 0, t]
    i_h = int(np.nonzero(axis == 1)[0][0])
    ang = float(pos[1, 0, t]) * float(inv[i_h])
    assert abs(cs[0, t, i_h, 0] - np.cos(ang)) < 1e-12 and abs(cs[0, t, i_h, 1] - np.sin(ang)) < 1e-12
