"""Seeded synthetic inputs for the compact-prefill path (shapes of the Qwen3-VL workloads).

This module is the ONLY code shared by the HIP path's tests/bench and the CPU oracle's
tests.  It holds no arithmetic of the method: it draws random numbers, lays out text and
visual spans in a sequence, fills M-RoPE id triples, and converts fp32 draws to bf16 bit
patterns.  Anything the method computes (kept count, selection, compaction, attention) is
passed in by the caller or computed elsewhere.

The workloads stand in for the paper's Qwen3-VL-2B-Instruct single-image runs
(Experimental Setup, Table 1) and for the multi-image / video settings its Limitations
section names as future work: the path's cost depends on shapes and on the score
distribution only, so no dataset item and no trained weight is needed.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    """One synthetic configuration.  Pure shape data; `kept` is the tabulated keep count
    (max of budget and the sum of the floors) used only to size Q/K/V and outputs."""
    name: str
    index: int                 # seed = 1000 * index + trial
    batch: int
    frames: int
    height: int
    width: int
    cell_h: int
    cell_w: int
    cell_floor: int
    frame_floor: int
    budget: int
    text_len: int
    dim: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str                 # "fp32" | "bf16"
    causal: bool
    score_dist: str            # "normal" | "lognormal" | "uniform" | "normal_frame_offset"
    images: int                # number of separate visual spans (frames split evenly)
    kept: int                  # tabulated K for this grid (checked by tests on both sides)

    @property
    def n_visual(self) -> int:
        return self.frames * self.height * self.width

    @property
    def seq_len(self) -> int:
        return self.text_len + self.n_visual

    @property
    def seq_compact(self) -> int:
        return self.text_len + self.kept

    def grid_tuple(self) -> Tuple[int, ...]:
        return (self.frames, self.height, self.width, self.cell_h, self.cell_w,
                self.cell_floor, self.frame_floor, self.budget)


WORKLOADS: Dict[str, Workload] = {
    w.name: w for w in [
        Workload("tiny", 0, 1, 1, 16, 16, 4, 4, 2, 0, 85, 32, 256, 4, 2, 64,
                 "fp32", True, "normal", 1, 85),
        Workload("2b", 1, 1, 1, 32, 32, 4, 4, 1, 0, 341, 128, 2048, 16, 8, 128,
                 "bf16", True, "normal", 1, 341),
        Workload("8b", 2, 4, 2, 32, 32, 4, 4, 1, 0, 682, 256, 4096, 32, 8, 128,
                 "bf16", True, "lognormal", 2, 682),
        Workload("vit", 3, 2, 1, 64, 64, 8, 8, 1, 0, 1365, 0, 1152, 16, 16, 72,
                 "bf16", False, "uniform", 1, 1365),
        Workload("video", 4, 1, 16, 24, 24, 4, 4, 1, 16, 3072, 512, 4096, 32, 8, 128,
                 "bf16", True, "normal_frame_offset", 1, 3072),
    ]
}


def rng_for(w: Workload, trial: int, stream: int = 0) -> np.random.Generator:
    """Independent generator per (workload, trial, stream); stream separates tensors."""
    return np.random.Generator(np.random.PCG64([1000 * w.index + trial, stream]))


# ----------------------------------------------------------------------------- bf16 bits
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite input)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize(x: np.ndarray, dtype: str) -> Tuple[np.ndarray, np.ndarray]:
    """Returns (storage, widened): the array as the device stores it (fp32 values or bf16
    bit patterns as uint16) and the exact fp32 values those bits represent."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "fp32":
        return x, x
    if dtype == "bf16":
        bits = f32_to_bf16_bits(x)
        return bits, bf16_bits_to_f32(bits)
    raise ValueError(dtype)


# ----------------------------------------------------------------------- sequence layout
def frame_starts(w: Workload) -> np.ndarray:
    """Sequence index of the first token of every frame (int64, ascending).

    One span (image or video): floor(L/2) text tokens, the frames back to back, the rest
    of the text.  Two images: L/4 text, image 0, L/4 text, image 1, L/2 text.
    """
    hw = w.height * w.width
    if w.images == 1:
        lead = w.text_len // 2
        return np.asarray([lead + f * hw for f in range(w.frames)], dtype=np.int64)
    per = w.frames // w.images
    assert per * w.images == w.frames
    gap = w.text_len // (2 * w.images)
    starts: List[int] = []
    pos = 0
    for _ in range(w.images):
        pos += gap
        for f in range(per):
            starts.append(pos + f * hw)
        pos += per * hw
    return np.asarray(starts, dtype=np.int64)


def position_ids(w: Workload) -> np.ndarray:
    """M-RoPE id triples, int32 [3, batch, S]; axis 0 = (temporal, height, width).

    Text token: all three ids equal the running position p.  A run of adjacent frames
    starting at running position p0: frame k of the run, row r, column c gets
    (p0 + k, p0 + r, p0 + c); the running position after the run is p0 + max(run length,
    height, width).  Every batch item has the same layout.
    """
    hw = w.height * w.width
    starts = frame_starts(w)
    ids = np.zeros((3, w.seq_len), dtype=np.int32)
    t = 0
    p = 0
    f = 0
    rr, cc = np.divmod(np.arange(hw, dtype=np.int32), np.int32(w.width))
    while t < w.seq_len:
        if f < w.frames and t == starts[f]:
            run = 1
            while f + run < w.frames and starts[f + run] == starts[f] + run * hw:
                run += 1
            for k in range(run):
                sl = slice(t + k * hw, t + (k + 1) * hw)
                ids[0, sl] = p + k
                ids[1, sl] = p + rr
                ids[2, sl] = p + cc
            t += run * hw
            p += max(run, w.height, w.width)
            f += run
        else:
            ids[:, t] = p
            t += 1
            p += 1
    return np.ascontiguousarray(np.broadcast_to(ids[:, None, :], (3, w.batch, w.seq_len)))


# ------------------------------------------------------------------------------- tensors
def scores(w: Workload, trial: int) -> np.ndarray:
    """fp32 importance scores [batch, N_v] with the workload's distribution."""
    g = rng_for(w, trial, 1)
    shape = (w.batch, w.n_visual)
    if w.score_dist == "normal":
        s = g.standard_normal(shape, dtype=np.float32)
    elif w.score_dist == "lognormal":
        s = np.exp(g.standard_normal(shape, dtype=np.float32))
    elif w.score_dist == "uniform":
        s = g.random(shape, dtype=np.float32)
    elif w.score_dist == "normal_frame_offset":
        s = g.standard_normal(shape, dtype=np.float32)
        off = (0.5 * g.standard_normal((w.batch, w.frames), dtype=np.float32))
        s = s + np.repeat(off, w.height * w.width, axis=1)
    else:
        raise ValueError(w.score_dist)
    return np.ascontiguousarray(s, dtype=np.float32)


def hidden(w: Workload, trial: int) -> Tuple[np.ndarray, np.ndarray]:
    """Hidden rows [batch, S, dim] ~ N(0,1): (device storage, exact fp32 widening)."""
    g = rng_for(w, trial, 2)
    x = g.standard_normal((w.batch, w.seq_len, w.dim), dtype=np.float32)
    return quantize(x, w.dtype)


def anchor(w: Workload, trial: int) -> np.ndarray:
    """A raw (un-normalised) anchor vector [dim] ~ N(0,1) + 0.25, fp32."""
    g = rng_for(w, trial, 3)
    return (g.standard_normal(w.dim, dtype=np.float32) + np.float32(0.25)).astype(np.float32)


def qkv(w: Workload, trial: int, seq: int | None = None):
    """Q [batch, seq, H_q, d], K and V [batch, seq, H_kv, d] ~ N(0,1).  Returns three
    (storage, widened) pairs.  `seq` defaults to the tabulated compact length."""
    seq = w.seq_compact if seq is None else seq
    g = rng_for(w, trial, 4)
    q = g.standard_normal((w.batch, seq, w.n_q_heads, w.head_dim), dtype=np.float32)
    k = g.standard_normal((w.batch, seq, w.n_kv_heads, w.head_dim), dtype=np.float32)
    v = g.standard_normal((w.batch, seq, w.n_kv_heads, w.head_dim), dtype=np.float32)
    return quantize(q, w.dtype), quantize(k, w.dtype), quantize(v, w.dtype)


def small_grid_cases() -> List[Tuple[int, ...]]:
    """Grid tuples (frames, H, W, cell_h, cell_w, cell_floor, frame_floor, budget) that span
    the degenerate cases of the selection: ragged cells, floors above the budget, zero and
    full budgets, one cell, several frames."""
    return [
        (1, 4, 4, 2, 2, 1, 0, 5),
        (1, 4, 4, 2, 2, 1, 0, 0),
        (1, 4, 4, 2, 2, 0, 0, 0),
        (1, 4, 4, 2, 2, 2, 0, 3),      # floors (8) above budget (3)
        (1, 4, 4, 4, 4, 3, 0, 16),     # one cell, keep everything
        (1, 5, 7, 2, 3, 1, 0, 11),     # ragged edge cells
        (1, 5, 7, 2, 3, 9, 0, 4),      # floor larger than any cell
        (2, 3, 5, 2, 2, 1, 2, 9),      # frame floor on top of cell floors
        (3, 4, 6, 4, 3, 1, 3, 20),
        (3, 4, 6, 4, 3, 0, 5, 7),      # frame floor only; sum of floors above budget
        (4, 9, 9, 3, 3, 1, 4, 81),
        (1, 1, 1, 1, 1, 1, 1, 1),
        (1, 1, 64, 1, 8, 2, 0, 21),
        (2, 33, 17, 5, 4, 2, 7, 400),
        (1, 70, 70, 7, 7, 1, 0, 1633), # spans several 1024-token tiles with a ragged tail
        (5, 31, 29, 4, 4, 1, 16, 1498),
        (1, 24, 24, 24, 24, 40, 0, 100),  # one cell per frame larger than a wavefront
        (2, 48, 48, 16, 16, 70, 100, 1536),
    ]
