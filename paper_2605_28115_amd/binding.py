"""Thin ctypes binding of libcivic.so (include/civic.h): argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI; PyTorch is used for device
memory and the current stream, nothing else.  There is no CPU fallback: if the library is not
built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcivic.so")

CIVIC_OK, ERR_INVALID_ARG, ERR_WORKSPACE, ERR_UNSUPPORTED, ERR_HIP = 0, -1, -2, -3, -4
CIVIC_F32, CIVIC_BF16 = 0, 1
MAX_VISUAL_TOKENS, MAX_FRAMES, MAX_SCORE_DIM, MAX_HEAD_DIM = 32768, 128, 8192, 256

EXPORTS = ("civic_last_hip_error", "civic_time_next_kernel", "civic_kept_count", "civic_select_workspace_bytes",
           "civic_compact_workspace_bytes", "civic_anchor_normalize", "civic_score", "civic_score_visual", "civic_select",
           "civic_compact", "civic_compact_prefill", "civic_prefill_attn", "civic_kv_write", "civic_prefill_attn_kv",
           "civic_decode_attn_workspace_bytes", "civic_decode_attn", "civic_decode_attn_noalloc",
           "civic_mrope_table", "civic_mrope_apply", "civic_kv_write_rope", "civic_prefill_attn_rope",
           "civic_anchor_aggregate_workspace_bytes", "civic_anchor_aggregate", "civic_kv_compress_workspace_bytes",
           "civic_kv_compress", "civic_cross_attn", "civic_kv_compress_ragged_workspace_bytes",
           "civic_kv_compress_ragged", "civic_cross_attn_ragged", "civic_ragged_offsets", "civic_compact_prefill_ragged",
           "civic_prefill_attn_ragged", "civic_decode_attn_ragged_workspace_bytes", "civic_decode_attn_ragged")


class CivicError(RuntimeError):
    def __init__(self, call: str, code: int, hip: int = 0):
        names = {ERR_INVALID_ARG: "CIVIC_ERR_INVALID_ARG", ERR_WORKSPACE: "CIVIC_ERR_WORKSPACE",
                 ERR_UNSUPPORTED: "CIVIC_ERR_UNSUPPORTED", ERR_HIP: "CIVIC_ERR_HIP"}
        super().__init__(f"{call} failed: {names.get(code, code)}" + (f" (hipError {hip})" if code == ERR_HIP else ""))
        self.code = code


class Grid(C.Structure):
    """Mirror of civic_grid."""
    _fields_ = [(n, C.c_int32) for n in ("frames", "height", "width", "cell_h", "cell_w",
                                         "cell_floor", "frame_floor", "budget")]

    @property
    def n_visual(self) -> int:
        return self.frames * self.height * self.width


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2605_28115_amd.build` (no CPU fallback exists)")

lib = C.CDLL(LIB_PATH)
_P = C.c_void_p
lib.civic_last_hip_error.restype = C.c_int
lib.civic_time_next_kernel.restype = C.c_int
lib.civic_time_next_kernel.argtypes = [_P, _P]
lib.civic_ragged_offsets.restype = C.c_int
lib.civic_ragged_offsets.argtypes = [C.c_int32, _P, C.POINTER(Grid), _P, _P, _P]
lib.civic_compact_prefill_ragged.restype = C.c_int
lib.civic_compact_prefill_ragged.argtypes = [_P, C.c_int, C.c_int32, _P, C.c_int32, _P, C.POINTER(Grid), _P, _P, C.c_float, _P, _P, _P, _P, _P, _P]
lib.civic_prefill_attn_ragged.restype = C.c_int
lib.civic_prefill_attn_ragged.argtypes = [_P, _P, _P, _P, C.c_int, C.c_int32, _P, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int64),
                                          C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.c_int32, C.c_float, _P, _P, C.c_int64, C.c_int64, _P]
lib.civic_decode_attn_ragged_workspace_bytes.restype = C.c_size_t
lib.civic_decode_attn_ragged_workspace_bytes.argtypes = [C.c_int, C.c_int32, _P, C.c_int32, C.c_int32, C.c_int32]
lib.civic_decode_attn_ragged.restype = C.c_int
lib.civic_decode_attn_ragged.argtypes = [_P, _P, _P, _P, C.c_int, C.c_int32, _P, C.c_int32, C.c_int32, C.c_int32, C.c_int64, C.c_float, _P,
                                         C.c_size_t, _P]
lib.civic_kept_count.restype = C.c_int64
lib.civic_kept_count.argtypes = [C.POINTER(Grid)]
lib.civic_select_workspace_bytes.restype = C.c_size_t
lib.civic_select_workspace_bytes.argtypes = [C.POINTER(Grid), C.c_int32]
lib.civic_compact_workspace_bytes.restype = C.c_size_t
lib.civic_compact_workspace_bytes.argtypes = [C.c_int32, C.c_int64]
lib.civic_anchor_normalize.restype = C.c_int
lib.civic_anchor_normalize.argtypes = [_P, C.c_int32, _P]
lib.civic_score.restype = C.c_int
lib.civic_score.argtypes = [_P, C.c_int, C.c_int64, C.c_int64, C.c_int32, _P, C.c_float, _P, _P]
lib.civic_score_visual.restype = C.c_int
lib.civic_score_visual.argtypes = [_P, C.c_int, C.c_int32, C.c_int64, C.c_int32, C.POINTER(Grid), _P, _P, C.c_float, _P, _P]
lib.civic_select.restype = C.c_int
lib.civic_select.argtypes = [_P, C.c_int32, C.POINTER(Grid), _P, _P, _P, C.c_size_t, _P]
lib.civic_compact.restype = C.c_int
lib.civic_compact.argtypes = [_P, C.c_int, C.c_int32, _P, C.c_int32, C.c_int64, C.POINTER(Grid), _P, _P, C.c_int64,
                              _P, _P, _P, _P, C.c_size_t, _P]
lib.civic_compact_prefill.restype = C.c_int
lib.civic_compact_prefill.argtypes = [_P, C.c_int, C.c_int32, C.c_int64, C.c_int32, _P, C.POINTER(Grid), _P, _P, C.c_float,
                                      _P, _P, _P, _P, _P, _P, C.c_size_t, _P]
lib.civic_prefill_attn.restype = C.c_int
lib.civic_prefill_attn.argtypes = [_P, _P, _P, _P, C.c_int, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                   _P, _P, _P, C.c_int32, C.c_float, _P]
lib.civic_kv_write.restype = C.c_int
lib.civic_kv_write.argtypes = [_P, _P, _P, C.c_int, _P, _P, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int64,
                               C.c_int64, _P]
lib.civic_prefill_attn_kv.restype = C.c_int
lib.civic_prefill_attn_kv.argtypes = [_P, _P, _P, _P, _P, _P, C.c_int, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                      _P, _P, _P, C.c_int64, C.c_int64, C.c_int32, C.c_float, _P]


lib.civic_decode_attn_workspace_bytes.restype = C.c_size_t
lib.civic_decode_attn_workspace_bytes.argtypes = [C.c_int, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int64]
lib.civic_decode_attn.restype = C.c_int
lib.civic_decode_attn.argtypes = [_P, _P, _P, _P, C.c_int, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int64, C.c_int64,
                                  C.c_float, _P, C.c_size_t, _P]
lib.civic_decode_attn_noalloc.restype = C.c_int
lib.civic_decode_attn_noalloc.argtypes = [_P, _P, _P, _P, C.c_int, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int64, C.c_int64,
                                          C.c_float, _P]
DECODE_NOALLOC_MAX_BYTES = 4 << 20
lib.civic_anchor_aggregate_workspace_bytes.restype = C.c_size_t
lib.civic_anchor_aggregate_workspace_bytes.argtypes = [C.c_int32] * 4
lib.civic_anchor_aggregate.restype = C.c_int
lib.civic_anchor_aggregate.argtypes = [_P, _P, C.c_int, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_float, _P, _P, _P,
                                       C.c_size_t, _P]
lib.civic_kv_compress_workspace_bytes.restype = C.c_size_t
lib.civic_kv_compress_workspace_bytes.argtypes = [C.c_int32] * 4
lib.civic_kv_compress.restype = C.c_int
lib.civic_kv_compress.argtypes = [_P, _P, C.c_int, _P, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _P, _P, _P, C.c_size_t, _P]
lib.civic_cross_attn.restype = C.c_int
lib.civic_cross_attn.argtypes = [_P, _P, _P, _P, C.c_int, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                 _P, _P, _P, C.c_float, _P]
lib.civic_kv_compress_ragged_workspace_bytes.restype = C.c_size_t
lib.civic_kv_compress_ragged_workspace_bytes.argtypes = [C.c_int32, _P, C.c_int32, C.c_int32]
lib.civic_kv_compress_ragged.restype = C.c_int
lib.civic_kv_compress_ragged.argtypes = [_P, _P, C.c_int, _P, C.c_int32, _P, C.c_int32, C.c_int32, _P, _P, _P, C.c_size_t, _P]
lib.civic_cross_attn_ragged.restype = C.c_int
lib.civic_cross_attn_ragged.argtypes = [_P, _P, _P, _P, C.c_int, C.c_int32, _P, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _P, _P, _P,
                                        C.c_float, _P]
lib.civic_mrope_table.restype = C.c_int
lib.civic_mrope_table.argtypes = [_P, C.c_int32, C.c_int64, C.c_int32, _P, _P, _P, _P]
lib.civic_mrope_apply.restype = C.c_int
lib.civic_mrope_apply.argtypes = [_P, _P, C.c_int, C.c_int32, C.c_int64, C.c_int32, C.c_int32, _P, _P, _P, _P]
lib.civic_kv_write_rope.restype = C.c_int
lib.civic_kv_write_rope.argtypes = [_P, _P, _P, C.c_int, _P, _P, _P, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int64,
                                    C.c_int64, _P]
lib.civic_prefill_attn_rope.restype = C.c_int
lib.civic_prefill_attn_rope.argtypes = [_P, _P, _P, _P, C.c_int, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                        _P, _P, _P, C.c_int32, C.c_float, _P, _P]


def _check(call: str, rc: int) -> None:
    if rc != CIVIC_OK:
        raise CivicError(call, rc, lib.civic_last_hip_error() if rc == ERR_HIP else 0)


def make_grid(grid) -> Grid:
    return grid if isinstance(grid, Grid) else Grid(*[int(x) for x in grid])


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return CIVIC_F32
    if t.dtype == torch.bfloat16:
        return CIVIC_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _dev(t: Optional[torch.Tensor]) -> C.c_void_p:
    if t is None:
        return C.c_void_p(0)
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    return C.c_void_p(t.data_ptr())


def _strides3(t: torch.Tensor):
    if t.dim() != 4 or t.stride(3) != 1:
        raise ValueError("expected [batch, seq, heads, head_dim] with contiguous head_dim")
    return (C.c_int64 * 3)(t.stride(0), t.stride(1), t.stride(2))


# ------------------------------------------------------------------------------ host functions
def civic_time_next_kernel(start: Optional[torch.cuda.Event], stop: Optional[torch.cuda.Event]) -> None:
    """Arms the one-shot kernel timer with two timing events that have been recorded at least once (torch creates an
    event's handle at its first record), or disarms it with (None, None)."""
    handle = lambda ev: None if ev is None else C.c_void_p(ev.cuda_event)
    _check("civic_time_next_kernel", lib.civic_time_next_kernel(handle(start), handle(stop)))


def civic_kept_count(grid) -> int:
    k = int(lib.civic_kept_count(C.byref(make_grid(grid))))
    if k < 0:
        raise CivicError("civic_kept_count", k)
    return k


def civic_select_workspace_bytes(grid, batch: int) -> int:
    return int(lib.civic_select_workspace_bytes(C.byref(make_grid(grid)), batch))


def civic_compact_workspace_bytes(batch: int, seq_len: int) -> int:
    return int(lib.civic_compact_workspace_bytes(batch, seq_len))


def civic_anchor_normalize(anchor: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(anchor, dtype=np.float32)
    q = np.empty_like(a)
    _check("civic_anchor_normalize", lib.civic_anchor_normalize(C.c_void_p(a.ctypes.data), a.shape[0], C.c_void_p(q.ctypes.data)))
    return q


# ---------------------------------------------------------------------------- device functions
def civic_score(hidden: torch.Tensor, anchor_q: torch.Tensor, inv_tau: float = 1.0,
                scores: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """hidden [..., dim] with contiguous last axis and one uniform row stride -> fp32 scores [...]."""
    dim = hidden.shape[-1]
    rows = hidden.reshape(-1, dim) if hidden.is_contiguous() else hidden
    if rows.dim() != 2 or rows.stride(1) != 1:
        raise ValueError("hidden must be viewable as [n_rows, dim] rows")
    if scores is None:
        scores = torch.empty(hidden.shape[:-1], dtype=torch.float32, device=hidden.device)
    _check("civic_score", lib.civic_score(_dev(rows), _dtype_code(rows), rows.shape[0], rows.stride(0), dim,
                                          _dev(anchor_q), float(inv_tau), _dev(scores), _stream(stream)))
    return scores


def civic_score_visual(hidden: torch.Tensor, grid, frame_start: Sequence[int], anchor_q: torch.Tensor, inv_tau: float = 1.0,
                       scores: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """hidden [batch, S, dim] contiguous; the frames' rows are scored where they lie -> fp32 scores [batch, N_v]."""
    g = make_grid(grid)
    if hidden.dim() != 3 or not hidden.is_contiguous():
        raise ValueError("hidden must be contiguous [batch, S, dim]")
    batch, seq_len, dim = hidden.shape
    fs = np.ascontiguousarray(np.asarray(frame_start, dtype=np.int64))
    if fs.shape != (g.frames,):
        raise ValueError("frame_start must have one entry per frame")
    if scores is None:
        scores = torch.empty((batch, g.n_visual), dtype=torch.float32, device=hidden.device)
    _check("civic_score_visual", lib.civic_score_visual(_dev(hidden), _dtype_code(hidden), batch, seq_len, dim, C.byref(g),
                                                        C.c_void_p(fs.ctypes.data), _dev(anchor_q), float(inv_tau),
                                                        _dev(scores), _stream(stream)))
    return scores


def civic_select(scores: torch.Tensor, grid, kept_idx: Optional[torch.Tensor] = None,
                 keep_flags: Optional[torch.Tensor] = None, want_flags: bool = False,
                 workspace: Optional[torch.Tensor] = None, stream=None) -> Tuple[torch.Tensor, Optional[torch.Tensor]]:
    g = make_grid(grid)
    if scores.dim() != 2 or scores.shape[1] != g.n_visual or not scores.is_contiguous() or scores.dtype != torch.float32:
        raise ValueError("scores must be contiguous fp32 [batch, N_v]")
    batch = scores.shape[0]
    k = civic_kept_count(g)
    if kept_idx is None:
        kept_idx = torch.empty((batch, k), dtype=torch.int32, device=scores.device)
    if keep_flags is None and want_flags:
        keep_flags = torch.empty((batch, g.n_visual), dtype=torch.uint8, device=scores.device)
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check("civic_select", lib.civic_select(_dev(scores), batch, C.byref(g), _dev(kept_idx), _dev(keep_flags),
                                            _dev(workspace), ws_bytes, _stream(stream)))
    return kept_idx, keep_flags


def civic_compact(hidden: torch.Tensor, pos_ids: torch.Tensor, grid, frame_start: Sequence[int],
                  kept_idx: torch.Tensor, hidden_c: Optional[torch.Tensor] = None,
                  pos_c: Optional[torch.Tensor] = None, src_idx: Optional[torch.Tensor] = None,
                  workspace: Optional[torch.Tensor] = None, stream=None):
    g = make_grid(grid)
    if hidden.dim() != 3 or not hidden.is_contiguous() or not pos_ids.is_contiguous() or not kept_idx.is_contiguous():
        raise ValueError("hidden [batch, S, dim], pos_ids [3, batch, S] and kept_idx [batch, K] must be contiguous")
    batch, seq_len, dim = hidden.shape
    if tuple(pos_ids.shape) != (3, batch, seq_len) or pos_ids.dtype != torch.int32 or kept_idx.dtype != torch.int32:
        raise ValueError("pos_ids must be int32 [3, batch, S] and kept_idx int32")
    n_kept = kept_idx.shape[1]
    seq_c = seq_len - g.n_visual + n_kept
    fs = np.ascontiguousarray(np.asarray(frame_start, dtype=np.int64))
    if fs.shape != (g.frames,):
        raise ValueError("frame_start must have one entry per frame")
    if hidden_c is None:
        hidden_c = torch.empty((batch, seq_c, dim), dtype=hidden.dtype, device=hidden.device)
    if pos_c is None:
        pos_c = torch.empty((3, batch, seq_c), dtype=torch.int32, device=hidden.device)
    if src_idx is None:
        src_idx = torch.empty((batch, seq_c), dtype=torch.int32, device=hidden.device)
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check("civic_compact", lib.civic_compact(_dev(hidden), _dtype_code(hidden), dim, _dev(pos_ids), batch, seq_len,
                                              C.byref(g), C.c_void_p(fs.ctypes.data), _dev(kept_idx), n_kept,
                                              _dev(hidden_c), _dev(pos_c), _dev(src_idx), _dev(workspace), ws_bytes,
                                              _stream(stream)))
    return hidden_c, pos_c, src_idx


def civic_compact_prefill(hidden: torch.Tensor, pos_ids: torch.Tensor, grid, frame_start: Sequence[int],
                          anchor_q: torch.Tensor, inv_tau: float = 1.0, scores: Optional[torch.Tensor] = None,
                          kept_idx: Optional[torch.Tensor] = None, hidden_c: Optional[torch.Tensor] = None,
                          pos_c: Optional[torch.Tensor] = None, src_idx: Optional[torch.Tensor] = None, stream=None):
    """Scores, selection and compact merge in one library call -> (scores, kept_idx, hidden_c, pos_c, src_idx)."""
    g = make_grid(grid)
    if hidden.dim() != 3 or not hidden.is_contiguous() or not pos_ids.is_contiguous():
        raise ValueError("hidden [batch, S, dim] and pos_ids [3, batch, S] must be contiguous")
    batch, seq_len, dim = hidden.shape
    if tuple(pos_ids.shape) != (3, batch, seq_len) or pos_ids.dtype != torch.int32:
        raise ValueError("pos_ids must be int32 [3, batch, S]")
    n_kept = civic_kept_count(grid)
    seq_c = seq_len - g.n_visual + n_kept
    fs = np.ascontiguousarray(np.asarray(frame_start, dtype=np.int64))
    if fs.shape != (g.frames,):
        raise ValueError("frame_start must have one entry per frame")
    dev = hidden.device
    if scores is None:
        scores = torch.empty((batch, g.n_visual), dtype=torch.float32, device=dev)
    if kept_idx is None:
        kept_idx = torch.empty((batch, n_kept), dtype=torch.int32, device=dev)
    if hidden_c is None:
        hidden_c = torch.empty((batch, seq_c, dim), dtype=hidden.dtype, device=dev)
    if pos_c is None:
        pos_c = torch.empty((3, batch, seq_c), dtype=torch.int32, device=dev)
    if src_idx is None:
        src_idx = torch.empty((batch, seq_c), dtype=torch.int32, device=dev)
    _check("civic_compact_prefill", lib.civic_compact_prefill(
        _dev(hidden), _dtype_code(hidden), batch, seq_len, dim, _dev(pos_ids), C.byref(g), C.c_void_p(fs.ctypes.data),
        _dev(anchor_q), float(inv_tau), _dev(scores), _dev(kept_idx), _dev(hidden_c), _dev(pos_c), _dev(src_idx),
        None, 0, _stream(stream)))
    return scores, kept_idx, hidden_c, pos_c, src_idx


def civic_ragged_offsets(seq_lens: Sequence[int], grids):
    """Row offsets of the packed tensors of a ragged batch -> (seq, visual, kept, compact), int64 [batch + 1] each."""
    gs = (Grid * len(grids))(*[make_grid(g) for g in grids])
    seq = np.concatenate([[0], np.cumsum(np.asarray(seq_lens, dtype=np.int64))]).astype(np.int64)
    vis, kept, comp = (np.zeros(len(grids) + 1, dtype=np.int64) for _ in range(3))
    _check("civic_ragged_offsets", lib.civic_ragged_offsets(len(grids), C.c_void_p(seq.ctypes.data), gs, C.c_void_p(vis.ctypes.data),
                                                            C.c_void_p(kept.ctypes.data), C.c_void_p(comp.ctypes.data)))
    return seq, vis, kept, comp


def civic_compact_prefill_ragged(hidden: torch.Tensor, pos_ids: torch.Tensor, seq_lens: Sequence[int], grids,
                                 frame_starts: Sequence[Sequence[int]], anchor_q: torch.Tensor, inv_tau: float = 1.0, stream=None):
    """Samples of different length and grid packed along the token axis: hidden [total, dim], pos_ids int32 [3, total],
    one grid and one list of (sample-local) frame starts per sample -> (scores, kept_idx, hidden_c, pos_c, src_idx), packed."""
    if hidden.dim() != 2 or not hidden.is_contiguous() or not pos_ids.is_contiguous() or pos_ids.dtype != torch.int32:
        raise ValueError("hidden [total, dim] and pos_ids int32 [3, total] must be contiguous")
    seq, vis, kept, comp = civic_ragged_offsets(seq_lens, grids)
    total, dim = hidden.shape
    if seq[-1] != total or tuple(pos_ids.shape) != (3, total) or len(frame_starts) != len(grids):
        raise ValueError("the samples' lengths must add up to the packed rows, with one frame-start list per sample")
    gs = (Grid * len(grids))(*[make_grid(g) for g in grids])
    for g, f in zip(gs, frame_starts):
        if len(f) != g.frames:
            raise ValueError("frame_starts must have one entry per frame of its sample")
    fs = np.ascontiguousarray(np.concatenate([np.asarray(f, dtype=np.int64) for f in frame_starts]) if len(grids) else np.zeros(0, np.int64))
    dev = hidden.device
    scores = torch.empty(int(vis[-1]), dtype=torch.float32, device=dev)
    kept_idx = torch.empty(int(kept[-1]), dtype=torch.int32, device=dev)
    hidden_c = torch.empty((int(comp[-1]), dim), dtype=hidden.dtype, device=dev)
    pos_c = torch.empty((3, int(comp[-1])), dtype=torch.int32, device=dev)
    src_idx = torch.empty(int(comp[-1]), dtype=torch.int32, device=dev)
    _check("civic_compact_prefill_ragged", lib.civic_compact_prefill_ragged(
        _dev(hidden), _dtype_code(hidden), len(grids), C.c_void_p(seq.ctypes.data), dim, _dev(pos_ids), gs, C.c_void_p(fs.ctypes.data),
        _dev(anchor_q), float(inv_tau), _dev(scores), _dev(kept_idx), _dev(hidden_c), _dev(pos_c), _dev(src_idx), _stream(stream)))
    return scores, kept_idx, hidden_c, pos_c, src_idx


def civic_prefill_attn_ragged(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, row_offsets: Sequence[int], causal: bool = True,
                              softmax_scale: float = 0.0, k_cache: Optional[torch.Tensor] = None,
                              v_cache: Optional[torch.Tensor] = None, pos0: int = 0, out: Optional[torch.Tensor] = None,
                              stream=None) -> torch.Tensor:
    """q [total, H_q, d], k and v [total, H_kv, d] packed (sample b owning rows [row_offsets[b], row_offsets[b+1])); with
    caches [batch, H_kv, s_max, d] every sample's K and V rows are written to its own cache rows from pos0."""
    if k.shape != v.shape or k.stride() != v.stride() or q.dtype != k.dtype or q.dim() != 3 or k.dim() != 3 or q.stride(2) != 1 or k.stride(2) != 1:
        raise ValueError("q [total, H_q, d]; k and v [total, H_kv, d] of one shape, strides and dtype")
    off = np.ascontiguousarray(np.asarray(row_offsets, dtype=np.int64))
    batch = off.size - 1
    total, hq, d = q.shape
    if out is None:
        out = torch.empty((total, hq, d), dtype=q.dtype, device=q.device)
    s_max = 0
    if k_cache is not None:
        if v_cache is None or k_cache.shape != v_cache.shape or not k_cache.is_contiguous() or not v_cache.is_contiguous() or \
                tuple(k_cache.shape[:2]) != (batch, k.shape[1]) or k_cache.shape[3] != d:
            raise ValueError("k_cache and v_cache must be contiguous [batch, H_kv, s_max, d]")
        s_max = k_cache.shape[2]
    qs = (C.c_int64 * 3)(0, q.stride(0), q.stride(1))
    ks = (C.c_int64 * 3)(0, k.stride(0), k.stride(1))
    os_ = (C.c_int64 * 3)(0, out.stride(0), out.stride(1))
    _check("civic_prefill_attn_ragged", lib.civic_prefill_attn_ragged(
        _dev(q), _dev(k), _dev(v), _dev(out), _dtype_code(q), batch, C.c_void_p(off.ctypes.data), hq, k.shape[1], d, qs, ks, os_,
        int(bool(causal)), float(softmax_scale), _dev(k_cache), _dev(v_cache), s_max, int(pos0), _stream(stream)))
    return out


def civic_prefill_attn(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, causal: bool = True,
                       softmax_scale: float = 0.0, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """q [batch, seq, H_q, d]; k, v [batch, seq, H_kv, d] with identical strides; strided views are fine."""
    if k.shape != v.shape or k.stride() != v.stride() or q.dtype != k.dtype or q.dtype != v.dtype:
        raise ValueError("k and v must share shape, strides and dtype with q's dtype")
    batch, seq, hq, d = q.shape
    if out is None:
        out = torch.empty((batch, seq, hq, d), dtype=q.dtype, device=q.device)
    _check("civic_prefill_attn", lib.civic_prefill_attn(_dev(q), _dev(k), _dev(v), _dev(out), _dtype_code(q), batch, seq,
                                                        hq, k.shape[2], d, _strides3(q), _strides3(k), _strides3(out),
                                                        int(bool(causal)), float(softmax_scale), _stream(stream)))
    return out


def civic_kv_write(k: torch.Tensor, v: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor, pos0: int = 0,
                   stream=None) -> None:
    """k, v [batch, seq, H_kv, d] -> caches [batch, H_kv, s_max, d] (contiguous) at rows [pos0, pos0 + seq)."""
    if k.shape != v.shape or k.stride() != v.stride() or k.dtype != v.dtype:
        raise ValueError("k and v must share shape, strides and dtype")
    batch, seq, hkv, d = k.shape
    if (not k_cache.is_contiguous() or not v_cache.is_contiguous() or k_cache.shape != v_cache.shape
            or k_cache.dtype != k.dtype or v_cache.dtype != k.dtype
            or k_cache.shape[0] != batch or k_cache.shape[1] != hkv or k_cache.shape[3] != d):
        raise ValueError("caches must be contiguous [batch, H_kv, s_max, d] of the inputs' dtype")
    _check("civic_kv_write", lib.civic_kv_write(_dev(k), _dev(v), _strides3(k), _dtype_code(k), _dev(k_cache), _dev(v_cache),
                                                batch, seq, hkv, d, k_cache.shape[2], int(pos0), _stream(stream)))


def civic_prefill_attn_kv(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                          pos0: int = 0, causal: bool = True, softmax_scale: float = 0.0,
                          out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """civic_prefill_attn and civic_kv_write on the same k, v as one call (same arguments, same results)."""
    if k.shape != v.shape or k.stride() != v.stride() or q.dtype != k.dtype or q.dtype != v.dtype:
        raise ValueError("k and v must share shape, strides and dtype with q's dtype")
    batch, seq, hq, d = q.shape
    hkv = k.shape[2]
    if (not k_cache.is_contiguous() or not v_cache.is_contiguous() or k_cache.shape != v_cache.shape
            or k_cache.dtype != k.dtype or v_cache.dtype != k.dtype
            or k_cache.shape[0] != batch or k_cache.shape[1] != hkv or k_cache.shape[3] != d):
        raise ValueError("caches must be contiguous [batch, H_kv, s_max, d] of the inputs' dtype")
    if out is None:
        out = torch.empty((batch, seq, hq, d), dtype=q.dtype, device=q.device)
    _check("civic_prefill_attn_kv", lib.civic_prefill_attn_kv(
        _dev(q), _dev(k), _dev(v), _dev(out), _dev(k_cache), _dev(v_cache), _dtype_code(q), batch, seq, hq, hkv, d,
        _strides3(q), _strides3(k), _strides3(out), k_cache.shape[2], int(pos0), int(bool(causal)), float(softmax_scale),
        _stream(stream)))
    return out


def civic_decode_attn_workspace_bytes(dtype: torch.dtype, batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
                                      n_ctx: int) -> int:
    code = CIVIC_F32 if dtype == torch.float32 else CIVIC_BF16
    return int(lib.civic_decode_attn_workspace_bytes(code, batch, n_q_heads, n_kv_heads, head_dim, n_ctx))


def _decode_shapes(q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor):
    if q.dim() != 3 or not q.is_contiguous() or not k_cache.is_contiguous() or not v_cache.is_contiguous():
        raise ValueError("q [batch, H_q, d] and the caches [batch, H_kv, s_max, d] must be contiguous")
    if k_cache.shape != v_cache.shape or k_cache.dim() != 4 or k_cache.dtype != q.dtype or v_cache.dtype != q.dtype:
        raise ValueError("caches must share shape and q's dtype")
    batch, hq, d = q.shape
    if k_cache.shape[0] != batch or k_cache.shape[3] != d:
        raise ValueError("caches must be [batch, H_kv, s_max, d]")
    return batch, hq, k_cache.shape[1], d, k_cache.shape[2]


def civic_decode_attn(q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor, n_ctx: int, softmax_scale: float = 0.0,
                      out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """q [batch, H_q, d] against rows [0, n_ctx) of the caches [batch, H_kv, s_max, d] -> out [batch, H_q, d]."""
    batch, hq, hkv, d, s_max = _decode_shapes(q, k_cache, v_cache)
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        need = civic_decode_attn_workspace_bytes(q.dtype, batch, hq, hkv, d, n_ctx)
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device) if need else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check("civic_decode_attn", lib.civic_decode_attn(_dev(q), _dev(k_cache), _dev(v_cache), _dev(out), _dtype_code(q), batch,
                                                      hq, hkv, d, s_max, int(n_ctx), float(softmax_scale), _dev(workspace),
                                                      ws_bytes, _stream(stream)))
    return out


def civic_decode_attn_ragged(q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor, n_ctx: Sequence[int], softmax_scale: float = 0.0,
                             out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """The decode step with one context length per sample: q [batch, H_q, d] over rows [0, n_ctx[b]) of the caches."""
    batch, hq, hkv, d, s_max = _decode_shapes(q, k_cache, v_cache)
    ctx = np.ascontiguousarray(np.asarray(n_ctx, dtype=np.int32))
    if ctx.shape != (batch,):
        raise ValueError("one context length per sample")
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        need = int(lib.civic_decode_attn_ragged_workspace_bytes(_dtype_code(q), batch, C.c_void_p(ctx.ctypes.data), hq, hkv, d))
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    _check("civic_decode_attn_ragged", lib.civic_decode_attn_ragged(
        _dev(q), _dev(k_cache), _dev(v_cache), _dev(out), _dtype_code(q), batch, C.c_void_p(ctx.ctypes.data), hq, hkv, d, s_max,
        float(softmax_scale), _dev(workspace), workspace.numel(), _stream(stream)))
    return out


def civic_decode_attn_noalloc(q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor, n_ctx: int, out: torch.Tensor,
                              softmax_scale: float = 0.0, stream=None) -> torch.Tensor:
    """civic_decode_attn without a workspace argument (the library's own static scratch); `out` is the caller's."""
    batch, hq, hkv, d, s_max = _decode_shapes(q, k_cache, v_cache)
    _check("civic_decode_attn_noalloc", lib.civic_decode_attn_noalloc(_dev(q), _dev(k_cache), _dev(v_cache), _dev(out),
                                                                      _dtype_code(q), batch, hq, hkv, d, s_max, int(n_ctx),
                                                                      float(softmax_scale), _stream(stream)))
    return out


def civic_mrope_table(pos_ids: torch.Tensor, axis_of_pair, inv_freq, cos_sin: Optional[torch.Tensor] = None,
                      stream=None) -> torch.Tensor:
    """pos_ids int32 [3, batch, seq] (device); axis_of_pair / inv_freq host arrays [n_pairs] -> fp32 [batch, seq, n_pairs, 2]."""
    if pos_ids.dim() != 3 or pos_ids.shape[0] != 3 or pos_ids.dtype != torch.int32 or not pos_ids.is_contiguous():
        raise ValueError("pos_ids must be contiguous int32 [3, batch, seq]")
    ax = np.ascontiguousarray(np.asarray(axis_of_pair, dtype=np.int32))
    fr = np.ascontiguousarray(np.asarray(inv_freq, dtype=np.float32))
    if ax.ndim != 1 or ax.shape != fr.shape:
        raise ValueError("axis_of_pair and inv_freq must be 1-D of one length")
    _, batch, seq = pos_ids.shape
    if cos_sin is None:
        cos_sin = torch.empty((batch, seq, ax.shape[0], 2), dtype=torch.float32, device=pos_ids.device)
    _check("civic_mrope_table", lib.civic_mrope_table(_dev(pos_ids), batch, seq, ax.shape[0], C.c_void_p(ax.ctypes.data),
                                                      C.c_void_p(fr.ctypes.data), _dev(cos_sin), _stream(stream)))
    return cos_sin


def civic_mrope_apply(x: torch.Tensor, cos_sin: torch.Tensor, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """x [batch, seq, heads, d] (strided views are fine) rotated into out (default: a new dense tensor; may be x itself)."""
    batch, seq, heads, d = x.shape
    if out is None:
        out = torch.empty((batch, seq, heads, d), dtype=x.dtype, device=x.device)
    if not cos_sin.is_contiguous() or tuple(cos_sin.shape) != (batch, seq, d // 2, 2) or cos_sin.dtype != torch.float32:
        raise ValueError("cos_sin must be contiguous fp32 [batch, seq, d/2, 2]")
    _check("civic_mrope_apply", lib.civic_mrope_apply(_dev(x), _dev(out), _dtype_code(x), batch, seq, heads, d, _strides3(x),
                                                      _strides3(out), _dev(cos_sin), _stream(stream)))
    return out


def civic_kv_write_rope(k: torch.Tensor, v: torch.Tensor, cos_sin: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                        pos0: int = 0, stream=None) -> None:
    """civic_kv_write with K rotated by cos_sin [batch, seq, d/2, 2] on its way into the cache."""
    if k.shape != v.shape or k.stride() != v.stride() or k.dtype != v.dtype:
        raise ValueError("k and v must share shape, strides and dtype")
    batch, seq, hkv, d = k.shape
    if (not k_cache.is_contiguous() or not v_cache.is_contiguous() or k_cache.shape != v_cache.shape
            or k_cache.dtype != k.dtype or v_cache.dtype != k.dtype
            or k_cache.shape[0] != batch or k_cache.shape[1] != hkv or k_cache.shape[3] != d):
        raise ValueError("caches must be contiguous [batch, H_kv, s_max, d] of the inputs' dtype")
    if not cos_sin.is_contiguous() or tuple(cos_sin.shape) != (batch, seq, d // 2, 2) or cos_sin.dtype != torch.float32:
        raise ValueError("cos_sin must be contiguous fp32 [batch, seq, d/2, 2]")
    _check("civic_kv_write_rope", lib.civic_kv_write_rope(_dev(k), _dev(v), _strides3(k), _dtype_code(k), _dev(cos_sin),
                                                          _dev(k_cache), _dev(v_cache), batch, seq, hkv, d, k_cache.shape[2],
                                                          int(pos0), _stream(stream)))


def civic_prefill_attn_rope(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, q_cos_sin: torch.Tensor, causal: bool = True,
                            softmax_scale: float = 0.0, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """civic_prefill_attn with Q rotated on the fly; k (already rotated) and v [batch, seq, H_kv, d] may be views of the caches."""
    if k.shape != v.shape or k.stride() != v.stride() or q.dtype != k.dtype or q.dtype != v.dtype:
        raise ValueError("k and v must share shape, strides and dtype with q's dtype")
    batch, seq, hq, d = q.shape
    if not q_cos_sin.is_contiguous() or tuple(q_cos_sin.shape) != (batch, seq, d // 2, 2) or q_cos_sin.dtype != torch.float32:
        raise ValueError("q_cos_sin must be contiguous fp32 [batch, seq, d/2, 2]")
    if out is None:
        out = torch.empty((batch, seq, hq, d), dtype=q.dtype, device=q.device)
    _check("civic_prefill_attn_rope", lib.civic_prefill_attn_rope(_dev(q), _dev(k), _dev(v), _dev(out), _dtype_code(q), batch, seq,
                                                                  hq, k.shape[2], d, _strides3(q), _strides3(k), _strides3(out),
                                                                  int(bool(causal)), float(softmax_scale), _dev(q_cos_sin),
                                                                  _stream(stream)))
    return out


def civic_anchor_aggregate(x0: torch.Tensor, anchors: torch.Tensor, inv_tau: float = 1.0, want_token_weight: bool = False,
                           z0: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None):
    """Eq. 8: x0 [batch, T, D], anchors [M, D] (bf16) -> z0 [batch, M, D] (and the per-token weight [batch, T] fp32)."""
    if x0.dim() != 3 or anchors.dim() != 2 or not x0.is_contiguous() or not anchors.is_contiguous() or x0.dtype != anchors.dtype:
        raise ValueError("x0 [batch, T, D] and anchors [M, D] must be contiguous and of one dtype")
    batch, t, d = x0.shape
    m = anchors.shape[0]
    if anchors.shape[1] != d:
        raise ValueError("anchors must be [M, D]")
    if z0 is None:
        z0 = torch.empty((batch, m, d), dtype=x0.dtype, device=x0.device)
    tw = torch.empty((batch, t), dtype=torch.float32, device=x0.device) if want_token_weight else None
    if workspace is None:
        workspace = torch.empty(int(lib.civic_anchor_aggregate_workspace_bytes(batch, t, m, d)), dtype=torch.uint8, device=x0.device)
    _check("civic_anchor_aggregate", lib.civic_anchor_aggregate(_dev(x0), _dev(anchors), _dtype_code(x0), batch, t, m, d,
                                                                float(inv_tau), _dev(z0), _dev(tw), _dev(workspace),
                                                                workspace.numel(), _stream(stream)))
    return (z0, tw) if want_token_weight else z0


def civic_kv_compress(k: torch.Tensor, v: torch.Tensor, r: torch.Tensor, k_c: Optional[torch.Tensor] = None,
                      v_c: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None):
    """Eq. 9: k, v [batch, M, ...] (trailing axes flattened to the width), r fp32 [M, S] -> k_c, v_c [batch, S, ...]."""
    if k.shape != v.shape or not k.is_contiguous() or not v.is_contiguous() or not r.is_contiguous() or r.dtype != torch.float32:
        raise ValueError("k and v must be contiguous of one shape, r contiguous fp32 [M, S]")
    batch, m = k.shape[0], k.shape[1]
    width = int(np.prod(k.shape[2:]))
    if r.shape[0] != m:
        raise ValueError("r must be [M, S]")
    s_mem = r.shape[1]
    if k_c is None:
        k_c = torch.empty((batch, s_mem) + tuple(k.shape[2:]), dtype=k.dtype, device=k.device)
    if v_c is None:
        v_c = torch.empty_like(k_c)
    if workspace is None:
        workspace = torch.empty(int(lib.civic_kv_compress_workspace_bytes(batch, m, s_mem, width)), dtype=torch.uint8, device=k.device)
    _check("civic_kv_compress", lib.civic_kv_compress(_dev(k), _dev(v), _dtype_code(k), _dev(r), batch, m, s_mem, width, _dev(k_c),
                                                      _dev(v_c), _dev(workspace), workspace.numel(), _stream(stream)))
    return k_c, v_c


def civic_cross_attn(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, softmax_scale: float = 0.0,
                     out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """q [batch, n_q, H_q, d] over k, v [batch, n_kv, H_kv, d], no mask."""
    if k.shape != v.shape or k.stride() != v.stride() or q.dtype != k.dtype or q.dtype != v.dtype:
        raise ValueError("k and v must share shape, strides and dtype with q's dtype")
    batch, n_q, hq, d = q.shape
    if out is None:
        out = torch.empty((batch, n_q, hq, d), dtype=q.dtype, device=q.device)
    _check("civic_cross_attn", lib.civic_cross_attn(_dev(q), _dev(k), _dev(v), _dev(out), _dtype_code(q), batch, n_q, k.shape[1], hq,
                                                    k.shape[2], d, _strides3(q), _strides3(k), _strides3(out), float(softmax_scale),
                                                    _stream(stream)))
    return out


def civic_kv_compress_ragged(k: torch.Tensor, v: torch.Tensor, r: torch.Tensor, row_offsets: Sequence[int],
                             k_c: Optional[torch.Tensor] = None, v_c: Optional[torch.Tensor] = None,
                             workspace: Optional[torch.Tensor] = None, stream=None):
    """Eq. 9 for packed items: k, v [total, ...] (trailing axes flattened to the width), r fp32 [total, S], item b owning
    rows [row_offsets[b], row_offsets[b+1]) -> k_c, v_c [batch, S, ...]."""
    if k.shape != v.shape or not k.is_contiguous() or not v.is_contiguous() or not r.is_contiguous() or r.dtype != torch.float32:
        raise ValueError("k and v must be contiguous of one shape, r contiguous fp32 [total, S]")
    off = np.ascontiguousarray(np.asarray(row_offsets, dtype=np.int64))
    batch = off.size - 1
    width = int(np.prod(k.shape[1:]))
    s_mem = r.shape[1]
    if r.shape[0] != k.shape[0] or off[-1] != k.shape[0]:
        raise ValueError("r and the offsets must cover the packed rows")
    if k_c is None:
        k_c = torch.empty((batch, s_mem) + tuple(k.shape[1:]), dtype=k.dtype, device=k.device)
    if v_c is None:
        v_c = torch.empty_like(k_c)
    if workspace is None:
        need = int(lib.civic_kv_compress_ragged_workspace_bytes(batch, C.c_void_p(off.ctypes.data), s_mem, width))
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=k.device)
    _check("civic_kv_compress_ragged", lib.civic_kv_compress_ragged(
        _dev(k), _dev(v), _dtype_code(k), _dev(r), batch, C.c_void_p(off.ctypes.data), s_mem, width, _dev(k_c), _dev(v_c),
        _dev(workspace), workspace.numel(), _stream(stream)))
    return k_c, v_c


def civic_cross_attn_ragged(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, q_offsets: Sequence[int],
                            softmax_scale: float = 0.0, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """q [total, H_q, d] packed (item b owning rows [q_offsets[b], q_offsets[b+1])) over k, v [batch, n_kv, H_kv, d]."""
    if k.shape != v.shape or k.stride() != v.stride() or q.dtype != k.dtype or q.dim() != 3 or q.stride(2) != 1:
        raise ValueError("q [total, H_q, d]; k and v [batch, n_kv, H_kv, d] of one shape, strides and dtype")
    off = np.ascontiguousarray(np.asarray(q_offsets, dtype=np.int64))
    batch = off.size - 1
    total, hq, d = q.shape
    if out is None:
        out = torch.empty((total, hq, d), dtype=q.dtype, device=q.device)
    qs = (C.c_int64 * 3)(0, q.stride(0), q.stride(1))
    os_ = (C.c_int64 * 3)(0, out.stride(0), out.stride(1))
    _check("civic_cross_attn_ragged", lib.civic_cross_attn_ragged(
        _dev(q), _dev(k), _dev(v), _dev(out), _dtype_code(q), batch, C.c_void_p(off.ctypes.data), k.shape[1], hq, k.shape[2], d,
        qs, _strides3(k), os_, float(softmax_scale), _stream(stream)))
    return out
