// civic_compact: Merge of Eq. 13.  Builds the contiguous, order-preserving compact sequence (all
// text tokens + kept visual tokens) and carries the position ids along unchanged.  HBM-bound row
// gather: only kept rows are ever read.
//
// One launch, no scratch.  A block owns a run of consecutive compact rows of one batch item and
// derives their dense source indices itself:
//   - kept_idx is ascending, so the number of kept tokens before frame f (kb[f]) is the position
//     where the frame id of consecutive entries steps past f; every thread looks at one entry and
//     its predecessor and fills the table in LDS.  The same pass drops the source index of every
//     kept visual token whose compact slot falls into the block's run.
//   - in compact space frame f starts at cs[f] = frame_start[f] - f*HW + kb[f] (text before it plus
//     kept tokens before it); a slot not claimed by a visual token is text and maps back by adding
//     the visual tokens dropped before it.
// A kept list of more than 1024 entries is not read whole by every block: a probe of one entry out of
// P brackets each frame boundary, the entries that can land in the block's rows are a small window,
// and a second round trip searches the bracketed stretches (see the kernel).
// The rows are then moved with the widest vector the row size allows (16 bytes for every Qwen3-VL
// shape), several rows in flight per thread so that loads are issued back to back before any store.
#include "civic_internal.h"

namespace civic {

constexpr int kCompactThreads = 256;
constexpr int kCompactMaxRows = 64;   // compact rows per block (LDS table size)
constexpr int kCompactUnroll = 4;
#ifndef CIVIC_COMPACT_BLOCKS_PER_CU
#define CIVIC_COMPACT_BLOCKS_PER_CU 8   // target number of workgroups per compute unit (a build-time knob for A/B runs)
#endif

struct FrameTable {
    int32_t n;                          // frames
    int32_t hw;                         // tokens per frame
    int32_t start[CIVIC_MAX_FRAMES];    // sequence index of each frame's first token
};

// U > 0: the launch guarantees rows_per_block == U * (kCompactThreads / threads_per_row) and a row
// length that is a multiple of 2 * threads_per_row vectors, so a block with all its rows (every block
// but a sample's last) copies them without a per-row or per-column condition.  U == 0: no such promise.
// LONG: the kept list is searched in two round trips instead of read whole (the launch guarantees
// that the probes' stretches and a block's window of entries each fit one batch of 4 per thread).
// pos_axis_in / pos_axis_out: elements between the three id axes of pos_ids and of pos_c (batch * seq_len and
// batch * seq_c for the rectangular tensors; the packed totals when the samples of a ragged batch are merged one by one).
// The block's work for batch item `b` of the tensors the pointers name; FT is a frame table (n, hw, start[]).
template <typename V, int U, bool LONG, typename FT>
__device__ __forceinline__ void compact_rows(
    const uint8_t* __restrict__ hidden, int64_t row_bytes, const int32_t* __restrict__ pos_ids,
    int32_t seq_len, const FT& ft, const int32_t* __restrict__ kept_idx, int32_t n_kept, int32_t seq_c,
    int32_t rows_per_block, int32_t threads_per_row, uint8_t* __restrict__ hidden_c, int32_t* __restrict__ pos_c,
    int32_t* __restrict__ src_idx, int64_t pos_axis_in, int64_t pos_axis_out, const int b)
{
    __shared__ int32_t kb[CIVIC_MAX_FRAMES + 1];
    __shared__ int32_t row_src[kCompactMaxRows];
    __shared__ int32_t fstart[CIVIC_MAX_FRAMES];   // frame_start - f*HW: text tokens before frame f
    __shared__ int32_t stretch[CIVIC_MAX_FRAMES];  // long lists: the probe at whose entry, or in the P - 1 before it, frame f's boundary lies

    const int tid = threadIdx.x;
    const int32_t j0 = blockIdx.x * rows_per_block;
    const int32_t nrows = min(rows_per_block, seq_c - j0);
    const int32_t* kept = kept_idx + static_cast<int64_t>(b) * n_kept;
    const int32_t F = ft.n, hw = ft.hw;
    auto frame_of = [&](int32_t v) { return min(max(v / hw, 0), F - 1); };

    // A block whose rows all lie before the first frame or behind the last kept visual token holds text only,
    // and the sources of such rows follow from the counts alone (nothing is dropped before the first frame,
    // everything that is dropped lies before the text at the end): no look at the list.  These blocks start
    // to move rows at once, which fills the memory system while the others are still reading the list.
    const int32_t first_vis = ft.start[0];
    const int32_t after_vis = ft.start[F - 1] - (F - 1) * hw + n_kept;
    const bool text_only = j0 + nrows <= first_vis || j0 >= after_vis;
    if (text_only) {
        const int32_t shift = j0 >= after_vis ? F * hw - n_kept : 0;
        for (int32_t r = tid; r < nrows; r += kCompactThreads) row_src[r] = j0 + r + shift;
        __syncthreads();
    } else {
    // Long kept lists (more than one batch below): reading the whole list in every block would cost a
    // memory round trip per batch and more L2 traffic than the rows themselves.  Two round trips
    // suffice: (1) every thread probes one entry out of P, which brackets each frame boundary between
    // two probes, together with the entries that can land in this block's rows (slot j holds entry
    // j - fstart[f], and fstart only grows with f, so they are a window of nrows plus the text between
    // the first and the last frame); (2) the bracketed stretches are searched for the boundaries.
    // Used when the window and the stretches fit one batch (decided at launch); otherwise the full pass below.
    if constexpr (LONG) {
        const int32_t probe_step = (n_kept + kCompactThreads - 1) / kCompactThreads;
        const int32_t win_lo = max(j0 - (ft.start[F - 1] - (F - 1) * hw), 0);
        const int32_t win_hi = min(j0 + nrows - ft.start[0], n_kept);
        const int32_t n_probes = (n_kept + probe_step - 1) / probe_step;
        const int32_t ip = tid * probe_step;
        int32_t probe = 0, probe_prev = 0, own[4];
        if (tid < n_probes) { probe = kept[ip]; probe_prev = tid > 0 ? kept[ip - probe_step] : 0; }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int32_t i = win_lo + u * kCompactThreads + tid;
            own[u] = i < win_hi ? kept[i] : 0;
        }
        if (tid < F) { fstart[tid] = ft.start[tid] - tid * hw; stretch[tid] = n_probes; }
        if (tid <= F) kb[tid] = tid == 0 ? 0 : n_kept;              // a boundary that no entry reaches stays at the end
        __syncthreads();
        if (tid < n_probes) {                                        // boundary f lies in (ip - P, ip] for f in (frame before, this frame]
            const int32_t f_hi = frame_of(probe), f_lo = tid > 0 ? frame_of(probe_prev) : -1;
            for (int32_t f = f_lo + 1; f <= f_hi; ++f) stretch[f] = tid;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int32_t i = win_lo + u * kCompactThreads + tid;
            if (i < win_hi) {
                const int32_t f = frame_of(own[u]), j = fstart[f] + i - j0;
                if (j >= 0 && j < nrows) row_src[j] = fstart[f] + own[u];
            }
        }
        __syncthreads();
        int32_t cur[4], prev[4], at[4], fr[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {                                // candidate u of this thread: entry `at` for boundary `fr`
            const int32_t c = u * kCompactThreads + tid;
            fr[u] = min(1 + c / probe_step, F - 1);
            at[u] = probe_step * (stretch[fr[u]] - 1) + 1 + (c - (fr[u] - 1) * probe_step);
            const bool live = c < (F - 1) * probe_step && at[u] >= 0 && at[u] < n_kept;
            if (!live) at[u] = -1;
            cur[u] = live ? kept[at[u]] : 0;
            prev[u] = live && at[u] > 0 ? kept[at[u] - 1] : 0;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (at[u] >= 0 && fr[u] <= frame_of(cur[u]) && (at[u] == 0 || frame_of(prev[u]) < fr[u])) kb[fr[u]] = at[u];
        __syncthreads();
    } else {
    // Entries are visited four strided positions per thread at a time, all loads of a batch issued
    // before any is used (one memory latency per batch instead of one per entry).  The first batch goes
    // out together with this thread's word of the frame table (a per-thread index into the kernel
    // arguments is a memory load too), so the block waits for memory once before it knows its rows.
    int32_t cur[4], prev[4];
    auto load_batch = [&](int32_t base) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int32_t i = base + u * kCompactThreads + tid;
            cur[u] = i < n_kept ? kept[i] : 0;
            prev[u] = (i > 0 && i <= n_kept) ? kept[i - 1] : 0;
        }
    };
    load_batch(0);
    if (tid < F) fstart[tid] = ft.start[tid] - tid * hw;
    __syncthreads();
    for (int32_t base = 0;;) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int32_t i = base + u * kCompactThreads + tid;
            if (i > n_kept) continue;
            int32_t f_prev = -1, f_cur = F;
            if (i > 0) f_prev = min(max(prev[u] / hw, 0), F - 1);
            if (i < n_kept) {
                const int32_t v = cur[u];
                f_cur = min(max(v / hw, 0), F - 1);
                const int32_t j = fstart[f_cur] + i - j0;                  // compact slot of this kept token
                if (j >= 0 && j < nrows) row_src[j] = fstart[f_cur] + v;
            }
            for (int32_t f = f_prev + 1; f <= f_cur; ++f) kb[f] = i;
        }
        base += kCompactThreads * 4;
        if (base > n_kept) break;
        load_batch(base);
    }
    __syncthreads();
    }

    for (int32_t r = tid; r < nrows; r += kCompactThreads) {
        const int32_t j = j0 + r;
        // number of frames whose compact start is <= j (cs is non-decreasing in f)
        int32_t lo = 0, hi = F;
        while (lo < hi) {
            const int32_t mid = (lo + hi) >> 1;
            if (fstart[mid] + kb[mid] <= j) lo = mid + 1; else hi = mid;
        }
        if (lo == 0) {
            row_src[r] = j;                                           // text before the first frame
        } else {
            const int32_t f = lo - 1;
            const int32_t vis_end = fstart[f] + kb[f + 1];              // end of frame f's kept tokens
            if (j >= vis_end) row_src[r] = j + lo * hw - kb[lo];      // text: add the dropped tokens back
        }
    }
    __syncthreads();
    }

    for (int32_t r = tid; r < nrows; r += kCompactThreads) {
        const int32_t src = min(max(row_src[r], 0), seq_len - 1);
        const int64_t o = static_cast<int64_t>(b) * seq_c + j0 + r;
        src_idx[o] = src;
#pragma unroll
        for (int a = 0; a < 3; ++a)
            pos_c[a * pos_axis_out + static_cast<int64_t>(b) * seq_c + j0 + r] =
                pos_ids[a * pos_axis_in + static_cast<int64_t>(b) * seq_len + src];
    }

    const int32_t vpr = static_cast<int32_t>(row_bytes / sizeof(V));    // vectors per row
    const int32_t rows_per_pass = kCompactThreads / threads_per_row;
    const int32_t rr = tid / threads_per_row, c0 = tid - rr * threads_per_row;
    const uint8_t* in_b = hidden + static_cast<int64_t>(b) * seq_len * row_bytes;
    uint8_t* out_b = hidden_c + (static_cast<int64_t>(b) * seq_c + j0) * row_bytes;
    if (U > 0 && nrows == rows_per_block) {
        // Straight-line copy: 2 * U independent 16-byte loads per column step, then the stores.  With
        // conditions around the accesses the compiler cannot count the loads in flight and waits for
        // all of them, and for the stores before them, at every step.
        const int Un = U > 0 ? U : 1;
        int32_t src[Un];
#pragma unroll
        for (int u = 0; u < Un; ++u) src[u] = min(max(row_src[u * rows_per_pass + rr], 0), seq_len - 1);
        for (int32_t c = c0; c < vpr; c += 2 * threads_per_row) {
            V val[2][Un];
#pragma unroll
            for (int u = 0; u < Un; ++u) {
                const V* in = reinterpret_cast<const V*>(in_b + static_cast<int64_t>(src[u]) * row_bytes) + c;
                val[0][u] = load_streaming(in);
                val[1][u] = load_streaming(in + threads_per_row);
            }
#pragma unroll
            for (int u = 0; u < Un; ++u) {
                V* out = reinterpret_cast<V*>(out_b + static_cast<int64_t>(u * rows_per_pass + rr) * row_bytes) + c;
                out[0] = val[0][u];
                out[threads_per_row] = val[1][u];
            }
        }
        return;
    }
    for (int32_t rbase = 0; rbase < nrows; rbase += rows_per_pass * kCompactUnroll) {
        // Rows as byte offsets from the two kernel-argument bases plus a flag (a pointer that may be null
        // would turn every access into a flat one, which the compiler fences off from its neighbours).
        int64_t in_off[kCompactUnroll], out_off[kCompactUnroll];
        bool live[kCompactUnroll];
#pragma unroll
        for (int u = 0; u < kCompactUnroll; ++u) {
            const int32_t r = rbase + u * rows_per_pass + rr;
            live[u] = r < nrows;
            const int32_t src = live[u] ? min(max(row_src[r], 0), seq_len - 1) : 0;
            in_off[u] = static_cast<int64_t>(src) * row_bytes;
            out_off[u] = static_cast<int64_t>(r) * row_bytes;
        }
        // two column steps x kCompactUnroll rows: up to 8 independent 16-byte loads before the first store
        for (int32_t c = c0; c < vpr; c += 2 * threads_per_row) {
            V val[2][kCompactUnroll];
            const bool second = c + threads_per_row < vpr;
#pragma unroll
            for (int u = 0; u < kCompactUnroll; ++u)
                if (live[u]) {
                    const V* in = reinterpret_cast<const V*>(in_b + in_off[u]) + c;
                    val[0][u] = load_streaming(in);
                    if (second) val[1][u] = load_streaming(in + threads_per_row);
                }
#pragma unroll
            for (int u = 0; u < kCompactUnroll; ++u)
                if (live[u]) {
                    V* out = reinterpret_cast<V*>(out_b + out_off[u]) + c;
                    out[0] = val[0][u];
                    if (second) out[threads_per_row] = val[1][u];
                }
        }
    }

}

template <typename V, int U, bool LONG>
__global__ __launch_bounds__(kCompactThreads) void compact_kernel(
    const uint8_t* __restrict__ hidden, int64_t row_bytes, const int32_t* __restrict__ pos_ids, int32_t batch,
    int32_t seq_len, FrameTable ft, const int32_t* __restrict__ kept_idx, int32_t n_kept, int32_t seq_c,
    int32_t rows_per_block, int32_t threads_per_row, uint8_t* __restrict__ hidden_c, int32_t* __restrict__ pos_c,
    int32_t* __restrict__ src_idx, int64_t pos_axis_in, int64_t pos_axis_out)
{
    (void)batch;
    compact_rows<V, U, LONG>(hidden, row_bytes, pos_ids, seq_len, ft, kept_idx, n_kept, seq_c, rows_per_block, threads_per_row,
                             hidden_c, pos_c, src_idx, pos_axis_in, pos_axis_out, blockIdx.y);
}

// Samples of different length and grid in one launch (the ragged front): grid y = sample, described by an entry of a
// table in the kernel arguments - where its rows, kept indices and compact rows begin in the packed tensors, and its
// frame table (up to kCompactRaggedFrames frames; samples with more are merged by a launch of their own).  Grid x
// covers the longest sample; a block past its sample's compact rows has nothing to do.
struct CompactItem {
    int32_t row0, comp0, kept0, n_kept, seq_len, seq_c;
    int32_t n, hw, start[kCompactRaggedFrames];              // the sample's frame table
};
struct CompactTable {
    CompactItem item[kCompactRaggedItems];
};
template <typename V, int U>
__global__ __launch_bounds__(kCompactThreads) void compact_ragged_kernel(
    const uint8_t* __restrict__ hidden, int64_t row_bytes, const int32_t* __restrict__ pos_ids, CompactTable t,
    const int32_t* __restrict__ kept_idx, int32_t rows_per_block, int32_t threads_per_row, uint8_t* __restrict__ hidden_c,
    int32_t* __restrict__ pos_c, int32_t* __restrict__ src_idx, int64_t pos_axis_in, int64_t pos_axis_out)
{
    const CompactItem& it = t.item[blockIdx.y];
    if (static_cast<int64_t>(blockIdx.x) * rows_per_block >= it.seq_c) return;
    compact_rows<V, U, false>(hidden + static_cast<int64_t>(it.row0) * row_bytes, row_bytes, pos_ids + it.row0, it.seq_len, it,
                              kept_idx + it.kept0, it.n_kept, it.seq_c, rows_per_block, threads_per_row,
                              hidden_c + static_cast<int64_t>(it.comp0) * row_bytes, pos_c + it.comp0, src_idx + it.comp0,
                              pos_axis_in, pos_axis_out, 0);
}

}  // namespace civic

namespace civic {

// The argument checks of civic_compact (host only, nothing is launched).
int compact_check(const void* hidden, int dtype, int32_t dim, const int32_t* pos_ids, int32_t batch, int64_t seq_len,
                  const civic_grid* grid, const int64_t* frame_start, const int32_t* kept_idx, int64_t n_kept,
                  const void* hidden_c, const int32_t* pos_c, const int32_t* src_idx)
{
    const int esz = dtype_size(dtype);
    GridInfo gi;
    if (grid_info(grid, &gi) != CIVIC_OK) return CIVIC_ERR_INVALID_ARG;
    if (!esz || !frame_start) return CIVIC_ERR_INVALID_ARG;
    if (dim <= 0 || batch < 0 || seq_len < gi.nv || n_kept < 0 || n_kept > gi.nv) return CIVIC_ERR_INVALID_ARG;
    // a tensor without elements (batch 0; nothing kept and no text) needs no pointer
    const bool some_out = batch > 0 && seq_len - gi.nv + n_kept > 0;
    if (batch > 0 && (!hidden || !pos_ids || (n_kept > 0 && !kept_idx))) return CIVIC_ERR_INVALID_ARG;
    if (some_out && (!hidden_c || !pos_c || !src_idx)) return CIVIC_ERR_INVALID_ARG;
    int64_t prev_end = 0;
    for (int32_t f = 0; f < gi.frames; ++f) {
        if (frame_start[f] < prev_end || frame_start[f] + gi.hw > seq_len) return CIVIC_ERR_INVALID_ARG;
        prev_end = frame_start[f] + gi.hw;
    }
    const int64_t row_bytes = static_cast<int64_t>(dim) * esz;
    int vec = 16;
    while (row_bytes % vec) vec >>= 1;
    const uintptr_t both = reinterpret_cast<uintptr_t>(hidden) | reinterpret_cast<uintptr_t>(hidden_c);
    if (both & static_cast<uintptr_t>(vec - 1)) return CIVIC_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(pos_ids) | reinterpret_cast<uintptr_t>(pos_c) |
         reinterpret_cast<uintptr_t>(src_idx) | reinterpret_cast<uintptr_t>(kept_idx)) & 3u)
        return CIVIC_ERR_INVALID_ARG;
    if (gi.frames > CIVIC_MAX_FRAMES || seq_len > INT32_MAX || batch > 65535) return CIVIC_ERR_UNSUPPORTED;
    return CIVIC_OK;
}

}  // namespace civic

namespace civic {

// How a launch copies rows of `row_bytes` bytes when it has `total_rows` of them to move.
struct CompactGeom {
    int vec;        // bytes per vector
    int tpr;        // threads per row
    int unroll;     // passes of the condition-free copy (0: the general loop)
    int64_t rpb;    // rows per block
};
static CompactGeom compact_geom(int64_t row_bytes, int64_t total_rows)
{
    int vec = 16;
    while (row_bytes % vec) vec >>= 1;
    // Threads per row: the power of two in [16, 256] that wastes the fewest lanes on this row length; among
    // equals the largest whose double divides the row, which is what the condition-free copy needs.
    const int64_t vpr = row_bytes / vec;
    int tpr = 256;
    int64_t best = -1;
    bool best_even = false;
    for (int t = 256; t >= 16; t >>= 1) {
        const int64_t slots = (vpr + t - 1) / t * t;
        const bool even = vpr % (2 * t) == 0;
        if (best < 0 || slots < best || (slots == best && even && !best_even)) { best = slots; tpr = t; best_even = even; }
    }
    // Rows per block: small blocks win (about 8 per CU on 256 CUs keep more loads in flight, and the
    // per-block pass over kept_idx is a few KB of L2 hits), as long as every thread has a vector to move.
    int64_t rpb = total_rows / (256 * CIVIC_COMPACT_BLOCKS_PER_CU);
    const int64_t min_rows = 256 / tpr > 2 ? 256 / tpr : 2;
    if (rpb < min_rows) rpb = min_rows;
    if (rpb > kCompactMaxRows) rpb = kCompactMaxRows;
    // Condition-free copy: 1, 2 or 4 passes of 256 / tpr rows per block (more rows per block go the general way).
    const int64_t rpp = 256 / tpr;
    int unroll = 0;
    if (best_even && rpb <= 4 * rpp) {
        unroll = rpb <= rpp ? 1 : rpb <= 2 * rpp ? 2 : 4;
        rpb = unroll * rpp;
    }
    return CompactGeom{vec, tpr, unroll, rpb};
}

// The launch of civic_compact for arguments that compact_check has passed.
int compact_launch(const void* hidden, int dtype, int32_t dim, const int32_t* pos_ids, int32_t batch, int64_t seq_len,
                   const civic_grid* grid, const int64_t* frame_start, const int32_t* kept_idx, int64_t n_kept, void* hidden_c,
                   int32_t* pos_c, int32_t* src_idx, int64_t pos_axis_in, int64_t pos_axis_out, void* stream)
{
    const int esz = dtype_size(dtype);
    GridInfo gi;
    grid_info(grid, &gi);
    const int64_t row_bytes = static_cast<int64_t>(dim) * esz;
    int vec = 16;
    while (row_bytes % vec) vec >>= 1;
    const int64_t seq_c = seq_len - gi.nv + n_kept;
    if (batch == 0 || seq_c == 0) return CIVIC_OK;

    FrameTable ft;
    ft.n = gi.frames; ft.hw = gi.hw;
    for (int32_t f = 0; f < CIVIC_MAX_FRAMES; ++f) ft.start[f] = f < gi.frames ? static_cast<int32_t>(frame_start[f]) : 0;

    const CompactGeom geom = compact_geom(row_bytes, seq_c * batch);
    const int tpr = geom.tpr, unroll = geom.unroll;
    const int64_t rpb = geom.rpb;
    const int64_t blocks = (seq_c + rpb - 1) / rpb;
    // Long kept lists (more than one batch of 4 entries per thread) are searched instead of read whole when
    // the stretches between the probes, (frames - 1) * ceil(n_kept / 256) entries, and the entries that can land
    // in one block, its rows plus the text between the first and the last frame, each fit one batch.
    const int64_t probe_step = (n_kept + kCompactThreads - 1) / kCompactThreads;
    const int64_t text_between = (frame_start[gi.frames - 1] - frame_start[0]) - static_cast<int64_t>(gi.frames - 1) * gi.hw;
    const bool long_list = vec == 16 && n_kept > 4 * kCompactThreads && (gi.frames - 1) * probe_step <= 4 * kCompactThreads &&
                           rpb + text_between <= 4 * kCompactThreads;

    const uint8_t* h = static_cast<const uint8_t*>(hidden);
    uint8_t* hc = static_cast<uint8_t*>(hidden_c);
    const dim3 g(static_cast<unsigned>(blocks), static_cast<unsigned>(batch)), blk(kCompactThreads);
    hipStream_t s = static_cast<hipStream_t>(stream);
#define CIVIC_COMPACT_LAUNCH(V, U, LONG)                                                                      \
    civic::launch((compact_kernel<V, U, LONG>), g, blk, 0, s, h, row_bytes, pos_ids, batch,                \
                       static_cast<int32_t>(seq_len), ft, kept_idx, static_cast<int32_t>(n_kept),               \
                       static_cast<int32_t>(seq_c), static_cast<int32_t>(rpb), tpr, hc, pos_c, src_idx, pos_axis_in, pos_axis_out)
    switch (vec) {
        case 16:
            if (long_list) {
                switch (unroll) {
                    case 1: CIVIC_COMPACT_LAUNCH(u32x4, 1, true); break;
                    case 2: CIVIC_COMPACT_LAUNCH(u32x4, 2, true); break;
                    case 4: CIVIC_COMPACT_LAUNCH(u32x4, 4, true); break;
                    default: CIVIC_COMPACT_LAUNCH(u32x4, 0, true); break;
                }
            } else {
                switch (unroll) {
                    case 1: CIVIC_COMPACT_LAUNCH(u32x4, 1, false); break;
                    case 2: CIVIC_COMPACT_LAUNCH(u32x4, 2, false); break;
                    case 4: CIVIC_COMPACT_LAUNCH(u32x4, 4, false); break;
                    default: CIVIC_COMPACT_LAUNCH(u32x4, 0, false); break;
                }
            }
            break;
        case 8: CIVIC_COMPACT_LAUNCH(u32x2, 0, false); break;
        case 4: CIVIC_COMPACT_LAUNCH(uint32_t, 0, false); break;
        default: CIVIC_COMPACT_LAUNCH(uint16_t, 0, false); break;
    }
#undef CIVIC_COMPACT_LAUNCH
    return check_launch();
}

// Up to kCompactRaggedItems samples of different length and grid merged by ONE launch (the ragged front).  Every sample
// has passed compact_check on its own and has at most kCompactRaggedFrames frames; row numbers fit 32 bits.
int compact_samples_launch(const void* hidden, int dtype, int32_t dim, const int32_t* pos_ids, const int32_t* kept_idx, void* hidden_c,
                           int32_t* pos_c, int32_t* src_idx, const RaggedSample* samples, int32_t n, int64_t pos_axis_in,
                           int64_t pos_axis_out, void* stream)
{
    const int64_t row_bytes = static_cast<int64_t>(dim) * dtype_size(dtype);
    CompactTable t;
    int64_t total_rows = 0, longest = 0;
    for (int i = 0; i < kCompactRaggedItems; ++i) {
        CompactItem& it = t.item[i];
        if (i >= n) { it = t.item[0]; it.seq_c = 0; continue; }   // (never read: the grid has n samples)
        const RaggedSample& x = samples[i];
        GridInfo gi;
        grid_info(x.grid, &gi);
        it.row0 = static_cast<int32_t>(x.row0); it.comp0 = static_cast<int32_t>(x.comp0); it.kept0 = static_cast<int32_t>(x.kept0);
        it.n_kept = static_cast<int32_t>(x.n_kept); it.seq_len = static_cast<int32_t>(x.seq_len);
        it.seq_c = static_cast<int32_t>(x.seq_len - gi.nv + x.n_kept);
        it.n = gi.frames; it.hw = gi.hw;
        for (int f = 0; f < kCompactRaggedFrames; ++f) it.start[f] = f < gi.frames ? static_cast<int32_t>(x.frame_start[f]) : 0;
        total_rows += it.seq_c;
        longest = it.seq_c > longest ? it.seq_c : longest;
    }
    if (longest == 0) return CIVIC_OK;
    const CompactGeom geom = compact_geom(row_bytes, total_rows);
    const int64_t blocks = (longest + geom.rpb - 1) / geom.rpb;
    const uint8_t* h = static_cast<const uint8_t*>(hidden);
    uint8_t* hc = static_cast<uint8_t*>(hidden_c);
    const dim3 g(static_cast<unsigned>(blocks), static_cast<unsigned>(n)), blk(kCompactThreads);
    hipStream_t s = static_cast<hipStream_t>(stream);
#define CIVIC_COMPACT_RAGGED(V, U)                                                                                  \
    civic::launch((compact_ragged_kernel<V, U>), g, blk, 0, s, h, row_bytes, pos_ids, t, kept_idx,                    \
                  static_cast<int32_t>(geom.rpb), geom.tpr, hc, pos_c, src_idx, pos_axis_in, pos_axis_out)
    switch (geom.vec) {
        case 16:
            switch (geom.unroll) {
                case 1: CIVIC_COMPACT_RAGGED(u32x4, 1); break;
                case 2: CIVIC_COMPACT_RAGGED(u32x4, 2); break;
                case 4: CIVIC_COMPACT_RAGGED(u32x4, 4); break;
                default: CIVIC_COMPACT_RAGGED(u32x4, 0); break;
            }
            break;
        case 8: CIVIC_COMPACT_RAGGED(u32x2, 0); break;
        case 4: CIVIC_COMPACT_RAGGED(uint32_t, 0); break;
        default: CIVIC_COMPACT_RAGGED(uint16_t, 0); break;
    }
#undef CIVIC_COMPACT_RAGGED
    return check_launch();
}

}  // namespace civic

extern "C" int civic_compact(const void* hidden, int dtype, int32_t dim, const int32_t* pos_ids, int32_t batch,
                             int64_t seq_len, const civic_grid* grid, const int64_t* frame_start,
                             const int32_t* kept_idx, int64_t n_kept, void* hidden_c, int32_t* pos_c,
                             int32_t* src_idx, void* workspace, size_t workspace_bytes, void* stream)
{
    using namespace civic;
    (void)workspace; (void)workspace_bytes;
    const int rc_check = compact_check(hidden, dtype, dim, pos_ids, batch, seq_len, grid, frame_start, kept_idx, n_kept,
                                       hidden_c, pos_c, src_idx);
    if (rc_check != CIVIC_OK) return rc_check;
    GridInfo gi;
    grid_info(grid, &gi);
    return compact_launch(hidden, dtype, dim, pos_ids, batch, seq_len, grid, frame_start, kept_idx, n_kept, hidden_c, pos_c,
                          src_idx, static_cast<int64_t>(batch) * seq_len, static_cast<int64_t>(batch) * (seq_len - gi.nv + n_kept), stream);
}
