// civic_compact_prefill: the front of the path in one call - anchor scores of the visual rows (Eq. 8), token
// selection under the budget and the floors, compact merge (Eq. 13).  No arithmetic of its own: the three
// stages' kernels are enqueued back to back on the caller's stream.  What it saves is host time: one crossing
// of the language boundary instead of three, which is most of a step on shapes whose kernels take a few
// microseconds each.
#include "civic_internal.h"

#include <cstring>

extern "C" int civic_compact_prefill(const void* hidden, int dtype, int32_t batch, int64_t seq_len, int32_t dim,
                                     const int32_t* pos_ids, const civic_grid* grid, const int64_t* frame_start,
                                     const float* anchor_q, float inv_tau, float* scores, int32_t* kept_idx,
                                     void* hidden_c, int32_t* pos_c, int32_t* src_idx, void* workspace,
                                     size_t workspace_bytes, void* stream)
{
    using namespace civic;
    // every check of every stage before the first launch
    int rc = score_visual_check(hidden, dtype, batch, seq_len, dim, grid, frame_start, anchor_q, inv_tau, scores);
    if (rc != CIVIC_OK) return rc;
    rc = select_check(scores, batch, grid, kept_idx);
    if (rc != CIVIC_OK) return rc;
    const int64_t n_kept = civic_kept_count(grid);                // >= 0: the grid has passed the checks above
    rc = compact_check(hidden, dtype, dim, pos_ids, batch, seq_len, grid, frame_start, kept_idx, n_kept, hidden_c, pos_c, src_idx);
    if (rc != CIVIC_OK) return rc;
    const size_t need = civic_select_workspace_bytes(grid, batch);
    if (need > 0 && (!workspace || workspace_bytes < need)) return CIVIC_ERR_INVALID_ARG;

    rc = civic_score_visual(hidden, dtype, batch, seq_len, dim, grid, frame_start, anchor_q, inv_tau, scores, stream);
    if (rc != CIVIC_OK) return rc;
    rc = civic_select(scores, batch, grid, kept_idx, nullptr, workspace, workspace_bytes, stream);
    if (rc != CIVIC_OK) return rc;
    return civic_compact(hidden, dtype, dim, pos_ids, batch, seq_len, grid, frame_start, kept_idx, n_kept, hidden_c, pos_c,
                         src_idx, workspace, workspace_bytes, stream);
}

// ------------------------------------------------------------------------------------------------ ragged batches
// Samples of different length and grid (images of different grid sizes in one batch), packed along the token axis.
extern "C" int civic_ragged_offsets(int32_t batch, const int64_t* seq_offsets, const civic_grid* grids, int64_t* visual_offsets,
                                    int64_t* kept_offsets, int64_t* compact_offsets)
{
    using namespace civic;
    if (batch < 0 || !seq_offsets || seq_offsets[0] != 0 || (batch > 0 && !grids)) return CIVIC_ERR_INVALID_ARG;
    int64_t vis = 0, kept = 0, comp = 0;
    if (visual_offsets) visual_offsets[0] = 0;
    if (kept_offsets) kept_offsets[0] = 0;
    if (compact_offsets) compact_offsets[0] = 0;
    for (int32_t b = 0; b < batch; ++b) {
        GridInfo gi;
        if (grid_info(&grids[b], &gi) != CIVIC_OK) return CIVIC_ERR_INVALID_ARG;
        const int64_t len = seq_offsets[b + 1] - seq_offsets[b];
        if (len < gi.nv) return CIVIC_ERR_INVALID_ARG;        // (which also makes the offsets non-decreasing)
        vis += gi.nv; kept += gi.kept; comp += len - gi.nv + gi.kept;
        if (visual_offsets) visual_offsets[b + 1] = vis;
        if (kept_offsets) kept_offsets[b + 1] = kept;
        if (compact_offsets) compact_offsets[b + 1] = comp;
    }
    return CIVIC_OK;
}

extern "C" int civic_compact_prefill_ragged(const void* hidden, int dtype, int32_t batch, const int64_t* seq_offsets, int32_t dim,
                                            const int32_t* pos_ids, const civic_grid* grids, const int64_t* frame_start,
                                            const float* anchor_q, float inv_tau, float* scores, int32_t* kept_idx,
                                            void* hidden_c, int32_t* pos_c, int32_t* src_idx, void* stream)
{
    using namespace civic;
    const int esz = dtype_size(dtype);
    if (!esz || dim <= 0) return CIVIC_ERR_INVALID_ARG;
    int rc = civic_ragged_offsets(batch, seq_offsets, grids, nullptr, nullptr, nullptr);
    if (rc != CIVIC_OK) return rc;
    if (batch == 0) return CIVIC_OK;
    if (!frame_start) return CIVIC_ERR_INVALID_ARG;
    // Per sample: where its rows, scores, kept indices, compact rows and frame starts begin in the packed tensors.
    // The id axes of the packed pos_ids / pos_c are the packed totals apart.
    struct Sample {
        const char* hidden; const int32_t* pos; const int64_t* frames; float* scores; int32_t* kept; char* hidden_c;
        int32_t* pos_c; int32_t* src; int64_t len, n_kept;
    };
    auto sample = [&](int32_t b, int64_t vis, int64_t kept, int64_t comp, int64_t frames_before) {
        Sample x;
        const int64_t row0 = seq_offsets[b];
        x.hidden = hidden ? static_cast<const char*>(hidden) + row0 * dim * esz : nullptr;
        x.pos = pos_ids ? pos_ids + row0 : nullptr;
        x.frames = frame_start + frames_before;
        x.scores = scores ? scores + vis : nullptr;
        x.kept = kept_idx ? kept_idx + kept : nullptr;
        x.hidden_c = hidden_c ? static_cast<char*>(hidden_c) + comp * dim * esz : nullptr;
        x.pos_c = pos_c ? pos_c + comp : nullptr;
        x.src = src_idx ? src_idx + comp : nullptr;
        x.len = seq_offsets[b + 1] - row0;
        x.n_kept = civic_kept_count(&grids[b]);
        return x;
    };
    int64_t total_c = 0;
    for (int32_t b = 0; b < batch; ++b) total_c += (seq_offsets[b + 1] - seq_offsets[b]) - static_cast<int64_t>(grids[b].frames) * grids[b].height * grids[b].width + civic_kept_count(&grids[b]);
    const int64_t total = seq_offsets[batch];
    // A run of consecutive samples of one shape (same grid, length and frame starts) is a rectangular batch where it
    // lies in the packed tensors, so it goes through the kernels as one: `n` samples per launch.
    auto run_length = [&](int32_t b, int64_t frames_before) {
        const civic_grid& g = grids[b];
        const int64_t len = seq_offsets[b + 1] - seq_offsets[b];
        int32_t n = 1;
        while (b + n < batch && n < 65535) {
            const civic_grid& h = grids[b + n];
            if (std::memcmp(&g, &h, sizeof(civic_grid)) != 0 || seq_offsets[b + n + 1] - seq_offsets[b + n] != len) break;
            if (std::memcmp(frame_start + frames_before, frame_start + frames_before + static_cast<int64_t>(n) * g.frames,
                            sizeof(int64_t) * g.frames) != 0)
                break;
            ++n;
        }
        return n;
    };
    // every check of every run before the first launch
    {
        int64_t vis = 0, kept = 0, comp = 0, frames_before = 0;
        for (int32_t b = 0; b < batch;) {
            const civic_grid* g = &grids[b];
            const Sample x = sample(b, vis, kept, comp, frames_before);
            const int32_t n = run_length(b, frames_before);
            rc = score_visual_check(x.hidden, dtype, n, x.len, dim, g, x.frames, anchor_q, inv_tau, x.scores);
            if (rc == CIVIC_OK) rc = select_check(x.scores, n, g, x.kept);
            if (rc == CIVIC_OK) rc = compact_check(x.hidden, dtype, dim, x.pos, n, x.len, g, x.frames, x.kept, x.n_kept, x.hidden_c, x.pos_c, x.src);
            if (rc != CIVIC_OK) return rc;
            const int64_t nv = static_cast<int64_t>(g->frames) * g->height * g->width;
            vis += n * nv; kept += n * x.n_kept; comp += n * (x.len - nv + x.n_kept); frames_before += static_cast<int64_t>(n) * g->frames;
            b += n;
        }
        if (total > INT32_MAX || vis > INT32_MAX) return CIVIC_ERR_UNSUPPORTED;     // (row numbers travel as 32-bit kernel arguments)
    }
    // Scores: the frames of all samples, 64 spans per launch.  Selection: 16 samples per launch, each workgroup with its
    // own sample's grid.  Merge: run by run.
    {
        constexpr int kSlices = 64, kSamples = 16;
        int32_t first[kSlices], count[kSlices], out[kSlices], n_sl = 0, longest = 0;
        auto flush_scores = [&]() {
            const int r = n_sl ? score_slices_launch(hidden, dtype, dim, anchor_q, inv_tau, scores, first, count, out, n_sl, longest, stream) : CIVIC_OK;
            n_sl = 0; longest = 0;
            return r;
        };
        int64_t vis = 0, frames_before = 0;
        for (int32_t b = 0; b < batch; ++b) {
            const civic_grid& g = grids[b];
            const int32_t hw = g.height * g.width;
            for (int32_t f = 0; f < g.frames; ++f) {
                first[n_sl] = static_cast<int32_t>(seq_offsets[b] + frame_start[frames_before + f]);
                count[n_sl] = hw;
                out[n_sl] = static_cast<int32_t>(vis + static_cast<int64_t>(f) * hw);
                longest = hw > longest ? hw : longest;
                if (++n_sl == kSlices && (rc = flush_scores()) != CIVIC_OK) return rc;
            }
            vis += static_cast<int64_t>(g.frames) * hw;
            frames_before += g.frames;
        }
        if ((rc = flush_scores()) != CIVIC_OK) return rc;

        const float* sc[kSamples];
        int32_t* kp[kSamples];
        const civic_grid* gp[kSamples];
        int32_t n_sm = 0;
        int64_t kept = 0;
        vis = 0;
        for (int32_t b = 0; b < batch; ++b) {
            sc[n_sm] = scores + vis; kp[n_sm] = kept_idx + kept; gp[n_sm] = &grids[b];
            vis += static_cast<int64_t>(grids[b].frames) * grids[b].height * grids[b].width;
            kept += civic_kept_count(&grids[b]);
            if (++n_sm == kSamples || b + 1 == batch) {
                if ((rc = select_samples_launch(sc, kp, gp, n_sm, stream)) != CIVIC_OK) return rc;
                n_sm = 0;
            }
        }
    }
    // Merge: samples with few frames 24 per launch (a table of sample descriptions in the kernel arguments); a sample
    // with more frames than the table holds per sample goes out by itself, together with its run of equal samples.
    {
        RaggedSample rs[kCompactRaggedItems];
        int32_t n_rs = 0;
        auto flush_merge = [&]() {
            const int r = n_rs ? compact_samples_launch(hidden, dtype, dim, pos_ids, kept_idx, hidden_c, pos_c, src_idx, rs, n_rs, total,
                                                        total_c, stream)
                               : CIVIC_OK;
            n_rs = 0;
            return r;
        };
        int64_t vis = 0, kept = 0, comp = 0, frames_before = 0;
        for (int32_t b = 0; b < batch;) {
            const civic_grid* g = &grids[b];
            const Sample x = sample(b, vis, kept, comp, frames_before);
            const int64_t nv = static_cast<int64_t>(g->frames) * g->height * g->width;
            int32_t n = 1;
            if (g->frames > kCompactRaggedFrames) {
                n = run_length(b, frames_before);
                rc = compact_launch(x.hidden, dtype, dim, x.pos, n, x.len, g, x.frames, x.kept, x.n_kept, x.hidden_c, x.pos_c, x.src, total,
                                    total_c, stream);
                if (rc != CIVIC_OK) return rc;
            } else {
                rs[n_rs++] = RaggedSample{seq_offsets[b], comp, kept, x.n_kept, x.len, g, x.frames};
                if (n_rs == kCompactRaggedItems && (rc = flush_merge()) != CIVIC_OK) return rc;
            }
            vis += n * nv; kept += n * x.n_kept; comp += n * (x.len - nv + x.n_kept); frames_before += static_cast<int64_t>(n) * g->frames;
            b += n;
        }
        if ((rc = flush_merge()) != CIVIC_OK) return rc;
    }
    return CIVIC_OK;
}
