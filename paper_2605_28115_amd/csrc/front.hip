// civic_compact_prefill: the front of the path in one call - anchor scores of the visual rows (Eq. 8), token
// selection under the budget and the floors, compact merge (Eq. 13).  No arithmetic of its own: the three
// stages' kernels are enqueued back to back on the caller's stream.  What it saves is host time: one crossing
// of the language boundary instead of three, which is most of a step on shapes whose kernels take a few
// microseconds each.
#include "civic_internal.h"

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
