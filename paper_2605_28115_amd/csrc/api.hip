// Host-only entry points: error state, grid arithmetic, workspace queries, anchor preparation.
#include <atomic>
#include <cmath>
#include <vector>

#include "civic_internal.h"

namespace civic {

static std::atomic<int> g_last_hip_error{0};

int record_hip_error(hipError_t e)
{
    g_last_hip_error.store(static_cast<int>(e));
    return CIVIC_ERR_HIP;
}

int allow_dynamic_lds(const void* kernel, size_t bytes, std::atomic<uint64_t>* done)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return record_hip_error(e);
    const uint64_t bit = dev >= 0 && dev < 64 ? uint64_t{1} << dev : 0;   // devices beyond 63 set it on every call
    if (bit && (done->load(std::memory_order_acquire) & bit)) return CIVIC_OK;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
    if (e != hipSuccess) return record_hip_error(e);
    done->fetch_or(bit, std::memory_order_release);
    return CIVIC_OK;
}

KernelTimer& kernel_timer()
{
    static thread_local KernelTimer t;
    return t;
}

int grid_info(const civic_grid* g, GridInfo* out)
{
    if (!g || !out) return CIVIC_ERR_INVALID_ARG;
    if (g->frames <= 0 || g->height <= 0 || g->width <= 0 || g->cell_h <= 0 || g->cell_w <= 0)
        return CIVIC_ERR_INVALID_ARG;
    if (g->cell_floor < 0 || g->frame_floor < 0 || g->budget < 0) return CIVIC_ERR_INVALID_ARG;
    const int64_t hw = static_cast<int64_t>(g->height) * g->width;
    const int64_t nv = hw * g->frames;
    if (nv > INT32_MAX || g->budget > nv) return CIVIC_ERR_INVALID_ARG;

    // Floors of one frame: full cells, a ragged right column of cells, a ragged bottom row, a corner.
    const int64_t full_r = g->height / g->cell_h, rem_r = g->height % g->cell_h;
    const int64_t full_c = g->width / g->cell_w, rem_c = g->width % g->cell_w;
    auto floor_of = [&](int64_t size) { return size < g->cell_floor ? size : static_cast<int64_t>(g->cell_floor); };
    int64_t per_frame = full_r * full_c * floor_of(static_cast<int64_t>(g->cell_h) * g->cell_w);
    if (rem_c) per_frame += full_r * floor_of(static_cast<int64_t>(g->cell_h) * rem_c);
    if (rem_r) per_frame += full_c * floor_of(rem_r * g->cell_w);
    if (rem_r && rem_c) per_frame += floor_of(rem_r * rem_c);
    out->cell_kept_frame = static_cast<int32_t>(per_frame);
    const int64_t left = hw - per_frame;
    per_frame += left < g->frame_floor ? left : static_cast<int64_t>(g->frame_floor);
    const int64_t floor_sum = per_frame * g->frames;

    out->frames = g->frames; out->height = g->height; out->width = g->width;
    out->cell_h = g->cell_h; out->cell_w = g->cell_w;
    out->cell_floor = g->cell_floor; out->frame_floor = g->frame_floor; out->budget = g->budget;
    out->hw = static_cast<int32_t>(hw);
    out->nv = static_cast<int32_t>(nv);
    out->floor_sum = static_cast<int32_t>(floor_sum);
    out->kept = static_cast<int32_t>(floor_sum > g->budget ? floor_sum : g->budget);
    out->fill = static_cast<int32_t>(g->budget > floor_sum ? g->budget - floor_sum : 0);
    return CIVIC_OK;
}

}  // namespace civic

extern "C" {

int civic_last_hip_error(void) { return civic::g_last_hip_error.load(); }

int civic_time_next_kernel(void* start_event, void* stop_event)
{
    civic::KernelTimer& t = civic::kernel_timer();
    if (!start_event && !stop_event) { t = civic::KernelTimer{}; return CIVIC_OK; }
    if (!start_event || !stop_event || start_event == stop_event) return CIVIC_ERR_INVALID_ARG;
    t.start = static_cast<hipEvent_t>(start_event);
    t.stop = static_cast<hipEvent_t>(stop_event);
    t.armed = true;
    return CIVIC_OK;
}

int64_t civic_kept_count(const civic_grid* grid)
{
    civic::GridInfo gi;
    const int rc = civic::grid_info(grid, &gi);
    return rc == CIVIC_OK ? gi.kept : rc;
}

size_t civic_select_workspace_bytes(const civic_grid* grid, int32_t batch)
{
    (void)grid; (void)batch;
    return 0;   // the selection keeps all of its state in LDS
}

size_t civic_compact_workspace_bytes(int32_t batch, int64_t seq_len)
{
    (void)batch; (void)seq_len;
    return 0;   // the compact merge derives every source index inside the copy kernel
}

int civic_anchor_normalize(const float* anchor, int32_t dim, float* anchor_q)
{
    if (!anchor || !anchor_q || dim <= 0) return CIVIC_ERR_INVALID_ARG;
    long double sum = 0.0L;
    for (int32_t j = 0; j < dim; ++j) sum += anchor[j];
    const double mean = static_cast<double>(sum / dim);
    // LN divides by sqrt(var + eps) and Norm divides by the norm of the result: the first factor
    // cancels, leaving the centred vector over its own l2 norm.
    long double ss = 0.0L;
    for (int32_t j = 0; j < dim; ++j) { const double c = anchor[j] - mean; ss += c * c; }
    const double nrm = std::sqrt(static_cast<double>(ss));
    if (!(nrm > 0.0) || !std::isfinite(nrm)) return CIVIC_ERR_INVALID_ARG;
    for (int32_t j = 0; j < dim; ++j) anchor_q[j] = static_cast<float>((anchor[j] - mean) / nrm);
    return CIVIC_OK;
}

}  // extern "C"
