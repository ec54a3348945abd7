// Internal helpers shared by the translation units of libcivic (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <atomic>
#include <type_traits>

#include "civic.h"

namespace civic {

// Records a failing HIP status for civic_last_hip_error() and maps it to the ABI code.
int record_hip_error(hipError_t e);

// Raises a kernel's dynamic LDS limit to `bytes` on the current device; the attribute belongs to the device's
// copy of the kernel, so it is set once per device (bit d of *done: device d has it).  CIVIC_OK or an error code.
int allow_dynamic_lds(const void* kernel, size_t bytes, std::atomic<uint64_t>* done);

// One-shot kernel timer of the calling thread (civic_time_next_kernel arms it).
struct KernelTimer {
    hipEvent_t start = nullptr, stop = nullptr;
    bool armed = false;
};
KernelTimer& kernel_timer();

// Every kernel of the library is launched through here.  The arguments are converted to the kernel's own
// parameter types first, so both launch forms pack the same bytes.  When the thread's timer is armed, this launch
// carries its two events (recorded by the command processor at the kernel's start and end) and disarms it.
template <typename... Params, typename... Args>
static inline void launch(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds, hipStream_t s, Args&&... args)
{
    static_assert(sizeof...(Params) == sizeof...(Args), "kernel argument count");
    KernelTimer& t = kernel_timer();
    if (__builtin_expect(t.armed, 0)) {
        t.armed = false;
        hipExtLaunchKernelGGL(kernel, grid, block, static_cast<uint32_t>(lds), s, t.start, t.stop, 0u,
                              static_cast<Params>(args)...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, lds, s, static_cast<Params>(args)...);
    }
}

static inline int check_launch()
{
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? CIVIC_OK : record_hip_error(e);
}

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static inline int dtype_size(int dtype) { return dtype == CIVIC_F32 ? 4 : dtype == CIVIC_BF16 ? 2 : 0; }

// Validated view of a civic_grid with the derived counts every stage needs.
struct GridInfo {
    int32_t frames, height, width, cell_h, cell_w, cell_floor, frame_floor, budget;
    int32_t hw;          // tokens per frame
    int32_t nv;          // visual tokens per sample
    int32_t cell_kept_frame;   // tokens the cell floors protect in one frame
    int32_t floor_sum;   // tokens the floors protect, per sample
    int32_t kept;        // K = max(budget, floor_sum)
    int32_t fill;        // tokens the budget adds after the floors
};

// CIVIC_OK and a filled GridInfo, or CIVIC_ERR_INVALID_ARG.
int grid_info(const civic_grid* g, GridInfo* out);

// Argument checks of the three front stages, each a host function that launches nothing (the stage's entry
// point runs it first; civic_compact_prefill runs all three before the first launch).
int score_visual_check(const void* hidden, int dtype, int32_t batch, int64_t seq_len, int32_t dim, const civic_grid* grid,
                       const int64_t* frame_start, const float* anchor_q, float inv_tau, const float* scores);
int select_check(const float* scores, int32_t batch, const civic_grid* grid, const int32_t* kept_idx);
int compact_check(const void* hidden, int dtype, int32_t dim, const int32_t* pos_ids, int32_t batch, int64_t seq_len,
                  const civic_grid* grid, const int64_t* frame_start, const int32_t* kept_idx, int64_t n_kept,
                  const void* hidden_c, const int32_t* pos_c, const int32_t* src_idx);

// The launch of civic_compact for arguments that compact_check has passed; pos_axis_in / pos_axis_out are the element
// distances between the three id axes of pos_ids and of pos_c.
int compact_launch(const void* hidden, int dtype, int32_t dim, const int32_t* pos_ids, int32_t batch, int64_t seq_len,
                   const civic_grid* grid, const int64_t* frame_start, const int32_t* kept_idx, int64_t n_kept, void* hidden_c,
                   int32_t* pos_c, int32_t* src_idx, int64_t pos_axis_in, int64_t pos_axis_out, void* stream);

// Up to 64 spans of rows of a packed tensor scored in one launch (the ragged front); arguments checked by the caller.
int score_slices_launch(const void* hidden, int dtype, int32_t dim, const float* anchor_q, float inv_tau, float* scores,
                        const int32_t* first, const int32_t* count, const int32_t* out, int32_t n_slices, int32_t longest, void* stream);

// Up to 16 samples of different grids selected in one launch (the ragged front); every sample checked by the caller.
int select_samples_launch(const float* const* scores, int32_t* const* kept_idx, const civic_grid* const* grids, int32_t n, void* stream);

// One sample of a ragged batch for compact_samples_launch: where its rows, kept indices and compact rows begin in the
// packed tensors, its kept count, length, grid and (sample-local) frame starts.
struct RaggedSample {
    int64_t row0, comp0, kept0, n_kept, seq_len;
    const civic_grid* grid;
    const int64_t* frame_start;
};
constexpr int kCompactRaggedItems = 24, kCompactRaggedFrames = 8;
// Up to kCompactRaggedItems samples (each checked by the caller, at most kCompactRaggedFrames frames) merged by one launch.
int compact_samples_launch(const void* hidden, int dtype, int32_t dim, const int32_t* pos_ids, const int32_t* kept_idx, void* hidden_c,
                           int32_t* pos_c, int32_t* src_idx, const RaggedSample* samples, int32_t n, int64_t pos_axis_in,
                           int64_t pos_axis_out, void* stream);

constexpr int kWave = 64;

// Native vector types (the nontemporal load builtin does not take HIP's struct vectors).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <typename T>
__device__ __forceinline__ T load_streaming(const T* p) { return __builtin_nontemporal_load(p); }

// Sum over the 64 lanes of a wavefront, returned in every lane.  Data-parallel-primitive (DPP) adds:
// an inclusive scan inside each row of 16 lanes (row_shr 1, 2, 4, 8), then the row totals are carried
// across rows (row_bcast 15 into rows 1 and 3, row_bcast 31 into rows 2 and 3) so that lane 63 holds
// the total; no LDS traffic, unlike a shuffle.
__device__ __forceinline__ float wave_sum(float v)
{
    auto dpp_add = [](float x, auto ctrl, auto row_mask) {
        const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(x), decltype(ctrl)::value,
                                                      decltype(row_mask)::value, 0xF, false);
        return x + __int_as_float(moved);
    };
    using std::integral_constant;
    v = dpp_add(v, integral_constant<int, 0x111>{}, integral_constant<int, 0xF>{});   // row_shr:1
    v = dpp_add(v, integral_constant<int, 0x112>{}, integral_constant<int, 0xF>{});   // row_shr:2
    v = dpp_add(v, integral_constant<int, 0x114>{}, integral_constant<int, 0xF>{});   // row_shr:4
    v = dpp_add(v, integral_constant<int, 0x118>{}, integral_constant<int, 0xF>{});   // row_shr:8
    v = dpp_add(v, integral_constant<int, 0x142>{}, integral_constant<int, 0xA>{});   // row_bcast:15 -> rows 1, 3
    v = dpp_add(v, integral_constant<int, 0x143>{}, integral_constant<int, 0xC>{});   // row_bcast:31 -> rows 2, 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// One frequency pair of the rotary embedding: (x0, x1) turned by the angle whose (cos, sin) is (c, s).  Written
// with explicit fused multiply-adds so that every kernel that rotates rounds the same way.
__device__ __forceinline__ void rope_pair(float x0, float x1, float c, float s, float& y0, float& y1)
{
    y0 = __builtin_fmaf(x0, c, -(x1 * s));
    y1 = __builtin_fmaf(x1, c, x0 * s);
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

}  // namespace civic
