// Internal helpers shared by the translation units of libcivic (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "civic.h"

namespace civic {

// Records a failing HIP status for civic_last_hip_error() and maps it to the ABI code.
int record_hip_error(hipError_t e);

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
    int32_t floor_sum;   // tokens the floors protect, per sample
    int32_t kept;        // K = max(budget, floor_sum)
    int32_t fill;        // tokens the budget adds after the floors
};

// CIVIC_OK and a filled GridInfo, or CIVIC_ERR_INVALID_ARG.
int grid_info(const civic_grid* g, GridInfo* out);

constexpr int kWave = 64;

// Native vector types (the nontemporal load builtin does not take HIP's struct vectors).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <typename T>
__device__ __forceinline__ T load_streaming(const T* p) { return __builtin_nontemporal_load(p); }

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

}  // namespace civic
