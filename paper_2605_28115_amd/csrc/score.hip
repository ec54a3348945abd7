// civic_score: anchor logit of Eq. 8 for every hidden row.  HBM-bound row reduction.
//
// One wavefront owns a row at a time.  The row is fetched once with 16-byte loads (lane l takes
// chunks l, l+64, ...) and held in registers, so the centred second pass (norm and dot product of
// x - mean) costs no second trip to memory and has none of the cancellation a one-pass
// sum-of-squares formula would have.  The anchor chunks a lane needs are the same for every row
// and stay in registers for the lifetime of the wave.
#include "civic_internal.h"

namespace civic {

template <bool BF16> struct Chunk;
template <> struct Chunk<true> {
    static constexpr int kElems = 8;
    static __device__ __forceinline__ void unpack(const u32x4& raw, float* x)
    {
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i]     = __uint_as_float(w[i] << 16);
            x[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
};
template <> struct Chunk<false> {
    static constexpr int kElems = 4;
    static __device__ __forceinline__ void unpack(const u32x4& raw, float* x)
    {
        x[0] = __uint_as_float(raw.x); x[1] = __uint_as_float(raw.y);
        x[2] = __uint_as_float(raw.z); x[3] = __uint_as_float(raw.w);
    }
};

template <int CHUNKS, bool BF16>
__global__ __launch_bounds__(256) void score_kernel(const uint8_t* __restrict__ hidden, int64_t n_rows,
                                                    int64_t row_stride_bytes, int32_t dim,
                                                    const float* __restrict__ anchor_q, float inv_tau,
                                                    float* __restrict__ scores)
{
    constexpr int E = Chunk<BF16>::kElems;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave = (static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x) >> 6;
    const int64_t n_waves = (static_cast<int64_t>(gridDim.x) * blockDim.x) >> 6;
    const int n_chunks = dim / E;
    const float inv_dim = 1.0f / static_cast<float>(dim);

    float q[CHUNKS][E];
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
        const int ch = c * kWave + lane;
#pragma unroll
        for (int e = 0; e < E; e += 4) {
            float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
            if (ch < n_chunks) t = *reinterpret_cast<const float4*>(anchor_q + ch * E + e);
            q[c][e] = t.x; q[c][e + 1] = t.y; q[c][e + 2] = t.z; q[c][e + 3] = t.w;
        }
    }

    for (int64_t row = wave; row < n_rows; row += n_waves) {
        const u32x4* src = reinterpret_cast<const u32x4*>(hidden + row * row_stride_bytes);
        u32x4 raw[CHUNKS];
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) {
            const int ch = c * kWave + lane;
            raw[c] = u32x4{0u, 0u, 0u, 0u};
            if (ch < n_chunks) raw[c] = load_streaming(src + ch);
        }
        // first element of the row, for the exact "no variance" test (equal elements <=> max == min)
        const float first = __uint_as_float(__builtin_amdgcn_readfirstlane(BF16 ? (raw[0].x << 16) : raw[0].x));
        float sum = 0.f;
        bool same = true;
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) {
            const bool live = (c * kWave + lane) < n_chunks;
            float x[E];
            Chunk<BF16>::unpack(raw[c], x);
#pragma unroll
            for (int e = 0; e < E; ++e) { sum += x[e]; same = same && (!live || x[e] == first); }
        }
        const bool constant_row = __ballot(!same) == 0ull;
        const float mean = wave_sum(sum) * inv_dim;
        float n2 = 0.f, dot = 0.f;
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) {
            const bool live = (c * kWave + lane) < n_chunks;
            float x[E];
            Chunk<BF16>::unpack(raw[c], x);
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const float d = live ? x[e] - mean : 0.f;
                n2 = fmaf(d, d, n2);
                dot = fmaf(q[c][e], d, dot);
            }
        }
        n2 = wave_sum(n2);
        dot = wave_sum(dot);
        if (lane == 0) scores[row] = (n2 > 0.f && !constant_row) ? inv_tau * dot / sqrtf(n2) : 0.f;
    }
}

template <int CHUNKS>
static int launch_score(bool bf16, const void* hidden, int64_t n_rows, int64_t row_stride_bytes, int32_t dim,
                        const float* anchor_q, float inv_tau, float* scores, hipStream_t stream)
{
    // 16 resident waves per CU on 256 CUs keep enough 16-byte loads in flight to cover HBM latency.
    const int64_t max_waves = 256 * 16;
    int64_t waves = n_rows < max_waves ? n_rows : max_waves;
    const unsigned blocks = static_cast<unsigned>((waves + 3) / 4);
    const uint8_t* h = static_cast<const uint8_t*>(hidden);
    if (bf16)
        hipLaunchKernelGGL((score_kernel<CHUNKS, true>), dim3(blocks), dim3(256), 0, stream, h, n_rows,
                           row_stride_bytes, dim, anchor_q, inv_tau, scores);
    else
        hipLaunchKernelGGL((score_kernel<CHUNKS, false>), dim3(blocks), dim3(256), 0, stream, h, n_rows,
                           row_stride_bytes, dim, anchor_q, inv_tau, scores);
    return check_launch();
}

}  // namespace civic

extern "C" int civic_score(const void* hidden, int dtype, int64_t n_rows, int64_t row_stride, int32_t dim,
                           const float* anchor_q, float inv_tau, float* scores, void* stream)
{
    using namespace civic;
    const int esz = dtype_size(dtype);
    if (!esz || !hidden || !anchor_q || !scores) return CIVIC_ERR_INVALID_ARG;
    if (n_rows < 0 || dim <= 0 || row_stride < dim) return CIVIC_ERR_INVALID_ARG;
    const int elems = 16 / esz;
    if (dim % elems) return CIVIC_ERR_INVALID_ARG;
    if (!aligned16(hidden) || !aligned16(anchor_q) || (row_stride * esz) % 16) return CIVIC_ERR_INVALID_ARG;
    if (!(inv_tau == inv_tau)) return CIVIC_ERR_INVALID_ARG;
    if (static_cast<int64_t>(dim) * esz > static_cast<int64_t>(CIVIC_MAX_SCORE_DIM) * 2) return CIVIC_ERR_UNSUPPORTED;
    if (n_rows == 0) return CIVIC_OK;

    const int chunks = (dim / elems + kWave - 1) / kWave;   // 16-byte chunks per lane
    const bool bf16 = dtype == CIVIC_BF16;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t rsb = row_stride * esz;
#define CIVIC_SCORE_CASE(N) \
    if (chunks <= N) return launch_score<N>(bf16, hidden, n_rows, rsb, dim, anchor_q, inv_tau, scores, s)
    CIVIC_SCORE_CASE(1); CIVIC_SCORE_CASE(2); CIVIC_SCORE_CASE(3); CIVIC_SCORE_CASE(4);
    CIVIC_SCORE_CASE(6); CIVIC_SCORE_CASE(8); CIVIC_SCORE_CASE(12); CIVIC_SCORE_CASE(16);
#undef CIVIC_SCORE_CASE
    return CIVIC_ERR_UNSUPPORTED;
}
