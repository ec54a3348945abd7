// civic_score: anchor logit of Eq. 8 for every hidden row.  HBM-bound row reduction.
//
// One wavefront owns a row at a time.  The row is fetched once with 16-byte loads (lane l takes
// chunks l, l+64, ...) and held in registers, so the centred second pass (norm and dot product of
// x - mean) costs no second trip to memory and has none of the cancellation a one-pass
// sum-of-squares formula would have.  The anchor is staged once per 16-wave block in LDS; the three
// wave-wide sums are DPP reductions.  The next row's loads are issued before the reductions of the
// current one.
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

#ifndef CIVIC_SCORE_THREADS
#define CIVIC_SCORE_THREADS 512
#endif
#ifndef CIVIC_SCORE_BLOCKS_PER_CU
#define CIVIC_SCORE_BLOCKS_PER_CU 2
#endif
constexpr int kScoreThreads = CIVIC_SCORE_THREADS;    // wavefronts of a block share one copy of the anchor in LDS
constexpr int kScoreBlocksPerCu = CIVIC_SCORE_BLOCKS_PER_CU;

template <int CHUNKS, bool BF16>
__global__ __launch_bounds__(kScoreThreads, kScoreBlocksPerCu) void score_kernel(const uint8_t* __restrict__ hidden, int64_t n_rows,
                                                              int64_t row_stride_bytes, int32_t dim,
                                                              const float* __restrict__ anchor_q, float inv_tau,
                                                              float* __restrict__ scores)
{
    constexpr int E = Chunk<BF16>::kElems;
    extern __shared__ __attribute__((aligned(16))) float q_s[];      // [dim]
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int n_chunks = dim / E;
    const float inv_dim = 1.0f / static_cast<float>(dim);
    const int64_t first = static_cast<int64_t>(blockIdx.x) * (kScoreThreads / kWave) + wave;
    const int64_t step = static_cast<int64_t>(gridDim.x) * (kScoreThreads / kWave);

    // The first row's loads go out before anything else; the anchor is staged while they are in flight.
    u32x4 raw[CHUNKS];
    auto fetch = [&](int64_t row) {
        const u32x4* src = reinterpret_cast<const u32x4*>(hidden + row * row_stride_bytes);
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) {
            const int ch = c * kWave + lane;
            raw[c] = u32x4{0u, 0u, 0u, 0u};
            if (ch < n_chunks) raw[c] = load_streaming(src + ch);
        }
    };
    if (first < n_rows) fetch(first);
    for (int i = threadIdx.x * 4; i < dim; i += kScoreThreads * 4)
        *reinterpret_cast<float4*>(q_s + i) = *reinterpret_cast<const float4*>(anchor_q + i);
    __syncthreads();

    for (int64_t row = first; row < n_rows; row += step) {
        // Pass 1: row sum, and the exact "no variance" test (every 32-bit word equals the first one
        // with its halves equal, i.e. every element carries the same bits).
        const uint32_t w0 = __builtin_amdgcn_readfirstlane(raw[0].x);
        const bool w0_uniform = !BF16 || (w0 >> 16) == (w0 & 0xFFFFu);
        float sum = 0.f;
        bool same = w0_uniform;
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) {
            const bool live = (c * kWave + lane) < n_chunks;
            same = same && (!live || (raw[c].x == w0 && raw[c].y == w0 && raw[c].z == w0 && raw[c].w == w0));
            float x[E];
            Chunk<BF16>::unpack(raw[c], x);                   // dead chunks are zero filled and add nothing
#pragma unroll
            for (int e = 0; e < E; ++e) sum += x[e];
        }
        const bool constant_row = __ballot(!same) == 0ull;
        const float mean = wave_sum(sum) * inv_dim;
        float n2 = 0.f, dot = 0.f;
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) {
            const int ch = c * kWave + lane;
            if (ch < n_chunks) {
                float x[E], q[E];
                Chunk<BF16>::unpack(raw[c], x);
#pragma unroll
                for (int e = 0; e < E; e += 4) {
                    const float4 t = *reinterpret_cast<const float4*>(q_s + ch * E + e);
                    q[e] = t.x; q[e + 1] = t.y; q[e + 2] = t.z; q[e + 3] = t.w;
                }
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const float d = x[e] - mean;
                    n2 = fmaf(d, d, n2);
                    dot = fmaf(q[e], d, dot);
                }
            }
        }
        if (row + step < n_rows) fetch(row + step);          // next row in flight during the reductions
        n2 = wave_sum(n2);
        dot = wave_sum(dot);
        if (lane == 0) scores[row] = (n2 > 0.f && !constant_row) ? inv_tau * dot / sqrtf(n2) : 0.f;
    }
}

template <int CHUNKS>
static int launch_score(bool bf16, const void* hidden, int64_t n_rows, int64_t row_stride_bytes, int32_t dim,
                        const float* anchor_q, float inv_tau, float* scores, hipStream_t stream)
{
    // Two 8-wave blocks per CU on 256 CUs; a wavefront loops over its rows with the next row's loads in
    // flight while the current one is reduced, so the vector work overlaps the stream from HBM.
    constexpr int rows_per_block = kScoreThreads / kWave;
    int64_t blocks = (n_rows + rows_per_block - 1) / rows_per_block;
    if (blocks > 256 * kScoreBlocksPerCu) blocks = 256 * kScoreBlocksPerCu;
    const uint8_t* h = static_cast<const uint8_t*>(hidden);
    const size_t lds = sizeof(float) * static_cast<size_t>(dim);
    if (bf16)
        hipLaunchKernelGGL((score_kernel<CHUNKS, true>), dim3(static_cast<unsigned>(blocks)), dim3(kScoreThreads), lds,
                           stream, h, n_rows, row_stride_bytes, dim, anchor_q, inv_tau, scores);
    else
        hipLaunchKernelGGL((score_kernel<CHUNKS, false>), dim3(static_cast<unsigned>(blocks)), dim3(kScoreThreads), lds,
                           stream, h, n_rows, row_stride_bytes, dim, anchor_q, inv_tau, scores);
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
