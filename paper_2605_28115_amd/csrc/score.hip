// civic_score: anchor logit of Eq. 8 for every hidden row.  HBM-bound row reduction.
//
// One wavefront owns a row at a time and fetches it with 16-byte loads (lane l takes chunks l, l+64,
// ...); the anchor is staged once per block in LDS and the wave-wide sums are DPP reductions.
//
// fp32 rows: the row is held in registers, so the centred second pass (norm and dot product of
// x - mean) costs no second trip to memory and has none of the cancellation a one-pass
// sum-of-squares formula would have.  The next row's loads are issued before the reductions.
//
// bf16 rows: at 8 rows per SIMD that two-pass arithmetic (7 vector instructions per element) takes as
// long as the row's trip from HBM, so the common case runs in one pass on the packed words with
// v_dot2c_f32_bf16, two elements per instruction: sum x (against a word of ones), sum x^2 (a word
// against itself) and sum q*x with the anchor split into a bf16 head and a bf16 tail (16 mantissa
// bits).  Then n2 = sum x^2 - N*mean^2 and dot = sum q*x - mean * sum q.  A chunk's register is
// refilled with the next row's chunk as soon as it is consumed.  The one-pass result is only used
// when the subtraction cancels at most one bit (N*mean^2 <= half of sum x^2, i.e. |mean| <= the
// standard deviation); any other row - large offset, constant, Inf/NaN - is re-read (from L2) and
// takes the centred two-pass arithmetic.
#include "civic_internal.h"

namespace civic {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), acc, false);
}

// The 8 bf16 elements of a 16-byte chunk, widened.
__device__ __forceinline__ void unpack_bf16(const u32x4& raw, float* x)
{
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x[2 * i]     = __uint_as_float(w[i] << 16);
        x[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
}

#ifndef CIVIC_SCORE_THREADS
#define CIVIC_SCORE_THREADS 512
#endif
#ifndef CIVIC_SCORE_BLOCKS_PER_CU
#define CIVIC_SCORE_BLOCKS_PER_CU 2
#endif
constexpr int kScoreThreads = CIVIC_SCORE_THREADS;    // wavefronts of a block share one copy of the anchor in LDS
constexpr int kScoreBlocksPerCu = CIVIC_SCORE_BLOCKS_PER_CU;
#ifndef CIVIC_SCORE_WAVES_PER_SIMD
#define CIVIC_SCORE_WAVES_PER_SIMD 4
#endif
constexpr int kScoreWavesPerSimd = CIVIC_SCORE_WAVES_PER_SIMD;   // register budget of the bf16 kernel: 512 / this

// Where the rows of a launch live.  PlainRows: n_rows rows at a uniform stride from `hidden` (grid y = 1).
// SpanRows (civic_score_visual): grid y runs over (batch item, frame); a block scores rows of ONE frame span
// of the dense sequence, so all it needs is that span's first row, found once per block, and the kernels below
// stay what they are: a uniform-stride walk over n_rows = height * width rows.
constexpr int kRaggedSlices = 64;       // frame spans of one ragged launch
struct PlainRows {
    static constexpr bool kSpans = false;
};
struct SpanRows {
    static constexpr bool kSpans = true;
    int32_t frames;                     // per sample
    int32_t hw;                         // tokens per frame
    int64_t seq_len;                    // rows per sample in the dense sequence
    int32_t start[CIVIC_MAX_FRAMES];    // sequence index of each frame's first token
    __device__ __forceinline__ int64_t first_row(uint32_t y) const
    {
        const uint32_t b = y / static_cast<uint32_t>(frames), f = y - b * static_cast<uint32_t>(frames);
        return static_cast<int64_t>(b) * seq_len + start[f];
    }
    __device__ __forceinline__ int64_t out_offset(uint32_t y) const { return static_cast<int64_t>(y) * hw; }
    __device__ __forceinline__ int64_t rows(uint32_t, int64_t n_rows) const { return n_rows; }
};
// RaggedRows (the ragged front): grid y runs over the frames of samples of different grids packed along the token
// axis; every slice brings its own first row, row count and place in the packed scores.
struct RaggedRows {
    static constexpr bool kSpans = true;
    int32_t first[kRaggedSlices], count[kRaggedSlices], out[kRaggedSlices];
    __device__ __forceinline__ int64_t first_row(uint32_t y) const { return first[y]; }
    __device__ __forceinline__ int64_t out_offset(uint32_t y) const { return out[y]; }
    __device__ __forceinline__ int64_t rows(uint32_t y, int64_t) const { return count[y]; }
};

// fp32 rows: two passes over a row held in registers.
template <int CHUNKS, typename MAP>
__global__ __launch_bounds__(kScoreThreads, kScoreBlocksPerCu) void score_f32_kernel(
    const uint8_t* __restrict__ hidden, int64_t n_rows, int64_t row_stride_bytes, int32_t dim,
    const float* __restrict__ anchor_q, float inv_tau, float* __restrict__ scores, MAP map)
{
    if constexpr (MAP::kSpans) {
        hidden += map.first_row(blockIdx.y) * row_stride_bytes;
        scores += map.out_offset(blockIdx.y);
        n_rows = map.rows(blockIdx.y, n_rows);
    }
    constexpr int E = 4;
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
        // Pass 1: row sum, and the exact "no variance" test (every element carries the bits of the first).
        const uint32_t w0 = __builtin_amdgcn_readfirstlane(raw[0].x);
        float sum = 0.f;
        bool same = true;
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) {
            const bool live = (c * kWave + lane) < n_chunks;
            same = same && (!live || (raw[c].x == w0 && raw[c].y == w0 && raw[c].z == w0 && raw[c].w == w0));
            const float x[E] = {__uint_as_float(raw[c].x), __uint_as_float(raw[c].y), __uint_as_float(raw[c].z),
                                __uint_as_float(raw[c].w)};   // dead chunks are zero filled and add nothing
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
                const float x[E] = {__uint_as_float(raw[c].x), __uint_as_float(raw[c].y), __uint_as_float(raw[c].z),
                                    __uint_as_float(raw[c].w)};
                const float4 t = *reinterpret_cast<const float4*>(q_s + ch * E);
                const float q[E] = {t.x, t.y, t.z, t.w};
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

// bf16 rows, one pass on packed words (see the file header).  LDS: q_hi[dim/2] and q_lo[dim/2] words
// (element pairs packed like the row's own words), then the per-wave partial sums of q.
template <int CHUNKS, typename MAP>
__global__ __launch_bounds__(kScoreThreads, kScoreWavesPerSimd) void score_bf16_kernel(
    const uint8_t* __restrict__ hidden, int64_t n_rows, int64_t row_stride_bytes, int32_t dim,
    const float* __restrict__ anchor_q, float inv_tau, float* __restrict__ scores, MAP map)
{
    if constexpr (MAP::kSpans) {
        hidden += map.first_row(blockIdx.y) * row_stride_bytes;
        scores += map.out_offset(blockIdx.y);
        n_rows = map.rows(blockIdx.y, n_rows);
    }
    constexpr int kWaves = kScoreThreads / kWave;
    extern __shared__ __attribute__((aligned(16))) uint32_t q_w[];
    uint32_t* q_hi = q_w;
    uint32_t* q_lo = q_w + dim / 2;
    float* q_part = reinterpret_cast<float*>(q_w + dim);          // [kWaves]
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int n_chunks = dim / 8;
    const float inv_dim = 1.0f / static_cast<float>(dim);
    const int64_t first = static_cast<int64_t>(blockIdx.x) * kWaves + wave;
    const int64_t step = static_cast<int64_t>(gridDim.x) * kWaves;

    u32x4 raw[CHUNKS];
    auto fetch_chunk = [&](int64_t row, int c) {
        const int ch = c * kWave + lane;
        raw[c] = u32x4{0u, 0u, 0u, 0u};                            // a dead chunk adds nothing to any sum
        if (ch < n_chunks) raw[c] = load_streaming(reinterpret_cast<const u32x4*>(hidden + row * row_stride_bytes) + ch);
    };
    if (first < n_rows) {
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) fetch_chunk(first, c);
    }

    // Anchor: head = bf16(q), tail = bf16(q - head), both rounded to nearest even; sum_q is the sum of what the
    // two words represent.
    float q_sum = 0.f;
    for (int i = threadIdx.x * 4; i < dim; i += kScoreThreads * 4) {
        const float4 t = *reinterpret_cast<const float4*>(anchor_q + i);
        const float v[4] = {t.x, t.y, t.z, t.w};
        uint32_t hw[2], lw[2];                                     // packed pairs (v_cvt_pk_bf16_f32 rounds to nearest even)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const bf16x2 hp = {static_cast<__bf16>(v[2 * e]), static_cast<__bf16>(v[2 * e + 1])};
            hw[e] = __builtin_bit_cast(uint32_t, hp);
            const float h0 = __uint_as_float(hw[e] << 16), h1 = __uint_as_float(hw[e] & 0xFFFF0000u);
            const bf16x2 lp = {static_cast<__bf16>(v[2 * e] - h0), static_cast<__bf16>(v[2 * e + 1] - h1)};
            lw[e] = __builtin_bit_cast(uint32_t, lp);
            q_sum += (h0 + __uint_as_float(lw[e] << 16)) + (h1 + __uint_as_float(lw[e] & 0xFFFF0000u));
        }
        *reinterpret_cast<u32x2*>(q_hi + i / 2) = u32x2{hw[0], hw[1]};
        *reinterpret_cast<u32x2*>(q_lo + i / 2) = u32x2{lw[0], lw[1]};
    }
    q_sum = wave_sum(q_sum);
    if (lane == 0) q_part[wave] = q_sum;
    __syncthreads();
    q_sum = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) q_sum += q_part[w];

    constexpr uint32_t kOnes = 0x3F803F80u;                        // two bf16 ones
    for (int64_t row = first; row < n_rows; row += step) {
        const bool more = row + step < n_rows;
        float sum = 0.f, sq = 0.f, dh = 0.f, dl = 0.f;
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) {
            int qw = min(c * kWave + lane, n_chunks - 1) * 4;      // dead chunks read a valid anchor word and multiply it by 0
            asm volatile("" : "+v"(qw));                           // re-read per row: 64 registers of anchor would halve the occupancy
            const u32x4 qh = *reinterpret_cast<const u32x4*>(q_hi + qw);
            const u32x4 ql = *reinterpret_cast<const u32x4*>(q_lo + qw);
            const uint32_t w[4] = {raw[c].x, raw[c].y, raw[c].z, raw[c].w};
            const uint32_t a[4] = {qh.x, qh.y, qh.z, qh.w}, b[4] = {ql.x, ql.y, ql.z, ql.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                sum = dot2_bf16(w[e], kOnes, sum);
                sq = dot2_bf16(w[e], w[e], sq);
                dh = dot2_bf16(w[e], a[e], dh);
                dl = dot2_bf16(w[e], b[e], dl);
            }
            if (more) {
                // The register is free again.  The refill is tied to the sums above so that the chunks are
                // consumed and refilled one after the other, never all 8 fetched into fresh registers.
                int64_t next = row + step;
                asm volatile("" : "+v"(next) : "v"(sum), "v"(sq), "v"(dh), "v"(dl));
                fetch_chunk(next, c);
            }
        }
        sum = wave_sum(sum);
        sq = wave_sum(sq);
        const float qx = wave_sum(dh + dl);
        const float mean = sum * inv_dim;
        float n2 = sq - sum * mean;
        float dot = qx - mean * q_sum;
        if (!(n2 >= 0.5f * sq && sq >= 1e-30f)) {                 // also rows whose squares leave the normal range
            // Centred two passes over the row, re-read chunk by chunk (wave-uniform branch: every
            // operand of the test is a wave-wide sum).
            const u32x4* src = reinterpret_cast<const u32x4*>(hidden + row * row_stride_bytes);
            const uint32_t w0 = __builtin_amdgcn_readfirstlane(src[0].x);
            bool same = (w0 >> 16) == (w0 & 0xFFFFu);
            float s1 = 0.f;
            for (int ch = lane; ch < n_chunks; ch += kWave) {
                const u32x4 r = src[ch];
                same = same && r.x == w0 && r.y == w0 && r.z == w0 && r.w == w0;
                float x[8];
                unpack_bf16(r, x);
#pragma unroll
                for (int e = 0; e < 8; ++e) s1 += x[e];
            }
            const bool constant_row = __ballot(!same) == 0ull;
            const float mean2 = wave_sum(s1) * inv_dim;
            float n2c = 0.f, dotc = 0.f;
            for (int ch = lane; ch < n_chunks; ch += kWave) {
                float x[8], qa[8], qb[8];
                unpack_bf16(src[ch], x);
                unpack_bf16(*reinterpret_cast<const u32x4*>(q_hi + ch * 4), qa);
                unpack_bf16(*reinterpret_cast<const u32x4*>(q_lo + ch * 4), qb);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float d = x[e] - mean2;
                    n2c = fmaf(d, d, n2c);
                    dotc = fmaf(qa[e] + qb[e], d, dotc);
                }
            }
            n2 = constant_row ? 0.f : wave_sum(n2c);
            dot = wave_sum(dotc);
        }
        if (lane == 0) scores[row] = n2 > 0.f ? inv_tau * dot / sqrtf(n2) : 0.f;
    }
}

// n_rows rows per grid-y slice (`slices` of them: 1 for a plain call, batch * frames for the spans of a dense
// sequence).
template <int CHUNKS, typename MAP>
static int launch_score(bool bf16, const void* hidden, int64_t n_rows, int64_t slices, int64_t row_stride_bytes, int32_t dim,
                        const float* anchor_q, float inv_tau, float* scores, const MAP& map, hipStream_t stream)
{
    // Two 8-wave blocks per CU on 256 CUs; a wavefront loops over its rows with the next row's loads in
    // flight while the current one is reduced, so the vector work overlaps the stream from HBM.
    constexpr int rows_per_block = kScoreThreads / kWave;
    int64_t blocks = (n_rows + rows_per_block - 1) / rows_per_block;
    int64_t cap = 256 * kScoreBlocksPerCu / slices;
    if (cap < 1) cap = 1;
    if (blocks > cap) blocks = cap;
    const uint8_t* h = static_cast<const uint8_t*>(hidden);
    const size_t lds = sizeof(float) * static_cast<size_t>(dim);
    const dim3 grid(static_cast<unsigned>(blocks), static_cast<unsigned>(slices));
    if (bf16)
        civic::launch((score_bf16_kernel<CHUNKS, MAP>), grid, dim3(kScoreThreads),
                           lds + sizeof(float) * rows_per_block, stream, h, n_rows, row_stride_bytes, dim, anchor_q,
                           inv_tau, scores, map);
    else
        civic::launch((score_f32_kernel<CHUNKS, MAP>), grid, dim3(kScoreThreads), lds,
                           stream, h, n_rows, row_stride_bytes, dim, anchor_q, inv_tau, scores, map);
    return check_launch();
}

// Shared by civic_score and civic_score_visual once their own arguments are checked.
template <typename MAP>
static int score_rows(const void* hidden, int dtype, int64_t n_rows, int64_t slices, int64_t row_stride, int32_t dim,
                      const float* anchor_q, float inv_tau, float* scores, const MAP& map, void* stream)
{
    const int esz = dtype_size(dtype);
    const int elems = 16 / esz;
    const int chunks = (dim / elems + kWave - 1) / kWave;   // 16-byte chunks per lane
    const bool bf16 = dtype == CIVIC_BF16;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t rsb = row_stride * esz;
#define CIVIC_SCORE_CASE(N) \
    if (chunks <= N) return launch_score<N, MAP>(bf16, hidden, n_rows, slices, rsb, dim, anchor_q, inv_tau, scores, map, s)
    CIVIC_SCORE_CASE(1); CIVIC_SCORE_CASE(2); CIVIC_SCORE_CASE(3); CIVIC_SCORE_CASE(4);
    CIVIC_SCORE_CASE(6); CIVIC_SCORE_CASE(8); CIVIC_SCORE_CASE(12); CIVIC_SCORE_CASE(16);
#undef CIVIC_SCORE_CASE
    return CIVIC_ERR_UNSUPPORTED;
}

}  // namespace civic

extern "C" int civic_score(const void* hidden, int dtype, int64_t n_rows, int64_t row_stride, int32_t dim,
                           const float* anchor_q, float inv_tau, float* scores, void* stream)
{
    using namespace civic;
    const int esz = dtype_size(dtype);
    if (!esz || !anchor_q) return CIVIC_ERR_INVALID_ARG;
    if (n_rows < 0 || dim <= 0 || row_stride < dim) return CIVIC_ERR_INVALID_ARG;
    if (n_rows > 0 && (!hidden || !scores)) return CIVIC_ERR_INVALID_ARG;   // no rows: nothing to point at
    const int elems = 16 / esz;
    if (dim % elems) return CIVIC_ERR_INVALID_ARG;
    if (!aligned16(hidden) || !aligned16(anchor_q) || (row_stride * esz) % 16) return CIVIC_ERR_INVALID_ARG;
    if (!(inv_tau == inv_tau)) return CIVIC_ERR_INVALID_ARG;
    if (static_cast<int64_t>(dim) * esz > static_cast<int64_t>(CIVIC_MAX_SCORE_DIM) * 2) return CIVIC_ERR_UNSUPPORTED;
    if (n_rows == 0) return CIVIC_OK;

    return score_rows(hidden, dtype, n_rows, 1, row_stride, dim, anchor_q, inv_tau, scores, PlainRows{}, stream);
}

namespace civic {

// The argument checks of civic_score_visual (host only, nothing is launched).
int score_visual_check(const void* hidden, int dtype, int32_t batch, int64_t seq_len, int32_t dim, const civic_grid* grid,
                       const int64_t* frame_start, const float* anchor_q, float inv_tau, const float* scores)
{
    const int esz = dtype_size(dtype);
    GridInfo gi;
    if (grid_info(grid, &gi) != CIVIC_OK) return CIVIC_ERR_INVALID_ARG;
    if (!esz || !anchor_q || !frame_start) return CIVIC_ERR_INVALID_ARG;
    if (batch < 0 || dim <= 0 || seq_len < gi.nv) return CIVIC_ERR_INVALID_ARG;
    if (batch > 0 && (!hidden || !scores)) return CIVIC_ERR_INVALID_ARG;
    int64_t prev_end = 0;
    for (int32_t f = 0; f < gi.frames; ++f) {
        if (frame_start[f] < prev_end || frame_start[f] + gi.hw > seq_len) return CIVIC_ERR_INVALID_ARG;
        prev_end = frame_start[f] + gi.hw;
    }
    const int elems = 16 / esz;
    if (dim % elems) return CIVIC_ERR_INVALID_ARG;
    if (!aligned16(hidden) || !aligned16(anchor_q)) return CIVIC_ERR_INVALID_ARG;
    if (!(inv_tau == inv_tau)) return CIVIC_ERR_INVALID_ARG;
    if (static_cast<int64_t>(dim) * esz > static_cast<int64_t>(CIVIC_MAX_SCORE_DIM) * 2) return CIVIC_ERR_UNSUPPORTED;
    const int64_t slices = static_cast<int64_t>(batch) * gi.frames;
    if (gi.frames > CIVIC_MAX_FRAMES || seq_len > INT32_MAX || slices > 65535) return CIVIC_ERR_UNSUPPORTED;
    return CIVIC_OK;
}

// The frames of `n_slices` (<= kRaggedSlices) spans of a packed tensor in one launch: slice i is `count[i]` rows from
// row `first[i]`, scored into scores[out[i] ..]; `longest` is the largest count.  Arguments checked by the caller.
int score_slices_launch(const void* hidden, int dtype, int32_t dim, const float* anchor_q, float inv_tau, float* scores,
                        const int32_t* first, const int32_t* count, const int32_t* out, int32_t n_slices, int32_t longest, void* stream)
{
    RaggedRows map;
    for (int i = 0; i < kRaggedSlices; ++i) {
        map.first[i] = i < n_slices ? first[i] : 0;
        map.count[i] = i < n_slices ? count[i] : 0;
        map.out[i] = i < n_slices ? out[i] : 0;
    }
    return score_rows(hidden, dtype, longest, n_slices, dim, dim, anchor_q, inv_tau, scores, map, stream);
}

}  // namespace civic

extern "C" int civic_score_visual(const void* hidden, int dtype, int32_t batch, int64_t seq_len, int32_t dim,
                                  const civic_grid* grid, const int64_t* frame_start, const float* anchor_q,
                                  float inv_tau, float* scores, void* stream)
{
    using namespace civic;
    const int rc = score_visual_check(hidden, dtype, batch, seq_len, dim, grid, frame_start, anchor_q, inv_tau, scores);
    if (rc != CIVIC_OK) return rc;
    if (batch == 0) return CIVIC_OK;
    GridInfo gi;
    grid_info(grid, &gi);
    const int64_t slices = static_cast<int64_t>(batch) * gi.frames;
    SpanRows map;
    map.frames = gi.frames; map.hw = gi.hw; map.seq_len = seq_len;
    for (int32_t f = 0; f < CIVIC_MAX_FRAMES; ++f) map.start[f] = f < gi.frames ? static_cast<int32_t>(frame_start[f]) : 0;
    return score_rows(hidden, dtype, gi.hw, slices, dim, dim, anchor_q, inv_tau, scores, map, stream);
}
