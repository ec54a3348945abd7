// civic_select: exact constrained top-k (cell floors, frame floors, global budget) with ascending,
// order-preserving output.  Latency-bound: a sample's scores are 8-128 KB.
//
// One 1024-thread workgroup per sample keeps everything in LDS: a 32-bit sort key per token and one
// mark bit per token.  The strict order "higher score first, equal scores to the lower index" becomes
// (key ascending, index ascending) after mapping the float bits to an unsigned key (with -0 folded
// onto +0).
//   cells   small cells: every token counts the members of its cell that precede it (all pairs in
//           LDS); the wavefront ballot of "rank < floor" IS the 64-bit mark word of those 64 tokens.
//           large cells: one wavefront per cell runs the radix select below.
//   frames  one wavefront per frame: radix select (4 passes of 8 bits over a per-wave LDS histogram)
//           finds the key of the frame_floor-th unmarked token; equal keys are admitted in index
//           order with ballot prefix counts.
//   budget  the same radix select run by the whole workgroup over the unmarked tokens of the sample.
//   output  popcounts of the 64-bit mark words -> LDS prefix scan -> every set bit writes its index
//           at (prefix of its word + set bits below it): ascending kept_idx without any sort.
#include "civic_internal.h"

namespace civic {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kSmallCell = 256;        // cells up to this many tokens use the all-pairs rank

struct SelArgs {
    const float* scores;
    int32_t* kept_idx;
    uint8_t* keep_flags;
    int32_t frames, height, width, hw, nv, nv_pad;
    int32_t cell_h, cell_w, cell_floor, frame_floor;
    int32_t cells_y, cells_x;
    int32_t fill;          // tokens the global budget adds after the floors
    int32_t kept;          // K
    int32_t big_cells;     // 1: cells go through the per-wave radix select
};

__device__ __forceinline__ uint32_t order_key(float s)
{
    uint32_t u = __float_as_uint(s);
    if (u == 0x80000000u) u = 0u;                               // -0 ties with +0
    const uint32_t asc = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return ~asc;                                                 // higher score -> smaller key
}

// A rectangle of one frame in raster order: token i -> base + (i / w) * pitch + i % w.
struct Region {
    int32_t base, w, pitch, count;
    __device__ __forceinline__ int32_t token(int32_t i) const { return base + (i / w) * pitch + (i % w); }
};

__device__ __forceinline__ bool is_marked(const uint32_t* marks, int32_t v) { return (marks[v >> 5] >> (v & 31)) & 1u; }
__device__ __forceinline__ void set_mark(uint32_t* marks, int32_t v) { atomicOr(&marks[v >> 5], 1u << (v & 31)); }

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v, int lane)
{
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t t = __shfl_up(v, off, kWave);
        if (lane >= off) v += t;
    }
    return v;
}

// Orders LDS traffic of the team: a workgroup barrier, or for a single wavefront (whose LDS
// operations already execute in program order) a compiler-level fence.
template <bool BLOCK>
__device__ __forceinline__ void team_sync()
{
    if constexpr (BLOCK) {
        __syncthreads();
    } else {
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

// Marks the first m tokens, in (key, index) order, among the eligible tokens of `reg`; eligible means
// not marked yet when only_unmarked is set.  Run by one wavefront (BLOCK = false) or by the whole
// workgroup (BLOCK = true; every thread must call it with the same arguments).
//   hist  256 counters owned by the team;  bc  4 words owned by the team.
template <bool BLOCK>
__device__ void select_first(const uint32_t* keys, uint32_t* marks, uint32_t* hist, uint32_t* bc, const Region reg,
                             int32_t m, bool only_unmarked)
{
    constexpr int TEAM = BLOCK ? kSelThreads : kWave;
    const int rank = BLOCK ? threadIdx.x : (threadIdx.x & (kWave - 1));
    const int lane = threadIdx.x & (kWave - 1);
    const int32_t n_iter = (reg.count + TEAM - 1) / TEAM;
    if (m <= 0) return;

    // eligible count
    if (rank == 0) bc[0] = 0;
    team_sync<BLOCK>();
    for (int32_t it = 0; it < n_iter; ++it) {
        const int32_t i = it * TEAM + rank;
        bool e = false;
        if (i < reg.count) { const int32_t v = reg.token(i); e = !(only_unmarked && is_marked(marks, v)); }
        const uint64_t bal = __ballot(e);
        if (lane == 0 && bal) atomicAdd(&bc[0], static_cast<uint32_t>(__popcll(bal)));
    }
    team_sync<BLOCK>();
    const int32_t eligible = static_cast<int32_t>(bc[0]);
    team_sync<BLOCK>();
    if (m >= eligible) {                                         // floor covers everything that is left
        for (int32_t it = 0; it < n_iter; ++it) {
            const int32_t i = it * TEAM + rank;
            if (i < reg.count) { const int32_t v = reg.token(i); if (!(only_unmarked && is_marked(marks, v))) set_mark(marks, v); }
        }
        team_sync<BLOCK>();
        return;
    }

    // Radix select of the m-th smallest key among the eligible tokens: 4 digits of 8 bits, high first.
    uint32_t prefix = 0, remaining = static_cast<uint32_t>(m), ties = 0;
#pragma unroll 1
    for (int shift = 24; shift >= 0; shift -= 8) {
        for (int i = rank; i < 256; i += TEAM) hist[i] = 0;
        team_sync<BLOCK>();
        const uint32_t hi_mask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
        for (int32_t it = 0; it < n_iter; ++it) {
            const int32_t i = it * TEAM + rank;
            if (i < reg.count) {
                const int32_t v = reg.token(i);
                const uint32_t k = keys[v];
                if (!(only_unmarked && is_marked(marks, v)) && (k & hi_mask) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1u);
            }
        }
        team_sync<BLOCK>();
        if (!BLOCK || threadIdx.x < kWave) {                     // one wavefront scans the 256 bins
            uint32_t c[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) c[t] = hist[lane * 4 + t];
            const uint32_t mine = c[0] + c[1] + c[2] + c[3];
            const uint32_t incl = wave_incl_scan(mine, lane);
            uint32_t before = incl - mine;
            if (before < remaining && remaining <= incl) {       // exactly one lane
                int t = 0;
                while (before + c[t] < remaining) { before += c[t]; ++t; }
                bc[0] = static_cast<uint32_t>(lane * 4 + t);       // digit
                bc[1] = before;                                   // eligible tokens below that digit
                bc[2] = c[t];                                     // tokens with that digit
            }
        }
        team_sync<BLOCK>();
        prefix |= bc[0] << shift;
        remaining -= bc[1];
        ties = bc[2];
        team_sync<BLOCK>();
    }
    // prefix is now the threshold key; `remaining` of the `ties` tokens that carry it are admitted.

    if (ties == remaining) {                                     // no contested tie: order does not matter
        for (int32_t it = 0; it < n_iter; ++it) {
            const int32_t i = it * TEAM + rank;
            if (i < reg.count) {
                const int32_t v = reg.token(i);
                if (!(only_unmarked && is_marked(marks, v)) && keys[v] <= prefix) set_mark(marks, v);
            }
        }
        team_sync<BLOCK>();
        return;
    }

    // Contested tie: admit equal keys in index order.  Tokens are visited in ascending index; the
    // ballot prefix inside a wavefront plus a running count across wavefronts gives each its rank.
    uint32_t running = 0;
    uint32_t* wave_cnt = hist;                                   // reuse: kSelWaves counters
    for (int32_t it = 0; it < n_iter; ++it) {
        const int32_t i = it * TEAM + rank;
        bool eq = false;
        int32_t v = 0;
        if (i < reg.count) {
            v = reg.token(i);
            if (!(only_unmarked && is_marked(marks, v))) {
                const uint32_t k = keys[v];
                if (k < prefix) set_mark(marks, v);
                eq = k == prefix;
            }
        }
        const uint64_t bal = __ballot(eq);
        uint32_t below = static_cast<uint32_t>(__popcll(bal & ((1ull << lane) - 1ull)));
        if constexpr (BLOCK) {
            const int w = threadIdx.x >> 6;
            if (lane == 0) wave_cnt[w] = static_cast<uint32_t>(__popcll(bal));
            __syncthreads();
            uint32_t tile_total = 0;
            for (int x = 0; x < kSelWaves; ++x) { const uint32_t cx = wave_cnt[x]; if (x < w) below += cx; tile_total += cx; }
            __syncthreads();
            if (eq && running + below < remaining) set_mark(marks, v);
            running += tile_total;
        } else {
            if (eq && running + below < remaining) set_mark(marks, v);
            running += static_cast<uint32_t>(__popcll(bal));
        }
    }
    team_sync<BLOCK>();
}

__global__ __launch_bounds__(kSelThreads) void select_kernel(SelArgs a)
{
    extern __shared__ uint32_t smem[];
    uint32_t* keys = smem;                                   // [nv_pad]
    uint32_t* marks = keys + a.nv_pad;                       // [nv_pad / 32]
    uint32_t* hist = marks + a.nv_pad / 32;                  // [kSelWaves][256]
    uint32_t* bcast = hist + kSelWaves * 256;                // [kSelWaves][4]
    uint32_t* word_prefix = bcast + kSelWaves * 4;           // [nv_pad / 64]

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int b = blockIdx.x;
    const float* s = a.scores + static_cast<int64_t>(b) * a.nv;

    for (int32_t v = tid; v < a.nv_pad; v += kSelThreads) keys[v] = v < a.nv ? order_key(s[v]) : 0xFFFFFFFFu;
    for (int32_t w = tid; w < a.nv_pad / 32; w += kSelThreads) marks[w] = 0u;
    __syncthreads();

    // ---- (1) cell floors
    if (a.cell_floor > 0) {
        if (!a.big_cells) {
            for (int32_t v0 = 0; v0 < a.nv_pad; v0 += kSelThreads) {
                const int32_t v = v0 + tid;
                bool mark = false;
                if (v < a.nv) {
                    const int32_t f = v / a.hw, rem = v - f * a.hw;
                    const int32_t r = rem / a.width, c = rem - r * a.width;
                    const int32_t r0 = (r / a.cell_h) * a.cell_h, c0 = (c / a.cell_w) * a.cell_w;
                    const int32_t r1 = min(r0 + a.cell_h, a.height), c1 = min(c0 + a.cell_w, a.width);
                    if ((r1 - r0) * (c1 - c0) <= a.cell_floor) {
                        mark = true;
                    } else {
                        const uint32_t kv = keys[v];
                        int32_t ahead = 0;
                        for (int32_t rr = r0; rr < r1; ++rr) {
                            const int32_t u0 = f * a.hw + rr * a.width;
                            for (int32_t cc = c0; cc < c1; ++cc) {
                                const uint32_t ku = keys[u0 + cc];
                                ahead += (ku < kv || (ku == kv && u0 + cc < v)) ? 1 : 0;
                            }
                        }
                        mark = ahead < a.cell_floor;
                    }
                }
                const uint64_t bal = __ballot(mark);
                if (lane == 0 && v < a.nv_pad) {
                    marks[v >> 5] = static_cast<uint32_t>(bal);
                    marks[(v >> 5) + 1] = static_cast<uint32_t>(bal >> 32);
                }
            }
        } else {
            const int32_t cells = a.frames * a.cells_y * a.cells_x;
            for (int32_t cell = wave; cell < cells; cell += kSelWaves) {
                const int32_t f = cell / (a.cells_y * a.cells_x), rem = cell - f * a.cells_y * a.cells_x;
                const int32_t cy = rem / a.cells_x, cx = rem - cy * a.cells_x;
                const int32_t r0 = cy * a.cell_h, c0 = cx * a.cell_w;
                const int32_t hgt = min(a.cell_h, a.height - r0), wid = min(a.cell_w, a.width - c0);
                const Region reg{f * a.hw + r0 * a.width + c0, wid, a.width, hgt * wid};
                select_first<false>(keys, marks, hist + wave * 256, bcast + wave * 4, reg, a.cell_floor, false);
            }
        }
        __syncthreads();
    }

    // ---- (2) frame floors
    if (a.frame_floor > 0) {
        for (int32_t f = wave; f < a.frames; f += kSelWaves) {
            const Region reg{f * a.hw, a.hw, a.hw, a.hw};
            select_first<false>(keys, marks, hist + wave * 256, bcast + wave * 4, reg, a.frame_floor, true);
        }
        __syncthreads();
    }

    // ---- (3) global budget
    if (a.fill > 0) {
        const Region reg{0, a.nv, a.nv, a.nv};
        select_first<true>(keys, marks, hist, bcast, reg, a.fill, true);
    }
    __syncthreads();

    // ---- (4) ascending output
    const int32_t words = a.nv_pad / 64;                     // <= 512, one per thread
    uint32_t pc = 0;
    if (tid < words) pc = __popc(marks[2 * tid]) + __popc(marks[2 * tid + 1]);
    const uint32_t incl = wave_incl_scan(pc, lane);
    if (lane == kWave - 1) bcast[wave] = incl;
    __syncthreads();
    uint32_t wave_base = 0;
    for (int x = 0; x < wave; ++x) wave_base += bcast[x];
    if (tid < words) word_prefix[tid] = wave_base + incl - pc;
    __syncthreads();

    int32_t* out = a.kept_idx + static_cast<int64_t>(b) * a.kept;
    for (int32_t v = tid; v < a.nv_pad; v += kSelThreads) {
        const uint32_t lo = marks[(v >> 6) * 2], hi = marks[(v >> 6) * 2 + 1];
        const uint64_t word = (static_cast<uint64_t>(hi) << 32) | lo;
        const bool bit = (word >> lane) & 1ull;
        if (bit) {
            const uint32_t pos = word_prefix[v >> 6] + static_cast<uint32_t>(__popcll(word & ((1ull << lane) - 1ull)));
            if (pos < static_cast<uint32_t>(a.kept)) out[pos] = v;
        }
        if (a.keep_flags && v < a.nv) a.keep_flags[static_cast<int64_t>(b) * a.nv + v] = bit ? 1 : 0;
    }
}

}  // namespace civic

extern "C" int civic_select(const float* scores, int32_t batch, const civic_grid* grid, int32_t* kept_idx,
                            uint8_t* keep_flags, void* workspace, size_t workspace_bytes, void* stream)
{
    using namespace civic;
    (void)workspace; (void)workspace_bytes;
    GridInfo gi;
    if (grid_info(grid, &gi) != CIVIC_OK) return CIVIC_ERR_INVALID_ARG;
    if (!scores || batch < 0) return CIVIC_ERR_INVALID_ARG;
    if (gi.kept > 0 && !kept_idx) return CIVIC_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(scores) | reinterpret_cast<uintptr_t>(kept_idx)) & 3u) return CIVIC_ERR_INVALID_ARG;
    if (gi.nv > CIVIC_MAX_VISUAL_TOKENS) return CIVIC_ERR_UNSUPPORTED;
    if (batch == 0) return CIVIC_OK;

    SelArgs a;
    a.scores = scores; a.kept_idx = kept_idx; a.keep_flags = keep_flags;
    a.frames = gi.frames; a.height = gi.height; a.width = gi.width; a.hw = gi.hw; a.nv = gi.nv;
    a.nv_pad = (gi.nv + 63) / 64 * 64;
    a.cell_h = gi.cell_h < gi.height ? gi.cell_h : gi.height;
    a.cell_w = gi.cell_w < gi.width ? gi.cell_w : gi.width;
    a.cell_floor = gi.cell_floor; a.frame_floor = gi.frame_floor;
    a.cells_y = (gi.height + a.cell_h - 1) / a.cell_h;
    a.cells_x = (gi.width + a.cell_w - 1) / a.cell_w;
    a.fill = gi.fill; a.kept = gi.kept;
    a.big_cells = static_cast<int64_t>(a.cell_h) * a.cell_w > kSmallCell ? 1 : 0;

    const size_t lds = sizeof(uint32_t) * (static_cast<size_t>(a.nv_pad) + a.nv_pad / 32 + kSelWaves * 256 +
                                           kSelWaves * 4 + a.nv_pad / 64 + 2);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(select_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (e != hipSuccess) return record_hip_error(e);
    }
    hipLaunchKernelGGL(select_kernel, dim3(static_cast<unsigned>(batch)), dim3(kSelThreads), lds, s, a);
    return check_launch();
}
