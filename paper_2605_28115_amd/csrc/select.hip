// civic_select: exact constrained top-k (cell floors, frame floors, global budget) with ascending,
// order-preserving output.  Latency-bound: a sample's scores are 8-128 KB.
//
// One 1024-thread workgroup per sample keeps everything in LDS: a 32-bit sort key per token and one
// mark bit per token.  The strict order "higher score first, equal scores to the lower index" becomes
// (key ascending, index ascending) after mapping the float bits to an unsigned key (with -0 folded
// onto +0).
//   cells   small cells: one thread per cell picks the cell's best remaining member cell_floor times
//           (members scanned in index order, strict key comparison = the tie rule).
//           large cells: one wavefront per cell runs the radix select below.
//   frames  one wavefront per frame: radix select (digits of 8 bits, high first, over a per-wave LDS
//           histogram) finds the key of the frame_floor-th unmarked token; equal keys are admitted
//           in index order with ballot prefix counts.
//   budget  the same radix select run by the whole workgroup over the unmarked tokens of the sample,
//           with digits of 11 bits.  A select stops after the first digit whose bin is admitted
//           whole (typically the second of three), because the threshold's low bits no longer matter.
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
    int32_t floor_sum;     // tokens the floors protect
    int32_t fill;          // tokens the global budget adds after the floors
    int32_t kept;          // K
    int32_t big_cells;     // 1: cells go through the per-wave radix select
    uint32_t magic_cells_f, magic_cells_x;   // ceil(2^32 / d) for d = cells per frame, cells per grid row (0 for d = 1)
};

// n / d for 0 <= n, n * d < 2^32, with magic = ceil(2^32 / d) for d >= 2 and magic = 0 for d = 1.
__device__ __forceinline__ int32_t div_magic(int32_t n, uint32_t magic)
{
    return magic ? static_cast<int32_t>(__umulhi(static_cast<uint32_t>(n), magic)) : n;
}

__device__ __forceinline__ uint32_t order_key(float s)
{
    uint32_t u = __float_as_uint(s);
    if (u == 0x80000000u) u = 0u;                               // -0 ties with +0
    const uint32_t asc = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return ~asc;                                                 // higher score -> smaller key
}

// A rectangle of one frame in raster order: token i -> base + (i / w) * pitch + i % w.  CONTIG: the
// rectangle spans whole grid rows (w == pitch), so token i is simply base + i.
struct Region {
    int32_t base, w, pitch, count;
    template <bool CONTIG>
    __device__ __forceinline__ int32_t token(int32_t i) const
    {
        if constexpr (CONTIG) return base + i;
        else return base + (i / w) * pitch + (i % w);
    }
};

__device__ __forceinline__ bool is_marked(const uint32_t* marks, int32_t v) { return (marks[v >> 5] >> (v & 31)) & 1u; }
__device__ __forceinline__ void set_mark(uint32_t* marks, int32_t v) { atomicOr(&marks[v >> 5], 1u << (v & 31)); }

// Inclusive prefix sum over the 64 lanes with DPP adds: scan inside each row of 16 lanes (row_shr 1, 2,
// 4, 8; lanes without a source keep their value), then carry row totals forward (row_bcast 15 into rows
// 1 and 3, row_bcast 31 into rows 2 and 3).
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v, int)
{
    auto step = [](uint32_t x, auto ctrl, auto row_mask) {
        return x + static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), decltype(ctrl)::value,
                                                                      decltype(row_mask)::value, 0xF, false));
    };
    using std::integral_constant;
    v = step(v, integral_constant<int, 0x111>{}, integral_constant<int, 0xF>{});
    v = step(v, integral_constant<int, 0x112>{}, integral_constant<int, 0xF>{});
    v = step(v, integral_constant<int, 0x114>{}, integral_constant<int, 0xF>{});
    v = step(v, integral_constant<int, 0x118>{}, integral_constant<int, 0xF>{});
    v = step(v, integral_constant<int, 0x142>{}, integral_constant<int, 0xA>{});
    v = step(v, integral_constant<int, 0x143>{}, integral_constant<int, 0xC>{});
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
// workgroup (BLOCK = true; every thread must call it with the same arguments, and `eligible` must be
// given).  eligible < 0 (wavefront only): counted here.
//   hist  counters owned by the team: 2 x 2048 for the workgroup (double buffered, so the next pass's
//         clear hides behind the scan; both must be zero on entry and are left dirty), 256 for a
//         wavefront (cleared here, left zero);  bc  8 words owned by the team, 16 for the workgroup.
template <bool BLOCK, bool CONTIG>
__device__ void select_first(const uint32_t* keys, uint32_t* marks, uint32_t* hist, uint32_t* bc, const Region reg,
                             int32_t m, bool only_unmarked, int32_t eligible)
{
    constexpr int TEAM = BLOCK ? kSelThreads : kWave;
    const int rank = BLOCK ? threadIdx.x : (threadIdx.x & (kWave - 1));
    const int lane = threadIdx.x & (kWave - 1);
    const int32_t n_iter = (reg.count + TEAM - 1) / TEAM;
    if (m <= 0) return;

    if (!BLOCK && eligible < 0) {                                // wave-uniform count from ballots
        eligible = 0;
        for (int32_t it = 0; it < n_iter; ++it) {
            const int32_t i = it * TEAM + rank;
            bool e = false;
            if (i < reg.count) { const int32_t v = reg.token<CONTIG>(i); e = !(only_unmarked && is_marked(marks, v)); }
            eligible += __popcll(__ballot(e));
        }
    }
    if (m >= eligible) {                                         // floor covers everything that is left
        for (int32_t it = 0; it < n_iter; ++it) {
            const int32_t i = it * TEAM + rank;
            if (i < reg.count) { const int32_t v = reg.token<CONTIG>(i); if (!(only_unmarked && is_marked(marks, v))) set_mark(marks, v); }
        }
        team_sync<BLOCK>();
        return;
    }

    // Radix select of the m-th smallest key among the eligible tokens, high digit first.
    constexpr int BITS = BLOCK ? 11 : 8;
    constexpr int BINS = 1 << BITS;
    constexpr int PASSES = (32 + BITS - 1) / BITS;
    constexpr int CH = BINS / 256;                               // the scanning wavefront takes 4 bins per lane and chunk
    static_assert(CH <= 8, "chunk totals are read as two quads");
    if constexpr (!BLOCK) {                                      // the workgroup's histograms are clear on entry (see the kernel)
        for (int i = rank; i < BINS; i += TEAM) hist[i] = 0;
        team_sync<false>();
    }
    uint32_t prefix = 0, remaining = static_cast<uint32_t>(m), ties = 0;
    int done_shift = 0;                                          // key bits below this were never looked at
#pragma unroll 1
    for (int pass = 0; pass < PASSES; ++pass) {
        const int shift = 32 - BITS * (pass + 1) > 0 ? 32 - BITS * (pass + 1) : 0;
        const int width = 32 - BITS * pass < BITS ? 32 - BITS * pass : BITS;
        const uint32_t digit_mask = (1u << width) - 1u;
        uint32_t* h = hist + (BLOCK ? (pass & 1) * BINS : 0);
        const uint32_t hi_mask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + width));
        for (int32_t it = 0; it < n_iter; ++it) {
            const int32_t i = it * TEAM + rank;
            if (i < reg.count) {
                const int32_t v = reg.token<CONTIG>(i);
                const uint32_t k = keys[v];
                if ((k & hi_mask) == prefix && !(only_unmarked && is_marked(marks, v))) atomicAdd(&h[(k >> shift) & digit_mask], 1u);
            }
        }
        team_sync<BLOCK>();
        // Scan: every 256-bin chunk has a wavefront of its own (4 bins per lane); the workgroup-wide
        // select passes the chunk totals through bc[8..].
        const int chunk = BLOCK ? static_cast<int>(threadIdx.x >> 6) : 0;
        const bool scanner = chunk < CH;
        uint32_t c[4] = {0u, 0u, 0u, 0u}, mine = 0, incl = 0, base = 0;
        if (scanner) {
            const u32x4 t = *reinterpret_cast<const u32x4*>(h + chunk * 256 + lane * 4);
            c[0] = t.x; c[1] = t.y; c[2] = t.z; c[3] = t.w;
            mine = t.x + t.y + t.z + t.w;
            incl = wave_incl_scan(mine, lane);
        }
        if constexpr (BLOCK) {
            if (scanner) {
                if (lane == kWave - 1) bc[8 + chunk] = incl;
            } else {
                // meanwhile the other wavefronts clear the other histogram for the next pass
                for (int i = threadIdx.x - CH * kWave; i < BINS; i += kSelThreads - CH * kWave) hist[((pass + 1) & 1) * BINS + i] = 0;
            }
            __syncthreads();
            if (scanner) {
                const u32x4 t0 = *reinterpret_cast<const u32x4*>(bc + 8), t1 = *reinterpret_cast<const u32x4*>(bc + 12);
                const uint32_t tot[8] = {t0.x, t0.y, t0.z, t0.w, t1.x, t1.y, t1.z, t1.w};
#pragma unroll
                for (int x = 0; x < CH; ++x) base += x < chunk ? tot[x] : 0u;
            }
        }
        if (scanner) {
            uint32_t before = base + incl - mine;
            if (before < remaining && remaining <= base + incl) {   // exactly one lane of one chunk
                int t = 0;
                while (before + c[t] < remaining) { before += c[t]; ++t; }
                bc[(pass & 1) * 4 + 0] = static_cast<uint32_t>(chunk * 256 + lane * 4 + t);   // digit
                bc[(pass & 1) * 4 + 1] = before;                                                // eligible tokens below that digit
                bc[(pass & 1) * 4 + 2] = c[t];                                                  // tokens with that digit
            }
        }
        if constexpr (BLOCK) {
            __syncthreads();
        } else {
            team_sync<false>();
            for (int i = lane; i < BINS; i += kWave) hist[i] = 0;     // a wavefront orders its own LDS traffic for free
            team_sync<false>();
        }
        prefix |= bc[(pass & 1) * 4 + 0] << shift;
        remaining -= bc[(pass & 1) * 4 + 1];
        ties = bc[(pass & 1) * 4 + 2];
        done_shift = shift;
        if (ties == remaining) break;                            // the whole bin is admitted: its lower bits decide nothing
    }
    // prefix (above done_shift) is now the threshold; `remaining` of the `ties` tokens that carry it are admitted.

    if (ties == remaining) {                                     // no contested tie: order does not matter
        const uint32_t limit = prefix >> done_shift;
        if (BLOCK && CONTIG && (reg.base & (kWave - 1)) == 0) {
            // A wavefront covers 64 consecutive tokens = its own two mark words: one ballot, no atomics.
            for (int32_t it = 0; it < n_iter; ++it) {
                const int32_t i = it * TEAM + rank;
                const int32_t v = reg.base + i;
                const bool admit = i < reg.count && !(only_unmarked && is_marked(marks, v)) && (keys[v] >> done_shift) <= limit;
                const uint64_t bal = __ballot(admit);
                if (lane == 0 && bal) {                          // i - lane < reg.count here, so the words exist
                    marks[v >> 5] |= static_cast<uint32_t>(bal);
                    marks[(v >> 5) + 1] |= static_cast<uint32_t>(bal >> 32);
                }
            }
        } else {
            for (int32_t it = 0; it < n_iter; ++it) {
                const int32_t i = it * TEAM + rank;
                if (i < reg.count) {
                    const int32_t v = reg.token<CONTIG>(i);
                    if (!(only_unmarked && is_marked(marks, v)) && (keys[v] >> done_shift) <= limit) set_mark(marks, v);
                }
            }
        }
        team_sync<BLOCK>();
        return;
    }

    // Contested tie: admit equal keys in index order.  Tokens are visited in ascending index; the
    // ballot prefix inside a wavefront plus a running count across wavefronts gives each its rank.
    uint32_t running = 0;
    uint32_t* wave_cnt = hist;                                   // reuse: kSelWaves counters
    team_sync<BLOCK>();
    for (int32_t it = 0; it < n_iter; ++it) {
        const int32_t i = it * TEAM + rank;
        bool eq = false;
        int32_t v = 0;
        if (i < reg.count) {
            v = reg.token<CONTIG>(i);
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
    extern __shared__ __attribute__((aligned(16))) uint32_t smem[];
    uint32_t* keys = smem;                                   // [nv_pad]; this and the next start on 16-byte boundaries
    uint32_t* hist = keys + a.nv_pad;                        // [kSelWaves][256]; the workgroup-wide select uses all of it as 2 x 2048
    uint32_t* bcast = hist + kSelWaves * 256;                // [kSelWaves][8]
    uint32_t* marks = bcast + kSelWaves * 8;                 // [nv_pad / 32]
    uint32_t* word_prefix = marks + a.nv_pad / 32;           // [nv_pad / 64]

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int b = blockIdx.x;
    const float* s = a.scores + static_cast<int64_t>(b) * a.nv;

    for (int32_t v = tid; v < a.nv_pad; v += kSelThreads) keys[v] = v < a.nv ? order_key(s[v]) : 0xFFFFFFFFu;
    for (int32_t w = tid; w < a.nv_pad / 32; w += kSelThreads) marks[w] = 0u;
    // The budget select wants zeroed histograms; the per-wavefront selects before it leave theirs zeroed.
    for (int i = tid; i < kSelWaves * 256; i += kSelThreads) hist[i] = 0u;
    __syncthreads();

    // ---- (1) cell floors
    if (a.cell_floor > 0) {
        if (!a.big_cells) {
            // One thread per cell: cell_floor rounds of "best member after the previous winner".  Members
            // are scanned in ascending index with a strict key comparison, which is the tie rule.  The
            // work is cells * floor * size instead of tokens * size for an all-pairs rank.
            const int32_t cells_f = a.cells_y * a.cells_x, cells = a.frames * cells_f;
            const bool quad_rows = (a.cell_w & 3) == 0 && a.cells_x * a.cell_w == a.width;   // every cell row is made of aligned quads of keys
            for (int32_t cell = tid; cell < cells; cell += kSelThreads) {
                const int32_t f = div_magic(cell, a.magic_cells_f), rem = cell - f * cells_f;
                const int32_t cy = div_magic(rem, a.magic_cells_x), cx = rem - cy * a.cells_x;
                const int32_t r0 = cy * a.cell_h, c0 = cx * a.cell_w;
                const int32_t r1 = min(r0 + a.cell_h, a.height), c1 = min(c0 + a.cell_w, a.width);
                const int32_t base = f * a.hw;
                const int32_t rounds = min(a.cell_floor, (r1 - r0) * (c1 - c0));
                uint32_t last_key = 0;
                int32_t last_idx = -1;                             // nothing chosen yet
                for (int32_t k = 0; k < rounds; ++k) {
                    uint32_t best_key = 0xFFFFFFFFu;
                    int32_t best_idx = -1;
                    if (quad_rows) {
                        // The cell as a row-major list of aligned quads of keys, four 16-byte LDS reads
                        // at a time (consecutive cells read consecutive quads, so a wavefront's reads do
                        // not collide on banks).  The first round has no previous winner to stay behind.
                        auto scan = [&](auto first_round) {
                            const int32_t qpr = a.cell_w >> 2, quads = (r1 - r0) * qpr;
                            int32_t row_u = base + r0 * a.width + c0, q = 0;        // next quad: row start, quad in row
                            for (int32_t t0 = 0; t0 < quads; t0 += 4) {
                                u32x4 kv[4];
                                int32_t u0[4];
#pragma unroll
                                for (int z = 0; z < 4; ++z) {
                                    u0[z] = row_u + 4 * q;
                                    kv[z] = *reinterpret_cast<const u32x4*>(keys + (t0 + z < quads ? u0[z] : row_u));
                                    if (++q == qpr) { q = 0; row_u += a.width; }
                                    if (t0 + z + 1 >= quads) { q = 0; row_u = base + r0 * a.width + c0; }   // stay inside the cell
                                }
#pragma unroll
                                for (int z = 0; z < 4; ++z) {
                                    const uint32_t ku[4] = {kv[z].x, kv[z].y, kv[z].z, kv[z].w};
                                    const bool quad_ok = t0 + z < quads;
#pragma unroll
                                    for (int x = 0; x < 4; ++x) {
                                        const int32_t u = u0[z] + x;
                                        bool ok = quad_ok && (best_idx < 0 || ku[x] < best_key);
                                        if constexpr (!decltype(first_round)::value)
                                            ok = ok && (ku[x] > last_key || (ku[x] == last_key && u > last_idx));
                                        if (ok) { best_key = ku[x]; best_idx = u; }
                                    }
                                }
                            }
                        };
                        if (k == 0) scan(std::true_type{}); else scan(std::false_type{});
                    } else
                    for (int32_t rr = r0; rr < r1; ++rr) {
                        const int32_t u0 = base + rr * a.width;
                        for (int32_t cc = c0; cc < c1; cc += 4) {           // 4 independent LDS reads at a time
                            uint32_t ku[4];
#pragma unroll
                            for (int x = 0; x < 4; ++x) ku[x] = cc + x < c1 ? keys[u0 + cc + x] : 0xFFFFFFFFu;
#pragma unroll
                            for (int x = 0; x < 4; ++x) {
                                const int32_t u = u0 + cc + x;
                                const bool after_last = last_idx < 0 || ku[x] > last_key || (ku[x] == last_key && u > last_idx);
                                const bool better = best_idx < 0 || ku[x] < best_key;
                                if (cc + x < c1 && after_last && better) { best_key = ku[x]; best_idx = u; }
                            }
                        }
                    }
                    if (best_idx >= 0) set_mark(marks, best_idx);
                    last_key = best_key; last_idx = best_idx;
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
                select_first<false, false>(keys, marks, hist + wave * 256, bcast + wave * 8, reg, a.cell_floor, false, hgt * wid);
            }
        }
        __syncthreads();
    }

    // ---- (2) frame floors
    if (a.frame_floor > 0) {
        for (int32_t f = wave; f < a.frames; f += kSelWaves) {
            const Region reg{f * a.hw, a.hw, a.hw, a.hw};
            select_first<false, true>(keys, marks, hist + wave * 256, bcast + wave * 8, reg, a.frame_floor, true, -1);
        }
        __syncthreads();
    }

    // ---- (3) global budget
    if (a.fill > 0) {
        const Region reg{0, a.nv, a.nv, a.nv};
        select_first<true, true>(keys, marks, hist, bcast, reg, a.fill, true, a.nv - a.floor_sum);
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
    {
        uint32_t tot[kSelWaves];                             // independent reads; a loop to `wave` would wait on each in turn
#pragma unroll
        for (int x = 0; x < kSelWaves; x += 4) {
            const u32x4 t = *reinterpret_cast<const u32x4*>(bcast + x);
            tot[x] = t.x; tot[x + 1] = t.y; tot[x + 2] = t.z; tot[x + 3] = t.w;
        }
#pragma unroll
        for (int x = 0; x < kSelWaves; ++x) wave_base += x < wave ? tot[x] : 0u;
    }
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
    if (batch < 0) return CIVIC_ERR_INVALID_ARG;
    if (batch > 0 && (!scores || (gi.kept > 0 && !kept_idx))) return CIVIC_ERR_INVALID_ARG;
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
    a.floor_sum = gi.floor_sum; a.fill = gi.fill; a.kept = gi.kept;
    a.big_cells = static_cast<int64_t>(a.cell_h) * a.cell_w > kSmallCell ? 1 : 0;
    auto magic = [](int64_t d) { return d <= 1 ? 0u : static_cast<uint32_t>(((int64_t{1} << 32) + d - 1) / d); };
    a.magic_cells_f = magic(static_cast<int64_t>(a.cells_y) * a.cells_x);
    a.magic_cells_x = magic(a.cells_x);

    const size_t lds = sizeof(uint32_t) * (static_cast<size_t>(a.nv_pad) + a.nv_pad / 32 + kSelWaves * 256 +
                                           kSelWaves * 8 + a.nv_pad / 64 + 2);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(select_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (e != hipSuccess) return record_hip_error(e);
    }
    hipLaunchKernelGGL(select_kernel, dim3(static_cast<unsigned>(batch)), dim3(kSelThreads), lds, s, a);
    return check_launch();
}
