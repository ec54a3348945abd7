// civic_select: exact constrained top-k (cell floors, frame floors, global budget) with ascending,
// order-preserving output.  Latency-bound: a sample's scores are 8-128 KB.
//
// One 1024-thread workgroup per sample keeps everything in LDS: a 32-bit sort key per token and one
// mark bit per token.  The strict order "higher score first, equal scores to the lower index" becomes
// (key ascending, index ascending) after mapping the float bits to an unsigned key (with -0 folded
// onto +0).
//   cells   small cells: one thread per cell picks the cell's best remaining member cell_floor times
//           (members scanned in index order, strict key comparison = the tie rule).
//           large cells: one wavefront per cell runs the select below.
//   frames  one wavefront per frame: the select below over the frame's unmarked tokens (256 bins).
//   budget  the same select run by the whole workgroup over the unmarked tokens of the sample (2048
//           bins).
//   select  one histogram pass over buckets that are linear in the score, a scan for the bucket that
//           holds the m-th token, one marking pass; the few tokens of that bucket are ranked against
//           each other directly.  Degenerate score distributions fall back to an exact radix select
//           over the key digits (see select_first).
//   output  popcounts of the 64-bit mark words -> LDS prefix scan -> every set bit writes its index
//           at (prefix of its word + set bits below it): ascending kept_idx without any sort.
#include <cmath>

#include "civic_internal.h"

namespace civic {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kSmallCell = 256;        // cells up to this many tokens are scanned by one thread each
constexpr int kSelBatch = 4;           // tokens per thread whose LDS reads are in flight together

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
    int32_t cell_kept_frame;   // tokens the cell floors protect in one frame
    int32_t quad_scores;   // 1: every sample's scores can be read as aligned groups of four
    int32_t lds_words;     // size of the dynamic LDS allocation in 32-bit words
    uint32_t magic_cells_f, magic_cells_x;   // ceil(2^32 / d) for d = cells per frame, cells per grid row (0 for d = 1)
    uint32_t magic_qpr;                      // the same for d = quads of four tokens per cell row
    int32_t cell_team, cell_team_shift;      // lanes per small cell (a power of two up to 16) and its log2; 0: one thread per cell
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

// Reduction over the 64 lanes with an idempotent operation (min, max), result in lane 63: the same DPP
// moves as the scan above; a lane without a source combines with its own value.
template <typename Op>
__device__ __forceinline__ float wave_reduce(float v, Op op)
{
    auto step = [&](float x, auto ctrl, auto row_mask) {
        const int xi = __float_as_int(x);
        return op(x, __int_as_float(__builtin_amdgcn_update_dpp(xi, xi, decltype(ctrl)::value, decltype(row_mask)::value, 0xF, false)));
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
// workgroup (BLOCK = true; every thread must call it with the same arguments, `eligible` must be
// given, and the caller synchronises the workgroup before anyone reads the marks: the function ends
// without a barrier of its own).  eligible < 0 (wavefront only): counted here.
//   hist  counters owned by the team: 2 x 2048 for the workgroup (double buffered, so the next pass's
//         clear hides behind the scan; both must be zero on entry and are left dirty), 256 for a
//         wavefront (cleared here, left zero);  bc  8 words owned by the team, 16 for the workgroup.
//   smax, range  largest score of the sample and its distance to the smallest one (any value is safe:
//         they only steer the first pass).
// First a histogram over buckets that are linear in the score, from the sample's largest down to its
// smallest, a monotone map that spreads the usual score distributions over all bins (the leading bits of a float
// key do not: they are sign and exponent).  Everything below the bucket that holds the m-th token is
// admitted, and when that bucket holds few tokens they are ranked against each other directly, so the
// select is over after one pass.  Otherwise (few distinct values, an outlier that squeezes everything
// into one bucket, infinities) an exact radix select over the key digits, high digit first, decides.
template <bool BLOCK, bool CONTIG>
__device__ void select_first(const uint32_t* keys, uint32_t* marks, uint32_t* hist, uint32_t* bc, const Region reg,
                             int32_t m, bool only_unmarked, int32_t eligible, float smax, float range)
{
    constexpr int TEAM = BLOCK ? kSelThreads : kWave;
    const int rank = BLOCK ? threadIdx.x : (threadIdx.x & (kWave - 1));
    const int lane = threadIdx.x & (kWave - 1);
    const int32_t n_iter = (reg.count + TEAM - 1) / TEAM;
    const int32_t n_batch = (n_iter + kSelBatch - 1) / kSelBatch;
    if (m <= 0 || reg.count <= 0) return;

    // The passes over the region take kSelBatch tokens per thread at a time, with all LDS reads of a
    // batch issued before the first is used (from clamped indices, so that none is conditional).  A
    // contiguous region that starts on a multiple of four gives a thread four consecutive tokens: one
    // 16-byte read for the keys, one mark word, and later one LDS atomic for the four new mark bits;
    // otherwise the four tokens are a team-width apart.
    const bool quad = CONTIG && (reg.base & 3) == 0;
    auto fetch = [&](int32_t bi, int32_t (&tok)[kSelBatch], uint32_t (&key)[kSelBatch], bool (&el)[kSelBatch]) {
        if (quad) {
            const int32_t i0 = kSelBatch * (bi * TEAM + rank);
            const int32_t v0 = reg.base + min(i0, (reg.count - 1) & ~(kSelBatch - 1));   // the array is padded to 64 tokens
            const u32x4 k = *reinterpret_cast<const u32x4*>(keys + v0);
            const uint32_t mw = marks[v0 >> 5] >> (v0 & 31);
            key[0] = k.x; key[1] = k.y; key[2] = k.z; key[3] = k.w;
#pragma unroll
            for (int u = 0; u < kSelBatch; ++u) {
                tok[u] = v0 + u;
                el[u] = i0 + u < reg.count && !(only_unmarked && ((mw >> u) & 1u));
            }
        } else {
            uint32_t mw[kSelBatch];
#pragma unroll
            for (int u = 0; u < kSelBatch; ++u) {
                const int32_t i = (bi * kSelBatch + u) * TEAM + rank;
                tok[u] = reg.token<CONTIG>(min(i, reg.count - 1));
                key[u] = keys[tok[u]];
                mw[u] = marks[tok[u] >> 5];
            }
#pragma unroll
            for (int u = 0; u < kSelBatch; ++u) {
                const int32_t i = (bi * kSelBatch + u) * TEAM + rank;
                el[u] = i < reg.count && !(only_unmarked && ((mw[u] >> (tok[u] & 31)) & 1u));
            }
        }
    };
    // Sets the mark bits of the batch's admitted tokens (a token is admitted at most once, and a pass
    // reads a token's own bit only, so the order of reads and writes between tokens does not matter).
    auto mark = [&](const int32_t (&tok)[kSelBatch], const bool (&adm)[kSelBatch]) {
        if (quad) {
            uint32_t nib = 0;
#pragma unroll
            for (int u = 0; u < kSelBatch; ++u) nib |= adm[u] ? 1u << u : 0u;
            if (nib) atomicOr(&marks[tok[0] >> 5], nib << (tok[0] & 31));   // an admitted token means tok[0] was not clamped
        } else {
#pragma unroll
            for (int u = 0; u < kSelBatch; ++u)
                if (adm[u]) set_mark(marks, tok[u]);
        }
    };
    int32_t tok[kSelBatch];
    uint32_t key[kSelBatch];
    bool el[kSelBatch], adm[kSelBatch];

    if (!BLOCK && eligible < 0) {                                // wave-uniform count from ballots
        eligible = 0;
        for (int32_t bi = 0; bi < n_batch; ++bi) {
            fetch(bi, tok, key, el);
#pragma unroll
            for (int u = 0; u < kSelBatch; ++u) eligible += __popcll(__ballot(el[u]));
        }
    }
    if (m >= eligible) {                                         // floor covers everything that is left
        for (int32_t bi = 0; bi < n_batch; ++bi) {
            fetch(bi, tok, key, el);
            mark(tok, el);
        }
        team_sync<false>();
        return;
    }

    constexpr int BITS = BLOCK ? 11 : 8;
    constexpr int BINS = 1 << BITS;
    constexpr int PASSES = (32 + BITS - 1) / BITS;
    constexpr int CH = BINS / 256;                               // the scanning wavefront takes 4 bins per lane and chunk
    constexpr uint32_t CAND = BLOCK ? 256 : 64;                  // tokens of one bucket that are ranked directly
    static_assert(CH <= 8, "chunk totals are read as two quads");
    static_assert(2 * CAND <= BINS, "the candidates live in a histogram buffer");
    if constexpr (!BLOCK) {                                      // the workgroup's histograms are clear on entry (see the kernel)
        for (int i = rank; i < BINS; i += TEAM) hist[i] = 0;
        team_sync<false>();
    }

    // Finds the bin that holds the `want`-th counted token of histogram `pass & 1` (the workgroup's; a
    // wavefront has one): bin, tokens in lower bins, tokens in the bin.  Every 256-bin chunk has a
    // wavefront of its own (4 bins per lane); the workgroup-wide select passes the chunk totals through
    // bc[8..] and clears the other histogram meanwhile; a wavefront clears its histogram afterwards.
    auto scan = [&](int pass, uint32_t want, uint32_t& bin, uint32_t& below, uint32_t& count) {
        uint32_t* h = hist + (BLOCK ? (pass & 1) * BINS : 0);
        uint32_t* res = bc + (pass & 1) * 4;
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
            if (before < want && want <= base + incl) {          // exactly one lane of one chunk
                int t = 0;
                while (before + c[t] < want) { before += c[t]; ++t; }
                res[0] = static_cast<uint32_t>(chunk * 256 + lane * 4 + t);
                res[1] = before;
                res[2] = c[t];
                res[3] = 0;                                      // the candidate counter of the first pass
            }
        }
        if constexpr (BLOCK) {
            __syncthreads();
        } else {
            team_sync<false>();
            for (int i = lane; i < BINS; i += kWave) hist[i] = 0;     // a wavefront orders its own LDS traffic for free
            team_sync<false>();
        }
        bin = res[0]; below = res[1]; count = res[2];
    };

    uint32_t remaining = static_cast<uint32_t>(m);
    int first = 0;                                               // 1: the radix passes start on the second histogram
    if (range > 0.0f && range < INFINITY) {
        // ---- one pass over score-linear buckets
        const float scale = static_cast<float>(BINS) / range;
        auto bucket = [&](uint32_t k) {                          // never decreases with the key; any input lands inside the histogram
            const uint32_t asc = ~k;
            const float s = __uint_as_float((asc & 0x80000000u) ? (asc & 0x7FFFFFFFu) : ~asc);
            return static_cast<uint32_t>(min(max(static_cast<int32_t>((smax - s) * scale), 0), BINS - 1));
        };
        for (int32_t bi = 0; bi < n_batch; ++bi) {
            fetch(bi, tok, key, el);
#pragma unroll
            for (int u = 0; u < kSelBatch; ++u)
                if (el[u]) atomicAdd(&hist[bucket(key[u])], 1u);
        }
        team_sync<BLOCK>();
        uint32_t bin, below, count;
        scan(0, remaining, bin, below, count);
        const uint32_t want = remaining - below;                  // of the `count` tokens in the bucket
        if (count == want || count <= CAND) {
            uint32_t* cand = hist + (BLOCK ? BINS : 0);          // (key, token) pairs; this histogram is clear by now
            for (int32_t bi = 0; bi < n_batch; ++bi) {
                fetch(bi, tok, key, el);
#pragma unroll
                for (int u = 0; u < kSelBatch; ++u) {
                    const uint32_t bk = bucket(key[u]);
                    adm[u] = el[u] && (bk < bin || (count == want && bk == bin));
                    if (count != want && el[u] && bk == bin) {
                        const uint32_t slot = atomicAdd(&bc[3], 1u);
                        *reinterpret_cast<u32x2*>(cand + 2 * slot) = u32x2{key[u], static_cast<uint32_t>(tok[u])};
                    }
                }
                mark(tok, adm);
            }
            if (count == want) { team_sync<false>(); return; }
            team_sync<BLOCK>();
            {
                // Thread j ranks candidate j among all of them by (key, token): the strict order itself.
                if ((static_cast<uint32_t>(rank) & ~static_cast<uint32_t>(kWave - 1)) < count) {   // wavefronts that own a candidate
                    const u32x2 me = *reinterpret_cast<const u32x2*>(cand + 2 * min(static_cast<uint32_t>(rank), count - 1));
                    uint32_t ahead = 0;
                    for (uint32_t i0 = 0; i0 < count; i0 += 8) {   // eight broadcast reads in flight (a clamped index repeats the last pair)
                        u32x2 other[8];
#pragma unroll
                        for (uint32_t u = 0; u < 8; ++u) other[u] = *reinterpret_cast<const u32x2*>(cand + 2 * min(i0 + u, count - 1));
#pragma unroll
                        for (uint32_t u = 0; u < 8; ++u)
                            ahead += (i0 + u < count && (other[u].x < me.x || (other[u].x == me.x && other[u].y < me.y))) ? 1u : 0u;
                    }
                    if (static_cast<uint32_t>(rank) < count && ahead < want) set_mark(marks, static_cast<int32_t>(me.y));
                }
                team_sync<false>();
                if constexpr (!BLOCK) {
                    for (int i = lane; i < 2 * static_cast<int>(CAND); i += kWave) hist[i] = 0;
                    team_sync<false>();
                }
            }
            return;
        }
        first = 1;
    }

    // ---- radix select of the m-th smallest key among the eligible tokens, high digit first
    uint32_t prefix = 0, ties = 0;
    int done_shift = 0;                                          // key bits below this were never looked at
#pragma unroll 1
    for (int pass = first; pass < first + PASSES; ++pass) {
        const int digit = pass - first;
        const int shift = 32 - BITS * (digit + 1) > 0 ? 32 - BITS * (digit + 1) : 0;
        const int width = 32 - BITS * digit < BITS ? 32 - BITS * digit : BITS;
        const uint32_t digit_mask = (1u << width) - 1u;
        uint32_t* h = hist + (BLOCK ? (pass & 1) * BINS : 0);
        const uint32_t hi_mask = digit == 0 ? 0u : (0xFFFFFFFFu << (shift + width));
        for (int32_t bi = 0; bi < n_batch; ++bi) {
            fetch(bi, tok, key, el);
#pragma unroll
            for (int u = 0; u < kSelBatch; ++u)
                if (el[u] && (key[u] & hi_mask) == prefix) atomicAdd(&h[(key[u] >> shift) & digit_mask], 1u);
        }
        team_sync<BLOCK>();
        uint32_t bin, below;
        scan(pass, remaining, bin, below, ties);
        prefix |= bin << shift;
        remaining -= below;
        done_shift = shift;
        if (ties == remaining) break;                            // the whole bin is admitted: its lower bits decide nothing
    }
    // prefix (above done_shift) is now the threshold; `remaining` of the `ties` tokens that carry it are admitted.

    if (ties == remaining) {                                     // no contested tie: order does not matter
        const uint32_t limit = prefix >> done_shift;
        for (int32_t bi = 0; bi < n_batch; ++bi) {
            fetch(bi, tok, key, el);
#pragma unroll
            for (int u = 0; u < kSelBatch; ++u) adm[u] = el[u] && (key[u] >> done_shift) <= limit;
            mark(tok, adm);
        }
        team_sync<false>();
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
    team_sync<false>();
}

// One workgroup selects one sample: `a` describes it, `b` is its place in the tensors a.scores, a.kept_idx and
// a.keep_flags point at.
__device__ __forceinline__ void select_sample(const SelArgs& a, const int b)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t smem[];
    uint32_t* keys = smem;                                   // [nv_pad]; this and the next start on 16-byte boundaries
    uint32_t* hist = keys + a.nv_pad;                        // [kSelWaves][256]; the workgroup-wide select uses all of it as 2 x 2048
    uint32_t* bcast = hist + kSelWaves * 256;                // [kSelWaves][8]
    uint32_t* marks = bcast + kSelWaves * 8;                 // [nv_pad / 32]
    uint32_t* word_prefix = marks + a.nv_pad / 32;           // [nv_pad / 64]
    float* extremes = reinterpret_cast<float*>(smem + a.lds_words - 2 * kSelWaves);   // [2][kSelWaves], 16-byte aligned

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const float* s = a.scores + static_cast<int64_t>(b) * a.nv;

    // Keys into LDS; on the way the sample's smallest and largest score (NaN ignored), which steer the
    // first pass of the selects.
    float lo = INFINITY, hi = -INFINITY;
    if (a.quad_scores) {                                     // 16-byte loads: the sample starts on a 16-byte boundary, nv % 4 == 0
        for (int32_t q = tid; q < a.nv / 4; q += kSelThreads) {
            const float4 x = reinterpret_cast<const float4*>(s)[q];
            const u32x4 k = {order_key(x.x), order_key(x.y), order_key(x.z), order_key(x.w)};
            *reinterpret_cast<u32x4*>(keys + 4 * q) = k;
            lo = fminf(fminf(lo, x.x), fminf(fminf(x.y, x.z), x.w));
            hi = fmaxf(fmaxf(hi, x.x), fmaxf(fmaxf(x.y, x.z), x.w));
        }
        for (int32_t v = a.nv + tid; v < a.nv_pad; v += kSelThreads) keys[v] = 0xFFFFFFFFu;
    } else {
        for (int32_t v0 = tid; v0 < a.nv_pad; v0 += kSelBatch * kSelThreads) {
            float x[kSelBatch];
#pragma unroll
            for (int u = 0; u < kSelBatch; ++u) x[u] = s[min(v0 + u * kSelThreads, a.nv - 1)];   // a clamped index repeats a real score
#pragma unroll
            for (int u = 0; u < kSelBatch; ++u) {
                const int32_t v = v0 + u * kSelThreads;
                if (v < a.nv_pad) keys[v] = v < a.nv ? order_key(x[u]) : 0xFFFFFFFFu;
                lo = fminf(lo, x[u]);
                hi = fmaxf(hi, x[u]);
            }
        }
    }
    lo = wave_reduce(lo, [](float p, float q) { return fminf(p, q); });
    hi = wave_reduce(hi, [](float p, float q) { return fmaxf(p, q); });
    if (lane == kWave - 1) { extremes[wave] = lo; extremes[kSelWaves + wave] = hi; }
    for (int32_t w = tid; w < a.nv_pad / 32; w += kSelThreads) marks[w] = 0u;
    // The budget select wants zeroed histograms; the per-wavefront selects before it leave theirs zeroed.
    for (int i = tid; i < kSelWaves * 256; i += kSelThreads) hist[i] = 0u;
    __syncthreads();
    float smin = INFINITY, smax = -INFINITY;
#pragma unroll
    for (int x = 0; x < kSelWaves; x += 4) {
        const float4 l4 = *reinterpret_cast<const float4*>(extremes + x), h4 = *reinterpret_cast<const float4*>(extremes + kSelWaves + x);
        smin = fminf(fminf(smin, l4.x), fminf(fminf(l4.y, l4.z), l4.w));
        smax = fmaxf(fmaxf(smax, h4.x), fmaxf(fmaxf(h4.y, h4.z), h4.w));
    }
    const float range = smax - smin;                         // 0, infinite or NaN: the selects go straight to the key digits

    // ---- (1) cell floors
    if (a.cell_floor > 0) {
        if (!a.big_cells) {
            // cell_floor rounds of "best member after the previous winner"; members are compared in
            // ascending index with a strict key comparison, which is the tie rule.  The work is
            // cells * floor * size instead of tokens * size for an all-pairs rank.
            const int32_t cells_f = a.cells_y * a.cells_x, cells = a.frames * cells_f;
            if (a.cell_team > 0) {
                // Every cell row is made of aligned quads of keys (cell width a multiple of 4 that divides
                // the grid width).  A team of 16 adjacent lanes takes a cell, a lane the quads q0, q0 + team,
                // ... of its row-major quad list (one 16-byte LDS read each), and the lanes' candidates meet
                // in the team's last lane through DPP row shifts.  All loops have wave-uniform bounds so
                // that every lane is active at the shifts.
                const int team = a.cell_team, q0 = tid & (team - 1);
                const int32_t qpr = a.cell_w >> 2, quads_full = a.cell_h * qpr;
                const int32_t rounds_full = min(a.cell_floor, a.cell_h * a.cell_w);
                for (int32_t cell0 = 0; cell0 < cells; cell0 += kSelThreads >> a.cell_team_shift) {
                    const int32_t cell = cell0 + (tid >> a.cell_team_shift);
                    const bool live = cell < cells;
                    const int32_t cc = live ? cell : 0;
                    const int32_t f = div_magic(cc, a.magic_cells_f), rem = cc - f * cells_f;
                    const int32_t cy = div_magic(rem, a.magic_cells_x), cx = rem - cy * a.cells_x;
                    const int32_t r0 = cy * a.cell_h, rows = min(a.cell_h, a.height - r0);
                    const int32_t first = f * a.hw + r0 * a.width + cx * a.cell_w;       // the cell's first token
                    const int32_t quads = live ? rows * qpr : 0, rounds = min(a.cell_floor, rows * a.cell_w);
                    uint32_t last_key = 0;
                    int32_t last_idx = -1;
                    for (int32_t k = 0; k < rounds_full; ++k) {
                        uint32_t best_key = 0xFFFFFFFFu;
                        int32_t best_idx = INT32_MAX;                  // no candidate
                        for (int32_t q = q0; q < quads_full; q += team) {
                            const bool quad_ok = q < quads && k < rounds;
                            const int32_t qr = div_magic(q, a.magic_qpr), u0 = first + qr * a.width + 4 * (q - qr * qpr);
                            const u32x4 kv = *reinterpret_cast<const u32x4*>(keys + (quad_ok ? u0 : 0));
                            const uint32_t ku[4] = {kv.x, kv.y, kv.z, kv.w};
#pragma unroll
                            for (int x = 0; x < 4; ++x) {
                                const int32_t u = u0 + x;
                                const bool after_last = k == 0 || ku[x] > last_key || (ku[x] == last_key && u > last_idx);
                                if (quad_ok && after_last && (best_idx == INT32_MAX || ku[x] < best_key)) { best_key = ku[x]; best_idx = u; }
                            }
                        }
                        auto meet = [&](auto ctrl) {                   // take the better of mine and the lane `shift` to the left
                            const uint32_t ok = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(
                                static_cast<int>(best_key), static_cast<int>(best_key), decltype(ctrl)::value, 0xF, 0xF, false));
                            const int32_t oi = __builtin_amdgcn_update_dpp(best_idx, best_idx, decltype(ctrl)::value, 0xF, 0xF, false);
                            if (ok < best_key || (ok == best_key && oi < best_idx)) { best_key = ok; best_idx = oi; }
                        };
                        using std::integral_constant;
                        if (team > 1) meet(integral_constant<int, 0x111>{});   // row_shr:1
                        if (team > 2) meet(integral_constant<int, 0x112>{});   // row_shr:2
                        if (team > 4) meet(integral_constant<int, 0x114>{});   // row_shr:4
                        if (team > 8) meet(integral_constant<int, 0x118>{});   // row_shr:8
                        if (q0 == team - 1 && best_idx != INT32_MAX) set_mark(marks, best_idx);
                        if (k + 1 < rounds_full) {                     // the winner back to the whole team
                            last_key = static_cast<uint32_t>(__shfl(static_cast<int>(best_key), lane | (team - 1)));
                            last_idx = __shfl(best_idx, lane | (team - 1));
                        }
                    }
                }
            } else {
            // One thread per cell.
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
            }
        } else {
            const int32_t cells = a.frames * a.cells_y * a.cells_x;
            for (int32_t cell = wave; cell < cells; cell += kSelWaves) {
                const int32_t f = cell / (a.cells_y * a.cells_x), rem = cell - f * a.cells_y * a.cells_x;
                const int32_t cy = rem / a.cells_x, cx = rem - cy * a.cells_x;
                const int32_t r0 = cy * a.cell_h, c0 = cx * a.cell_w;
                const int32_t hgt = min(a.cell_h, a.height - r0), wid = min(a.cell_w, a.width - c0);
                const Region reg{f * a.hw + r0 * a.width + c0, wid, a.width, hgt * wid};
                select_first<false, false>(keys, marks, hist + wave * 256, bcast + wave * 8, reg, a.cell_floor, false, hgt * wid, smax, range);
            }
        }
        __syncthreads();
    }

    // ---- (2) frame floors
    if (a.frame_floor > 0) {
        for (int32_t f = wave; f < a.frames; f += kSelWaves) {
            const Region reg{f * a.hw, a.hw, a.hw, a.hw};
            select_first<false, true>(keys, marks, hist + wave * 256, bcast + wave * 8, reg, a.frame_floor, true,
                                      a.hw - a.cell_kept_frame, smax, range);
        }
        __syncthreads();
    }

    // ---- (3) global budget
    if (a.fill > 0) {
        const Region reg{0, a.nv, a.nv, a.nv};
        select_first<true, true>(keys, marks, hist, bcast, reg, a.fill, true, a.nv - a.floor_sum, smax, range);
    }
    __syncthreads();

    // ---- (4) ascending output
    const int32_t words = a.nv_pad / 64;                     // <= 512, one per thread
    int32_t* out = a.kept_idx + static_cast<int64_t>(b) * a.kept;
    if (words <= kWave) {
        // Up to 4096 tokens: the mark words fit one per lane, so every wavefront scans all of them itself and
        // takes the prefixes of its own words from the scan's lanes; nothing goes through LDS, no barrier.
        const u32x2 mine = *reinterpret_cast<const u32x2*>(marks + 2 * min(lane, words - 1));
        const uint32_t cnt = lane < words ? __popc(mine.x) + __popc(mine.y) : 0u;
        const uint32_t before = wave_incl_scan(cnt, lane) - cnt;
#pragma unroll
        for (int u = 0; u < kWave / kSelWaves; ++u) {        // the wavefront's tokens: 64 per 1024, word wave + 16 u
            const int w = wave + u * kSelWaves;
            if (w >= words) break;
            const uint32_t lo = __builtin_amdgcn_readlane(mine.x, w), hi = __builtin_amdgcn_readlane(mine.y, w);
            const uint32_t base = __builtin_amdgcn_readlane(before, w);
            const uint64_t word = (static_cast<uint64_t>(hi) << 32) | lo;
            const int32_t v = w * kWave + lane;
            const bool bit = (word >> lane) & 1ull;
            if (bit) {
                const uint32_t pos = base + static_cast<uint32_t>(__popcll(word & ((1ull << lane) - 1ull)));
                if (pos < static_cast<uint32_t>(a.kept)) out[pos] = v;
            }
            if (a.keep_flags && v < a.nv) a.keep_flags[static_cast<int64_t>(b) * a.nv + v] = bit ? 1 : 0;
        }
        return;
    }
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

    for (int32_t v0 = tid; v0 < a.nv_pad; v0 += kSelBatch * kSelThreads) {
        u32x2 mw[kSelBatch];
        uint32_t wp[kSelBatch];
#pragma unroll
        for (int u = 0; u < kSelBatch; ++u) {                // a batch of reads from clamped indices, then the stores
            const int32_t w = min(v0 + u * kSelThreads, a.nv_pad - 1) >> 6;
            mw[u] = *reinterpret_cast<const u32x2*>(marks + 2 * w);
            wp[u] = word_prefix[w];
        }
#pragma unroll
        for (int u = 0; u < kSelBatch; ++u) {
            const int32_t v = v0 + u * kSelThreads;
            if (v >= a.nv_pad) break;
            const uint64_t word = (static_cast<uint64_t>(mw[u].y) << 32) | mw[u].x;
            const bool bit = (word >> lane) & 1ull;
            if (bit) {
                const uint32_t pos = wp[u] + static_cast<uint32_t>(__popcll(word & ((1ull << lane) - 1ull)));
                if (pos < static_cast<uint32_t>(a.kept)) out[pos] = v;
            }
            if (a.keep_flags && v < a.nv) a.keep_flags[static_cast<int64_t>(b) * a.nv + v] = bit ? 1 : 0;
        }
    }
}

__global__ __launch_bounds__(kSelThreads) void select_kernel(SelArgs a)
{
    select_sample(a, blockIdx.x);
}

// Samples of different grids in one launch (the ragged front): workgroup i takes the i-th description of a table in
// the kernel arguments, each with its own pointers, so its place in them is 0.
constexpr int kSelRaggedItems = 16;
struct SelTable {
    SelArgs item[kSelRaggedItems];
};
__global__ __launch_bounds__(kSelThreads) void select_ragged_kernel(SelTable t)
{
    select_sample(t.item[blockIdx.x], 0);
}


}  // namespace civic

namespace civic {

// The argument checks of civic_select (host only, nothing is launched).
int select_check(const float* scores, int32_t batch, const civic_grid* grid, const int32_t* kept_idx)
{
    GridInfo gi;
    if (grid_info(grid, &gi) != CIVIC_OK) return CIVIC_ERR_INVALID_ARG;
    if (batch < 0) return CIVIC_ERR_INVALID_ARG;
    if (batch > 0 && (!scores || (gi.kept > 0 && !kept_idx))) return CIVIC_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(scores) | reinterpret_cast<uintptr_t>(kept_idx)) & 3u) return CIVIC_ERR_INVALID_ARG;
    if (gi.nv > CIVIC_MAX_VISUAL_TOKENS) return CIVIC_ERR_UNSUPPORTED;
    return CIVIC_OK;
}

}  // namespace civic

namespace civic {

// What the kernel needs to know about a sample of grid `gi` (checked), and the dynamic LDS it takes in bytes.
static SelArgs make_sel_args(const float* scores, int32_t* kept_idx, uint8_t* keep_flags, const GridInfo& gi, size_t* lds_bytes)
{
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
    a.cell_kept_frame = gi.cell_kept_frame;
    a.quad_scores = (reinterpret_cast<uintptr_t>(scores) & 15u) == 0 && gi.nv % 4 == 0;
    auto magic = [](int64_t d) { return d <= 1 ? 0u : static_cast<uint32_t>(((int64_t{1} << 32) + d - 1) / d); };
    a.magic_cells_f = magic(static_cast<int64_t>(a.cells_y) * a.cells_x);
    a.magic_cells_x = magic(a.cells_x);
    a.magic_qpr = magic(a.cell_w / 4);
    a.cell_team = 0; a.cell_team_shift = 0;
    // Cells of 64-256 tokens whose rows are made of aligned quads of keys get 16 lanes each; smaller ones are
    // faster with a thread of their own (measured: 4 x 4 cells 1.0 us against 1.3 us, 8 x 8 cells 2.4 against 1.5).
    if (a.cell_w % 4 == 0 && a.cells_x * a.cell_w == a.width && !a.big_cells && a.cell_h * (a.cell_w / 4) >= 16) {
        a.cell_team = 16; a.cell_team_shift = 4;
    }
    // keys | histograms | per-team words | mark bits | word prefixes, rounded up to 16 bytes | per-wavefront extremes
    const size_t lds_words = (static_cast<size_t>(a.nv_pad) + kSelWaves * 256 + kSelWaves * 8 + a.nv_pad / 32 + a.nv_pad / 64 + 3) / 4 * 4 +
                             2 * kSelWaves;
    a.lds_words = static_cast<int32_t>(lds_words);
    *lds_bytes = sizeof(uint32_t) * lds_words;
    return a;
}

// The limit of dynamic LDS is raised once per device and kernel, for the largest sample there is.
static int allow_select_lds(const void* kernel, std::atomic<uint64_t>* done)
{
    constexpr size_t max_pad = (CIVIC_MAX_VISUAL_TOKENS + 63) / 64 * 64;
    constexpr size_t max_lds = sizeof(uint32_t) * ((max_pad + kSelWaves * 256 + kSelWaves * 8 + max_pad / 32 + max_pad / 64 + 3) / 4 * 4 +
                                                   2 * kSelWaves);
    return allow_dynamic_lds(kernel, max_lds, done);
}

// `n` (<= 16) samples of different grids in one launch: sample i reads scores[i], writes kept_idx[i] (arguments checked
// by the caller with select_check, one sample each).
int select_samples_launch(const float* const* scores, int32_t* const* kept_idx, const civic_grid* const* grids, int32_t n, void* stream)
{
    SelTable t;
    size_t lds = 0;
    for (int i = 0; i < kSelRaggedItems; ++i) {
        const int at = i < n ? i : 0;                             // (entries past the launch repeat the first; never read)
        GridInfo gi;
        grid_info(grids[at], &gi);
        size_t one = 0;
        t.item[i] = make_sel_args(scores[at], kept_idx[at], nullptr, gi, &one);
        if (i < n && one > lds) lds = one;
    }
    if (lds > 64 * 1024) {
        static std::atomic<uint64_t> allowed{0};
        const int rc = allow_select_lds(reinterpret_cast<const void*>(select_ragged_kernel), &allowed);
        if (rc != CIVIC_OK) return rc;
    }
    civic::launch(select_ragged_kernel, dim3(static_cast<unsigned>(n)), dim3(kSelThreads), lds, static_cast<hipStream_t>(stream), t);
    return check_launch();
}

}  // namespace civic

extern "C" int civic_select(const float* scores, int32_t batch, const civic_grid* grid, int32_t* kept_idx,
                            uint8_t* keep_flags, void* workspace, size_t workspace_bytes, void* stream)
{
    using namespace civic;
    (void)workspace; (void)workspace_bytes;
    const int rc_check = select_check(scores, batch, grid, kept_idx);
    if (rc_check != CIVIC_OK) return rc_check;
    if (batch == 0) return CIVIC_OK;
    GridInfo gi;
    grid_info(grid, &gi);
    size_t lds = 0;
    const SelArgs a = make_sel_args(scores, kept_idx, keep_flags, gi, &lds);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (lds > 64 * 1024) {
        static std::atomic<uint64_t> allowed{0};
        const int rc = allow_select_lds(reinterpret_cast<const void*>(select_kernel), &allowed);
        if (rc != CIVIC_OK) return rc;
    }
    civic::launch(select_kernel, dim3(static_cast<unsigned>(batch)), dim3(kSelThreads), lds, s, a);
    return check_launch();
}
