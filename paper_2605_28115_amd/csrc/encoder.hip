// Encoder-side compaction of CIVIC, the paper's own (learned, soft) route to a compact sequence:
//   civic_anchor_aggregate  Eq. 8: Z_0 = softmax(Q_A K_0^T / tau) X_0 with K_0 = Norm(LN(X_0)), Q_A = Norm(LN(A)),
//                           softmax over the dense tokens
//   civic_kv_compress       Eq. 9: K_c = Rbar^T K, V_c = Rbar^T V with the column-normalised assignment matrix
// (the attention over the compressed keys, softmax(Q K_c^T / sqrt(d)) V_c, is civic_cross_attn in attn.hip).
//
// Both are dense contractions and run on the bf16 MFMA pipe through one kernel, C = alpha * A B^T, whose B operand
// may be stored either way round: like A, with the contraction index contiguous (the logits Q_A K_0^T), or with the
// contraction index as the row index, which is how X_0 lies in Z_0 = W_A X_0 and how K and V lie in Eq. 9; those are
// read where they are (transposing LDS reads), no transposed copy is made.  A is always contraction-contiguous and
// zero-padded to a multiple of 64 in that direction (W_A and Rbar^T are written that way), so the GEMM has no tail
// there; row and column tails are clamped loads and masked stores.
//   - 128 x 128 output tile per 256-thread workgroup, 64 x 64 per wavefront (2 x 2 blocks of
//     v_mfma_f32_32x32x16_bf16, fp32 accumulators), 64 contraction elements per LDS tile.
//   - A and B tiles go from global memory straight into an LDS ring (global_load_lds_dwordx4), 16-byte chunks
//     XOR-swizzled by the row so that operand reads fall on distinct banks; explicit vmcnt waits, fence-free barriers;
//     the fragments of the next k-step are read while the MFMAs of the current one run, in a hand-written order.
//   - Two ring depths: two stages and two workgroups per compute unit for grids that fill the chip (the kernel is then
//     bound by the L2 -> LDS traffic of its tiles, 64 FLOP per byte; a deeper ring at one workgroup per unit was
//     slower, 46.6 against 35.3 us on the 1365 x 4096 x 1152 logits), four stages for grids that leave units without a
//     second workgroup anyway, where the latency of a tile is what a workgroup waits for.
//   - K_c and V_c of Eq. 9 come from one launch (grid z = batch item x tensor).
// The softmax of Eq. 8 runs over rows of 4096 logits and more, too long for a fused epilogue: the logits go to
// scratch in fp32, a row kernel turns them into bf16 weights, the second GEMM consumes those.
#include <cmath>

#include "civic_internal.h"

namespace civic {

typedef __bf16 enc_bf16x8 __attribute__((ext_vector_type(8)));
typedef float enc_f32x16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) char enc_lds_char;

constexpr int kGemmBM = 128, kGemmBN = 128, kGemmBK = 64;
constexpr int kGemmThreads = 256;
constexpr int kGemmTileBytes = kGemmBM * kGemmBK * 2;         // one operand tile: 16 KB

constexpr int kGroupItems = 64;    // items of one grouped launch (longer lists go out in several)

// Items of different row counts packed along the row axis (the ragged Eq. 9 calls): item i owns rows
// [row[i], row[i + 1]) of the packed tensors; pad_row counts the same rows with every item's length rounded up to 64,
// which is how the items' zero-padded Rbar^T blocks follow one another in scratch memory.
struct Group {
    int32_t row[kGroupItems + 1];
    int32_t pad_row[kGroupItems + 1];
};

struct GemmArgs {
    const __bf16* a; const __bf16* b; void* c;
    // a second (B, C) pair served by the same launch (grid z = 2 * batch item + pair), or null
    const __bf16* b_alt; void* c_alt;
    int64_t lda, ldb, ldc;             // elements between rows of A [m x k], of B as stored, of C [m x n]
    int64_t sa, sb, sc;                // elements between batch items (0 = shared)
    int32_t m, n, k;                   // k a multiple of 64 (A is zero-padded up to it)
    int32_t kb_rows;                   // B stored [k x n]: the rows that exist (<= k); rows beyond re-read the last one
    float alpha;
    // output tiles: counts per matrix, tiles of all matrices of the launch, n-tiles per panel (filled in by launch_gemm)
    int32_t tiles_m, tiles_n, total_tiles, panel;
    // GROUPED launches only: batch item i multiplies A_i = a + m * pad_row[i] (its own contraction length
    // pad_row[i + 1] - pad_row[i], which is also its row pitch) with the rows [row[i], row[i + 1]) of b
    Group grp;
};

template <int LDS_IMM>
__device__ __forceinline__ void enc_dma16(const void* base, uint32_t byte_off, uint32_t lds_addr)
{
    // 16 bytes per lane from base + byte_off (scalar base, per-lane offset) into LDS at lds_addr + LDS_IMM + lane * 16
    asm volatile("s_add_u32 m0, %0, %3\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(byte_off), "s"(base), "n"(LDS_IMM) : "memory", "scc");
}

__device__ __forceinline__ const char* enc_uniform(const void* p)
{
    const uint64_t bits = reinterpret_cast<uint64_t>(p);
    const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<uint32_t>(bits >> 32)));
    const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<uint32_t>(bits)));
    return reinterpret_cast<const char*>((static_cast<uint64_t>(hi) << 32) | lo);
}

// physical chunk = logical chunk ^ swz(row): rows 0..31 of a 128-byte-pitch tile, same logical chunk -> 32 banks groups
__device__ __forceinline__ int enc_swz(int row) { return (((row >> 1) & 1) << 2) | ((row >> 2) & 3); }
// the same for a 256-byte pitch (16 chunks per row): a tile stored with the contraction index as its rows
__device__ __forceinline__ int enc_swz16(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

typedef short enc_s16x4 __attribute__((ext_vector_type(4)));
typedef short enc_s16x8 __attribute__((ext_vector_type(8)));

// C = alpha * A B^T.  A is stored [m x k] (contraction index contiguous).  B_KROWS = false: B stored [n x k], the same
// way.  B_KROWS = true: B stored [k x n], contraction index as the row index - the layout of X_0 in Z_0 = W_A X_0 and of
// K, V in Eq. 9; its tiles (64 contraction rows x 128 columns, 256-byte pitch) are read with the transposing LDS read,
// which hands a lane one column and 4 consecutive contraction rows, so no transposed copy is ever made.
// STAGES: tiles in the LDS ring, all but one in flight ahead of the one consumed: 2 (two workgroups per compute unit)
// when the grid fills the chip, 4 (one workgroup per unit) when it does not and a tile's latency is what is waited for.
template <bool C_BF16, bool B_KROWS, int STAGES, bool GROUPED = false>
__global__ __launch_bounds__(kGemmThreads, STAGES == 2 ? 2 : 1) void gemm_kernel(GemmArgs g)
{
    extern __shared__ __attribute__((aligned(16))) char gemm_lds[];
    enc_lds_char* const lds = (enc_lds_char*)gemm_lds;       // the A stages, then the B stages
    const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    const int wm = w >> 1, wn = w & 1;                        // the wavefront's 64 x 64 quadrant
    // Workgroup -> output tile.  The hardware hands consecutive workgroups to the eight XCDs in turn, each with an L2
    // of its own, so workgroup p takes tile (p mod 8) * (workgroups / 8) + p / 8: every XCD owns a contiguous run of
    // tiles, and the tiles of a matrix are numbered panel by panel (a panel = `panel` tile columns, all tile rows), so
    // that run is a compact block whose A row slabs and B column slabs are shared inside one L2 as the workgroups
    // advance along the contraction together.  With the plain (x, y) numbering every XCD touches every slab and the
    // kernel runs at the speed of the memory behind the L2s.
    const uint32_t per_xcd = gridDim.x >> 3;
    const uint32_t tile = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
    if (tile >= static_cast<uint32_t>(g.total_tiles)) return;            // (the grid is padded to a multiple of 8)
    const uint32_t per_mat = static_cast<uint32_t>(g.tiles_m) * g.tiles_n;
    const uint32_t zi = tile / per_mat, rr = tile - zi * per_mat;
    const uint32_t pn = rr / (static_cast<uint32_t>(g.panel) * g.tiles_m);
    const uint32_t base_n = pn * g.panel;
    const uint32_t pw = min(static_cast<uint32_t>(g.panel), static_cast<uint32_t>(g.tiles_n) - base_n);
    const uint32_t within = rr - pn * g.panel * g.tiles_m;
    const int m0 = static_cast<int>(within / pw) * kGemmBM, n0 = static_cast<int>(base_n + within % pw) * kGemmBN;
    const bool alt = g.b_alt != nullptr && (zi & 1u);
    const int64_t bz = g.b_alt != nullptr ? (zi >> 1) : zi;
    const __bf16* const b_mat = alt ? g.b_alt : g.b;
    // contraction length, A's row pitch and the operands' first elements for this batch item
    int32_t k_len = g.k, kb_rows = g.kb_rows;
    int64_t lda = g.lda, a_first = bz * g.sa, b_first = bz * g.sb;
    if constexpr (GROUPED) {
        static_assert(B_KROWS, "grouped items differ in their contraction rows");
        const int32_t r0 = g.grp.row[bz], p0 = g.grp.pad_row[bz];
        k_len = g.grp.pad_row[bz + 1] - p0;
        kb_rows = g.grp.row[bz + 1] - r0;
        lda = k_len;
        a_first = static_cast<int64_t>(g.m) * p0;
        b_first = static_cast<int64_t>(r0) * g.ldb;
    }

    // global -> LDS: instruction j of wavefront w fills slots [(4 w + j) * 64, +64) of a tile; slot -> (row, physical chunk)
    const char* a_base = reinterpret_cast<const char*>(g.a + a_first + static_cast<int64_t>(m0) * lda);
    const char* b_base = B_KROWS ? reinterpret_cast<const char*>(b_mat + b_first + n0)
                                 : reinterpret_cast<const char*>(b_mat + b_first + static_cast<int64_t>(n0) * g.ldb);
    const int last_tile = k_len / kGemmBK - 1;
    uint32_t a_off[4], b_off[4], b_off_tail[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int slot = (w * 4 + j) * kWave + lane;
        const int row = slot >> 3;
        const int c = (slot & 7) ^ enc_swz(row);
        a_off[j] = static_cast<uint32_t>(min(row, g.m - 1 - m0)) * static_cast<uint32_t>(lda * 2) + c * 16;
        if constexpr (B_KROWS) {
            const int krow = slot >> 4;                       // contraction row inside the tile
            const int lc = (slot & 15) ^ enc_swz16(krow);     // logical chunk: columns n0 + 8 lc .. + 7
            const int cc = min(lc, (g.n - n0) / 8 - 1);       // (n is a multiple of 8; chunks past it re-read a valid one)
            b_off[j] = static_cast<uint32_t>(krow) * static_cast<uint32_t>(g.ldb * 2) + cc * 16;
            b_off_tail[j] = static_cast<uint32_t>(min(last_tile * kGemmBK + krow, kb_rows - 1) - last_tile * kGemmBK) *
                                static_cast<uint32_t>(g.ldb * 2) + cc * 16;
        } else {
            b_off[j] = static_cast<uint32_t>(min(row, g.n - 1 - n0)) * static_cast<uint32_t>(g.ldb * 2) + c * 16;
            b_off_tail[j] = b_off[j];
        }
    }
    const uint32_t lds_wave = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds)) + w * 4 * kWave * 16);
    auto issue = [&](int kt, auto stage_c) {
        constexpr int st = decltype(stage_c)::value;
        const char* ab = enc_uniform(a_base + static_cast<int64_t>(kt) * kGemmBK * 2);
        const char* bb = B_KROWS ? enc_uniform(b_base + static_cast<int64_t>(kt) * kGemmBK * g.ldb * 2)
                                 : enc_uniform(b_base + static_cast<int64_t>(kt) * kGemmBK * 2);
        const bool tail = B_KROWS && kt == last_tile;
        enc_dma16<st * kGemmTileBytes + 0 * 1024>(ab, a_off[0], lds_wave);
        enc_dma16<st * kGemmTileBytes + 1 * 1024>(ab, a_off[1], lds_wave);
        enc_dma16<st * kGemmTileBytes + 2 * 1024>(ab, a_off[2], lds_wave);
        enc_dma16<st * kGemmTileBytes + 3 * 1024>(ab, a_off[3], lds_wave);
        enc_dma16<(STAGES + st) * kGemmTileBytes + 0 * 1024>(bb, tail ? b_off_tail[0] : b_off[0], lds_wave);
        enc_dma16<(STAGES + st) * kGemmTileBytes + 1 * 1024>(bb, tail ? b_off_tail[1] : b_off[1], lds_wave);
        enc_dma16<(STAGES + st) * kGemmTileBytes + 2 * 1024>(bb, tail ? b_off_tail[2] : b_off[2], lds_wave);
        enc_dma16<(STAGES + st) * kGemmTileBytes + 3 * 1024>(bb, tail ? b_off_tail[3] : b_off[3], lds_wave);
    };

    // A reads: row (quadrant row 32 i + col), logical chunk 2 s + half; the swizzle depends on row bits 1..3 only, so the
    // second row block is the first plus a constant.  B the same when it is stored like A; when it is stored with the
    // contraction index as rows, two transposing reads per fragment: a block of 16 lanes fetches a patch of 4
    // contraction rows (8 half + 4 hi + 0..3 of the 16-row step) x 16 columns and every lane receives one column of it.
    enc_lds_char* a_addr[4];
    enc_lds_char* b_addr[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        a_addr[s] = lds + (wm * 64 + col) * 128 + (((2 * s + half) ^ enc_swz(col)) << 4);
        if constexpr (B_KROWS) {
            const int hi = s & 1, j = s >> 1;                 // (the four registers are the (hi, j) combinations)
            const int l16 = lane & 15, g16 = (lane >> 4) & 1;
            const int krow = 8 * half + 4 * hi + (l16 >> 2);
            const int el = wn * 64 + 32 * j + 16 * g16 + 4 * (l16 & 3);
            b_addr[s] = lds + STAGES * kGemmTileBytes + krow * 256 + (((el >> 3) ^ enc_swz16(krow)) << 4) + (el & 7) * 2;
        } else {
            b_addr[s] = lds + STAGES * kGemmTileBytes + (wn * 64 + col) * 128 + (((2 * s + half) ^ enc_swz(col)) << 4);
        }
        asm volatile("" : "+v"(a_addr[s]), "+v"(b_addr[s]));
    }

    enc_f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int n_tiles = k_len / kGemmBK;
#pragma unroll
    for (int t = 0; t < STAGES - 1; ++t)
        if (t == 0) issue(0, std::integral_constant<int, 0>{});
        else if (t == 1) { if (n_tiles > 1) issue(1, std::integral_constant<int, 1>{}); }
        else { if (n_tiles > 2) issue(2, std::integral_constant<int, 2>{}); }
    // Loads retire in order, 8 per tile and wavefront: tile kt has landed once at most 8 * (tiles issued after it)
    // loads are outstanding.
    auto wait_landed = [&](int younger) {
        if (younger >= 2) __builtin_amdgcn_s_waitcnt(0x4F70);            // vmcnt(16): the count's bits 5:4 sit in bits 15:14
        else if (younger == 1) __builtin_amdgcn_s_waitcnt(0x0F70 | 8);   // vmcnt(8)
        else __builtin_amdgcn_s_waitcnt(0x0F70);                         // vmcnt(0)
    };
    auto step = [&](int kt, auto stage_c) __attribute__((always_inline)) {
        constexpr int st = decltype(stage_c)::value;
        wait_landed(min(n_tiles - 1 - kt, STAGES - 2));
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();                         // landed for every wavefront; the stage of tile kt - 1 is free
        asm volatile("" ::: "memory");
        if (kt + STAGES - 1 < n_tiles) issue(kt + STAGES - 1, std::integral_constant<int, (st + STAGES - 1) % STAGES>{});
        // operand fragments of k-step s + 1 are read while the MFMAs of step s run (in the order written)
        auto read_a = [&](int s, int i) __attribute__((always_inline)) {
            return *reinterpret_cast<const __attribute__((address_space(3))) enc_bf16x8*>(a_addr[s] + st * kGemmTileBytes + i * 32 * 128);
        };
        auto read_b = [&](int s, int j) __attribute__((always_inline)) {
            if constexpr (B_KROWS) {
                const enc_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) enc_s16x4*)(b_addr[2 * j] + st * kGemmTileBytes + s * 16 * 256));
                const enc_s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) enc_s16x4*)(b_addr[2 * j + 1] + st * kGemmTileBytes + s * 16 * 256));
                const enc_s16x8 v8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                return __builtin_bit_cast(enc_bf16x8, v8);
            } else {
                return *reinterpret_cast<const __attribute__((address_space(3))) enc_bf16x8*>(b_addr[s] + st * kGemmTileBytes + j * 32 * 128);
            }
        };
        enc_bf16x8 af[2][2], bf[2][2];
        af[0][0] = read_a(0, 0); af[0][1] = read_a(0, 1); bf[0][0] = read_b(0, 0); bf[0][1] = read_b(0, 1);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int cur = s & 1, nxt = cur ^ 1;
            if (s + 1 < 4) { af[nxt][0] = read_a(s + 1, 0); af[nxt][1] = read_a(s + 1, 1); bf[nxt][0] = read_b(s + 1, 0); bf[nxt][1] = read_b(s + 1, 1); }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[cur][i], bf[cur][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    for (int kt = 0; kt < n_tiles; kt += STAGES) {
        step(kt, std::integral_constant<int, 0>{});
        if (kt + 1 < n_tiles) step(kt + 1, std::integral_constant<int, 1>{});
        if constexpr (STAGES == 4) {
            if (kt + 2 < n_tiles) step(kt + 2, std::integral_constant<int, 2>{});
            if (kt + 3 < n_tiles) step(kt + 3, std::integral_constant<int, 3>{});
        }
    }

    // register r of block (i, j): row 32 i + 8 (r / 4) + r % 4 + 4 half, column 32 j + col
    char* c_base = static_cast<char*>(alt ? g.c_alt : g.c) + (bz * g.sc) * (C_BF16 ? 2 : 4);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * 64 + 32 * i + 8 * (r >> 2) + (r & 3) + 4 * half;
                const int cc = n0 + wn * 64 + 32 * j + col;
                if (row < g.m && cc < g.n) {
                    const float val = acc[i][j][r] * g.alpha;
                    const int64_t idx = static_cast<int64_t>(row) * g.ldc + cc;
                    if constexpr (C_BF16) reinterpret_cast<__bf16*>(c_base)[idx] = static_cast<__bf16>(val);
                    else reinterpret_cast<float*>(c_base)[idx] = val;
                }
            }
}

template <bool C_BF16, bool B_KROWS, int STAGES, bool GROUPED = false>
static int launch_gemm_variant(const GemmArgs& g, unsigned blocks, hipStream_t s)
{
    const dim3 grid(blocks);
    constexpr size_t lds = 2 * STAGES * kGemmTileBytes;
    static std::atomic<uint64_t> allowed{0};
    const int rc = allow_dynamic_lds(reinterpret_cast<const void*>(gemm_kernel<C_BF16, B_KROWS, STAGES, GROUPED>), lds, &allowed);
    if (rc != CIVIC_OK) return rc;
    civic::launch((gemm_kernel<C_BF16, B_KROWS, STAGES, GROUPED>), grid, dim3(kGemmThreads), lds, s, g);
    return check_launch();
}

// `batch` batch items; with g.b_alt set every item runs twice, once per (B, C) pair.  b_krows: B is stored [k x n].
// grouped: g.grp describes the `batch` items (bf16 result, B stored [k x n] only).
static int launch_gemm(const GemmArgs& g_in, int batch, bool c_bf16, bool b_krows, hipStream_t s, bool grouped = false)
{
    GemmArgs g = g_in;
    const int64_t z = static_cast<int64_t>(batch) * (g.b_alt ? 2 : 1);
    g.tiles_n = (g.n + kGemmBN - 1) / kGemmBN;
    g.tiles_m = (g.m + kGemmBM - 1) / kGemmBM;
    const int64_t total = z * g.tiles_m * g.tiles_n;
    if (total > (int64_t{1} << 30)) return CIVIC_ERR_UNSUPPORTED;
    g.total_tiles = static_cast<int32_t>(total);
    const unsigned grid = static_cast<unsigned>((total + 7) / 8 * 8);
    // panel width: about the square root of an XCD's share of the tiles, so that its block is as tall as it is wide
    int panel = 1;
    while (static_cast<int64_t>(panel + 1) * (panel + 1) <= (total + 7) / 8) ++panel;
    g.panel = panel < g.tiles_n ? panel : g.tiles_n;
    // a grid that leaves compute units without a second workgroup takes the deeper ring
    const bool deep = total < 2 * 256;
    if (grouped) return deep ? launch_gemm_variant<true, true, 4, true>(g, grid, s) : launch_gemm_variant<true, true, 2, true>(g, grid, s);
    if (c_bf16) {
        if (b_krows) return deep ? launch_gemm_variant<true, true, 4>(g, grid, s) : launch_gemm_variant<true, true, 2>(g, grid, s);
        return deep ? launch_gemm_variant<true, false, 4>(g, grid, s) : launch_gemm_variant<true, false, 2>(g, grid, s);
    }
    if (b_krows) return deep ? launch_gemm_variant<false, true, 4>(g, grid, s) : launch_gemm_variant<false, true, 2>(g, grid, s);
    return deep ? launch_gemm_variant<false, false, 4>(g, grid, s) : launch_gemm_variant<false, false, 2>(g, grid, s);
}

// ------------------------------------------------------------------------------------------ row kernels
template <bool BF16>
__device__ __forceinline__ float enc_load(const void* p, int64_t i)
{
    if constexpr (BF16) return bf16_bits_to_float(static_cast<const uint16_t*>(p)[i]);
    else return static_cast<const float*>(p)[i];
}

// out[row, :] = Norm(LN(x[row, :])) = (x - mean) / ||x - mean|| as bf16 (a row without variance gives zeros); one
// wavefront per row.  Rows come from two matrices in one launch (the anchors, then the dense tokens): rows [0, rows_a)
// from xa into outa, the rest from xb into outb.  CH > 0: bf16 rows of up to 64 * 8 * CH elements, dim a multiple of 8
// and 16-byte aligned rows: the row is read once with 16-byte loads and stays in registers for the centred second pass
// and the store.  CH == 0: any row, three passes over a row that stays in L1/L2 after the first.
template <bool BF16, int CH>
__global__ __launch_bounds__(256) void ln_norm_rows_kernel(const void* __restrict__ xa, int64_t rows_a, const void* __restrict__ xb,
                                                           int64_t rows_b, int32_t dim, __bf16* __restrict__ outa,
                                                           __bf16* __restrict__ outb)
{
    const int lane = threadIdx.x & (kWave - 1);
    int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (row >= rows_a + rows_b) return;
    const void* x = xa;
    __bf16* out = outa;
    if (row >= rows_a) { row -= rows_a; x = xb; out = outb; }
    const int64_t base = row * dim;
    if constexpr (CH > 0) {
        static_assert(BF16, "the register-resident path reads packed bf16");
        const u32x4* src = reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(x) + base);
        const int n_chunks = dim >> 3;
        u32x4 v[CH];
        float sum = 0.f;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int k = c * kWave + lane;
            v[c] = u32x4{0u, 0u, 0u, 0u};
            if (k < n_chunks) v[c] = src[k];
#pragma unroll
            for (int e = 0; e < 4; ++e) sum += __uint_as_float(v[c][e] << 16) + __uint_as_float(v[c][e] & 0xFFFF0000u);
        }
        const float mean = wave_sum(sum) / static_cast<float>(dim);
        float n2 = 0.f;
#pragma unroll
        for (int c = 0; c < CH; ++c)
            if (c * kWave + lane < n_chunks) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float lo = __uint_as_float(v[c][e] << 16) - mean, hi = __uint_as_float(v[c][e] & 0xFFFF0000u) - mean;
                    n2 = fmaf(lo, lo, n2); n2 = fmaf(hi, hi, n2);
                }
            }
        n2 = wave_sum(n2);
        const float inv = n2 > 0.f ? 1.0f / sqrtf(n2) : 0.f;
        u32x4* dst = reinterpret_cast<u32x4*>(out + base);
#pragma unroll
        for (int c = 0; c < CH; ++c)
            if (c * kWave + lane < n_chunks) {
                u32x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const __bf16 lo = static_cast<__bf16>((__uint_as_float(v[c][e] << 16) - mean) * inv);
                    const __bf16 hi = static_cast<__bf16>((__uint_as_float(v[c][e] & 0xFFFF0000u) - mean) * inv);
                    o[e] = static_cast<uint32_t>(__builtin_bit_cast(uint16_t, lo)) | (static_cast<uint32_t>(__builtin_bit_cast(uint16_t, hi)) << 16);
                }
                dst[c * kWave + lane] = o;
            }
    } else {
        float sum = 0.f;
        for (int j = lane; j < dim; j += kWave) sum += enc_load<BF16>(x, base + j);
        const float mean = wave_sum(sum) / static_cast<float>(dim);
        float n2 = 0.f;
        for (int j = lane; j < dim; j += kWave) { const float c = enc_load<BF16>(x, base + j) - mean; n2 = fmaf(c, c, n2); }
        n2 = wave_sum(n2);
        const float inv = n2 > 0.f ? 1.0f / sqrtf(n2) : 0.f;
        for (int j = lane; j < dim; j += kWave) out[base + j] = static_cast<__bf16>((enc_load<BF16>(x, base + j) - mean) * inv);
    }
}

// p[row, 0..cols) = softmax(s[row, 0..cols)) as bf16, p[row, cols..ld_p) = 0; one wavefront per row.  Rows of up to
// 64 * 4 * CH logits (ld_s a multiple of 4) stay in registers between the maximum, the exponentials and the store: one
// trip to memory; longer rows take the three-pass loop.
template <int CH>
__global__ __launch_bounds__(256) void row_softmax_kernel(const float* __restrict__ s, int64_t rows, int32_t cols, int64_t ld_s,
                                                          __bf16* __restrict__ p, int64_t ld_p)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const float* src = s + row * ld_s;
    __bf16* dst = p + row * ld_p;
    if constexpr (CH > 0) {
        float4 v[CH];
        float mx = -INFINITY;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int j = (c * kWave + lane) * 4;
            v[c] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            if (j < cols) v[c] = *reinterpret_cast<const float4*>(src + j);   // (ld_s is padded: the vector stays inside the row)
            if (j + 1 >= cols) v[c].y = -INFINITY;
            if (j + 2 >= cols) v[c].z = -INFINITY;
            if (j + 3 >= cols) v[c].w = -INFINITY;
            mx = fmaxf(mx, fmaxf(fmaxf(v[c].x, v[c].y), fmaxf(v[c].z, v[c].w)));
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
        float sum = 0.f;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            v[c].x = __expf(v[c].x - mx); v[c].y = __expf(v[c].y - mx); v[c].z = __expf(v[c].z - mx); v[c].w = __expf(v[c].w - mx);
            sum += (v[c].x + v[c].y) + (v[c].z + v[c].w);
        }
        const float inv = 1.0f / wave_sum(sum);
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int j = (c * kWave + lane) * 4;
            if (j < ld_p) {                                                   // (ld_p is a multiple of 64)
                const __bf16 o[4] = {static_cast<__bf16>(v[c].x * inv), static_cast<__bf16>(v[c].y * inv),
                                     static_cast<__bf16>(v[c].z * inv), static_cast<__bf16>(v[c].w * inv)};
                u32x2 packed;
                packed.x = static_cast<uint32_t>(__builtin_bit_cast(uint16_t, o[0])) | (static_cast<uint32_t>(__builtin_bit_cast(uint16_t, o[1])) << 16);
                packed.y = static_cast<uint32_t>(__builtin_bit_cast(uint16_t, o[2])) | (static_cast<uint32_t>(__builtin_bit_cast(uint16_t, o[3])) << 16);
                *reinterpret_cast<u32x2*>(dst + j) = packed;
            }
        }
    } else {
        float mx = -INFINITY;
        for (int j = lane; j < cols; j += kWave) mx = fmaxf(mx, src[j]);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
        float sum = 0.f;
        for (int j = lane; j < cols; j += kWave) sum += __expf(src[j] - mx);
        const float inv = 1.0f / wave_sum(sum);
        for (int j = lane; j < ld_p; j += kWave) dst[j] = static_cast<__bf16>(j < cols ? __expf(src[j] - mx) * inv : 0.f);
    }
}

// out[b, j] = sum over rows of p[b, row, j]: the weight a dense token receives from all anchors together.
__global__ __launch_bounds__(256) void col_sum_kernel(const __bf16* __restrict__ p, int32_t rows, int32_t cols, int64_t ld_p,
                                                      int64_t batch_stride, float* __restrict__ out)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t b = blockIdx.y;
    if (j >= cols) return;
    const __bf16* src = p + b * batch_stride + j;
    float acc = 0.f;
    for (int r = 0; r < rows; ++r) acc += static_cast<float>(src[static_cast<int64_t>(r) * ld_p]);
    out[b * cols + j] = acc;
}

constexpr int kColParts = 32;             // partial column sums per column (col_part_sum_kernel below)

// out[b, c, r] = in[b, r, c] * inv[c] for r < rows, 0 for rows <= r < ld_out; 32 x 32 tiles through LDS.  inv[c] is one
// over column c's sum, taken here from its kColParts partial sums part[p, c] (0 for a column that sums to zero); with
// part null the values are copied unscaled.
template <typename TIN>
__device__ __forceinline__ void transpose_pad_block(const TIN* __restrict__ in, int32_t rows, int32_t cols, int64_t ld_in,
                                                    int64_t in_batch, const float* __restrict__ part,
                                                    __bf16* __restrict__ out, int64_t ld_out, int64_t out_batch, int64_t b)
{
    __shared__ float tile[32][33];
    __shared__ float inv_s[32];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
    const int r0 = blockIdx.x * 32, c0 = blockIdx.y * 32;
    if (part != nullptr && threadIdx.x < 32) {
        const int c = c0 + threadIdx.x;
        float t = 0.f;
        if (c < cols) {
#pragma unroll
            for (int p = 0; p < kColParts; ++p) t += part[static_cast<int64_t>(p) * cols + c];
        }
        inv_s[threadIdx.x] = t != 0.f ? 1.0f / t : 0.f;      // (read after the barrier below)
    }
    for (int k = ty; k < 32; k += 8) {
        const int r = r0 + k, c = c0 + tx;
        float v = 0.f;
        if (r < rows && c < cols) {
            if constexpr (std::is_same<TIN, float>::value) v = in[b * in_batch + static_cast<int64_t>(r) * ld_in + c];
            else v = static_cast<float>(in[b * in_batch + static_cast<int64_t>(r) * ld_in + c]);
        }
        tile[k][tx] = v;
    }
    __syncthreads();
    for (int k = ty; k < 32; k += 8) {
        const int c = c0 + k, r = r0 + tx;
        if (c < cols && r < ld_out) {
            const float sc = part ? inv_s[k] : 1.0f;
            out[b * out_batch + static_cast<int64_t>(c) * ld_out + r] = static_cast<__bf16>(tile[tx][k] * sc);
        }
    }
}

template <typename TIN>
__global__ __launch_bounds__(256) void transpose_pad_kernel(const TIN* __restrict__ in, int32_t rows, int32_t cols, int64_t ld_in,
                                                            int64_t in_batch, const float* __restrict__ part,
                                                            __bf16* __restrict__ out, int64_t ld_out, int64_t out_batch)
{
    transpose_pad_block<TIN>(in, rows, cols, ld_in, in_batch, part, out, ld_out, out_batch, blockIdx.z);
}

// The same for the items of a group (grid z): item i's rows of r [.., cols], every column over its own sum (the item's
// kColParts x cols partial sums), to the item's block of the padded Rbar^T scratch (cols x its padded length); blocks
// past an item's padded length write nothing.
__global__ __launch_bounds__(256) void transpose_pad_grouped_kernel(const float* __restrict__ r, int32_t cols,
                                                                    const float* __restrict__ part, __bf16* __restrict__ out, Group grp)
{
    const int i = blockIdx.z;
    const int32_t r0 = grp.row[i], p0 = grp.pad_row[i];
    transpose_pad_block<float>(r + static_cast<int64_t>(r0) * cols, grp.row[i + 1] - r0, cols, cols, 0,
                               part + static_cast<int64_t>(i) * kColParts * cols, out + static_cast<int64_t>(cols) * p0,
                               grp.pad_row[i + 1] - p0, 0, 0);
}

// Column sums of r [rows, cols], first step: block (x, y) adds the rows y, y + gridDim.y, ... of 64 columns (its four
// wavefronts four rows apart, coalesced 256-byte reads, meeting in LDS) into part[y, c]; the transposing kernel above
// adds a column's kColParts partial sums and inverts the total.
__device__ __forceinline__ void col_part_sum_block(const float* __restrict__ r, int32_t rows, int32_t cols, float* __restrict__ part)
{
    __shared__ float lds_part[4][kWave];
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
    const int c = blockIdx.x * kWave + lane;
    float acc = 0.f;
    if (c < cols)
        for (int m = blockIdx.y * 4 + wv; m < rows; m += 4 * kColParts) acc += r[static_cast<int64_t>(m) * cols + c];
    lds_part[wv][lane] = acc;
    __syncthreads();
    if (wv == 0 && c < cols)
        part[static_cast<int64_t>(blockIdx.y) * cols + c] = (lds_part[0][lane] + lds_part[1][lane]) + (lds_part[2][lane] + lds_part[3][lane]);
}

__global__ __launch_bounds__(256) void col_part_sum_kernel(const float* __restrict__ r, int32_t rows, int32_t cols, float* __restrict__ part)
{
    col_part_sum_block(r, rows, cols, part);
}

__global__ __launch_bounds__(256) void col_part_sum_grouped_kernel(const float* __restrict__ r, int32_t cols, float* __restrict__ part, Group grp)
{
    const int i = blockIdx.z;                                 // the item: its own rows, its own kColParts x cols partial sums
    const int32_t r0 = grp.row[i];
    col_part_sum_block(r + static_cast<int64_t>(r0) * cols, grp.row[i + 1] - r0, cols, part + static_cast<int64_t>(i) * kColParts * cols);
}

static int64_t pad64(int64_t x) { return (x + 63) / 64 * 64; }
static size_t align256(size_t x) { return (x + 255) / 256 * 256; }

struct AggPlan {                         // byte offsets into the workspace of civic_anchor_aggregate
    int64_t t_pad;
    size_t qa, k0, s, p, total;
};

static void agg_plan(int32_t batch, int32_t n_tokens, int32_t n_anchors, int32_t dim, AggPlan* p)
{
    p->t_pad = pad64(n_tokens);
    size_t off = 0;
    p->qa = off; off += align256(static_cast<size_t>(n_anchors) * dim * 2);
    p->k0 = off; off += align256(static_cast<size_t>(batch) * n_tokens * dim * 2);
    p->s = off;  off += align256(static_cast<size_t>(batch) * n_anchors * p->t_pad * 4);
    p->p = off;  off += align256(static_cast<size_t>(batch) * n_anchors * p->t_pad * 2);
    p->total = off;
}

struct CompressPlan {                    // byte offsets into the workspace of civic_kv_compress
    int64_t m_pad;
    size_t part, rt, xt, total;
};

static void compress_plan(int32_t batch, int32_t n_rows, int32_t n_mem, int32_t width, CompressPlan* p)
{
    p->m_pad = pad64(n_rows);
    size_t off = 0;
    p->part = off; off += align256(static_cast<size_t>(n_mem) * 4 * kColParts);
    p->rt = off;  off += align256(static_cast<size_t>(n_mem) * p->m_pad * 2);
    // (a transposed copy of K, then V, only for widths whose rows are not whole 16-byte chunks)
    p->xt = off;  off += width % 8 ? align256(static_cast<size_t>(batch) * width * p->m_pad * 2) : 0;
    p->total = off;
}

static bool agg_sizes_ok(int32_t batch, int32_t n_tokens, int32_t n_anchors, int32_t dim)
{
    return batch >= 0 && n_tokens > 0 && n_anchors > 0 && dim > 0;
}

}  // namespace civic

extern "C" size_t civic_anchor_aggregate_workspace_bytes(int32_t batch, int32_t n_tokens, int32_t n_anchors, int32_t dim)
{
    if (!civic::agg_sizes_ok(batch, n_tokens, n_anchors, dim)) return 0;
    civic::AggPlan p;
    civic::agg_plan(batch, n_tokens, n_anchors, dim, &p);
    return p.total;
}

extern "C" int civic_anchor_aggregate(const void* x0, const void* anchors, int dtype, int32_t batch, int32_t n_tokens,
                                      int32_t n_anchors, int32_t dim, float inv_tau, void* z0, float* token_weight,
                                      void* workspace, size_t workspace_bytes, void* stream)
{
    using namespace civic;
    const int esz = dtype_size(dtype);
    if (!esz || !agg_sizes_ok(batch, n_tokens, n_anchors, dim)) return CIVIC_ERR_INVALID_ARG;
    if (!(inv_tau >= 0.f) || std::isinf(inv_tau)) return CIVIC_ERR_INVALID_ARG;
    if (batch > 0 && (!x0 || !anchors || !z0)) return CIVIC_ERR_INVALID_ARG;
    if (!aligned16(x0) || !aligned16(anchors) || !aligned16(z0) || (reinterpret_cast<uintptr_t>(token_weight) & 3u)) return CIVIC_ERR_INVALID_ARG;
    if (dim % 64) return CIVIC_ERR_UNSUPPORTED;                          // the first contraction runs over dim in tiles of 64
    if (dtype != CIVIC_BF16) return CIVIC_ERR_UNSUPPORTED;               // z0 leaves the MFMA path as bf16
    if (batch > 65535 || static_cast<int64_t>(n_tokens) * dim * 2 >= (int64_t{1} << 32) ||
        static_cast<int64_t>(n_anchors) * pad64(n_tokens) * 2 >= (int64_t{1} << 32))
        return CIVIC_ERR_UNSUPPORTED;                                     // 32-bit row offsets inside one batch item
    AggPlan p;
    agg_plan(batch, n_tokens, n_anchors, dim, &p);
    if (!workspace || workspace_bytes < p.total || !aligned16(workspace)) return CIVIC_ERR_WORKSPACE;
    if (batch == 0) return CIVIC_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    __bf16* qa = reinterpret_cast<__bf16*>(ws + p.qa);
    __bf16* k0 = reinterpret_cast<__bf16*>(ws + p.k0);
    float* sl = reinterpret_cast<float*>(ws + p.s);
    __bf16* pw = reinterpret_cast<__bf16*>(ws + p.p);
    const int64_t rows_x = static_cast<int64_t>(batch) * n_tokens;

    // Q_A = Norm(LN(A)), K_0 = Norm(LN(X_0)): one launch over the rows of both
    {
        const dim3 grid(static_cast<unsigned>((n_anchors + rows_x + 3) / 4));
        const int chunks = (dim / 8 + kWave - 1) / kWave;                              // 16-byte pieces per lane
#define CIVIC_LN_CASE(N) civic::launch((ln_norm_rows_kernel<true, N>), grid, dim3(256), 0, s, anchors, static_cast<int64_t>(n_anchors), \
                                            x0, rows_x, dim, qa, k0)
        if (chunks <= 1) CIVIC_LN_CASE(1);
        else if (chunks <= 2) CIVIC_LN_CASE(2);
        else if (chunks <= 4) CIVIC_LN_CASE(4);
        else if (chunks <= 8) CIVIC_LN_CASE(8);
        else CIVIC_LN_CASE(0);
#undef CIVIC_LN_CASE
    }
    int rc = check_launch();
    if (rc != CIVIC_OK) return rc;
    // logits = Q_A K_0^T / tau  [n_anchors x n_tokens] per batch item, fp32
    GemmArgs g1;
    g1.b_alt = nullptr; g1.c_alt = nullptr; g1.kb_rows = 0;
    g1.a = qa; g1.b = k0; g1.c = sl;
    g1.lda = dim; g1.ldb = dim; g1.ldc = p.t_pad;
    g1.sa = 0; g1.sb = static_cast<int64_t>(n_tokens) * dim; g1.sc = static_cast<int64_t>(n_anchors) * p.t_pad;
    g1.m = n_anchors; g1.n = n_tokens; g1.k = dim; g1.alpha = inv_tau;
    rc = launch_gemm(g1, batch, false, false, s);
    if (rc != CIVIC_OK) return rc;
    // W_A = softmax over the dense tokens, bf16, zero in the padding
    const int64_t rows_w = static_cast<int64_t>(batch) * n_anchors;
    {
        const dim3 grid(static_cast<unsigned>((rows_w + 3) / 4));
        const int chunks = static_cast<int>((p.t_pad / 4 + kWave - 1) / kWave);       // float4 per lane
#define CIVIC_SOFTMAX_CASE(N) civic::launch((row_softmax_kernel<N>), grid, dim3(256), 0, s, sl, rows_w, n_tokens, p.t_pad, pw, p.t_pad)
        if (chunks <= 4) CIVIC_SOFTMAX_CASE(4);
        else if (chunks <= 8) CIVIC_SOFTMAX_CASE(8);
        else if (chunks <= 16) CIVIC_SOFTMAX_CASE(16);
        else if (chunks <= 32) CIVIC_SOFTMAX_CASE(32);
        else CIVIC_SOFTMAX_CASE(0);
#undef CIVIC_SOFTMAX_CASE
    }
    if (token_weight)
        civic::launch(col_sum_kernel, dim3(static_cast<unsigned>((n_tokens + 255) / 256), static_cast<unsigned>(batch)), dim3(256), 0, s,
                           pw, n_anchors, n_tokens, p.t_pad, static_cast<int64_t>(n_anchors) * p.t_pad, token_weight);
    rc = check_launch();
    if (rc != CIVIC_OK) return rc;
    // Z_0 = W_A X_0, X_0 read where it lies (tokens are its rows: the contraction index is the row index)
    GemmArgs g2;
    g2.b_alt = nullptr; g2.c_alt = nullptr;
    g2.a = pw; g2.b = static_cast<const __bf16*>(x0); g2.c = z0;
    g2.lda = p.t_pad; g2.ldb = dim; g2.ldc = dim;
    g2.sa = static_cast<int64_t>(n_anchors) * p.t_pad; g2.sb = static_cast<int64_t>(n_tokens) * dim; g2.sc = static_cast<int64_t>(n_anchors) * dim;
    g2.m = n_anchors; g2.n = dim; g2.k = static_cast<int32_t>(p.t_pad); g2.kb_rows = n_tokens; g2.alpha = 1.0f;
    return launch_gemm(g2, batch, true, true, s);
}

extern "C" size_t civic_kv_compress_workspace_bytes(int32_t batch, int32_t n_rows, int32_t n_mem, int32_t width)
{
    if (batch < 0 || n_rows <= 0 || n_mem <= 0 || width <= 0) return 0;
    civic::CompressPlan p;
    civic::compress_plan(batch, n_rows, n_mem, width, &p);
    return p.total;
}

extern "C" int civic_kv_compress(const void* k, const void* v, int dtype, const float* r, int32_t batch, int32_t n_rows,
                                 int32_t n_mem, int32_t width, void* k_c, void* v_c, void* workspace, size_t workspace_bytes,
                                 void* stream)
{
    using namespace civic;
    const int esz = dtype_size(dtype);
    if (!esz || batch < 0 || n_rows <= 0 || n_mem <= 0 || width <= 0) return CIVIC_ERR_INVALID_ARG;
    if (!r || (batch > 0 && (!k || !v || !k_c || !v_c))) return CIVIC_ERR_INVALID_ARG;
    if (!aligned16(k) || !aligned16(v) || !aligned16(k_c) || !aligned16(v_c) || !aligned16(r)) return CIVIC_ERR_INVALID_ARG;
    if (dtype != CIVIC_BF16) return CIVIC_ERR_UNSUPPORTED;
    if (batch > 65535 || pad64(n_rows) * static_cast<int64_t>(width) * 2 >= (int64_t{1} << 32) ||
        pad64(n_rows) * static_cast<int64_t>(n_mem) * 2 >= (int64_t{1} << 32))
        return CIVIC_ERR_UNSUPPORTED;
    CompressPlan p;
    compress_plan(batch, n_rows, n_mem, width, &p);
    if (!workspace || workspace_bytes < p.total || !aligned16(workspace)) return CIVIC_ERR_WORKSPACE;
    if (batch == 0) return CIVIC_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    __bf16* rt = reinterpret_cast<__bf16*>(ws + p.rt);
    __bf16* xt = reinterpret_cast<__bf16*>(ws + p.xt);
    // Rbar^T [n_mem x m_pad]: every column of R over its sum, transposed, zero beyond n_rows
    float* part = reinterpret_cast<float*>(ws + p.part);
    civic::launch(col_part_sum_kernel, dim3(static_cast<unsigned>((n_mem + kWave - 1) / kWave), kColParts), dim3(256), 0, s, r, n_rows,
                       n_mem, part);
    civic::launch((transpose_pad_kernel<float>), dim3(static_cast<unsigned>(p.m_pad / 32), static_cast<unsigned>((n_mem + 31) / 32), 1u),
                       dim3(256), 0, s, r, n_rows, n_mem, static_cast<int64_t>(n_mem), int64_t{0}, part, rt, p.m_pad, int64_t{0});
    int rc = check_launch();
    if (rc != CIVIC_OK) return rc;
    GemmArgs g;
    g.a = rt; g.lda = p.m_pad; g.ldc = width;
    g.sa = 0; g.sc = static_cast<int64_t>(n_mem) * width;
    g.m = n_mem; g.n = width; g.k = static_cast<int32_t>(p.m_pad); g.alpha = 1.0f;
    if (width % 8 == 0) {
        // X_c = Rbar^T X with X read where it lies (its rows are the contraction index); K and V in one launch
        g.b = static_cast<const __bf16*>(k); g.c = k_c; g.b_alt = static_cast<const __bf16*>(v); g.c_alt = v_c;
        g.ldb = width; g.sb = static_cast<int64_t>(n_rows) * width; g.kb_rows = n_rows;
        return launch_gemm(g, batch, true, true, s);
    }
    const void* src[2] = {k, v};
    void* dst[2] = {k_c, v_c};
    for (int t = 0; t < 2; ++t) {
        // X^T [width x m_pad] per batch item, then X_c = Rbar^T (X^T)^T
        civic::launch((transpose_pad_kernel<__bf16>), dim3(static_cast<unsigned>(p.m_pad / 32), static_cast<unsigned>((width + 31) / 32),
                                                                static_cast<unsigned>(batch)),
                           dim3(256), 0, s, static_cast<const __bf16*>(src[t]), n_rows, width, static_cast<int64_t>(width),
                           static_cast<int64_t>(n_rows) * width, static_cast<const float*>(nullptr), xt, p.m_pad,
                           static_cast<int64_t>(width) * p.m_pad);
        rc = check_launch();
        if (rc != CIVIC_OK) return rc;
        g.b = xt; g.c = dst[t]; g.b_alt = nullptr; g.c_alt = nullptr; g.kb_rows = 0;
        g.ldb = p.m_pad; g.sb = static_cast<int64_t>(width) * p.m_pad;
        rc = launch_gemm(g, batch, true, false, s);
        if (rc != CIVIC_OK) return rc;
    }
    return CIVIC_OK;
}

// ---------------------------------------------------------------------------------------------- ragged batches
namespace civic {

// host [batch + 1], starting at 0, strictly increasing (every item has at least one row)
static bool offsets_ok(const int64_t* off, int32_t batch)
{
    if (!off || off[0] != 0) return false;
    for (int32_t b = 0; b < batch; ++b)
        if (off[b + 1] <= off[b] || off[b + 1] - off[b] > INT32_MAX) return false;
    return true;
}

}  // namespace civic

namespace civic {

struct RaggedPlan {                      // byte offsets into the workspace of civic_kv_compress_ragged
    int64_t pad_total;                   // sum of the items' row counts, each rounded up to 64
    size_t part, rt, total;
};

static void ragged_plan(int32_t batch, const int64_t* off, int32_t n_mem, RaggedPlan* p)
{
    p->pad_total = 0;
    for (int32_t b = 0; b < batch; ++b) p->pad_total += pad64(off[b + 1] - off[b]);
    size_t at = 0;
    p->part = at; at += align256(static_cast<size_t>(batch) * n_mem * 4 * kColParts);
    p->rt = at;   at += align256(static_cast<size_t>(n_mem) * p->pad_total * 2);
    p->total = at;
}

}  // namespace civic

extern "C" size_t civic_kv_compress_ragged_workspace_bytes(int32_t batch, const int64_t* row_offsets, int32_t n_mem, int32_t width)
{
    if (batch <= 0 || n_mem <= 0 || width <= 0 || !civic::offsets_ok(row_offsets, batch)) return 0;
    civic::RaggedPlan p;                                      // every item keeps its own column sums and its own Rbar^T
    civic::ragged_plan(batch, row_offsets, n_mem, &p);
    return p.total;
}

extern "C" int civic_kv_compress_ragged(const void* k, const void* v, int dtype, const float* r, int32_t batch,
                                        const int64_t* row_offsets, int32_t n_mem, int32_t width, void* k_c, void* v_c,
                                        void* workspace, size_t workspace_bytes, void* stream)
{
    using namespace civic;
    const int esz = dtype_size(dtype);
    if (!esz || batch < 0 || n_mem <= 0 || width <= 0) return CIVIC_ERR_INVALID_ARG;
    if (batch == 0) return CIVIC_OK;
    if (!offsets_ok(row_offsets, batch)) return CIVIC_ERR_INVALID_ARG;
    if (!r || !k || !v || !k_c || !v_c) return CIVIC_ERR_INVALID_ARG;
    if (!aligned16(k) || !aligned16(v) || !aligned16(k_c) || !aligned16(v_c) || !aligned16(r)) return CIVIC_ERR_INVALID_ARG;
    if (dtype != CIVIC_BF16) return CIVIC_ERR_UNSUPPORTED;
    // every item's first row must be 16-byte aligned in K, V and R: whole 16-byte pieces per row
    if (width % 8 || n_mem % 4) return CIVIC_ERR_UNSUPPORTED;
    if (row_offsets[batch] > INT32_MAX) return CIVIC_ERR_UNSUPPORTED;       // (row numbers travel as 32-bit kernel arguments)
    for (int32_t b = 0; b < batch; ++b) {                                     // 32-bit row offsets inside one item, as in civic_kv_compress
        const int64_t padded = pad64(row_offsets[b + 1] - row_offsets[b]);
        if (padded * width * 2 >= (int64_t{1} << 32) || padded * n_mem * 2 >= (int64_t{1} << 32)) return CIVIC_ERR_UNSUPPORTED;
    }
    RaggedPlan p;
    ragged_plan(batch, row_offsets, n_mem, &p);
    if (p.pad_total > INT32_MAX) return CIVIC_ERR_UNSUPPORTED;                // (padded row numbers are 32-bit as well)
    if (!workspace || workspace_bytes < p.total || !aligned16(workspace)) return CIVIC_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    // Groups of up to kGroupItems items, three launches each: the partial column sums of every item's R rows,
    // Rbar^T of every item (transposed, scaled, zero-padded to a multiple of 64 contraction rows) and ONE grouped GEMM
    // for K_c and V_c of all items (grid z = item x tensor; an item's contraction length comes from the group's table).
    int64_t pad_done = 0;
    for (int32_t b0 = 0; b0 < batch; b0 += kGroupItems) {
        const int32_t nb = batch - b0 < kGroupItems ? batch - b0 : kGroupItems;
        GemmArgs g;
        int32_t longest_pad = 0;
        g.grp.pad_row[0] = 0;
        for (int32_t i = 0; i <= kGroupItems; ++i) {
            const int32_t at = i <= nb ? i : nb;                              // (entries past the group repeat its end)
            g.grp.row[i] = static_cast<int32_t>(row_offsets[b0 + at]);
            if (i > 0) {
                const int32_t padded = i <= nb ? static_cast<int32_t>(pad64(row_offsets[b0 + i] - row_offsets[b0 + i - 1])) : 0;
                g.grp.pad_row[i] = g.grp.pad_row[i - 1] + padded;
                longest_pad = padded > longest_pad ? padded : longest_pad;
            }
        }
        float* part = reinterpret_cast<float*>(ws + p.part) + static_cast<int64_t>(b0) * n_mem * kColParts;
        __bf16* rt = reinterpret_cast<__bf16*>(ws + p.rt) + static_cast<int64_t>(n_mem) * pad_done;
        civic::launch(col_part_sum_grouped_kernel, dim3(static_cast<unsigned>((n_mem + kWave - 1) / kWave), kColParts, static_cast<unsigned>(nb)),
                      dim3(256), 0, s, r, n_mem, part, g.grp);
        civic::launch(transpose_pad_grouped_kernel, dim3(static_cast<unsigned>(longest_pad / 32), static_cast<unsigned>((n_mem + 31) / 32),
                                                        static_cast<unsigned>(nb)),
                      dim3(256), 0, s, r, n_mem, part, rt, g.grp);
        int rc = check_launch();
        if (rc != CIVIC_OK) return rc;
        g.a = rt; g.lda = 0; g.sa = 0; g.k = 0; g.kb_rows = 0;                // (per item, from the table)
        g.b = static_cast<const __bf16*>(k); g.b_alt = static_cast<const __bf16*>(v); g.ldb = width; g.sb = 0;
        g.c = static_cast<__bf16*>(k_c) + static_cast<int64_t>(b0) * n_mem * width;
        g.c_alt = static_cast<__bf16*>(v_c) + static_cast<int64_t>(b0) * n_mem * width;
        g.ldc = width; g.sc = static_cast<int64_t>(n_mem) * width;
        g.m = n_mem; g.n = width; g.alpha = 1.0f;
        rc = launch_gemm(g, nb, true, true, s, true);
        if (rc != CIVIC_OK) return rc;
        pad_done += g.grp.pad_row[nb];
    }
    return CIVIC_OK;
}
