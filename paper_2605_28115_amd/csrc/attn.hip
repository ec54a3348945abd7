// civic_prefill_attn: dense grouped-query prefill attention over the compact sequence (the
// beta * N_l * (L+M_p)^2 * D_l term of Eq. 7; softmax(Q K^T / sqrt(d)) V as in Eq. 9).
//
// bf16 path (MFMA-bound): flash-style, one 512-thread workgroup = 8 wavefronts x 32 query rows over
// one KV head.  With four or more query heads per KV head the wavefronts are 4 heads x 2 row tiles
// (64 rows), so one K/V tile staged in LDS serves the whole group and all wavefronts share the
// causal extent; smaller groups put more row tiles of the same head in the workgroup.
//   - K/V tiles of 64 keys go from global memory straight into a small LDS ring
//     (global_load_lds_dwordx4, 16 bytes per lane), one tile ahead of the one being consumed; Q is
//     staged the same way, so the kernel has no register-destination global load, and the ring is
//     tracked with explicit vmcnt waits and fence-free workgroup barriers.  Rows keep a 256-byte
//     pitch and the 16-byte chunks are XOR-swizzled, so neither the 128-bit K reads nor the
//     transposing V reads hit a bank conflict.
//   - Scores are computed TRANSPOSED, S^T = K Q^T with v_mfma_f32_32x32x16_bf16: a lane owns one
//     query column, so softmax row statistics are in-lane reductions plus one exchange between the
//     two half-waves, and the rescale factor is a per-lane scalar.  The exponentiated tile, rounded
//     to bf16, is already laid out as the B operand of O^T += V^T P^T; the matching A operand comes
//     from the row-major V tile through the LDS transpose read ds_read_b64_tr_b16.
//   - Little vector work per score: a probability is exp2(fma(score, scale * log2 e, -offset)), one
//     fused multiply-add and one v_exp_f32; the offset is the first tile's row maximum and moves
//     later only when the row sums show that a tile outgrew it (no per-tile maximum pass).
//   - fp32 accumulation, row sums taken from the rounded probabilities with v_dot2c_f32_bf16, bf16
//     output (nearest even) staged through LDS into whole 16-byte row segments.
//   - Workgroups are ordered heaviest causal row tile first (row tile on grid y, the rest of the block
//     index decoded with multiply-high constants from the launch: no integer division ahead of Q's loads).
//   - Masking costs a compare and a select per score and only on tiles that cross the diagonal or the end
//     of the sequence; a wavefront that cannot see the second half of such a tile computes the first only.
//   - civic_prefill_attn_kv: the workgroup of a KV head's first head block also copies the K/V rows of its
//     own query rows into the caches (8 threads per row, same address for K and V).
//
// fp32 path and head sizes the MFMA path does not cover: a plain fp32 kernel, one wavefront per
// query row (lanes over keys for Q K^T, lanes over channels for P V).
#include <algorithm>
#include <array>
#include <cmath>
#include <type_traits>

#include "civic_internal.h"

// LDS fragments (K rows, transposed V) are read this many MFMAs ahead of the MFMA that consumes them (build-time
// knob for A/B runs; 2-4 measure within 1 % of each other, 2 needs the fewest registers).
#ifndef CIVIC_ATTN_DIST
#define CIVIC_ATTN_DIST 2
#endif

namespace civic {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kRaggedItems = 64;          // items of one ragged launch (longer lists go out in several)

struct AttnArgs {
    const void* q; const void* k; const void* v; void* out;
    int64_t qs[3], ks[3], os[3];          // element strides: batch, token, head
    int32_t batch, seq, n_q_heads, n_kv_heads, head_dim, causal;
    int32_t kv_seq;                       // keys per sample (= seq except for civic_cross_attn, which has no mask)
    float scale;                          // softmax scale (natural-exponent domain)
    int32_t heads_per_block, row_tiles;   // MFMA path: block shape and number of 32*rows_per_block tiles
    int32_t paired;                       // MFMA path: a workgroup walks two row tiles, a heavy and a light one
    // MFMA path, block index -> (head block, kv head, batch) without integer division: q heads per kv head,
    // head blocks per kv head, log2(heads_per_block), ceil(2^32 / d) for d = head blocks, kv heads (0 for d = 1)
    int32_t group, head_blocks, hb_shift;
    uint32_t magic_head_blocks, magic_kv_heads;
    // fused KV-cache write (MFMA path; null = none): caches are dense [batch, n_kv_heads, s_max, head_dim]
    void* k_cache; void* v_cache;
    int64_t s_max, pos0;
    // rotary embedding of Q from a (cos, sin) table [batch, seq, head_dim / 2] (null = none): civic_prefill_attn_rope
    const float2* q_cs;
    // ragged queries (civic_cross_attn_ragged; read by the RAGGED instantiations only): `batch` items packed along the
    // token axis, item b owning query and output rows [item_row[b], item_row[b + 1]); `seq` is the longest item
    int32_t item_row[kRaggedItems + 1];
    int32_t kv_packed;                    // ragged: keys and values are packed along the token axis like the queries
};

// ------------------------------------------------------------------------------------ fp32 ALU path
template <bool BF16>
__device__ __forceinline__ float load_elem(const void* p, int64_t i)
{
    if constexpr (BF16) return bf16_bits_to_float(static_cast<const uint16_t*>(p)[i]);
    else return static_cast<const float*>(p)[i];
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

template <bool BF16>
__global__ __launch_bounds__(256) void attn_plain_kernel(AttnArgs a)
{
    __shared__ float q_s[4][CIVIC_MAX_HEAD_DIM];
    __shared__ float p_s[4][kWave];
    const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x >> 6;
    const int i = blockIdx.x * 4 + w, h = blockIdx.y, b = blockIdx.z;
    if (i >= a.seq) return;                                   // no workgroup barrier below
    const int g = h / (a.n_q_heads / a.n_kv_heads), d = a.head_dim;
    const int64_t q_off = b * a.qs[0] + i * a.qs[1] + h * a.qs[2];
    const int64_t kv_off = b * a.ks[0] + g * a.ks[2];
    // KV-cache write of this query row's K and V row (the first head of every KV group does it; 16-byte pieces, loads
    // and stores fly under everything below), so that this path needs no second launch either
    if (a.k_cache != nullptr && h == g * (a.n_q_heads / a.n_kv_heads)) {
        constexpr int EPP = BF16 ? 8 : 4;                     // elements per piece
        const int64_t src = kv_off + static_cast<int64_t>(i) * a.ks[1];
        const int64_t dst = ((static_cast<int64_t>(b) * a.n_kv_heads + g) * a.s_max + a.pos0 + i) * d;
        for (int c = lane * EPP; c < d; c += kWave * EPP) {
            if constexpr (BF16) {
                *reinterpret_cast<uint4*>(static_cast<uint16_t*>(a.k_cache) + dst + c) = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(a.k) + src + c);
                *reinterpret_cast<uint4*>(static_cast<uint16_t*>(a.v_cache) + dst + c) = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(a.v) + src + c);
            } else {
                *reinterpret_cast<float4*>(static_cast<float*>(a.k_cache) + dst + c) = *reinterpret_cast<const float4*>(static_cast<const float*>(a.k) + src + c);
                *reinterpret_cast<float4*>(static_cast<float*>(a.v_cache) + dst + c) = *reinterpret_cast<const float4*>(static_cast<const float*>(a.v) + src + c);
            }
        }
    }
    for (int c = lane; c < d; c += kWave) q_s[w][c] = load_elem<BF16>(a.q, q_off + c) * a.scale;
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (a.q_cs) {                                             // rotary embedding: pairs (c, c + d/2) of the query row
        const float2* cs = a.q_cs + (static_cast<int64_t>(b) * a.seq + i) * (d / 2);
        for (int c = lane; c < d / 2; c += kWave) {
            const float x0 = q_s[w][c], x1 = q_s[w][c + d / 2];
            const float2 t = cs[c];
            rope_pair(x0, x1, t.x, t.y, q_s[w][c], q_s[w][c + d / 2]);
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }

    float acc[CIVIC_MAX_HEAD_DIM / kWave];
#pragma unroll
    for (int t = 0; t < CIVIC_MAX_HEAD_DIM / kWave; ++t) acc[t] = 0.f;
    float m = -INFINITY, l = 0.f;
    const int last = a.causal ? i : a.kv_seq - 1;
    for (int j0 = 0; j0 <= last; j0 += kWave) {
        const int j = j0 + lane;
        float z = -INFINITY;
        if (j <= last) {
            const int64_t base = kv_off + j * a.ks[1];
            float dot = 0.f;
            for (int c = 0; c < d; c += 8) {
                if constexpr (BF16) {
                    const uint4 raw = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(a.k) + base + c);
                    const uint32_t wds[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        dot = fmaf(q_s[w][c + 2 * e], __uint_as_float(wds[e] << 16), dot);
                        dot = fmaf(q_s[w][c + 2 * e + 1], __uint_as_float(wds[e] & 0xFFFF0000u), dot);
                    }
                } else {
                    const float4 lo = *reinterpret_cast<const float4*>(static_cast<const float*>(a.k) + base + c);
                    const float4 hi = *reinterpret_cast<const float4*>(static_cast<const float*>(a.k) + base + c + 4);
                    dot = fmaf(q_s[w][c], lo.x, dot); dot = fmaf(q_s[w][c + 1], lo.y, dot);
                    dot = fmaf(q_s[w][c + 2], lo.z, dot); dot = fmaf(q_s[w][c + 3], lo.w, dot);
                    dot = fmaf(q_s[w][c + 4], hi.x, dot); dot = fmaf(q_s[w][c + 5], hi.y, dot);
                    dot = fmaf(q_s[w][c + 6], hi.z, dot); dot = fmaf(q_s[w][c + 7], hi.w, dot);
                }
            }
            z = dot;
        }
        const float m_new = fmaxf(m, wave_max(z));           // finite: key j0 is always visible
        const float p = expf(z - m_new);
        const float alpha = expf(m - m_new);
        l = l * alpha + wave_sum(p);
        m = m_new;
        p_s[w][lane] = p;
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const int nk = min(kWave, last - j0 + 1);
#pragma unroll
        for (int t = 0; t < CIVIC_MAX_HEAD_DIM / kWave; ++t) {
            const int c = lane + t * kWave;
            if (c < d) {
                float s = acc[t] * alpha;
                for (int jj = 0; jj < nk; ++jj)
                    s = fmaf(p_s[w][jj], load_elem<BF16>(a.v, kv_off + (j0 + jj) * a.ks[1] + c), s);
                acc[t] = s;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    const float inv = 1.f / l;
    const int64_t o_off = b * a.os[0] + i * a.os[1] + h * a.os[2];
#pragma unroll
    for (int t = 0; t < CIVIC_MAX_HEAD_DIM / kWave; ++t) {
        const int c = lane + t * kWave;
        if (c < d) {
            const float o = acc[t] * inv;
            if constexpr (BF16) static_cast<__bf16*>(a.out)[o_off + c] = static_cast<__bf16>(o);
            else static_cast<float*>(a.out)[o_off + c] = o;
        }
    }
}

// --------------------------------------------------------------------------------------- MFMA path
constexpr int kBN = 64;                 // keys per LDS tile

typedef short s16x4 __attribute__((ext_vector_type(4)));

// LDS transpose read (gfx950): the 16 lanes of a group each name 4 consecutive bf16 of a 4 x 16 block
// (lane i -> row i/4, columns 4(i%4)..+3); lane i receives column i of the block, rows 0..3.
__device__ __forceinline__ s16x4 lds_read_tr16(const __bf16* p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (s16x4 __attribute__((address_space(3)))*)(const_cast<__bf16*>(p)));
}

// K/V tiles live in LDS with a fixed row pitch of PITCH 16-byte chunks and an XOR swizzle of the chunk
// index by a function of the row, so that no padding is needed (global -> LDS loads write 64
// consecutive 16-byte slots per wavefront instruction) and both the 128-bit K reads (16 lanes = 16
// consecutive rows, same logical chunk) and the transposing 64-bit V reads (32 lanes = 4 consecutive
// rows x 4 chunks) fall on distinct banks.
template <int PITCH>
__device__ __forceinline__ int swz(int row)
{
    if constexpr (PITCH == 16) return ((row & 3) << 2) | ((row >> 2) & 3);
    else return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
}


typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) char lds_char;

// 16 bytes per lane from global memory (scalar base + per-lane byte offset) straight into LDS at
// lds_addr + LDS_IMM + lane * 16 (lds_addr wave-uniform).  Issued as inline assembly on purpose: the pipeline
// tracks these loads with explicit s_waitcnt vmcnt(N), and an LDS read the compiler could see racing
// with an asynchronous LDS write would make it drain the whole load queue first.  m0 is written and not
// declared: the register is reserved (the compiler rejects it as a clobber), never allocated, and set by the
// compiler only directly in front of an instruction that reads it, of which this file has none.
template <int LDS_IMM>
__device__ __forceinline__ void dma16(const void* base, uint32_t byte_off, uint32_t lds_addr)
{
    // (the LDS address is lds_addr + LDS_IMM, added here so that one scalar register serves every instruction
    // of a tile instead of one register per instruction)
    asm volatile("s_add_u32 m0, %0, %3\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(byte_off), "s"(base), "n"(LDS_IMM) : "memory", "scc");
}

// dma16 with the LDS immediate BASE_IMM + j * 1024 for a loop index j that is a constant after unrolling
// (at most 16 instructions per wavefront and tile).
template <int BASE_IMM, int J = 0>
__device__ __forceinline__ void dma16_at(const void* base, uint32_t byte_off, uint32_t lds_addr,
                                         std::integral_constant<int, BASE_IMM> imm, int j)
{
    if constexpr (J < 16) {
        if (j == J) dma16<BASE_IMM + J * kWave * 16>(base, byte_off, lds_addr);
        else dma16_at<BASE_IMM, J + 1>(base, byte_off, lds_addr, imm, j);
    }
}

// Workgroup barrier without the memory fence __syncthreads() implies (which would wait for every
// outstanding load, including the prefetches that are meant to stay in flight).
__device__ __forceinline__ void block_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// The same pointer with both halves forced into scalar registers (the value must be wave-uniform).
__device__ __forceinline__ const char* uniform_ptr(const void* p)
{
    const uint64_t bits = reinterpret_cast<uint64_t>(p);
    // the builtin returns a signed int: widen each half as unsigned
    const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<uint32_t>(bits >> 32)));
    const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<uint32_t>(bits)));
    return reinterpret_cast<const char*>((static_cast<uint64_t>(hi) << 32) | lo);
}

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    // s_waitcnt immediate (gfx9): vmcnt = bits [3:0] and [15:14]; expcnt and lgkmcnt left at their maxima
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

// DP: head_dim rounded up to a multiple of 32; WAVES: wavefronts per workgroup (4 or 8); STAGES: K/V
// tiles in flight in LDS.
template <int DP, int WAVES, int STAGES>
struct AttnTile {
    static constexpr int THREADS = WAVES * kWave;
    static constexpr int KSTEPS = DP / 16;      // MFMA k-steps of Q K^T
    static constexpr int DT = DP / 32;          // 32-row tiles of O^T
    static constexpr int PITCH = DP == 64 ? 8 : 16;        // 16-byte chunks per LDS row
    static constexpr int PITCHB = PITCH * 16;              // ... in bytes
    static constexpr int TILEB = kBN * PITCHB;             // bytes per K (or V) tile
    static constexpr int NI = kBN * PITCH / THREADS;       // global->LDS instructions per wavefront, tile and tensor
    static constexpr int TLOADS = 2 * NI;                  // ... per tile (K and V)
    static constexpr int VBASE = STAGES * TILEB;           // byte offset of the V stages
    static constexpr int OROW = DP + 8;                    // elements per staged output row (padded against bank conflicts)
    // behind the rings every wavefront owns an area that first stages its Q tile (32 rows in the K tile layout)
    // and later its 32 x DP output tile
    static constexpr int QW = 32 * PITCHB;
    static constexpr int WAREA = QW > 32 * OROW * 2 ? QW : 32 * OROW * 2;
    static constexpr int LDS_BYTES = 2 * STAGES * TILEB + WAVES * WAREA;
    static_assert(WAVES == 4 || WAVES == 8, "block shapes are 4 or 8 wavefronts");
    static_assert(STAGES == 2, "every wait below is for all outstanding loads, which fits a ring of two");
};

// Waits until at most `younger` tiles' worth of loads (TL per tile) are outstanding, younger <= MAXY.
template <int MAXY, int TL>
__device__ __forceinline__ void wait_tiles(int younger)
{
    if constexpr (MAXY == 0) wait_vmcnt<0>();
    else {
        if (younger >= MAXY) wait_vmcnt<MAXY * TL>();
        else wait_tiles<MAXY - 1, TL>(younger);
    }
}

template <int DP, int WAVES, int STAGES, bool RAGGED = false>
__global__ __launch_bounds__(WAVES * kWave, 2) void attn_mfma_kernel(AttnArgs a)
{
    using T = AttnTile<DP, WAVES, STAGES>;
    constexpr int kAttnWaves = WAVES, kStages = STAGES;
    constexpr int KSTEPS = T::KSTEPS, DT = T::DT, PITCH = T::PITCH, PITCHB = T::PITCHB, TILEB = T::TILEB;
    constexpr int NI = T::NI, TLOADS = T::TLOADS, VBASE = T::VBASE;
    extern __shared__ __attribute__((aligned(16))) __bf16 smem[];
    lds_char* const lds = (lds_char*)smem;    // K stages at [0, VBASE), V stages at [VBASE, 2 VBASE), then the wavefronts' areas

    const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    const int HB = a.heads_per_block, RB = kAttnWaves >> a.hb_shift;   // heads and 32-row sub-tiles per block
    const int group = a.group, head_blocks = a.head_blocks;

    // blockIdx.y -> the workgroup's row tiles, the heaviest causal ones first (the linear dispatch order runs
    // through x first); blockIdx.x -> (head block, kv head, batch).  The quotients come from multiply-high with
    // constants prepared at launch: a chain of integer divisions here would delay the first load by half a
    // microsecond.  A paired launch gives workgroup y the row tiles n-1-y and then y (y-1 when n is odd, where
    // the heaviest tile stays alone): under the causal mask tile t has t+1 key tiles, so every workgroup gets
    // the same number of them, one workgroup per compute unit covers the launch, and the second tile's Q and
    // first K/V tile are fetched under the first one's last tiles and output stores.
    auto div_magic = [](uint32_t n, uint32_t magic) { return magic ? __umulhi(n, magic) : n; };
    int rt = a.row_tiles - 1 - static_cast<int>(blockIdx.y);
    int rt_next = a.paired ? static_cast<int>(blockIdx.y) - (a.row_tiles & 1) : -1;
    const uint32_t bid = blockIdx.x;
    const uint32_t bid_hb = div_magic(bid, a.magic_head_blocks);      // = kv head + n_kv_heads * batch
    const int hb = static_cast<int>(bid - bid_hb * head_blocks);
    const int b = static_cast<int>(div_magic(bid_hb, a.magic_kv_heads));
    const int g = static_cast<int>(bid_hb) - b * a.n_kv_heads;

    const int h = g * group + hb * HB + (w & (HB - 1));
    const int wrow = (w >> a.hb_shift) * 32;                  // this wavefront's first query row inside a row tile
    // Query rows of this sample and where they start.  Ragged launches (no mask, one row tile per workgroup): item b's
    // rows come from the table in the arguments, and a workgroup whose row tile lies past its item's end has nothing
    // to do (the grid covers the longest item); it leaves before any load or barrier.
    int seq_item = a.seq, kv_seq_item = a.kv_seq;
    int64_t q_first = b * a.qs[0], o_first = b * a.os[0], kv_first = b * a.ks[0];
    if constexpr (RAGGED) {
        const int32_t first = a.item_row[b];
        seq_item = a.item_row[b + 1] - first;
        q_first = static_cast<int64_t>(first) * a.qs[1];
        o_first = static_cast<int64_t>(first) * a.os[1];
        if (a.kv_packed) {                                    // keys and values packed like the queries (self-attention)
            kv_seq_item = seq_item;
            kv_first = static_cast<int64_t>(first) * a.ks[1];
        }
        if (rt * RB * 32 >= seq_item) return;
    }
    const int seq = seq_item, kv_seq = kv_seq_item;
    const float sl2 = a.scale * 1.4426950408889634f;          // scale * log2(e)

    // geometry of the row tile being computed
    int row0, block_row0, block_rows_end, qi, n_tiles;
    auto set_rows = [&](int t) {
        block_row0 = t * RB * 32;
        row0 = block_row0 + wrow;                             // this wavefront's first query row
        block_rows_end = min(block_row0 + RB * 32, seq);
        qi = row0 + col;                                      // this lane's query row
        const int kv_end = a.causal ? block_rows_end : kv_seq; // keys [0, kv_end) are visible to the block
        n_tiles = (kv_end + kBN - 1) / kBN;
    };
    set_rows(rt);
    const __bf16* kp = static_cast<const __bf16*>(a.k) + kv_first + g * a.ks[2];
    const __bf16* vp = static_cast<const __bf16*>(a.v) + kv_first + g * a.ks[2];
    const uint32_t row_bytes = static_cast<uint32_t>(a.ks[1]) * 2u;   // K/V token stride

    // Q first: its loads are the longest wait of the prologue, everything else is set up in their shadow.
    // Q goes through LDS as well (same swizzled layout as a K tile, 32 rows per wavefront, in the wavefront's
    // own area behind the rings), so that the main loop holds no register-destination global load: the
    // compiler then never emits a vmcnt wait of its own there.
    const uint32_t q_lds = 2 * VBASE + w * T::WAREA;
    const char* qb = reinterpret_cast<const char*>(static_cast<const __bf16*>(a.q) + q_first + h * a.qs[2]);
    const uint64_t qb_bits = reinterpret_cast<uint64_t>(qb);
    // (the builtin returns a signed int: widen each half as unsigned)
    const uint32_t qb_hi = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<uint32_t>(qb_bits >> 32)));
    const uint32_t qb_lo = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<uint32_t>(qb_bits)));
    const uint64_t qb_uni = (static_cast<uint64_t>(qb_hi) << 32) | qb_lo;
    const uint32_t q_row_bytes = static_cast<uint32_t>(a.qs[1]) * 2u;
    const uint32_t q_lds_uni = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds)) + q_lds);
    // Slot -> (row, physical chunk) as for a K tile: instruction j covers rows 4j .. 4j+3 when a row has 16
    // chunks (8j .. 8j+7 when it has 8), and the chunk swizzle repeats every 16 rows, so instructions j and
    // j + 16/rows-per-instruction differ by a constant row offset only.
    auto q_slot_off = [&](int j, int first_row, bool clamp) {
        const int slot = j * kWave + lane;
        const int row = slot / PITCH;
        const int c = (slot % PITCH) ^ swz<PITCH>(row);
        const uint32_t cb = (c * 8 < a.head_dim) ? c * 16 : 0;
        const int r = clamp ? min(first_row + row, seq - 1) : first_row + row;
        return static_cast<uint32_t>(r) * q_row_bytes + cb;
    };
    auto issue_q = [&](int first_row) {                       // any row tile: rows past the sequence re-read its last row
#pragma unroll
        for (int j = 0; j < PITCH / 2; ++j)
            dma16_at(reinterpret_cast<const void*>(qb_uni), q_slot_off(j, first_row, true), q_lds_uni, std::integral_constant<int, 0>{}, j);
    };
    // The Q rows of a workgroup's second row tile, which is never the last of the sequence (no clamping): the
    // offsets of the first 16 rows stay in registers, the tile's first row enters through the scalar base.
    constexpr int QJ = 16 * PITCH / kWave;                    // instructions per 16 rows
    uint32_t q_voff[QJ];
#pragma unroll
    for (int j = 0; j < QJ; ++j) q_voff[j] = q_slot_off(j, 0, false);
    auto issue_q_next = [&](int first_row) {
        const char* base0 = uniform_ptr(reinterpret_cast<const char*>(qb_uni) + static_cast<int64_t>(first_row) * q_row_bytes);
        const char* base1 = uniform_ptr(base0 + 16 * static_cast<int64_t>(q_row_bytes));
#pragma unroll
        for (int j = 0; j < PITCH / 2; ++j)
            dma16_at(j < QJ ? base0 : base1, q_voff[j % QJ], q_lds_uni, std::integral_constant<int, 0>{}, j);
    };
    issue_q(row0);
    // Global -> LDS: instruction j of wavefront w fills slots [(w*NI + j)*64, +64) of a tile; slot ->
    // (row, physical chunk); the lane fetches the logical chunk that belongs there.  Every lane always
    // loads: rows past the end of the sequence re-read the last row (their scores are masked), chunks past
    // head_dim re-read chunk 0 (they meet zero-filled Q columns, or produce output columns that are never
    // stored).  The tile's first key enters through the scalar base, so the per-lane offsets are loop
    // invariant; only the tile that holds the end of the sequence needs the clamped set.
    uint32_t ld_voff[NI], ld_voff_tail[NI];
    const int tail_tile = (kv_seq - 1) / kBN;               // the tile that may run past the keys
#pragma unroll
    for (int j = 0; j < NI; ++j) {
        const int slot = (w * NI + j) * kWave + lane;
        const int row = slot / PITCH;
        const int c = (slot % PITCH) ^ swz<PITCH>(row);
        const uint32_t cb = (c * 8 < a.head_dim) ? c * 16 : 0;
        ld_voff[j] = row * row_bytes + cb;
        ld_voff_tail[j] = (min(tail_tile * kBN + row, kv_seq - 1) - tail_tile * kBN) * row_bytes + cb;
    }
    const uint32_t lds_wave = __builtin_amdgcn_readfirstlane(
        static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds)) + w * NI * kWave * 16);
    auto issue_tile = [&](int kt, auto stage_c) {
        constexpr int st = decltype(stage_c)::value;
        // (wave-uniform by construction; made so explicitly because the load takes its base in scalar registers)
        const char* kb = uniform_ptr(reinterpret_cast<const char*>(kp) + static_cast<int64_t>(kt) * kBN * row_bytes);
        const char* vb = uniform_ptr(reinterpret_cast<const char*>(vp) + static_cast<int64_t>(kt) * kBN * row_bytes);
        const bool tail = kt == tail_tile;
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const uint32_t off = tail ? ld_voff_tail[j] : ld_voff[j];
            dma16_at(kb, off, lds_wave, std::integral_constant<int, st * TILEB>{}, j);
            dma16_at(vb, off, lds_wave, std::integral_constant<int, st * TILEB + VBASE>{}, j);
        }
    };

    // Start the pipeline: tile 0 (the ring runs one tile ahead of the one being consumed)
    issue_tile(0, std::integral_constant<int, 0>{});

    // Q^T as B operand: lane (col, half) holds Q[qi][16 s + 8 half .. +7] for every k-step s.
    bf16x8 qreg[KSTEPS];
    auto read_q = [&]() {
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            const bf16x8 t = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(
                lds + q_lds + col * PITCHB + (((2 * s + half) ^ swz<PITCH>(col & 15)) << 4));
            qreg[s] = t;
        }
        if (a.head_dim != DP) {                               // a padded head: the columns past head_dim count as zero
            const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) qreg[s] = (16 * s + 8 * half < a.head_dim) ? qreg[s] : zero;
        }
        // in registers before the area is written again
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (a.q_cs != nullptr) {
            // Rotary embedding of the query row in registers: the lane holds elements 16 s + 8 half + j, and with
            // head_dim a multiple of 32 the partner of an element, head_dim / 2 further on, sits KSTEPS / 2
            // k-steps later in the same lane.  (cos, sin) of the row's 8 consecutive pairs come as four 16-byte loads.
            constexpr int HS = KSTEPS / 2;
            const float2* cs_row = a.q_cs + (static_cast<int64_t>(b) * seq + min(qi, seq - 1)) * (DP / 2) + 8 * half;
#pragma unroll
            for (int s = 0; s < HS; ++s) {
                float2 cs[8];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float4 t = reinterpret_cast<const float4*>(cs_row + 16 * s)[v];
                    cs[2 * v] = make_float2(t.x, t.y);
                    cs[2 * v + 1] = make_float2(t.z, t.w);
                }
                bf16x8 lo = qreg[s], hi = qreg[s + HS];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float x0 = static_cast<float>(lo[j]), x1 = static_cast<float>(hi[j]);
                    float r0, r1;
                    rope_pair(x0, x1, cs[j].x, cs[j].y, r0, r1);
                    lo[j] = static_cast<__bf16>(r0);
                    hi[j] = static_cast<__bf16>(r1);
                }
                qreg[s] = lo; qreg[s + HS] = hi;
            }
        }
    };
    // Loads retire in order and Q was issued first: wait until only the tile's loads are outstanding.
    wait_vmcnt<TLOADS>();
    read_q();

    // Per-lane LDS read addresses (bytes) inside stage 0; stage, t, u add compile-time immediates.
    lds_char* kaddr[KSTEPS];              // K: row col, logical chunk 2s + half
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
        kaddr[s] = lds + col * PITCHB + (((2 * s + half) ^ swz<PITCH>(col & 15)) << 4);
        // opaque to the optimiser: one register per address, every use is register + immediate
        asm volatile("" : "+v"(kaddr[s]));
    }
    const int l16 = lane & 15, g16 = (lane >> 4) & 1;
    lds_char* vaddr[2][DT];               // V: row 4 half + 8 hi + l16/4 (+ 32t + 16u), columns 32dt + 16 g16 + 4 (l16 % 4)
#pragma unroll
    for (int hi = 0; hi < 2; ++hi)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const int low4 = 4 * half + 8 * hi + (l16 >> 2);
            const int el = 32 * dt + 16 * g16 + 4 * (l16 & 3);
            vaddr[hi][dt] = lds + VBASE + low4 * PITCHB + (((el >> 3) ^ swz<PITCH>(low4)) << 4) + (el & 7) * 2;
            asm volatile("" : "+v"(vaddr[hi][dt]));
        }

    constexpr int kDist = CIVIC_ATTN_DIST;                  // LDS fragments are read this many MFMAs ahead of their use
    f32x16 acc_o[DT];
    float m_run;                           // offset subtracted from the raw logits (a recent row maximum)
    float l_run[2];                        // running row sum, two partial accumulators
    const bf16x2 ones = {static_cast<__bf16>(1.0f), static_cast<__bf16>(1.0f)};

    // The arithmetic of one tile (stage ST of the ring) for this wavefront: NT = 2 for the whole tile, 1 for
    // its first 32 keys only.
    auto tile = [&](int kt, auto stage_c, auto nt_c) {
        constexpr int ST = decltype(stage_c)::value;
        constexpr int NT = decltype(nt_c)::value;
        const int key0 = kt * kBN;
        if (a.causal && key0 > row0 + 31) return;             // no key of the tile is visible to this wavefront
        // S^T tile: rows = keys (two 32-key sub-tiles), columns = this wavefront's 32 queries
        f32x16 acc_s[NT];                                     // raw logits
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_s[t][r] = 0.f;
        // (fragments are read two MFMAs ahead of their use, in the order written: a scheduling barrier per MFMA
        // keeps that order whatever the register pressure around it)
        {
            auto read_k = [&](int i) __attribute__((always_inline)) {     // MFMA i = (k-step i / NT, sub-tile i % NT)
                return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(
                    kaddr[i / NT] + ST * TILEB + 32 * (i % NT) * PITCHB);
            };
            bf16x8 kf[kDist + 1];
#pragma unroll
            for (int i = 0; i < kDist; ++i) kf[i] = read_k(i);
#pragma unroll
            for (int i = 0; i < NT * KSTEPS; ++i) {
                if (i + kDist < NT * KSTEPS) kf[(i + kDist) % (kDist + 1)] = read_k(i + kDist);
                acc_s[i % NT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i % (kDist + 1)], qreg[i / NT], acc_s[i % NT], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }

        // mask only where the tile crosses the diagonal or the end of the sequence (wave-uniform)
        if ((a.causal && key0 + kBN - 1 > row0) || key0 + kBN > kv_seq) {
            // The lane sees the tile's keys below `lim` (end of the sequence, and its own row under the causal
            // mask).  Register r of sub-tile t holds tile key 32 t + 8 (r / 4) + r % 4 + 4 half, so one
            // per-lane threshold against a constant per register decides: a compare and a select each.
            int lim = kv_seq - key0;
            if (a.causal) lim = min(lim, qi - key0 + 1);
            const int thr = lim - 4 * half;
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    acc_s[t][r] = 32 * t + 8 * (r >> 2) + (r & 3) < thr ? acc_s[t][r] : -INFINITY;
        }
        // P = exp2((acc_s - m_run) * scale * log2 e), rounded to bf16, laid out as the B operands; lt = the
        // lane's two partial row sums of the rounded probabilities (what the PV product actually uses).
        bf16x8 pb[NT][2];
        float lt[2];
        auto probs = [&]() __attribute__((always_inline)) {
            const float off = -m_run * sl2;
            lt[0] = 0.f; lt[1] = 0.f;
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    u32x4 packed;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float p0 = __builtin_amdgcn_exp2f(fmaf(acc_s[t][8 * u + 2 * e], sl2, off));
                        const float p1 = __builtin_amdgcn_exp2f(fmaf(acc_s[t][8 * u + 2 * e + 1], sl2, off));
                        const bf16x2 pp = {static_cast<__bf16>(p0), static_cast<__bf16>(p1)};
                        packed[e] = __builtin_bit_cast(uint32_t, pp);
                        lt[e & 1] = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, lt[e & 1], false);
                    }
                    pb[t][u] = __builtin_bit_cast(bf16x8, packed);
                }
        };
        // The offset m_run is not the exact running maximum.  The first tile sets it to that tile's
        // row maximum; afterwards it moves (never down) only when a tile's probabilities come out
        // large, a row maximum 2^20 or so above it, which the row sums reveal without a separate
        // maximum pass.  Until then every term stays far inside the fp32 and bf16 ranges, and since P,
        // the row sum and the output accumulator all carry the same factor 2^-m_run the result does
        // not depend on it.
        const bool first = kt == 0;
        if (!first) probs();
        if (first || __any(lt[0] + lt[1] > 1048576.f)) {
            float mq[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
            for (int c4 = 0; c4 < 2 * NT; ++c4) {
                const f32x16& x = acc_s[c4 >> 1];
                const int o = 8 * (c4 & 1);
                mq[c4] = fmaxf(max3(max3(x[o], x[o + 1], x[o + 2]), x[o + 3], x[o + 4]), max3(x[o + 5], x[o + 6], x[o + 7]));
            }
            float mx = fmaxf(fmaxf(mq[0], mq[1]), fmaxf(mq[2], mq[3]));
            mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));        // finite on the first tile: key 0 is visible to every row
            const float m_new = first ? mx : fmaxf(mx, m_run);
            if (!first) {
                const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * sl2);
                l_run[0] *= alpha; l_run[1] *= alpha;
#pragma unroll
                for (int t = 0; t < DT; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc_o[t][r] *= alpha;
            }
            m_run = m_new;
            probs();
        }
        l_run[0] += lt[0]; l_run[1] += lt[1];
        // O^T += V^T P^T.  The k-slot (half, e) of step (t, u) is key 32t + 16u + 8(e/4) + 4 half + e%4.
        {
            auto read_v = [&](int i) __attribute__((always_inline)) {     // MFMA i = (key step i / DT, output tile i % DT)
                const int dt = i % DT, row = 16 * (i / DT);
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4*)(vaddr[0][dt] + ST * TILEB + row * PITCHB));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4*)(vaddr[1][dt] + ST * TILEB + row * PITCHB));
                const s16x8 v8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                return __builtin_bit_cast(bf16x8, v8);
            };
            bf16x8 vf[kDist + 1];
#pragma unroll
            for (int i = 0; i < kDist; ++i) vf[i] = read_v(i);
#pragma unroll
            for (int i = 0; i < NT * 2 * DT; ++i) {
                if (i + kDist < NT * 2 * DT) vf[(i + kDist) % (kDist + 1)] = read_v(i + kDist);
                acc_o[i % DT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i % (kDist + 1)], pb[i / (2 * DT)][(i / DT) % 2], acc_o[i % DT], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    // The same arithmetic for an inner tile (not the first, nothing masked), written out so that one wavefront's
    // matrix and vector instructions alternate: the logits of the tile's second 32 keys are multiplied while the
    // probabilities of its first 32 keys are exponentiated, a pair of scores behind every MFMA, and those enter the
    // PV product while the second half is exponentiated.  The order below is the order wanted: a scheduling barrier
    // after every unit keeps the compiler from regrouping it, and bounds the registers it needs.  (Measured against
    // the plain order with the same explicit fragment prefetch: 1-2 % on the 8B-shaped launch, 2-3 % on long
    // sequences - the vector work mostly does not hide behind the MFMAs, whatever the order.)  The offset check runs
    // per half, before that half's probabilities are used; a half whose row sums come out large raises the offset,
    // rescales what has been accumulated (the first half's PV product included, which carried the old offset like
    // everything else) and redoes that half's exponentials.
    auto tile_fast = [&](auto stage_c) {
        constexpr int ST = decltype(stage_c)::value;
        auto read_k = [&](int s, int t) __attribute__((always_inline)) {
            return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(kaddr[s] + ST * TILEB + 32 * t * PITCHB);
        };
        auto read_v = [&](int i, int t) __attribute__((always_inline)) {      // fragment i = (u, dt) of key half t
            const int u = i / DT, dt = i % DT;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) s16x4*)(vaddr[0][dt] + ST * TILEB + (32 * t + 16 * u) * PITCHB));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) s16x4*)(vaddr[1][dt] + ST * TILEB + (32 * t + 16 * u) * PITCHB));
            const s16x8 v8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8, v8);
        };
        // scores 2i, 2i + 1 of a half -> word i of its packed probabilities, and the lane's partial row sums
        auto soft_pair = [&](const f32x16& x, int i, float off, uint32_t (&packed)[8], float (&lt)[2]) __attribute__((always_inline)) {
            const float p0 = __builtin_amdgcn_exp2f(fmaf(x[2 * i], sl2, off));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(x[2 * i + 1], sl2, off));
            const bf16x2 pp = {static_cast<__bf16>(p0), static_cast<__bf16>(p1)};
            packed[i] = __builtin_bit_cast(uint32_t, pp);
            lt[i & 1] = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, lt[i & 1], false);
        };
        auto operand = [&](const uint32_t (&packed)[8], int u) __attribute__((always_inline)) {
            const u32x4 w = {packed[4 * u], packed[4 * u + 1], packed[4 * u + 2], packed[4 * u + 3]};
            return __builtin_bit_cast(bf16x8, w);
        };
        auto raise_offset = [&](const f32x16& x, uint32_t (&packed)[8], float (&lt)[2]) __attribute__((always_inline)) {
            float mx = fmaxf(fmaxf(max3(x[0], x[1], x[2]), max3(x[3], x[4], x[5])),
                             fmaxf(max3(x[6], x[7], x[8]), max3(x[9], x[10], x[11])));
            mx = fmaxf(fmaxf(mx, max3(x[12], x[13], x[14])), x[15]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
            const float m_new = fmaxf(mx, m_run);
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * sl2);
            l_run[0] *= alpha; l_run[1] *= alpha;
            // (in place, tied operands: the accumulators stay in the registers they have on the common path)
#pragma unroll
            for (int t = 0; t < DT; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float y = acc_o[t][r];
                    asm volatile("v_mul_f32 %0, %0, %1" : "+v"(y) : "v"(alpha));
                    acc_o[t][r] = y;
                }
            m_run = m_new;
            const float off = -m_run * sl2;
            lt[0] = 0.f; lt[1] = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) soft_pair(x, i, off, packed, lt);
        };
        constexpr int NF = 2 * DT;                            // V fragments per key half
        f32x16 s0, s1;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s0[r] = 0.f; s1[r] = 0.f; }
        uint32_t pk0[8], pk1[8];
        float lt0[2] = {0.f, 0.f}, lt1[2] = {0.f, 0.f};
        // K fragments as one sequence of 2 KSTEPS reads (first half, then second), kDist MFMAs ahead of their use
        auto read_kseq = [&](int i) __attribute__((always_inline)) { return read_k(i % KSTEPS, i / KSTEPS); };
        bf16x8 kf[kDist + 1];
#pragma unroll
        for (int i = 0; i < kDist; ++i) kf[i] = read_kseq(i);
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {                    // logits of the first half
            kf[(s + kDist) % (kDist + 1)] = read_kseq(s + kDist);
            s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s % (kDist + 1)], qreg[s], s0, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        const float off0 = -m_run * sl2;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {                    // logits of the second half | exponentials of the first
            if (KSTEPS + s + kDist < 2 * KSTEPS) kf[(KSTEPS + s + kDist) % (kDist + 1)] = read_kseq(KSTEPS + s + kDist);
            s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[(KSTEPS + s) % (kDist + 1)], qreg[s], s1, 0, 0, 0);
#pragma unroll
            for (int i = s * 8 / KSTEPS; i < (s + 1) * 8 / KSTEPS; ++i) soft_pair(s0, i, off0, pk0, lt0);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (__builtin_expect(__any(lt0[0] + lt0[1] > 1048576.f), 0)) raise_offset(s0, pk0, lt0);
        l_run[0] += lt0[0]; l_run[1] += lt0[1];
        const float off1 = -m_run * sl2;
        auto read_vseq = [&](int i) __attribute__((always_inline)) { return read_v(i % NF, i / NF); };
        bf16x8 vf[kDist + 1];
#pragma unroll
        for (int i = 0; i < kDist; ++i) vf[i] = read_vseq(i);
#pragma unroll
        for (int i = 0; i < NF; ++i) {                        // PV of the first half | exponentials of the second
            vf[(i + kDist) % (kDist + 1)] = read_vseq(i + kDist);
            acc_o[i % DT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i % (kDist + 1)], operand(pk0, i / DT), acc_o[i % DT], 0, 0, 0);
#pragma unroll
            for (int j = i * 8 / NF; j < (i + 1) * 8 / NF; ++j) soft_pair(s1, j, off1, pk1, lt1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (__builtin_expect(__any(lt1[0] + lt1[1] > 1048576.f), 0)) raise_offset(s1, pk1, lt1);
        l_run[0] += lt1[0]; l_run[1] += lt1[1];
#pragma unroll
        for (int i = 0; i < NF; ++i) {                        // PV of the second half
            if (NF + i + kDist < 2 * NF) vf[(NF + i + kDist) % (kDist + 1)] = read_vseq(NF + i + kDist);
            acc_o[i % DT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[(NF + i) % (kDist + 1)], operand(pk1, i / DT), acc_o[i % DT], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // One step of the pipeline: wait until the tile has landed, release the previous one, refill the freed
    // stage, compute.  At step q_issue the Q rows of the workgroup's next row tile are requested as well (their
    // area has been free since Q moved into registers); they land with a later tile.
    int q_issue = -1, next_row0 = 0;
    auto advance = [&](int kt, auto stage_c) __attribute__((always_inline)) {
        constexpr int ST = decltype(stage_c)::value;
        wait_vmcnt<0>();
        block_barrier();                                      // landed for every wavefront; tile kt-1 is released
        if (kt + 1 < n_tiles) issue_tile(kt + 1, std::integral_constant<int, (ST + 1) % kStages>{});
        if (kt == q_issue) issue_q_next(next_row0);
    };
    // a tile that may be the first, cross the diagonal or hold the end of the sequence
    auto step = [&](int kt, auto stage_c) __attribute__((always_inline)) {
        advance(kt, stage_c);
        // On the diagonal a wavefront whose rows all precede the tile's second half computes the first half
        // only: half the MFMAs and exponentials of that tile for half of the wavefronts, which the other
        // wavefront of the SIMD turns into time.  The same holds for a last tile whose second half lies past
        // the end of the sequence.
        if ((a.causal && kt * kBN + 32 > row0 + 31) || kt * kBN + 32 >= kv_seq) tile(kt, stage_c, std::integral_constant<int, 1>{});
        else tile(kt, stage_c, std::integral_constant<int, 2>{});
    };
    // an inner tile: whole, visible to every row of the workgroup, not the first
    auto step_inner = [&](int kt, auto stage_c) __attribute__((always_inline)) {
        advance(kt, stage_c);
        tile_fast(stage_c);
    };

    constexpr int OROW = T::OROW;
    constexpr int CPR = DP / 8;
    constexpr int kKvJ = (DP / 8 + 7) / 8;                     // pieces per thread, row and tensor
    constexpr int kKvRows = WAVES * kWave / 8;                 // rows per pass of the workgroup (64 with 8 wavefronts)
    __bf16* const o_s = reinterpret_cast<__bf16*>(smem) + q_lds / 2;   // the wavefront's area, now its output tile

    for (;;) {
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_o[t][r] = 0.f;
        m_run = 0.f; l_run[0] = 0.f; l_run[1] = 0.f;
        const bool has_next = rt_next >= 0;
        q_issue = has_next ? max(n_tiles - 3, 0) : -1;
        next_row0 = rt_next * RB * 32 + wrow;

        // Tile 0, then the inner tiles in a loop of their own (one code path, so the accumulators keep their
        // registers across it), then whatever is left: the diagonal, the end of the sequence.
        const int inner_end = min(a.causal ? (block_row0 + 1) / kBN : kv_seq / kBN, n_tiles);
        step(0, std::integral_constant<int, 0>{});
        int kt = 1;
        for (; kt + 1 < inner_end; kt += kStages) {
            step_inner(kt, std::integral_constant<int, 1>{});
            step_inner(kt + 1, std::integral_constant<int, 0>{});
        }
        for (; kt < n_tiles; kt += kStages) {
            step(kt, std::integral_constant<int, 1>{});
            if (kt + 1 < n_tiles) step(kt + 1, std::integral_constant<int, 0>{});
        }
        if (has_next) wait_vmcnt<0>();                        // the next Q rows (a one-tile pass waits nowhere else)
        __syncthreads();                                      // every tile consumed: the rings are free

        // what the epilogue needs of the tile just computed
        const int e_row0 = row0, e_block_row0 = block_row0, e_rows_end = block_rows_end;
        float l_sum = l_run[0] + l_run[1];
        const float l_tot = l_sum + __shfl_xor(l_sum, 32, kWave);
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        if (has_next) {
            // the next row tile starts here: its first K/V tile flies while this one's output is stored, and
            // its Q rows move into registers before the area takes the output tile
            set_rows(rt_next);
            issue_tile(0, std::integral_constant<int, 0>{});
            read_q();
        }

        // Fused KV-cache write: the workgroup of the first head block copies the K and V rows of its own
        // query rows (which it has just streamed through LDS, so the reads hit L2) into the cache; the loads
        // of the first 64 rows go out before the output rows are stored and their stores after; taller blocks
        // take the rest in a plain loop at the end.
        // Copy layout: 8 threads per row, thread t takes row t / 8 of a 64-row group and the 16-byte pieces
        // t % 8, t % 8 + 8, ... of it, the same piece of K and of V (one address computation for both).
        u32x4 kv_piece[2 * kKvJ];
        // opaque copies: they keep the address arithmetic of the epilogue down here, instead of in registers
        // (or spilled) across the main loop
        int tid_late = tid, lane_late = lane;
        asm volatile("" : "+v"(tid_late), "+v"(lane_late));
        const int col_late = lane_late & 31, half_late = lane_late >> 5;
        const bool kv_fused = a.k_cache != nullptr && hb == 0;
        const int kv_cpr = a.head_dim / 8;                     // 16-byte pieces per row
        const int kv_rows = e_rows_end - e_block_row0;
        const int kv_r = tid_late >> 3, kv_c = tid_late & 7;
        // element offsets of piece (row r, chunk kv_c) from kp / vp and from the cache bases
        auto kv_src_off = [&](int r) { return static_cast<int64_t>(e_block_row0 + r) * a.ks[1] + kv_c * 8; };
        auto kv_dst_off = [&](int r) {
            const int64_t cache_row = (static_cast<int64_t>(b) * a.n_kv_heads + g) * a.s_max + a.pos0 + e_block_row0 + r;
            return cache_row * a.head_dim + kv_c * 8;
        };
        // Stage the wavefront's 32 x DP output tile in LDS and write it out as whole 16-byte row segments.
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                bf16x4 o4;
#pragma unroll
                for (int e = 0; e < 4; ++e) o4[e] = static_cast<__bf16>(acc_o[dt][4 * rq + e] * inv);
                *reinterpret_cast<bf16x4*>(&o_s[col_late * OROW + 32 * dt + 8 * rq + 4 * half_late]) = o4;
            }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (kv_fused) {                                       // (the accumulators are dead by now: registers are free)
            const int64_t so = kv_src_off(kv_r);
#pragma unroll
            for (int j = 0; j < kKvJ; ++j) {
                kv_piece[2 * j] = kv_piece[2 * j + 1] = u32x4{0u, 0u, 0u, 0u};
                if (kv_r < kv_rows && kv_c + 8 * j < kv_cpr) {
                    kv_piece[2 * j] = *reinterpret_cast<const u32x4*>(kp + so + 64 * j);
                    kv_piece[2 * j + 1] = *reinterpret_cast<const u32x4*>(vp + so + 64 * j);
                }
            }
        }
        __bf16* ob = static_cast<__bf16*>(a.out) + o_first + h * a.os[2];
        if (kWave % CPR == 0 && e_row0 + 32 <= seq && a.head_dim == DP) {
            // whole tile, unpadded head: the lane keeps its column, rows advance by 64 / CPR per store
            constexpr int RPI = kWave / CPR > 0 ? kWave / CPR : 1;
            const int r0 = lane_late / CPR, dc = lane_late - r0 * CPR;
            __bf16* dst = ob + static_cast<int64_t>(e_row0 + r0) * a.os[1] + dc * 8;
            const __bf16* src = &o_s[r0 * OROW + dc * 8];
            const int64_t stride = static_cast<int64_t>(RPI) * a.os[1];
#pragma unroll
            for (int it = 0; it < 32 * CPR / kWave; ++it)
                *reinterpret_cast<bf16x8*>(dst + it * stride) = *reinterpret_cast<const bf16x8*>(src + it * RPI * OROW);
        } else {
#pragma unroll
            for (int it = 0; it < 32 * CPR / kWave; ++it) {
                const int id = it * kWave + lane_late;
                const int r = id / CPR, dc = id - r * CPR;
                if (e_row0 + r < seq && dc * 8 < a.head_dim)
                    *reinterpret_cast<bf16x8*>(ob + static_cast<int64_t>(e_row0 + r) * a.os[1] + dc * 8) =
                        *reinterpret_cast<const bf16x8*>(&o_s[r * OROW + dc * 8]);
            }
        }
        if (kv_fused) {
            __bf16* const kc = static_cast<__bf16*>(a.k_cache);
            __bf16* const vc = static_cast<__bf16*>(a.v_cache);
            const int64_t d0 = kv_dst_off(kv_r);
#pragma unroll
            for (int j = 0; j < kKvJ; ++j)
                if (kv_r < kv_rows && kv_c + 8 * j < kv_cpr) {
                    *reinterpret_cast<u32x4*>(kc + d0 + 64 * j) = kv_piece[2 * j];
                    *reinterpret_cast<u32x4*>(vc + d0 + 64 * j) = kv_piece[2 * j + 1];
                }
            for (int r = kv_r + kKvRows; r < kv_rows; r += kKvRows) {   // taller blocks (fewer than 4 heads per block)
                const int64_t so = kv_src_off(r), dd = kv_dst_off(r);
#pragma unroll
                for (int j = 0; j < kKvJ; ++j)
                    if (kv_c + 8 * j < kv_cpr) {
                        *reinterpret_cast<u32x4*>(kc + dd + 64 * j) = *reinterpret_cast<const u32x4*>(kp + so + 64 * j);
                        *reinterpret_cast<u32x4*>(vc + dd + 64 * j) = *reinterpret_cast<const u32x4*>(vp + so + 64 * j);
                    }
            }
        }
        if (!has_next) break;
        rt = rt_next;
        rt_next = -1;
    }
}

// Block shape and grid of the MFMA kernel for these sizes; false if the grid does not fit (more than 65535
// row tiles, or a block index too large for the multiply-high decoding: n * d < 2^32 for n < per_rt).
template <int WAVES>
static bool mfma_geometry(AttnArgs& a, int64_t* per_rt)
{
    const int group = a.n_q_heads / a.n_kv_heads;
    a.heads_per_block = (group % 4 == 0) ? 4 : (group % 2 == 0) ? 2 : 1;
    const int rows_per_block = 32 * (WAVES / a.heads_per_block);
    const int64_t row_tiles = (static_cast<int64_t>(a.seq) + rows_per_block - 1) / rows_per_block;
    a.row_tiles = static_cast<int32_t>(row_tiles);
    a.group = group;
    a.head_blocks = group / a.heads_per_block;
    a.hb_shift = a.heads_per_block == 4 ? 2 : a.heads_per_block == 2 ? 1 : 0;
    *per_rt = static_cast<int64_t>(a.head_blocks) * a.n_kv_heads * a.batch;
    const int64_t d_max = a.head_blocks > a.n_kv_heads ? a.head_blocks : a.n_kv_heads;
    return *per_rt * d_max < (int64_t{1} << 32) && row_tiles <= 65535;
}

constexpr int64_t kComputeUnits = 256;

// Time (in arbitrary units) until the last workgroup of a causal launch ends when every compute unit runs one
// workgroup at a time and takes the next in dispatch order.  `paired`: workgroup y walks row tiles n-1-y and
// its partner (see the kernel).  A key tile costs 1.9 and a workgroup 5.5 around its tiles, 2 more for a
// second row tile whose start hides under the first one's end (microseconds measured on the 8B-shaped
// launch).  Only the ratio of the two results is used.
static double causal_makespan(int n_row_tiles, int64_t per_rt, int rows_per_block, int seq, bool paired)
{
    auto tiles_of = [&](int rt) {
        const int64_t end = std::min<int64_t>(static_cast<int64_t>(rt + 1) * rows_per_block, seq);
        return static_cast<double>((end + kBN - 1) / kBN);
    };
    const int items = paired ? (n_row_tiles + 1) / 2 : n_row_tiles;
    std::array<double, kComputeUnits> free_at;                // a min-heap of the units' free times
    free_at.fill(0.0);
    auto cmp = [](double x, double y) { return x > y; };
    double last = 0.0;
    for (int y = 0; y < items; ++y) {
        double cost = 5.5 + 1.9 * tiles_of(n_row_tiles - 1 - y);
        if (paired) {
            const int light = y - (n_row_tiles & 1);
            if (light >= 0) cost += 2.0 + 1.9 * tiles_of(light);
        }
        for (int64_t x = 0; x < per_rt; ++x) {
            std::pop_heap(free_at.begin(), free_at.end(), cmp);
            const double t = free_at.back() + cost;
            free_at.back() = t;
            std::push_heap(free_at.begin(), free_at.end(), cmp);
            if (t > last) last = t;
        }
    }
    return last;
}

// Whether the launch gives every workgroup two row tiles.  It pays under the causal mask when the row tiles
// do not all run at once anyway: the pairs are equally heavy, there are half as many workgroup starts, and a
// pair's second start is hidden.  Decided with the model above for grids small enough that the answer depends
// on how the workgroups fall onto the compute units; larger grids always pair.  The last answer is kept per
// thread so that a loop over layers does not model the same launch again.
static bool choose_paired(const AttnArgs& a, int64_t per_rt, int rows_per_block)
{
#ifdef CIVIC_ATTN_FORCE_PAIRED
    return CIVIC_ATTN_FORCE_PAIRED && a.row_tiles >= 2;           // build-time override for A/B measurements
#endif
    if (!a.causal || a.row_tiles < 2) return false;
    const int64_t blocks = per_rt * a.row_tiles;
    if (blocks <= kComputeUnits) return false;                // one generation as it is
    if (blocks > 16 * kComputeUnits) return true;
    struct Memo { int32_t row_tiles, rows_per_block, seq; int64_t per_rt; bool paired; };
    static thread_local Memo memo = {0, 0, 0, 0, false};
    if (memo.row_tiles == a.row_tiles && memo.rows_per_block == rows_per_block && memo.seq == a.seq && memo.per_rt == per_rt)
        return memo.paired;
    const bool paired = causal_makespan(a.row_tiles, per_rt, rows_per_block, a.seq, true) <
                        causal_makespan(a.row_tiles, per_rt, rows_per_block, a.seq, false);
    memo = {a.row_tiles, rows_per_block, a.seq, per_rt, paired};
    return paired;
}

template <int DP, int WAVES, int STAGES, bool RAGGED>
static int launch_mfma(AttnArgs& a, hipStream_t s)
{
    using T = AttnTile<DP, WAVES, STAGES>;
    int64_t per_rt = 0;
    if (!mfma_geometry<WAVES>(a, &per_rt)) return CIVIC_ERR_UNSUPPORTED;      // (the caller has checked)
    auto magic = [](int64_t d) { return d <= 1 ? 0u : static_cast<uint32_t>(((int64_t{1} << 32) + d - 1) / d); };
    a.magic_head_blocks = magic(a.head_blocks);
    a.magic_kv_heads = magic(a.n_kv_heads);
    a.paired = !RAGGED && choose_paired(a, per_rt, 32 * (WAVES / a.heads_per_block)) ? 1 : 0;   // (pairs assume one length)
    const unsigned grid_y = static_cast<unsigned>(a.paired ? (a.row_tiles + 1) / 2 : a.row_tiles);
    constexpr size_t lds = T::LDS_BYTES;
    if (lds > 64 * 1024) {
        static std::atomic<uint64_t> allowed{0};
        const int rc = allow_dynamic_lds(reinterpret_cast<const void*>(attn_mfma_kernel<DP, WAVES, STAGES, RAGGED>), lds, &allowed);
        if (rc != CIVIC_OK) return rc;
    }
    civic::launch((attn_mfma_kernel<DP, WAVES, STAGES, RAGGED>), dim3(static_cast<unsigned>(per_rt), grid_y),
                       dim3(T::THREADS), lds, s, a);
    return check_launch();
}

#ifndef CIVIC_ATTN_STAGES
#define CIVIC_ATTN_STAGES 2
#endif
template <int WAVES, bool RAGGED>
static int launch_mfma_for(AttnArgs& a, hipStream_t s)
{
    if (a.head_dim <= 64) return launch_mfma<64, WAVES, CIVIC_ATTN_STAGES, RAGGED>(a, s);
    if (a.head_dim <= 96) return launch_mfma<96, WAVES, CIVIC_ATTN_STAGES, RAGGED>(a, s);
    return launch_mfma<128, WAVES, CIVIC_ATTN_STAGES, RAGGED>(a, s);
}

}  // namespace civic

namespace civic {

// Attention, and the KV-cache write when k_cache is not null (inside the attention kernel where the
// MFMA path runs, as a second launch otherwise).
// item_row (host, batch + 1 ascending row numbers, or null): the queries and outputs of the `batch` items are packed
// along the token axis, item b owning rows [item_row[b], item_row[b + 1]) of q and out, and `seq` is the longest item;
// at most kRaggedItems items, no rotary table.  kv_packed: k and v are packed the same way (self-attention of every
// item over its own rows, `kv_seq` = `seq`; the mask and the caches are allowed); otherwise they are [batch, kv_seq]
// and there is neither.  dry_run: every check and nothing launched.
static int prefill_attn(const void* q, const void* k, const void* v, void* out, int dtype, int32_t batch, int32_t seq,
                        int32_t kv_seq, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, const int64_t* q_strides,
                        const int64_t* kv_strides, const int64_t* o_strides, int32_t causal, float softmax_scale,
                        void* k_cache, void* v_cache, int64_t s_max, int64_t pos0, const float* q_cos_sin, void* stream,
                        const int32_t* item_row = nullptr, bool dry_run = false, bool kv_packed = false)
{
    const int esz = dtype_size(dtype);
    if (!esz || !q_strides || !kv_strides || !o_strides) return CIVIC_ERR_INVALID_ARG;
    if (batch < 0 || seq < 0 || kv_seq < 0 || n_q_heads <= 0 || n_kv_heads <= 0 || head_dim <= 0) return CIVIC_ERR_INVALID_ARG;
    if (causal && kv_seq != seq) return CIVIC_ERR_INVALID_ARG;
    if (seq > 0 && kv_seq == 0) return CIVIC_ERR_INVALID_ARG;                             // a softmax over no key has no value
    if (batch > 0 && seq > 0 && (!q || !k || !v || !out)) return CIVIC_ERR_INVALID_ARG;   // no tokens: no tensors
    if (n_q_heads % n_kv_heads) return CIVIC_ERR_INVALID_ARG;
    if (head_dim % 8) return CIVIC_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return CIVIC_ERR_INVALID_ARG;
    for (int i = 0; i < 3; ++i) {
        if (q_strides[i] < 0 || kv_strides[i] < 0 || o_strides[i] < 0) return CIVIC_ERR_INVALID_ARG;
        if ((q_strides[i] * esz) % 16 || (kv_strides[i] * esz) % 16 || (o_strides[i] * esz) % 16) return CIVIC_ERR_INVALID_ARG;
    }
    if (!(softmax_scale >= 0.f) || std::isinf(softmax_scale)) return CIVIC_ERR_INVALID_ARG;
    if (k_cache) {
        if (!v_cache || !aligned16(k_cache) || !aligned16(v_cache)) return CIVIC_ERR_INVALID_ARG;
        if (pos0 < 0 || s_max < 0 || pos0 + seq > s_max) return CIVIC_ERR_INVALID_ARG;
        if (kv_strides[2] < head_dim && n_kv_heads > 1) return CIVIC_ERR_INVALID_ARG;
    }
    if (q_cos_sin && (!aligned16(q_cos_sin) || head_dim % 4)) return CIVIC_ERR_INVALID_ARG;
    if (head_dim > CIVIC_MAX_HEAD_DIM || batch > 65535 || n_q_heads > 65535) return CIVIC_ERR_UNSUPPORTED;
    if (item_row && (batch > kRaggedItems || q_cos_sin || (!kv_packed && (causal || k_cache)))) return CIVIC_ERR_INVALID_ARG;
    if (kv_packed && (!item_row || kv_seq != seq)) return CIVIC_ERR_INVALID_ARG;
    if (batch == 0 || seq == 0) return CIVIC_OK;

    AttnArgs a;
    a.q = q; a.k = k; a.v = v; a.out = out;
    for (int i = 0; i < 3; ++i) { a.qs[i] = q_strides[i]; a.ks[i] = kv_strides[i]; a.os[i] = o_strides[i]; }
    a.batch = batch; a.seq = seq; a.kv_seq = kv_seq; a.n_q_heads = n_q_heads; a.n_kv_heads = n_kv_heads; a.head_dim = head_dim;
    a.causal = causal ? 1 : 0;
    a.scale = softmax_scale > 0.f ? softmax_scale : 1.0f / std::sqrt(static_cast<float>(head_dim));
    a.heads_per_block = 1; a.row_tiles = 0; a.paired = 0;
    a.group = n_q_heads / n_kv_heads; a.head_blocks = 0; a.hb_shift = 0; a.magic_head_blocks = 0; a.magic_kv_heads = 0;
    a.k_cache = k_cache; a.v_cache = v_cache; a.s_max = s_max; a.pos0 = pos0;
    a.q_cs = reinterpret_cast<const float2*>(q_cos_sin);
    for (int i = 0; i <= kRaggedItems; ++i) a.item_row[i] = item_row && i <= batch ? item_row[i] : 0;
    a.kv_packed = kv_packed ? 1 : 0;
    hipStream_t s = static_cast<hipStream_t>(stream);

    // the MFMA path addresses a K/V tile, and a head's Q rows, with 32-bit per-lane byte offsets, and its grid
    // has limits of its own; whatever falls outside takes the plain kernel
    // Workgroups of 8 wavefronts (256 query rows x heads) share each K/V tile the most; when they would
    // leave at least half of the compute units without work, workgroups of 4 wavefronts spread it over twice
    // as many (measured: 32 workgroups of 8 wavefronts 15.4 us, 64 of 4 12.2 us; but 192 of 8 37.9 us against
    // 384 of 4, two per unit, 39.7 us).
    int64_t per_rt = 0;
    // (with a rotary table the MFMA kernel needs an unpadded head whose halves are whole k-step pairs)
    const bool rope_fits = !q_cos_sin || head_dim == 64 || head_dim == 96 || head_dim == 128;
    if (dtype == CIVIC_BF16 && head_dim <= 128 && rope_fits && kv_strides[1] * 2 < (1 << 25) &&
        static_cast<int64_t>(seq) * q_strides[1] * 2 < (int64_t{1} << 32) && mfma_geometry<8>(a, &per_rt)) {
        if (dry_run) return CIVIC_OK;
        const bool eight = 2 * per_rt * a.row_tiles > kComputeUnits || !mfma_geometry<4>(a, &per_rt);
        if (item_row) return eight ? launch_mfma_for<8, true>(a, s) : launch_mfma_for<4, true>(a, s);
        return eight ? launch_mfma_for<8, false>(a, s) : launch_mfma_for<4, false>(a, s);
    }
    if (dry_run) return CIVIC_OK;
    // everything else: the fp32 kernel (which also writes the caches when asked to); ragged items one launch each
    for (int32_t it = 0; it < (item_row ? batch : 1); ++it) {
        AttnArgs ai = a;
        if (item_row) {
            ai.batch = 1; ai.seq = item_row[it + 1] - item_row[it];
            ai.q = static_cast<const char*>(q) + static_cast<int64_t>(item_row[it]) * q_strides[1] * esz;
            ai.out = static_cast<char*>(out) + static_cast<int64_t>(item_row[it]) * o_strides[1] * esz;
            const int64_t kv_at = kv_packed ? static_cast<int64_t>(item_row[it]) * kv_strides[1] : static_cast<int64_t>(it) * kv_strides[0];
            ai.k = static_cast<const char*>(k) + kv_at * esz;
            ai.v = static_cast<const char*>(v) + kv_at * esz;
            if (kv_packed) ai.kv_seq = ai.seq;
            if (k_cache) {
                const int64_t cache_at = static_cast<int64_t>(it) * n_kv_heads * s_max * head_dim * esz;
                ai.k_cache = static_cast<char*>(k_cache) + cache_at;
                ai.v_cache = static_cast<char*>(v_cache) + cache_at;
            }
        }
        const dim3 grid(static_cast<unsigned>((ai.seq + 3) / 4), static_cast<unsigned>(n_q_heads), static_cast<unsigned>(ai.batch));
        if (dtype == CIVIC_BF16) civic::launch((attn_plain_kernel<true>), grid, dim3(256), 0, s, ai);
        else civic::launch((attn_plain_kernel<false>), grid, dim3(256), 0, s, ai);
        const int rc = check_launch();
        if (rc != CIVIC_OK) return rc;
    }
    return CIVIC_OK;
}

}  // namespace civic

extern "C" int civic_prefill_attn(const void* q, const void* k, const void* v, void* out, int dtype, int32_t batch,
                                  int32_t seq, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                  const int64_t* q_strides, const int64_t* kv_strides, const int64_t* o_strides,
                                  int32_t causal, float softmax_scale, void* stream)
{
    return civic::prefill_attn(q, k, v, out, dtype, batch, seq, seq, n_q_heads, n_kv_heads, head_dim, q_strides, kv_strides,
                               o_strides, causal, softmax_scale, nullptr, nullptr, 0, 0, nullptr, stream);
}

extern "C" int civic_prefill_attn_rope(const void* q, const void* k, const void* v, void* out, int dtype, int32_t batch,
                                       int32_t seq, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                       const int64_t* q_strides, const int64_t* kv_strides, const int64_t* o_strides,
                                       int32_t causal, float softmax_scale, const float* q_cos_sin, void* stream)
{
    if (!q_cos_sin && batch > 0 && seq > 0) return CIVIC_ERR_INVALID_ARG;
    return civic::prefill_attn(q, k, v, out, dtype, batch, seq, seq, n_q_heads, n_kv_heads, head_dim, q_strides, kv_strides,
                               o_strides, causal, softmax_scale, nullptr, nullptr, 0, 0, q_cos_sin, stream);
}

extern "C" int civic_prefill_attn_kv(const void* q, const void* k, const void* v, void* out, void* k_cache, void* v_cache,
                                     int dtype, int32_t batch, int32_t seq, int32_t n_q_heads, int32_t n_kv_heads,
                                     int32_t head_dim, const int64_t* q_strides, const int64_t* kv_strides,
                                     const int64_t* o_strides, int64_t s_max, int64_t pos0, int32_t causal,
                                     float softmax_scale, void* stream)
{
    if ((!k_cache || !v_cache) && batch > 0 && seq > 0) return CIVIC_ERR_INVALID_ARG;
    return civic::prefill_attn(q, k, v, out, dtype, batch, seq, seq, n_q_heads, n_kv_heads, head_dim, q_strides, kv_strides,
                               o_strides, causal, softmax_scale, k_cache, v_cache, s_max, pos0, nullptr, stream);
}

extern "C" int civic_cross_attn(const void* q, const void* k, const void* v, void* out, int dtype, int32_t batch, int32_t n_q,
                                int32_t n_kv, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, const int64_t* q_strides,
                                const int64_t* kv_strides, const int64_t* o_strides, float softmax_scale, void* stream)
{
    return civic::prefill_attn(q, k, v, out, dtype, batch, n_q, n_kv, n_q_heads, n_kv_heads, head_dim, q_strides, kv_strides,
                               o_strides, 0, softmax_scale, nullptr, nullptr, 0, 0, nullptr, stream);
}

extern "C" int civic_cross_attn_ragged(const void* q, const void* k, const void* v, void* out, int dtype, int32_t batch,
                                       const int64_t* q_offsets, int32_t n_kv, int32_t n_q_heads, int32_t n_kv_heads,
                                       int32_t head_dim, const int64_t* q_strides, const int64_t* kv_strides,
                                       const int64_t* o_strides, float softmax_scale, void* stream)
{
    const int esz = civic::dtype_size(dtype);
    if (!esz || batch < 0 || !q_strides || !kv_strides || !o_strides) return CIVIC_ERR_INVALID_ARG;
    if (batch == 0) return CIVIC_OK;
    if (!q_offsets || q_offsets[0] != 0 || !q || !k || !v || !out) return CIVIC_ERR_INVALID_ARG;
    for (int32_t b = 0; b < batch; ++b)
        if (q_offsets[b + 1] <= q_offsets[b] || q_offsets[b + 1] - q_offsets[b] > INT32_MAX) return CIVIC_ERR_INVALID_ARG;
    // q_strides[0] / o_strides[0] (the batch stride of the rectangular call) are not used: items are packed along the
    // token axis (a token stride that keeps rows 16-byte aligned keeps every item's first row aligned as well).  Up to
    // kRaggedItems items go out as ONE launch whose workgroups look their item's rows up in a table in the kernel
    // arguments; longer lists in several.  Every group is checked before the first one is launched.
    if (q_offsets[batch] > INT32_MAX) return CIVIC_ERR_UNSUPPORTED;
    for (int pass = 0; pass < 2; ++pass)
        for (int32_t b0 = 0; b0 < batch; b0 += civic::kRaggedItems) {
            const int32_t nb = batch - b0 < civic::kRaggedItems ? batch - b0 : civic::kRaggedItems;
            int32_t rows[civic::kRaggedItems + 1], longest = 0;
            for (int32_t i = 0; i <= nb; ++i) rows[i] = static_cast<int32_t>(q_offsets[b0 + i]);
            for (int32_t i = 0; i < nb; ++i) longest = rows[i + 1] - rows[i] > longest ? rows[i + 1] - rows[i] : longest;
            const int rc = civic::prefill_attn(q, static_cast<const char*>(k) + static_cast<int64_t>(b0) * kv_strides[0] * esz,
                                               static_cast<const char*>(v) + static_cast<int64_t>(b0) * kv_strides[0] * esz, out, dtype, nb,
                                               longest, n_kv, n_q_heads, n_kv_heads, head_dim, q_strides, kv_strides, o_strides, 0,
                                               softmax_scale, nullptr, nullptr, 0, 0, nullptr, stream, rows, pass == 0);
            if (rc != CIVIC_OK) return rc;
        }
    return CIVIC_OK;
}


extern "C" int civic_prefill_attn_ragged(const void* q, const void* k, const void* v, void* out, int dtype, int32_t batch,
                                         const int64_t* row_offsets, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                         const int64_t* q_strides, const int64_t* kv_strides, const int64_t* o_strides,
                                         int32_t causal, float softmax_scale, void* k_cache, void* v_cache, int64_t s_max,
                                         int64_t pos0, void* stream)
{
    const int esz = civic::dtype_size(dtype);
    if (!esz || batch < 0 || !q_strides || !kv_strides || !o_strides) return CIVIC_ERR_INVALID_ARG;
    if ((k_cache == nullptr) != (v_cache == nullptr)) return CIVIC_ERR_INVALID_ARG;
    if (batch == 0) return CIVIC_OK;
    if (!row_offsets || row_offsets[0] != 0 || !q || !k || !v || !out) return CIVIC_ERR_INVALID_ARG;
    for (int32_t b = 0; b < batch; ++b)
        if (row_offsets[b + 1] <= row_offsets[b] || row_offsets[b + 1] - row_offsets[b] > INT32_MAX) return CIVIC_ERR_INVALID_ARG;
    if (row_offsets[batch] > INT32_MAX) return CIVIC_ERR_UNSUPPORTED;
    // Groups of up to kRaggedItems samples, ONE launch each: attention of every sample over its own rows (the mask counts
    // from the sample's first row) and, with caches, the write of its K and V rows into its own cache rows.  Every
    // group is checked before the first one is launched.
    for (int pass = 0; pass < 2; ++pass)
        for (int32_t b0 = 0; b0 < batch; b0 += civic::kRaggedItems) {
            const int32_t nb = batch - b0 < civic::kRaggedItems ? batch - b0 : civic::kRaggedItems;
            int32_t rows[civic::kRaggedItems + 1], longest = 0;
            for (int32_t i = 0; i <= nb; ++i) rows[i] = static_cast<int32_t>(row_offsets[b0 + i]);
            for (int32_t i = 0; i < nb; ++i) longest = rows[i + 1] - rows[i] > longest ? rows[i + 1] - rows[i] : longest;
            const int64_t cache_at = static_cast<int64_t>(b0) * n_kv_heads * s_max * head_dim * esz;
            const int rc = civic::prefill_attn(q, k, v, out, dtype, nb, longest, longest, n_q_heads, n_kv_heads, head_dim, q_strides,
                                               kv_strides, o_strides, causal, softmax_scale,
                                               k_cache ? static_cast<char*>(k_cache) + cache_at : nullptr,
                                               v_cache ? static_cast<char*>(v_cache) + cache_at : nullptr, s_max, pos0, nullptr, stream,
                                               rows, pass == 0, true);
            if (rc != CIVIC_OK) return rc;
        }
    return CIVIC_OK;
}
