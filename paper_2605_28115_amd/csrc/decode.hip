// civic_decode_attn: one generated token attending to the compact prompt in the contiguous KV cache (the
// per-token work inside the autoregressive decoding cost C_dec of Eq. 2 / Eq. 7; the cache is the one
// civic_kv_write fills).  HBM-bound: every K and V row of the context is read once, 2 * H_kv * n_ctx * d
// elements per sample, and nothing else of size moves.
//
// The context of a (batch item, KV head) is split over several workgroups so that a launch of a few dozen
// (item, head) pairs still covers the chip; a workgroup serves all query heads of its KV head at once (up to 8
// per pass), so K and V are read once per group, not once per query head.
//   - A cache row is read by LPR adjacent lanes, 16 bytes each (LPR = row bytes / 16 rounded up to a power of two),
//     64 / LPR rows per wavefront instruction; a lane's loads of a round (U rows of K and the same rows of V) are
//     issued before anything is computed, so a workgroup whose share is one round makes a single trip to memory.
//   - Logits: packed bf16 dot products (v_dot2_f32_bf16) of the lane's 8 channels against every query head,
//     summed over the row's lanes; every lane of the row then holds the row's logits.
//   - Each (wavefront, row slot) runs its own online softmax over the rows it meets: no barrier and no LDS in
//     the loop.  The lane keeps the 8 output channels of its chunk for every head in fp32.
//   - At the end the 4 * 64 / LPR partial states of the workgroup meet in LDS; the workgroup writes the final
//     rows (one split) or its (max, sum, unnormalised output) into the workspace, which a second small launch
//     combines.
#include <cmath>

#include "civic_internal.h"

namespace civic {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / kWave;
constexpr int kDecU = 4;                 // cache rows per lane and round

constexpr int kDecRaggedItems = 256;     // samples of one launch when every sample has its own context length

struct DecodeArgs {
    const void* q; const void* kc; const void* vc; void* out; float* ws;
    int64_t s_max;
    int32_t batch, n_q_heads, n_kv_heads, head_dim, group, head_blocks;
    int32_t n_ctx, splits, keys_per_split;
    int32_t cpr;                          // 16-byte chunks per cache row
    float scale_log2;                     // softmax scale * log2(e)
    // civic_decode_attn_ragged: sample b attends to its cache rows [0, ctx_of[b]) (n_ctx is then the longest, which the
    // splits are laid out for; a split that starts past a sample's rows contributes an empty partial result)
    int32_t per_item;
    int32_t ctx_of[kDecRaggedItems];
};

typedef __bf16 dec_bf16x2 __attribute__((ext_vector_type(2)));

// acc + a.lo * b.lo + a.hi * b.hi for two words of packed bf16 pairs.  (The words come in as scalars on purpose:
// a bit cast applied directly to an element of a vector variable reads the vector's first element.)
__device__ __forceinline__ float dot2_words(uint32_t a, uint32_t b, float acc)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dec_bf16x2, a), __builtin_bit_cast(dec_bf16x2, b), acc, false);
}

// Sum over the LPR adjacent lanes that share a cache row; every one of them receives the total.  Inside a row of
// 16 lanes the exchange is a data-parallel-primitive (DPP) operand of the add itself: lane pairs, then the two
// pairs of a quad, then the mirrored lane of the other quad of a half row (whose four lanes all hold that quad's
// sum by then), then the mirrored lane of the other half row.  No LDS round trip: a shuffle through LDS per step
// made the logits of a round a chain of 64 dependent waits.  Rows wider than 16 lanes finish with shuffles.
template <int CTRL>
__device__ __forceinline__ float dpp_moved(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, false));
}

template <int LPR>
__device__ __forceinline__ float row_sum(float v)
{
    if constexpr (LPR >= 2) v += dpp_moved<0xB1>(v);        // quad_perm [1,0,3,2]
    if constexpr (LPR >= 4) v += dpp_moved<0x4E>(v);        // quad_perm [2,3,0,1]
    if constexpr (LPR >= 8) v += dpp_moved<0x141>(v);       // row_half_mirror
    if constexpr (LPR >= 16) v += dpp_moved<0x140>(v);      // row_mirror
    if constexpr (LPR >= 32) v += __shfl_xor(v, 16, kWave);
    if constexpr (LPR >= 64) v += __shfl_xor(v, 32, kWave);
    return v;
}

template <bool BF16, int HG, int LPR>
__global__ __launch_bounds__(kDecThreads) void decode_partial_kernel(DecodeArgs a)
{
    constexpr int E = BF16 ? 8 : 4;       // elements per 16-byte chunk
    constexpr int RPS = kWave / LPR;      // cache rows per wavefront instruction
    constexpr int SLOTS = kDecWaves * RPS;   // independent softmax streams per workgroup
    extern __shared__ __attribute__((aligned(16))) float dec_lds[];
    // [SLOTS][HG] maxima, [SLOTS][HG] sums, [SLOTS][HG][d] outputs
    float* sm_m = dec_lds;
    float* sm_l = dec_lds + SLOTS * HG;
    float* sm_o = dec_lds + 2 * SLOTS * HG;

    const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid >> 6;
    const int r = lane / LPR, c = lane % LPR;
    const bool chunk_live = c < a.cpr;
    const int split = blockIdx.x;
    const int g = blockIdx.y / a.head_blocks, hb = blockIdx.y - g * a.head_blocks;
    const int b = blockIdx.z;
    const int d = a.head_dim;
    const int k0 = split * a.keys_per_split;
    const int n_ctx = a.per_item ? a.ctx_of[b] : a.n_ctx;
    const int k1 = min(k0 + a.keys_per_split, n_ctx);

    // the lane's chunk of every query head of the pass (heads past the group repeat the last one; never written)
    u32x4 qw[HG];
#pragma unroll
    for (int hh = 0; hh < HG; ++hh) {
        const int hg = min(hb * HG + hh, a.group - 1);
        const int64_t row = static_cast<int64_t>(b) * a.n_q_heads + g * a.group + hg;
        qw[hh] = u32x4{0u, 0u, 0u, 0u};
        if (chunk_live) qw[hh] = *reinterpret_cast<const u32x4*>(static_cast<const char*>(a.q) + (row * d + c * E) * (BF16 ? 2 : 4));
    }
    const int64_t head_row0 = (static_cast<int64_t>(b) * a.n_kv_heads + g) * a.s_max;
    const char* kbase = static_cast<const char*>(a.kc) + (head_row0 * d + c * E) * (BF16 ? 2 : 4);
    const char* vbase = static_cast<const char*>(a.vc) + (head_row0 * d + c * E) * (BF16 ? 2 : 4);
    const int64_t row_bytes = static_cast<int64_t>(d) * (BF16 ? 2 : 4);

    float m[HG], l[HG], acc[HG][E];
#pragma unroll
    for (int hh = 0; hh < HG; ++hh) {
        m[hh] = -INFINITY; l[hh] = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) acc[hh][e] = 0.f;
    }

    // Round: the workgroup's next SLOTS * U rows; slot (w, r) takes rows key0 + (u * kDecWaves + w) * RPS + r.  The
    // loads of the next round are issued before the current one is computed.
    u32x4 kq[kDecU], vq[kDecU], kn[kDecU], vn[kDecU];
    auto fetch = [&](int key0, u32x4* kd, u32x4* vd) {
#pragma unroll
        for (int u = 0; u < kDecU; ++u) {
            const int key = key0 + (u * kDecWaves + w) * RPS + r;
            kd[u] = u32x4{0u, 0u, 0u, 0u};
            vd[u] = u32x4{0u, 0u, 0u, 0u};
            if (key < k1 && chunk_live) {
                kd[u] = load_streaming(reinterpret_cast<const u32x4*>(kbase + key * row_bytes));
                vd[u] = load_streaming(reinterpret_cast<const u32x4*>(vbase + key * row_bytes));
            }
        }
    };
    fetch(k0, kn, vn);
    for (int key0 = k0; key0 < k1; key0 += SLOTS * kDecU) {
#pragma unroll
        for (int u = 0; u < kDecU; ++u) { kq[u] = kn[u]; vq[u] = vn[u]; }
        if (key0 + SLOTS * kDecU < k1) fetch(key0 + SLOTS * kDecU, kn, vn);
        float s[kDecU][HG];
#pragma unroll
        for (int u = 0; u < kDecU; ++u) {
            const int key = key0 + (u * kDecWaves + w) * RPS + r;
#pragma unroll
            for (int hh = 0; hh < HG; ++hh) {
                float part = 0.f;
                if constexpr (BF16) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) part = dot2_words(kq[u][e], qw[hh][e], part);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) part = fmaf(__uint_as_float(kq[u][e]), __uint_as_float(qw[hh][e]), part);
                }
                const float tot = row_sum<LPR>(part) * a.scale_log2;
                s[u][hh] = key < k1 ? tot : -INFINITY;
            }
        }
#pragma unroll
        for (int hh = 0; hh < HG; ++hh) {
            float m_new = m[hh];
#pragma unroll
            for (int u = 0; u < kDecU; ++u) m_new = fmaxf(m_new, s[u][hh]);
            const float m_use = m_new == -INFINITY ? 0.f : m_new;       // a slot that has met no row yet
            const float alpha = __builtin_amdgcn_exp2f(m[hh] - m_use);  // exp2(-inf) = 0 on the first rows
            float p[kDecU], psum = 0.f;
#pragma unroll
            for (int u = 0; u < kDecU; ++u) { p[u] = __builtin_amdgcn_exp2f(s[u][hh] - m_use); psum += p[u]; }
            l[hh] = l[hh] * alpha + psum;
            m[hh] = m_new;
#pragma unroll
            for (int e = 0; e < E; ++e) {
                float o = acc[hh][e] * alpha;
#pragma unroll
                for (int u = 0; u < kDecU; ++u) {
                    float ve;
                    if constexpr (BF16) ve = (e & 1) ? __uint_as_float(vq[u][e >> 1] & 0xFFFF0000u) : __uint_as_float(vq[u][e >> 1] << 16);
                    else ve = __uint_as_float(vq[u][e]);
                    o = fmaf(p[u], ve, o);
                }
                acc[hh][e] = o;
            }
        }
    }

    // the workgroup's SLOTS states meet in LDS
    const int slot = w * RPS + r;
#pragma unroll
    for (int hh = 0; hh < HG; ++hh) {
        if (c == 0) { sm_m[slot * HG + hh] = m[hh]; sm_l[slot * HG + hh] = l[hh]; }
        if (chunk_live) {
            float* dst = sm_o + (static_cast<size_t>(slot) * HG + hh) * d + c * E;
#pragma unroll
            for (int e = 0; e < E; ++e) dst[e] = acc[hh][e];
        }
    }
    __syncthreads();
    for (int i = tid; i < HG * d; i += kDecThreads) {
        const int hh = i / d, ch = i - hh * d;
        const int hg = hb * HG + hh;
        if (hg >= a.group) continue;
        float mx = -INFINITY;
#pragma unroll
        for (int sidx = 0; sidx < SLOTS; ++sidx) mx = fmaxf(mx, sm_m[sidx * HG + hh]);
        float o = 0.f, lt = 0.f;
#pragma unroll
        for (int sidx = 0; sidx < SLOTS; ++sidx) {
            const float ms = sm_m[sidx * HG + hh];
            const float wgt = ms == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ms - mx);
            o = fmaf(wgt, sm_o[(static_cast<size_t>(sidx) * HG + hh) * d + ch], o);
            lt = fmaf(wgt, sm_l[sidx * HG + hh], lt);
        }
        const int64_t row = static_cast<int64_t>(b) * a.n_q_heads + g * a.group + hg;
        if (a.splits == 1) {
            const float val = o / lt;                              // n_ctx >= 1: at least one row was met
            if constexpr (BF16) static_cast<__bf16*>(a.out)[row * d + ch] = static_cast<__bf16>(val);
            else static_cast<float*>(a.out)[row * d + ch] = val;
        } else {
            float* dst = a.ws + (row * a.splits + split) * (d + 2);
            if (ch == 0) { dst[0] = mx; dst[1] = lt; }
            dst[2 + ch] = o;
        }
    }
}

// Combines the splits of one (batch item, query head): out = sum_s w_s o_s / sum_s w_s l_s, w_s = 2^(m_s - max m).
// The weights are prepared once per block (one thread per split, through LDS); the channel sums then run over
// independent loads, eight splits at a time.
constexpr int kDecMaxSplits = 1024;
template <bool BF16>
__global__ __launch_bounds__(128) void decode_merge_kernel(const float* __restrict__ ws, void* __restrict__ out, int32_t splits,
                                                           int32_t d)
{
    __shared__ float wgt[kDecMaxSplits];
    __shared__ float red[4];
    const int64_t row = blockIdx.x;
    const float* src = ws + row * splits * (d + 2);
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
    // everything the first eight splits contribute is requested at once: the thread's (max, sum) pair and its
    // channel of their outputs; the weights then need no further trip to memory
    float o_pre[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) o_pre[j] = (j < splits && tid < d) ? src[j * (d + 2) + 2 + tid] : 0.f;
    float mloc = -INFINITY;
    for (int s = tid; s < splits; s += 128) mloc = fmaxf(mloc, src[s * (d + 2)]);
    const float m_own = tid < splits ? src[tid * (d + 2)] : -INFINITY, l_own = tid < splits ? src[tid * (d + 2) + 1] : 0.f;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mloc = fmaxf(mloc, __shfl_xor(mloc, off, kWave));
    if (lane == 0) red[wv] = mloc;
    __syncthreads();
    const float mx = fmaxf(red[0], red[1]);
    float lsum = 0.f;
    for (int s = tid; s < splits; s += 128) {
        const float ms = s == tid ? m_own : src[s * (d + 2)];
        const float wt = ms == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ms - mx);
        wgt[s] = wt;
        lsum = fmaf(wt, s == tid ? l_own : src[s * (d + 2) + 1], lsum);
    }
    lsum = wave_sum(lsum);
    if (lane == 0) red[2 + wv] = lsum;
    __syncthreads();
    const float inv = 1.0f / (red[2] + red[3]);
    for (int ch = tid; ch < d; ch += 128) {
        float o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        int s = 0;
        if (ch == tid) {                                           // the first eight are in registers already
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] = j < splits ? wgt[j] * o_pre[j] : 0.f;
            s = splits < 8 ? splits : 8;
        }
        for (; s + 8 <= splits; s += 8) {
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] = fmaf(wgt[s + j], src[(s + j) * (d + 2) + 2 + ch], o[j]);
        }
        for (; s < splits; ++s) o[0] = fmaf(wgt[s], src[s * (d + 2) + 2 + ch], o[0]);
        const float val = (((o[0] + o[1]) + (o[2] + o[3])) + ((o[4] + o[5]) + (o[6] + o[7]))) * inv;
        if constexpr (BF16) static_cast<__bf16*>(out)[row * d + ch] = static_cast<__bf16>(val);
        else static_cast<float*>(out)[row * d + ch] = val;
    }
}

// Block shape and split count for these sizes (shared by the launch and the workspace query).
struct DecodePlan {
    int hg, lpr, head_blocks, splits, keys_per_split;
    size_t ws_bytes, lds_bytes;
};

static int decode_plan(int dtype, int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int64_t n_ctx,
                       DecodePlan* p)
{
    const int esz = dtype_size(dtype);
    if (!esz || batch < 0 || n_q_heads <= 0 || n_kv_heads <= 0 || head_dim <= 0 || n_ctx < 0) return CIVIC_ERR_INVALID_ARG;
    if (n_q_heads % n_kv_heads) return CIVIC_ERR_INVALID_ARG;
    if ((static_cast<int64_t>(head_dim) * esz) % 16) return CIVIC_ERR_INVALID_ARG;
    const int cpr = head_dim * esz / 16;
    if (cpr > kWave || n_ctx > INT32_MAX || batch > 65535) return CIVIC_ERR_UNSUPPORTED;
    const int group = n_q_heads / n_kv_heads;
    p->hg = group >= 8 ? 8 : group > 2 ? 4 : group;             // 1, 2, 4 or 8 query heads per pass
    p->head_blocks = (group + p->hg - 1) / p->hg;
    if (static_cast<int64_t>(n_kv_heads) * p->head_blocks > 65535) return CIVIC_ERR_UNSUPPORTED;
    p->lpr = 8;
    while (p->lpr < cpr) p->lpr *= 2;
    // About four workgroups per compute unit, and no split shorter than one round of the workgroup.
    const int64_t units = static_cast<int64_t>(batch > 0 ? batch : 1) * n_kv_heads * p->head_blocks;
    const int64_t round_keys = static_cast<int64_t>(kDecWaves) * (kWave / p->lpr) * kDecU;
    int64_t splits = (1024 + units - 1) / units;
    const int64_t max_splits = (n_ctx + round_keys - 1) / round_keys;
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    if (splits > kDecMaxSplits) splits = kDecMaxSplits;
    int64_t kps = (n_ctx + splits - 1) / splits;
    kps = (kps + round_keys - 1) / round_keys * round_keys;     // whole rounds
    if (kps < round_keys) kps = round_keys;
    splits = n_ctx > 0 ? (n_ctx + kps - 1) / kps : 1;
    p->splits = static_cast<int>(splits);
    p->keys_per_split = static_cast<int>(kps);
    p->ws_bytes = splits > 1 ? sizeof(float) * static_cast<size_t>(batch) * n_q_heads * splits * (head_dim + 2) : 0;
    const int slots = kDecWaves * (kWave / p->lpr);
    p->lds_bytes = sizeof(float) * static_cast<size_t>(slots) * p->hg * (head_dim + 2);
    return CIVIC_OK;
}

template <bool BF16, int HG>
static int launch_decode_lpr(const DecodeArgs& a, const DecodePlan& p, hipStream_t s)
{
    const dim3 grid(static_cast<unsigned>(p.splits), static_cast<unsigned>(a.n_kv_heads * p.head_blocks), static_cast<unsigned>(a.batch));
#define CIVIC_DEC_CASE(L)                                                                                              \
    case L: {                                                                                                          \
        if (p.lds_bytes > 64 * 1024) {                                                                                 \
            static std::atomic<uint64_t> allowed{0};                                                                   \
            const int rc = allow_dynamic_lds(reinterpret_cast<const void*>(decode_partial_kernel<BF16, HG, L>), p.lds_bytes, &allowed); \
            if (rc != CIVIC_OK) return rc;                                                                             \
        }                                                                                                              \
        civic::launch((decode_partial_kernel<BF16, HG, L>), grid, dim3(kDecThreads), p.lds_bytes, s, a);          \
        break;                                                                                                         \
    }
    switch (p.lpr) {
        CIVIC_DEC_CASE(8) CIVIC_DEC_CASE(16) CIVIC_DEC_CASE(32) CIVIC_DEC_CASE(64)
        default: return CIVIC_ERR_UNSUPPORTED;
    }
#undef CIVIC_DEC_CASE
    return check_launch();
}

template <bool BF16>
static int launch_decode(const DecodeArgs& a, const DecodePlan& p, hipStream_t s)
{
    switch (p.hg) {
        case 1: return launch_decode_lpr<BF16, 1>(a, p, s);
        case 2: return launch_decode_lpr<BF16, 2>(a, p, s);
        case 4: return launch_decode_lpr<BF16, 4>(a, p, s);
        default: return launch_decode_lpr<BF16, 8>(a, p, s);
    }
}

// Everything but the choice of the workspace: `ws` holds at least plan.ws_bytes when the plan splits.
static int decode_attn(const void* q, const void* k_cache, const void* v_cache, void* out, int dtype, int32_t batch,
                       int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int64_t s_max, int64_t n_ctx,
                       float softmax_scale, const DecodePlan& p, float* ws, void* stream, const int32_t* ctx_of = nullptr)
{
    DecodeArgs a;
    a.per_item = ctx_of ? 1 : 0;
    for (int i = 0; i < kDecRaggedItems; ++i) a.ctx_of[i] = ctx_of && i < batch ? ctx_of[i] : 0;
    a.q = q; a.kc = k_cache; a.vc = v_cache; a.out = out; a.ws = ws;
    a.s_max = s_max;
    a.batch = batch; a.n_q_heads = n_q_heads; a.n_kv_heads = n_kv_heads; a.head_dim = head_dim;
    a.group = n_q_heads / n_kv_heads; a.head_blocks = p.head_blocks;
    a.n_ctx = static_cast<int32_t>(n_ctx); a.splits = p.splits; a.keys_per_split = p.keys_per_split;
    a.cpr = head_dim * dtype_size(dtype) / 16;
    const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / std::sqrt(static_cast<float>(head_dim));
    a.scale_log2 = scale * 1.4426950408889634f;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int rc = dtype == CIVIC_BF16 ? launch_decode<true>(a, p, s) : launch_decode<false>(a, p, s);
    if (rc != CIVIC_OK || p.splits == 1) return rc;
    const unsigned rows = static_cast<unsigned>(batch) * static_cast<unsigned>(n_q_heads);
    if (dtype == CIVIC_BF16) civic::launch((decode_merge_kernel<true>), dim3(rows), dim3(128), 0, s, ws, out, p.splits, head_dim);
    else civic::launch((decode_merge_kernel<false>), dim3(rows), dim3(128), 0, s, ws, out, p.splits, head_dim);
    return check_launch();
}

// Argument checks shared by the two entry points (all before any HIP call).  CIVIC_OK with *nothing = true when
// there is no row to compute.
static int decode_check(const void* q, const void* k_cache, const void* v_cache, void* out, int dtype, int32_t batch,
                        int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int64_t s_max, int64_t n_ctx,
                        float softmax_scale, DecodePlan* p, bool* nothing)
{
    *nothing = false;
    const int rc = decode_plan(dtype, batch, n_q_heads, n_kv_heads, head_dim, n_ctx, p);
    if (rc != CIVIC_OK) return rc;
    if (s_max < 0 || n_ctx > s_max) return CIVIC_ERR_INVALID_ARG;
    if (!(softmax_scale >= 0.f) || std::isinf(softmax_scale)) return CIVIC_ERR_INVALID_ARG;
    if (batch == 0) { *nothing = true; return CIVIC_OK; }
    if (n_ctx < 1) return CIVIC_ERR_INVALID_ARG;                 // a softmax over no row has no value
    if (!q || !k_cache || !v_cache || !out) return CIVIC_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out)) return CIVIC_ERR_INVALID_ARG;
    return CIVIC_OK;
}

// ------------------------------------------------------------------------------ no allocation at all
// civic_decode_attn_noalloc keeps the partial results of the splits in a buffer that belongs to the library's
// code object instead of one the caller brings: every GPU that loads the library holds its own copy of this
// array, at its own address, until the process ends.
constexpr size_t kDecStaticBytes = CIVIC_DECODE_NOALLOC_MAX_BYTES;
static __device__ __align__(256) unsigned char dec_static_scratch[kDecStaticBytes];

// The array's address on the current device.  In host code the array's name stands for the symbol, not for
// device memory: its address is asked for once per device, with that device current, and kept.
static int static_scratch_ptr(void** ptr)
{
    constexpr int kMaxDevices = 64;
    static std::atomic<void*> cached[kMaxDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return record_hip_error(e);
    if (dev >= 0 && dev < kMaxDevices) {
        void* p = cached[dev].load(std::memory_order_acquire);
        if (p) { *ptr = p; return CIVIC_OK; }
    }
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(dec_static_scratch));
    if (e != hipSuccess || !p) return record_hip_error(e != hipSuccess ? e : hipErrorInvalidSymbol);
    if (dev >= 0 && dev < kMaxDevices) cached[dev].store(p, std::memory_order_release);
    *ptr = p;
    return CIVIC_OK;
}

}  // namespace civic

extern "C" int civic_decode_attn_noalloc(const void* q, const void* k_cache, const void* v_cache, void* out, int dtype,
                                         int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                         int64_t s_max, int64_t n_ctx, float softmax_scale, void* stream)
{
    using namespace civic;
    DecodePlan p;
    bool nothing = false;
    const int rc = decode_check(q, k_cache, v_cache, out, dtype, batch, n_q_heads, n_kv_heads, head_dim, s_max, n_ctx,
                                softmax_scale, &p, &nothing);
    if (rc != CIVIC_OK || nothing) return rc;
    if (p.ws_bytes > kDecStaticBytes) return CIVIC_ERR_WORKSPACE;      // more partial results than the array holds
    void* scratch = nullptr;
    if (p.ws_bytes > 0) {
        const int rs = static_scratch_ptr(&scratch);
        if (rs != CIVIC_OK) return rs;
    }
    // every element of the array that the combine launch reads is written by this call's first launch: nothing
    // has to start at zero
    return decode_attn(q, k_cache, v_cache, out, dtype, batch, n_q_heads, n_kv_heads, head_dim, s_max, n_ctx, softmax_scale,
                       p, static_cast<float*>(scratch), stream);
}

extern "C" size_t civic_decode_attn_workspace_bytes(int dtype, int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                                                    int32_t head_dim, int64_t n_ctx)
{
    civic::DecodePlan p;
    if (civic::decode_plan(dtype, batch, n_q_heads, n_kv_heads, head_dim, n_ctx, &p) != CIVIC_OK) return 0;
    return p.ws_bytes;
}

extern "C" int civic_decode_attn(const void* q, const void* k_cache, const void* v_cache, void* out, int dtype,
                                 int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int64_t s_max,
                                 int64_t n_ctx, float softmax_scale, void* workspace, size_t workspace_bytes, void* stream)
{
    using namespace civic;
    DecodePlan p;
    bool nothing = false;
    const int rc = decode_check(q, k_cache, v_cache, out, dtype, batch, n_q_heads, n_kv_heads, head_dim, s_max, n_ctx,
                                softmax_scale, &p, &nothing);
    if (rc != CIVIC_OK || nothing) return rc;
    if (p.ws_bytes > 0 && (!workspace || workspace_bytes < p.ws_bytes || !aligned16(workspace))) return CIVIC_ERR_WORKSPACE;
    return decode_attn(q, k_cache, v_cache, out, dtype, batch, n_q_heads, n_kv_heads, head_dim, s_max, n_ctx, softmax_scale,
                       p, static_cast<float*>(workspace), stream);
}

// ---------------------------------------------------------------------------------------------- ragged caches
namespace civic {

// The longest context of samples [b0, b0 + nb); -1 if one of them is shorter than one row or longer than the caches.
static int64_t longest_ctx(const int32_t* n_ctx, int32_t b0, int32_t nb, int64_t s_max)
{
    int64_t longest = 0;
    for (int32_t i = 0; i < nb; ++i) {
        const int64_t n = n_ctx[b0 + i];
        if (n < 1 || n > s_max) return -1;
        longest = n > longest ? n : longest;
    }
    return longest;
}

}  // namespace civic

extern "C" size_t civic_decode_attn_ragged_workspace_bytes(int dtype, int32_t batch, const int32_t* n_ctx, int32_t n_q_heads,
                                                           int32_t n_kv_heads, int32_t head_dim)
{
    using namespace civic;
    if (batch <= 0 || !n_ctx) return 0;
    size_t need = 0;                                          // the groups run one after the other and share the workspace
    for (int32_t b0 = 0; b0 < batch; b0 += kDecRaggedItems) {
        const int32_t nb = batch - b0 < kDecRaggedItems ? batch - b0 : kDecRaggedItems;
        const int64_t longest = longest_ctx(n_ctx, b0, nb, INT32_MAX);
        DecodePlan p;
        if (longest < 0 || decode_plan(dtype, nb, n_q_heads, n_kv_heads, head_dim, longest, &p) != CIVIC_OK) return 0;
        need = p.ws_bytes > need ? p.ws_bytes : need;
    }
    return need;
}

extern "C" int civic_decode_attn_ragged(const void* q, const void* k_cache, const void* v_cache, void* out, int dtype,
                                        int32_t batch, const int32_t* n_ctx, int32_t n_q_heads, int32_t n_kv_heads,
                                        int32_t head_dim, int64_t s_max, float softmax_scale, void* workspace,
                                        size_t workspace_bytes, void* stream)
{
    using namespace civic;
    const int esz = dtype_size(dtype);
    if (!esz || batch < 0) return CIVIC_ERR_INVALID_ARG;
    if (batch > 0 && !n_ctx) return CIVIC_ERR_INVALID_ARG;
    // Groups of up to kDecRaggedItems samples, each the two launches of civic_decode_attn laid out for the group's
    // longest context; every group is checked before the first launch.
    for (int pass = 0; pass < 2; ++pass)
        for (int32_t b0 = 0; b0 < batch; b0 += kDecRaggedItems) {
            const int32_t nb = batch - b0 < kDecRaggedItems ? batch - b0 : kDecRaggedItems;
            const int64_t longest = longest_ctx(n_ctx, b0, nb, s_max);
            if (longest < 0) return CIVIC_ERR_INVALID_ARG;
            const char* qb = static_cast<const char*>(q) + static_cast<int64_t>(b0) * n_q_heads * head_dim * esz;
            char* ob = static_cast<char*>(out) + static_cast<int64_t>(b0) * n_q_heads * head_dim * esz;
            const int64_t cache_at = static_cast<int64_t>(b0) * n_kv_heads * s_max * head_dim * esz;
            const char* kb = static_cast<const char*>(k_cache) + cache_at;
            const char* vb = static_cast<const char*>(v_cache) + cache_at;
            DecodePlan p;
            bool nothing = false;
            int rc = decode_check(q ? qb : nullptr, k_cache ? kb : nullptr, v_cache ? vb : nullptr, out ? ob : nullptr, dtype, nb, n_q_heads,
                                  n_kv_heads, head_dim, s_max, longest, softmax_scale, &p, &nothing);
            if (rc != CIVIC_OK) return rc;
            if (p.ws_bytes > 0 && (!workspace || workspace_bytes < p.ws_bytes || !aligned16(workspace))) return CIVIC_ERR_WORKSPACE;
            if (pass == 0 || nothing) continue;
            rc = decode_attn(qb, kb, vb, ob, dtype, nb, n_q_heads, n_kv_heads, head_dim, s_max, longest, softmax_scale, p,
                             static_cast<float*>(workspace), stream, n_ctx + b0);
            if (rc != CIVIC_OK) return rc;
        }
    return CIVIC_OK;
}
