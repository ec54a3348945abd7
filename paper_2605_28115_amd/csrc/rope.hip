// Rotary position embedding on three axes (temporal, height, width), driven by the position ids that the
// compact merge carries along unchanged ("text positions are preserved, compact visual positions are inherited",
// sentence after Eq. 14).  The paper does not print the rotary form; this is the published three-axis rotary
// embedding of the Qwen-VL family in its rotate-half layout: frequency pair i of a head row is
// (x[i], x[i + d/2]), turned by the angle pos[axis_of_pair[i]] * inv_freq[i]; which axis and which frequency a
// pair uses are tables of the caller (sections or interleaved, any base).
//
//   civic_mrope_table    (cos, sin) per (batch item, token, pair), once per prefill: every layer and every head
//                        uses the same angles.  Angles are formed and reduced in double precision, so the fp32
//                        (cos, sin) are correctly rounded to ~1 ulp however large the ids are.
//   civic_mrope_apply    rotates the head rows of one tensor (HBM-bound; Q of a decode step, or any tensor).
//   civic_kv_write_rope  civic_kv_write with K rotated on its way into the cache: the copy is HBM-bound, the
//                        rotation rides along.
// (civic_prefill_attn_rope, in attn.hip, rotates Q in registers from the same table.)
#include <cmath>

#include "civic_internal.h"

namespace civic {

constexpr int kRopeMaxPairs = CIVIC_MAX_HEAD_DIM / 2;

struct RopeTables {
    float inv_freq[kRopeMaxPairs];
    uint8_t axis[kRopeMaxPairs];
};

__global__ __launch_bounds__(256) void mrope_table_kernel(const int32_t* __restrict__ pos, int32_t batch, int64_t seq, int32_t n_pairs,
                                                          RopeTables tab, float2* __restrict__ cos_sin)
{
    const int64_t total = static_cast<int64_t>(batch) * seq * n_pairs;
    for (int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; idx < total;
         idx += static_cast<int64_t>(gridDim.x) * blockDim.x) {
        const int i = static_cast<int>(idx % n_pairs);
        const int64_t bt = idx / n_pairs;                           // = b * seq + t
        const int32_t p = pos[static_cast<int64_t>(tab.axis[i]) * batch * seq + bt];
        const double angle = static_cast<double>(p) * static_cast<double>(tab.inv_freq[i]);
        double sn, cs;
        sincos(angle, &sn, &cs);
        cos_sin[idx] = make_float2(static_cast<float>(cs), static_cast<float>(sn));
    }
}

// One 16-byte chunk of the first half of a head row and its partner chunk of the second half, rotated by the
// (cos, sin) of E consecutive pairs (E = 8 bf16 or 4 fp32 elements per chunk).
template <bool BF16>
__device__ __forceinline__ void rotate_chunks(u32x4& lo, u32x4& hi, const float2* cs)
{
    if constexpr (BF16) {
#pragma unroll
        for (int wd = 0; wd < 4; ++wd) {
            const uint32_t a = lo[wd], b = hi[wd];
            const float x0[2] = {__uint_as_float(a << 16), __uint_as_float(a & 0xFFFF0000u)};
            const float x1[2] = {__uint_as_float(b << 16), __uint_as_float(b & 0xFFFF0000u)};
            __bf16 y0[2], y1[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const float2 t = cs[2 * wd + e];
                float r0, r1;
                rope_pair(x0[e], x1[e], t.x, t.y, r0, r1);
                y0[e] = static_cast<__bf16>(r0);
                y1[e] = static_cast<__bf16>(r1);
            }
            lo[wd] = static_cast<uint32_t>(__builtin_bit_cast(uint16_t, y0[0])) | (static_cast<uint32_t>(__builtin_bit_cast(uint16_t, y0[1])) << 16);
            hi[wd] = static_cast<uint32_t>(__builtin_bit_cast(uint16_t, y1[0])) | (static_cast<uint32_t>(__builtin_bit_cast(uint16_t, y1[1])) << 16);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float x0 = __uint_as_float(lo[e]), x1 = __uint_as_float(hi[e]);
            const float2 t = cs[e];
            float r0, r1;
            rope_pair(x0, x1, t.x, t.y, r0, r1);
            lo[e] = __float_as_uint(r0);
            hi[e] = __float_as_uint(r1);
        }
    }
}

template <bool BF16>
__device__ __forceinline__ void load_cs(const float2* __restrict__ table, int64_t token, int32_t n_pairs, int chunk, float2* cs)
{
    constexpr int E = BF16 ? 8 : 4;
    const float4* src = reinterpret_cast<const float4*>(table + token * n_pairs + chunk * E);
#pragma unroll
    for (int v = 0; v < E / 2; ++v) {
        const float4 t = src[v];
        cs[2 * v] = make_float2(t.x, t.y);
        cs[2 * v + 1] = make_float2(t.z, t.w);
    }
}

struct RopeApplyArgs {
    const void* x; void* out; const float2* cos_sin;
    int64_t xs[3], os[3];               // element strides: batch, token, head
    int64_t seq;
    int32_t batch, heads, half_chunks;  // 16-byte chunks in half a head row
    int32_t n_pairs;
};

// Work item = (token, head, chunk of the first half); grid y = batch item.
template <bool BF16>
__global__ __launch_bounds__(256) void mrope_apply_kernel(RopeApplyArgs a)
{
    constexpr int E = BF16 ? 8 : 4, ESZ = BF16 ? 2 : 4;
    const int b = blockIdx.y;
    const int64_t per_token = static_cast<int64_t>(a.heads) * a.half_chunks;
    const int64_t total = a.seq * per_token;
    for (int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; idx < total;
         idx += static_cast<int64_t>(gridDim.x) * blockDim.x) {
        const int64_t t = idx / per_token;
        const int rem = static_cast<int>(idx - t * per_token);
        const int h = rem / a.half_chunks, c = rem - h * a.half_chunks;
        const char* src = static_cast<const char*>(a.x) + (b * a.xs[0] + t * a.xs[1] + h * a.xs[2] + c * E) * ESZ;
        u32x4 lo = load_streaming(reinterpret_cast<const u32x4*>(src));
        u32x4 hi = load_streaming(reinterpret_cast<const u32x4*>(src + static_cast<int64_t>(a.n_pairs) * ESZ));
        float2 cs[E];
        load_cs<BF16>(a.cos_sin, b * a.seq + t, a.n_pairs, c, cs);
        rotate_chunks<BF16>(lo, hi, cs);
        char* dst = static_cast<char*>(a.out) + (b * a.os[0] + t * a.os[1] + h * a.os[2] + c * E) * ESZ;
        *reinterpret_cast<u32x4*>(dst) = lo;
        *reinterpret_cast<u32x4*>(dst + static_cast<int64_t>(a.n_pairs) * ESZ) = hi;
    }
}

struct KvRopeArgs {
    const void* k; const void* v; void* kc; void* vc; const float2* cos_sin;
    int64_t ks[3];                      // element strides of k and v: batch, token, head
    int64_t s_max, pos0;
    int32_t seq, n_kv_heads, half_chunks, n_pairs, head_dim;
};

template <bool BF16>
__global__ __launch_bounds__(256) void kv_write_rope_kernel(KvRopeArgs a)
{
    constexpr int E = BF16 ? 8 : 4, ESZ = BF16 ? 2 : 4;
    const int b = blockIdx.y;
    const int64_t per_token = static_cast<int64_t>(a.n_kv_heads) * a.half_chunks;
    const int64_t total = static_cast<int64_t>(a.seq) * per_token;
    const int64_t half_bytes = static_cast<int64_t>(a.n_pairs) * ESZ;
    for (int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; idx < total;
         idx += static_cast<int64_t>(gridDim.x) * blockDim.x) {
        const int64_t t = idx / per_token;
        const int rem = static_cast<int>(idx - t * per_token);
        const int g = rem / a.half_chunks, c = rem - g * a.half_chunks;
        const int64_t src_off = (b * a.ks[0] + t * a.ks[1] + g * a.ks[2] + c * E) * ESZ;
        const char* ksrc = static_cast<const char*>(a.k) + src_off;
        const char* vsrc = static_cast<const char*>(a.v) + src_off;
        u32x4 klo = load_streaming(reinterpret_cast<const u32x4*>(ksrc));
        u32x4 khi = load_streaming(reinterpret_cast<const u32x4*>(ksrc + half_bytes));
        const u32x4 vlo = load_streaming(reinterpret_cast<const u32x4*>(vsrc));
        const u32x4 vhi = load_streaming(reinterpret_cast<const u32x4*>(vsrc + half_bytes));
        float2 cs[E];
        load_cs<BF16>(a.cos_sin, static_cast<int64_t>(b) * a.seq + t, a.n_pairs, c, cs);
        rotate_chunks<BF16>(klo, khi, cs);
        const int64_t cache_row = (static_cast<int64_t>(b) * a.n_kv_heads + g) * a.s_max + a.pos0 + t;
        const int64_t dst_off = (cache_row * a.head_dim + c * E) * ESZ;
        char* kdst = static_cast<char*>(a.kc) + dst_off;
        char* vdst = static_cast<char*>(a.vc) + dst_off;
        *reinterpret_cast<u32x4*>(kdst) = klo;
        *reinterpret_cast<u32x4*>(kdst + half_bytes) = khi;
        *reinterpret_cast<u32x4*>(vdst) = vlo;
        *reinterpret_cast<u32x4*>(vdst + half_bytes) = vhi;
    }
}

// head_dim must split into two halves of whole 16-byte chunks.
static bool rope_head_dim_ok(int32_t head_dim, int esz)
{
    return head_dim > 0 && head_dim % 2 == 0 && ((head_dim / 2) * esz) % 16 == 0;
}

static unsigned rope_blocks(int64_t items)
{
    int64_t blocks = (items + 255) / 256;
    if (blocks > 256 * 8) blocks = 256 * 8;                       // grid-stride beyond eight blocks per compute unit
    return static_cast<unsigned>(blocks > 0 ? blocks : 1);
}

}  // namespace civic

extern "C" int civic_mrope_table(const int32_t* pos_ids, int32_t batch, int64_t seq, int32_t n_pairs,
                                 const int32_t* axis_of_pair, const float* inv_freq, float* cos_sin, void* stream)
{
    using namespace civic;
    if (batch < 0 || seq < 0 || n_pairs <= 0 || !axis_of_pair || !inv_freq) return CIVIC_ERR_INVALID_ARG;
    if (n_pairs > kRopeMaxPairs) return CIVIC_ERR_UNSUPPORTED;
    RopeTables tab;
    for (int32_t i = 0; i < kRopeMaxPairs; ++i) {
        if (i < n_pairs) {
            if (axis_of_pair[i] < 0 || axis_of_pair[i] > 2 || !std::isfinite(inv_freq[i])) return CIVIC_ERR_INVALID_ARG;
            tab.axis[i] = static_cast<uint8_t>(axis_of_pair[i]);
            tab.inv_freq[i] = inv_freq[i];
        } else {
            tab.axis[i] = 0; tab.inv_freq[i] = 0.f;
        }
    }
    const int64_t total = static_cast<int64_t>(batch) * seq * n_pairs;
    if (total > 0 && (!pos_ids || !cos_sin)) return CIVIC_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(pos_ids) & 3u) || !aligned16(cos_sin)) return CIVIC_ERR_INVALID_ARG;
    if (total == 0) return CIVIC_OK;
    civic::launch(mrope_table_kernel, dim3(rope_blocks(total)), dim3(256), 0, static_cast<hipStream_t>(stream), pos_ids, batch,
                       seq, n_pairs, tab, reinterpret_cast<float2*>(cos_sin));
    return check_launch();
}

extern "C" int civic_mrope_apply(const void* x, void* out, int dtype, int32_t batch, int64_t seq, int32_t heads, int32_t head_dim,
                                 const int64_t* x_strides, const int64_t* out_strides, const float* cos_sin, void* stream)
{
    using namespace civic;
    const int esz = dtype_size(dtype);
    if (!esz || !x_strides || !out_strides) return CIVIC_ERR_INVALID_ARG;
    if (batch < 0 || seq < 0 || heads <= 0 || !rope_head_dim_ok(head_dim, esz)) return CIVIC_ERR_INVALID_ARG;
    const bool some = batch > 0 && seq > 0;
    if (some && (!x || !out || !cos_sin)) return CIVIC_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(out) || !aligned16(cos_sin)) return CIVIC_ERR_INVALID_ARG;
    for (int i = 0; i < 3; ++i) {
        if (x_strides[i] < 0 || out_strides[i] < 0) return CIVIC_ERR_INVALID_ARG;
        if ((x_strides[i] * esz) % 16 || (out_strides[i] * esz) % 16) return CIVIC_ERR_INVALID_ARG;
    }
    if (head_dim > CIVIC_MAX_HEAD_DIM || batch > 65535) return CIVIC_ERR_UNSUPPORTED;
    if (!some) return CIVIC_OK;
    RopeApplyArgs a;
    a.x = x; a.out = out; a.cos_sin = reinterpret_cast<const float2*>(cos_sin);
    for (int i = 0; i < 3; ++i) { a.xs[i] = x_strides[i]; a.os[i] = out_strides[i]; }
    a.seq = seq; a.batch = batch; a.heads = heads; a.n_pairs = head_dim / 2;
    a.half_chunks = (head_dim / 2) * esz / 16;
    const dim3 grid(rope_blocks(seq * heads * a.half_chunks), static_cast<unsigned>(batch));
    if (dtype == CIVIC_BF16) civic::launch((mrope_apply_kernel<true>), grid, dim3(256), 0, static_cast<hipStream_t>(stream), a);
    else civic::launch((mrope_apply_kernel<false>), grid, dim3(256), 0, static_cast<hipStream_t>(stream), a);
    return check_launch();
}

extern "C" int civic_kv_write_rope(const void* k, const void* v, const int64_t* kv_strides, int dtype, const float* cos_sin,
                                   void* k_cache, void* v_cache, int32_t batch, int32_t seq, int32_t n_kv_heads,
                                   int32_t head_dim, int64_t s_max, int64_t pos0, void* stream)
{
    using namespace civic;
    const int esz = dtype_size(dtype);
    if (!esz || !kv_strides) return CIVIC_ERR_INVALID_ARG;
    if (batch < 0 || seq < 0 || n_kv_heads <= 0 || !rope_head_dim_ok(head_dim, esz)) return CIVIC_ERR_INVALID_ARG;
    const bool some = batch > 0 && seq > 0;
    if (some && (!k || !v || !k_cache || !v_cache || !cos_sin)) return CIVIC_ERR_INVALID_ARG;
    if (pos0 < 0 || s_max < 0 || pos0 + seq > s_max) return CIVIC_ERR_INVALID_ARG;
    if (!aligned16(k) || !aligned16(v) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(cos_sin)) return CIVIC_ERR_INVALID_ARG;
    for (int i = 0; i < 3; ++i)
        if (kv_strides[i] < 0 || (kv_strides[i] * esz) % 16) return CIVIC_ERR_INVALID_ARG;
    if (kv_strides[2] < head_dim && n_kv_heads > 1) return CIVIC_ERR_INVALID_ARG;
    if (head_dim > CIVIC_MAX_HEAD_DIM || batch > 65535) return CIVIC_ERR_UNSUPPORTED;
    if (!some) return CIVIC_OK;
    KvRopeArgs a;
    a.k = k; a.v = v; a.kc = k_cache; a.vc = v_cache; a.cos_sin = reinterpret_cast<const float2*>(cos_sin);
    for (int i = 0; i < 3; ++i) a.ks[i] = kv_strides[i];
    a.s_max = s_max; a.pos0 = pos0; a.seq = seq; a.n_kv_heads = n_kv_heads; a.head_dim = head_dim;
    a.n_pairs = head_dim / 2; a.half_chunks = (head_dim / 2) * esz / 16;
    const dim3 grid(rope_blocks(static_cast<int64_t>(seq) * n_kv_heads * a.half_chunks), static_cast<unsigned>(batch));
    if (dtype == CIVIC_BF16) civic::launch((kv_write_rope_kernel<true>), grid, dim3(256), 0, static_cast<hipStream_t>(stream), a);
    else civic::launch((kv_write_rope_kernel<false>), grid, dim3(256), 0, static_cast<hipStream_t>(stream), a);
    return check_launch();
}
