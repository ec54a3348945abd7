// civic_kv_write: contiguous, un-paged KV-cache rows (storage term of Eq. 7).  HBM-bound copy with
// a (token, head) -> (head, token) transpose at head-row granularity.
//
// A block moves a tile of consecutive tokens for every KV head, K and V in the same launch
// (blockIdx.z).  Reads walk the token-major source in address order; for each head the writes of
// the tile form one contiguous run of tile_tokens * head_bytes in the cache.
#include "civic_internal.h"

namespace civic {

constexpr int kKvThreads = 256;
constexpr int kKvUnroll = 4;

struct KvArgs {
    const u32x4* src[2];
    u32x4* dst[2];
    int64_t stride_b, stride_t, stride_h;   // source strides in 16-byte units
    int64_t s_max, pos0;
    int32_t seq, n_kv_heads, chunks_per_head;
    int32_t chunks_per_token;                // n_kv_heads * chunks_per_head
    int32_t total;                           // seq * chunks_per_token (< 2^31)
};

__global__ __launch_bounds__(kKvThreads) void kv_write_kernel(KvArgs a)
{
    const int b = blockIdx.y;
    const u32x4* __restrict__ src = a.src[blockIdx.z] + b * a.stride_b;
    u32x4* __restrict__ dst = a.dst[blockIdx.z] + static_cast<int64_t>(b) * a.n_kv_heads * a.s_max * a.chunks_per_head;
    const uint32_t base = blockIdx.x * (kKvThreads * kKvUnroll) + threadIdx.x;
    const uint32_t cpt = a.chunks_per_token, cph = a.chunks_per_head;

    u32x4 val[kKvUnroll];
    int64_t out[kKvUnroll];
#pragma unroll
    for (int u = 0; u < kKvUnroll; ++u) {
        const uint32_t idx = base + u * kKvThreads;
        out[u] = -1;
        if (idx < static_cast<uint32_t>(a.total)) {
            const uint32_t tok = idx / cpt, rem = idx - tok * cpt;
            const uint32_t head = rem / cph, c = rem - head * cph;
            val[u] = load_streaming(src + tok * a.stride_t + head * a.stride_h + c);
            out[u] = (head * a.s_max + a.pos0 + tok) * cph + c;
        }
    }
#pragma unroll
    for (int u = 0; u < kKvUnroll; ++u)
        if (out[u] >= 0) dst[out[u]] = val[u];
}

}  // namespace civic

extern "C" int civic_kv_write(const void* k, const void* v, const int64_t* kv_strides, int dtype, void* k_cache,
                              void* v_cache, int32_t batch, int32_t seq, int32_t n_kv_heads, int32_t head_dim,
                              int64_t s_max, int64_t pos0, void* stream)
{
    using namespace civic;
    const int esz = dtype_size(dtype);
    if (!esz || !kv_strides) return CIVIC_ERR_INVALID_ARG;
    if (batch < 0 || seq < 0 || n_kv_heads <= 0 || head_dim <= 0) return CIVIC_ERR_INVALID_ARG;
    if (batch > 0 && seq > 0 && (!k || !v || !k_cache || !v_cache)) return CIVIC_ERR_INVALID_ARG;   // else nothing to copy
    if (pos0 < 0 || s_max < 0 || pos0 + seq > s_max) return CIVIC_ERR_INVALID_ARG;
    if ((static_cast<int64_t>(head_dim) * esz) % 16) return CIVIC_ERR_INVALID_ARG;
    if (!aligned16(k) || !aligned16(v) || !aligned16(k_cache) || !aligned16(v_cache)) return CIVIC_ERR_INVALID_ARG;
    for (int i = 0; i < 3; ++i)
        if (kv_strides[i] < 0 || (kv_strides[i] * esz) % 16) return CIVIC_ERR_INVALID_ARG;
    if (kv_strides[2] < head_dim && n_kv_heads > 1) return CIVIC_ERR_INVALID_ARG;
    if (batch > 65535) return CIVIC_ERR_UNSUPPORTED;
    if (batch == 0 || seq == 0) return CIVIC_OK;

    KvArgs a;
    a.src[0] = static_cast<const u32x4*>(k); a.src[1] = static_cast<const u32x4*>(v);
    a.dst[0] = static_cast<u32x4*>(k_cache); a.dst[1] = static_cast<u32x4*>(v_cache);
    a.stride_b = kv_strides[0] * esz / 16; a.stride_t = kv_strides[1] * esz / 16; a.stride_h = kv_strides[2] * esz / 16;
    a.s_max = s_max; a.pos0 = pos0;
    a.seq = seq; a.n_kv_heads = n_kv_heads;
    a.chunks_per_head = head_dim * esz / 16;
    a.chunks_per_token = n_kv_heads * a.chunks_per_head;
    const int64_t total = static_cast<int64_t>(seq) * a.chunks_per_token;
    if (total > INT32_MAX) return CIVIC_ERR_UNSUPPORTED;
    a.total = static_cast<int32_t>(total);
    const int64_t per_block = kKvThreads * kKvUnroll;
    const int64_t blocks = (total + per_block - 1) / per_block;
    if (blocks > INT32_MAX) return CIVIC_ERR_UNSUPPORTED;
    civic::launch(kv_write_kernel, dim3(static_cast<unsigned>(blocks), static_cast<unsigned>(batch), 2),
                       dim3(kKvThreads), 0, static_cast<hipStream_t>(stream), a);
    return check_launch();
}
