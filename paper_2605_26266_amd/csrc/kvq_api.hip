// Host layer of the C ABI: argument validation, the cache object, dispatch to the kernels.
// No device memory is allocated here; the cache storage is carved out of the caller's buffer.
#include <deque>
#include <new>

#include "kvq_internal.h"

struct kvq_block {
    int slot;        // index into the per-block metadata arrays
    int64_t start;   // logical position of the block's first token
    int64_t count;   // tokens of the block (shrinks when the cache is truncated)
};

struct kvq_cache {
    kvq_cache_desc desc;
    kvq::CacheView view;
    int64_t cap32;  // capacity rounded up to whole tiles
    int64_t base;   // logical position of the oldest live token (the storage is a ring)
    int64_t len;    // live tokens
    std::deque<kvq_block> blocks;   // KVQ_KEYS_PER_CHANNEL: live appended blocks, oldest first
    int next_slot;
    bool status_clean;   // the status block has been cleared on the device since the cache was created or reset

    // Forget blocks that lie wholly outside [base, base + len).
    void trim_blocks()
    {
        while (!blocks.empty() && blocks.front().start + blocks.front().count <= base) blocks.pop_front();
        while (!blocks.empty() && blocks.back().start >= base + len) {   // slots stay consecutive: reuse it next
            next_slot = blocks.back().slot;
            blocks.pop_back();
        }
        if (!blocks.empty() && blocks.back().start + blocks.back().count > base + len)
            blocks.back().count = base + len - blocks.back().start;
        if (len == 0) blocks.clear();
    }
};

namespace {

kvq_status check_desc(const kvq_cache_desc *d)
{
    if (!d) return KVQ_ERR_INVALID_ARG;
    if (d->num_heads < 1 || d->capacity_tokens < 1 || d->head_dim < 1 || d->bits < 1) return KVQ_ERR_INVALID_ARG;
    if (d->io_dtype != KVQ_BF16 && d->io_dtype != KVQ_FP32) return KVQ_ERR_INVALID_ARG;
    if (d->head_dim != 64 && d->head_dim != 128) return KVQ_ERR_UNSUPPORTED;
    if (d->bits != 2 && d->bits != 4) return KVQ_ERR_UNSUPPORTED;
    if (d->meta_format != KVQ_META_FP32 && d->meta_format != KVQ_META_FP8_BF16) return KVQ_ERR_INVALID_ARG;
    if (d->group_size != d->head_dim && d->group_size != 32 && d->group_size != 64) return KVQ_ERR_UNSUPPORTED;
    if (d->group_size > d->head_dim) return KVQ_ERR_UNSUPPORTED;
    if (d->group_size != d->head_dim && d->meta_format != KVQ_META_FP8_BF16) return KVQ_ERR_UNSUPPORTED;
    if (d->rotate != 1) return KVQ_ERR_UNSUPPORTED;
    if (d->key_axis != KVQ_KEYS_PER_TOKEN && d->key_axis != KVQ_KEYS_PER_CHANNEL) return KVQ_ERR_INVALID_ARG;
    if (d->key_axis == KVQ_KEYS_PER_CHANNEL && (d->meta_format != KVQ_META_FP32 || d->group_size != d->head_dim))
        return KVQ_ERR_UNSUPPORTED;
    if (d->capacity_tokens > ((int64_t)1 << 40)) return KVQ_ERR_INVALID_ARG;
    return KVQ_OK;
}

int64_t round_up_tile(int64_t n) { return (n + kvq::kTileTokens - 1) / kvq::kTileTokens * kvq::kTileTokens; }

int64_t max_blocks_of(int64_t cap32) { return cap32 / kvq::kTileTokens + 2; }

// Bytes of the per-channel key metadata that follow the ordinary storage (0 for per-token keys).
int64_t channel_bytes(const kvq_cache_desc *d, int64_t cap32)
{
    if (d->key_axis != KVQ_KEYS_PER_CHANNEL) return 0;
    const int64_t hd = (int64_t)d->num_heads * d->head_dim;
    const int64_t n = max_blocks_of(cap32) * hd * 8 + cap32 * 4 + hd * 32;
    return (n + 255) / 256 * 256;
}

size_t elt_bytes(int io_dtype) { return io_dtype == KVQ_BF16 ? 2 : 4; }

// Tensor arguments: 16-byte aligned base, strides that keep every (token, head) vector 16-byte aligned.
bool tensor_ok(const void *p, int64_t stride_token, int64_t stride_head, int head_dim, int io_dtype)
{
    if (!p) return false;
    if (reinterpret_cast<uintptr_t>(p) % 16 != 0) return false;
    const int64_t quantum = 16 / (int64_t)elt_bytes(io_dtype);
    if (stride_token < head_dim || stride_head < head_dim) return false;
    if (stride_token % quantum != 0 || stride_head % quantum != 0) return false;
    return true;
}

}  // namespace

extern "C" {

size_t kvq_cache_bytes(const kvq_cache_desc *desc)
{
    if (check_desc(desc) != KVQ_OK) return 0;
    const int64_t cap32 = round_up_tile(desc->capacity_tokens);
    const int64_t meta = desc->meta_format == KVQ_META_FP32 ? 8 : 3 * (desc->head_dim / desc->group_size);
    const int64_t per_token = desc->head_dim * desc->bits / 8 + meta;
    return (size_t)(2 * (int64_t)desc->num_heads * cap32 * per_token + channel_bytes(desc, cap32) + kvq::kStatusBytes);
}

kvq_status kvq_cache_create(const kvq_cache_desc *desc, void *dev_mem, size_t bytes, kvq_cache **out)
{
    if (!out) return KVQ_ERR_INVALID_ARG;
    *out = nullptr;
    const kvq_status st = check_desc(desc);
    if (st != KVQ_OK) return st;
    if (!dev_mem || reinterpret_cast<uintptr_t>(dev_mem) % 256 != 0) return KVQ_ERR_INVALID_ARG;
    if (bytes < kvq_cache_bytes(desc)) return KVQ_ERR_INVALID_ARG;
    kvq_cache *c = new (std::nothrow) kvq_cache;
    if (!c) return KVQ_ERR_INVALID_ARG;
    c->desc = *desc;
    c->cap32 = round_up_tile(desc->capacity_tokens);
    c->len = 0;
    c->base = 0;
    c->next_slot = 0;
    c->status_clean = false;
    const int64_t H = desc->num_heads;
    const int64_t code_bytes = H * c->cap32 * desc->head_dim * desc->bits / 8;  // multiple of 256
    const int64_t meta_bytes = H * c->cap32 * 4;                                // multiple of 128
    char *p = static_cast<char *>(dev_mem);
    kvq::CacheView &v = c->view;
    v.k_codes = reinterpret_cast<uint32_t *>(p); p += code_bytes;
    v.v_codes = reinterpret_cast<uint32_t *>(p); p += code_bytes;
    v.k_scale = v.k_negzero = v.v_scale = v.v_zero_off = nullptr;
    v.k_scale8 = v.v_scale8 = nullptr;
    v.k_zero16 = v.v_zero16 = nullptr;
    v.group_size = desc->group_size;
    v.meta_format = desc->meta_format;
    if (desc->meta_format == KVQ_META_FP32) {
        v.k_scale = reinterpret_cast<float *>(p); p += meta_bytes;
        v.k_negzero = reinterpret_cast<float *>(p); p += meta_bytes;
        v.v_scale = reinterpret_cast<float *>(p); p += meta_bytes;
        v.v_zero_off = reinterpret_cast<float *>(p);
    } else {
        const int64_t groups = H * c->cap32 * (desc->head_dim / desc->group_size);   // multiple of 32
        v.k_zero16 = reinterpret_cast<uint16_t *>(p); p += 2 * groups;
        v.v_zero16 = reinterpret_cast<uint16_t *>(p); p += 2 * groups;
        v.k_scale8 = reinterpret_cast<uint8_t *>(p); p += groups;
        v.v_scale8 = reinterpret_cast<uint8_t *>(p); p += groups;
    }
    v.key_axis = desc->key_axis;
    v.max_blocks = 0;
    v.kc_scale = v.kc_zero = nullptr;
    v.k_block = nullptr;
    v.kc_range = nullptr;
    v.kc_inv = v.kc_z = nullptr;
    if (desc->key_axis == KVQ_KEYS_PER_CHANNEL) {
        // p stands after the four fp32 arrays of KVQ_META_FP32: a multiple of 128 bytes from a 256-byte base
        p = static_cast<char *>(dev_mem) + 2 * code_bytes + 4 * meta_bytes;
        const int64_t hd = H * desc->head_dim;
        v.max_blocks = (int32_t)max_blocks_of(c->cap32);
        v.kc_range = reinterpret_cast<unsigned long long *>(p); p += hd * 16;   // 8-byte types first
        v.kc_inv = reinterpret_cast<double *>(p); p += hd * 8;
        v.kc_z = reinterpret_cast<double *>(p); p += hd * 8;
        v.kc_scale = reinterpret_cast<float *>(p); p += (int64_t)v.max_blocks * hd * 4;
        v.kc_zero = reinterpret_cast<float *>(p); p += (int64_t)v.max_blocks * hd * 4;
        v.k_block = reinterpret_cast<uint32_t *>(p);
    }
    // every part before it is a multiple of 128 bytes: the status block is 4-byte aligned (it holds 32-bit words)
    v.status = reinterpret_cast<uint32_t *>(static_cast<char *>(dev_mem) + kvq_cache_bytes(desc) - kvq::kStatusBytes);
    v.cap_tiles = c->cap32 / kvq::kTileTokens;
    v.num_heads = desc->num_heads;
    v.head_dim = desc->head_dim;
    v.bits = desc->bits;
    v.io_dtype = desc->io_dtype;
    for (uint32_t &w : v.sign_mask) w = 0u;
    *out = c;
    return KVQ_OK;
}

void kvq_cache_destroy(kvq_cache *cache) { delete cache; }

int64_t kvq_cache_len(const kvq_cache *cache) { return cache ? cache->len : -1; }

kvq_status kvq_cache_reset(kvq_cache *cache)
{
    if (!cache) return KVQ_ERR_INVALID_ARG;
    cache->len = 0;
    cache->base = 0;
    cache->blocks.clear();
    cache->status_clean = false;   // the next append clears the sticky flag before it writes
    return KVQ_OK;
}

kvq_status kvq_cache_set_rotation_signs(kvq_cache *cache, const uint8_t *negate)
{
    if (!cache) return KVQ_ERR_INVALID_ARG;
    if (cache->len != 0) return KVQ_ERR_INVALID_ARG;   // codes already stored belong to the old rotation
    for (uint32_t &w : cache->view.sign_mask) w = 0u;
    if (negate)
        for (int c = 0; c < cache->desc.head_dim; ++c)
            if (negate[c]) cache->view.sign_mask[c >> 5] |= 1u << (c & 31);
    return KVQ_OK;
}

kvq_status kvq_cache_evict(kvq_cache *cache, int64_t n_tokens)
{
    if (!cache || n_tokens < 0 || n_tokens > cache->len) return KVQ_ERR_INVALID_ARG;
    cache->base += n_tokens;
    cache->len -= n_tokens;
    if (cache->len == 0) cache->base = 0;   // an empty cache starts over at a tile boundary
    cache->trim_blocks();
    return KVQ_OK;
}

kvq_status kvq_cache_truncate(kvq_cache *cache, int64_t new_len)
{
    if (!cache || new_len < 0 || new_len > cache->len) return KVQ_ERR_INVALID_ARG;
    cache->len = new_len;
    cache->trim_blocks();
    return KVQ_OK;
}

static kvq_status quantize_append_common(kvq_cache *cache, const void *k, const void *v, int64_t n_tokens,
                                         int64_t stride_token, int64_t stride_head, void *hip_stream, bool static_scratch)
{
    if (!cache || n_tokens < 0) return KVQ_ERR_INVALID_ARG;
    if (static_scratch && (int64_t)cache->desc.num_heads * cache->desc.head_dim > kvq::kStaticScratchChannels)
        return KVQ_ERR_CAPACITY;
    if (n_tokens == 0) return KVQ_OK;
    const kvq_cache_desc &d = cache->desc;
    if (!tensor_ok(k, stride_token, stride_head, d.head_dim, d.io_dtype) ||
        !tensor_ok(v, stride_token, stride_head, d.head_dim, d.io_dtype))
        return KVQ_ERR_INVALID_ARG;
    if (n_tokens > d.capacity_tokens - cache->len) return KVQ_ERR_CAPACITY;
    // Ring storage: the tiles touched by the live tokens and the new ones must all be distinct.
    const int64_t first_tile = cache->base / kvq::kTileTokens;
    const int64_t last_tile = (cache->base + cache->len + n_tokens - 1) / kvq::kTileTokens;
    if (last_tile - first_tile + 1 > cache->view.cap_tiles) return KVQ_ERR_CAPACITY;
    int slot = 0;
    if (d.key_axis == KVQ_KEYS_PER_CHANNEL) {
        if ((int64_t)cache->blocks.size() >= cache->view.max_blocks) return KVQ_ERR_CAPACITY;
        slot = cache->next_slot;
    }
    if (!cache->status_clean) {
        if (kvq::launch_status_clear(cache->view, static_cast<hipStream_t>(hip_stream)) != hipSuccess) return KVQ_ERR_HIP;
        cache->status_clean = true;
    }
    const hipError_t e = kvq::launch_quantize_append(cache->view, k, v, cache->base + cache->len, n_tokens, stride_token,
                                                     stride_head, slot, static_cast<hipStream_t>(hip_stream), static_scratch);
    if (e != hipSuccess) return KVQ_ERR_HIP;
    if (d.key_axis == KVQ_KEYS_PER_CHANNEL) {
        cache->blocks.push_back(kvq_block{slot, cache->base + cache->len, n_tokens});
        cache->next_slot = (slot + 1) % cache->view.max_blocks;
    }
    cache->len += n_tokens;
    return KVQ_OK;
}

kvq_status kvq_quantize_append(kvq_cache *cache, const void *k, const void *v, int64_t n_tokens,
                               int64_t stride_token, int64_t stride_head, void *hip_stream)
{
    return quantize_append_common(cache, k, v, n_tokens, stride_token, stride_head, hip_stream, false);
}

kvq_status kvq_quantize_append_static(kvq_cache *cache, const void *k, const void *v, int64_t n_tokens,
                                      int64_t stride_token, int64_t stride_head, void *hip_stream)
{
    return quantize_append_common(cache, k, v, n_tokens, stride_token, stride_head, hip_stream, true);
}

static kvq_status attention_common(const kvq_cache *cache, int64_t cache_start, int64_t cache_len,
                                   const void *q, const void *k_cur, const void *v_cur, int64_t m,
                                   int64_t n_cur, int64_t stride_token, int64_t stride_head,
                                   float softmax_scale, int correction, void *out, float *mass_cached,
                                   void *hip_stream, bool force_vector, const kvq_attention_opts *opts = nullptr,
                                   const void *k_ref = nullptr, const void *v_ref = nullptr, float *diag = nullptr)
{
    // diag != nullptr: the diagnostics call (no out / mass_cached; k_ref, v_ref hold the cached tokens unquantized)
    kvq_attention_opts o = {1, 0, stride_token, stride_head};
    if (opts) {
        o = *opts;
        if (o.q_stride_token == 0 && o.q_stride_head == 0) {
            o.q_stride_token = stride_token;
            o.q_stride_head = stride_head;
        }
        if (o.q_heads_per_kv_head < 1 || o.q_heads_per_kv_head > 64) return KVQ_ERR_INVALID_ARG;
        if (o.causal != 0 && o.causal != 1) return KVQ_ERR_INVALID_ARG;
        if (o.causal && n_cur < m) return KVQ_ERR_INVALID_ARG;   // the queries are the last m current positions
    }
    if (!cache || m < 0 || n_cur < 0 || cache_len < 0 || cache_start < 0) return KVQ_ERR_INVALID_ARG;
    if (cache_start + cache_len > cache->len) return KVQ_ERR_INVALID_ARG;
    if (cache_len == 0 && n_cur == 0) return KVQ_ERR_INVALID_ARG;
    if (correction < 0 || correction > 2) return KVQ_ERR_INVALID_ARG;
    if (!(softmax_scale >= 0.0f) || !(softmax_scale < 3.0e38f)) return KVQ_ERR_INVALID_ARG;
    if (m == 0) return KVQ_OK;
    const kvq_cache_desc &d = cache->desc;
    if (!tensor_ok(q, o.q_stride_token, o.q_stride_head, d.head_dim, d.io_dtype)) return KVQ_ERR_INVALID_ARG;
    if (!diag && !tensor_ok(out, o.q_stride_token, o.q_stride_head, d.head_dim, d.io_dtype)) return KVQ_ERR_INVALID_ARG;
    if (diag && cache_len > 0 && (!tensor_ok(k_ref, stride_token, stride_head, d.head_dim, d.io_dtype) ||
                                  !tensor_ok(v_ref, stride_token, stride_head, d.head_dim, d.io_dtype)))
        return KVQ_ERR_INVALID_ARG;
    if (diag && reinterpret_cast<uintptr_t>(diag) % 4 != 0) return KVQ_ERR_INVALID_ARG;
    if (n_cur > 0 && (!tensor_ok(k_cur, stride_token, stride_head, d.head_dim, d.io_dtype) ||
                      !tensor_ok(v_cur, stride_token, stride_head, d.head_dim, d.io_dtype)))
        return KVQ_ERR_INVALID_ARG;
    if (mass_cached && reinterpret_cast<uintptr_t>(mass_cached) % 4 != 0) return KVQ_ERR_INVALID_ARG;
    if (!diag && (out == q || out == k_cur || out == v_cur)) return KVQ_ERR_INVALID_ARG;
    if (m > ((int64_t)1 << 31) - 256 || n_cur > ((int64_t)1 << 31) - 256) return KVQ_ERR_INVALID_ARG;

    kvq::AttentionArgs a;
    a.cv = cache->view;
    a.cache_start = cache->base + cache_start;
    a.cache_len = cache_len;
    a.phys_tile_first = (a.cache_start / kvq::kTileTokens) % cache->view.cap_tiles;
    a.q = q;
    a.k_cur = k_cur;
    a.v_cur = v_cur;
    a.m = m;
    a.n_cur = n_cur;
    a.stride_token = stride_token;
    a.stride_head = stride_head;
    a.q_stride_token = o.q_stride_token;
    a.q_stride_head = o.q_stride_head;
    a.q_per_kv = o.q_heads_per_kv_head;
    a.causal = o.causal;
    a.softmax_scale = softmax_scale > 0.0f ? softmax_scale : (d.head_dim == 64 ? 0.125f : 0.088388347648318f);
    a.correction = correction;
    a.out = out;
    a.mass_cached = mass_cached;
    a.n_key_blocks = 0;
    a.status = cache->status_clean && cache_len > 0 ? cache->view.status : nullptr;
    a.only_if_flagged = 0;
    // the exact (sinh) correction is a diagnostic mode: vector kernel only
    force_vector = force_vector || correction == 2;
    if (d.key_axis == KVQ_KEYS_PER_CHANNEL && !force_vector) {
        // The matrix-core kernel walks the window block by block: list the appended blocks it overlaps.  A window
        // without cached keys or with more blocks than the list holds goes to the vector kernel.
        const int64_t w0 = a.cache_start, w1 = a.cache_start + cache_len;
        int nb = 0;
        bool fits = cache_len > 0;
        for (const kvq_block &b : cache->blocks) {
            const int64_t s0 = b.start > w0 ? b.start : w0, s1 = b.start + b.count < w1 ? b.start + b.count : w1;
            if (s0 >= s1) continue;
            if (nb == kvq::kMaxKeyBlocks) { fits = false; break; }
            a.key_blocks[nb++] = kvq::KeyBlock{(int32_t)b.slot, (int32_t)(s0 - w0), (int32_t)(s1 - w0)};
        }
        a.n_key_blocks = nb;
        force_vector = !fits || nb == 0;
    }
    // (the matrix-core loaders do their ring arithmetic and their offsets inside a head in 32 bits)
    force_vector = force_vector || cache_len >= (int64_t(1) << 31) || cache->view.cap_tiles >= (int64_t(1) << 20);
    const bool matrix_path = !force_vector && d.io_dtype == KVQ_BF16 && d.head_dim == 128 &&
                             d.group_size == d.head_dim;   // one (scale, zero-point) per token, either format
    const hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (diag) return kvq::launch_diagnostics_simt(a, k_ref, v_ref, diag, s) == hipSuccess ? KVQ_OK : KVQ_ERR_HIP;
    const bool group_matrix_path = !force_vector && kvq::attention_mfma_group_supported(cache->view);
    hipError_t e = matrix_path         ? kvq::launch_attention_mfma(a, s)
                   : group_matrix_path ? kvq::launch_attention_mfma_group(a, s)
                                       : kvq::launch_attention_simt(a, s);
    if (e == hipSuccess && (matrix_path || group_matrix_path) && a.status) {
        // A cache that has ever stored a zero-point beyond the matrix-core kernels' domain carries a flag: the launch
        // above has then returned without writing anything, and this one, which otherwise returns at once, does the work.
        a.only_if_flagged = 1;
        e = kvq::launch_attention_simt(a, s);
    }
    return e == hipSuccess ? KVQ_OK : KVQ_ERR_HIP;
}

kvq_status kvq_chunk_attention(const kvq_cache *cache, int64_t cache_start, int64_t cache_len,
                               const void *q, const void *k_cur, const void *v_cur, int64_t m,
                               int64_t n_cur, int64_t stride_token, int64_t stride_head,
                               float softmax_scale, int correction, void *out, float *mass_cached,
                               void *hip_stream)
{
    return attention_common(cache, cache_start, cache_len, q, k_cur, v_cur, m, n_cur, stride_token, stride_head,
                            softmax_scale, correction, out, mass_cached, hip_stream, false);
}

kvq_status kvq_chunk_attention_fp32(const kvq_cache *cache, int64_t cache_start, int64_t cache_len,
                                    const void *q, const void *k_cur, const void *v_cur, int64_t m,
                                    int64_t n_cur, int64_t stride_token, int64_t stride_head,
                                    float softmax_scale, int correction, void *out, float *mass_cached,
                                    void *hip_stream)
{
    return attention_common(cache, cache_start, cache_len, q, k_cur, v_cur, m, n_cur, stride_token, stride_head,
                            softmax_scale, correction, out, mass_cached, hip_stream, true);
}

kvq_status kvq_chunk_attention_ex(const kvq_cache *cache, int64_t cache_start, int64_t cache_len,
                                  const void *q, const void *k_cur, const void *v_cur, int64_t m,
                                  int64_t n_cur, int64_t stride_token, int64_t stride_head,
                                  float softmax_scale, int correction, const kvq_attention_opts *opts,
                                  void *out, float *mass_cached, void *hip_stream)
{
    return attention_common(cache, cache_start, cache_len, q, k_cur, v_cur, m, n_cur, stride_token, stride_head,
                            softmax_scale, correction, out, mass_cached, hip_stream, false, opts);
}

kvq_status kvq_attention_diagnostics(const kvq_cache *cache, int64_t cache_start, int64_t cache_len, const void *q,
                                     const void *k_ref, const void *v_ref, const void *k_cur, const void *v_cur,
                                     int64_t m, int64_t n_cur, int64_t stride_token, int64_t stride_head,
                                     float softmax_scale, int correction, float *diag, void *hip_stream)
{
    if (!diag) return KVQ_ERR_INVALID_ARG;
    return attention_common(cache, cache_start, cache_len, q, k_cur, v_cur, m, n_cur, stride_token, stride_head,
                            softmax_scale, correction, nullptr, nullptr, hip_stream, true, nullptr, k_ref, v_ref, diag);
}

kvq_status kvq_cache_export(const kvq_cache *cache, int which, int64_t start, int64_t count, uint8_t *codes,
                            float *scales, float *zeros, void *hip_stream)
{
    if (!cache || (which != 0 && which != 1) || start < 0 || count < 0) return KVQ_ERR_INVALID_ARG;
    if (start + count > cache->len) return KVQ_ERR_INVALID_ARG;
    if (count == 0) return KVQ_OK;
    const hipError_t e = kvq::launch_export(cache->view, which, cache->base + start, count, codes, scales, zeros,
                                            static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? KVQ_OK : KVQ_ERR_HIP;
}

const char *kvq_status_string(kvq_status status)
{
    switch (status) {
        case KVQ_OK: return "ok";
        case KVQ_ERR_INVALID_ARG: return "invalid argument";
        case KVQ_ERR_UNSUPPORTED: return "unsupported configuration";
        case KVQ_ERR_CAPACITY: return "cache capacity exceeded";
        case KVQ_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

const char *kvq_version(void) { return "0.2"; }

}  // extern "C"
