// fp32 vector-ALU chunk attention: the reference-precision GPU path.
//
// Used for KVQ_FP32 caches, for head_dim 64, and by kvq_chunk_attention_fp32.  It follows
// Alg. 1 of the paper literally in single precision, one workgroup of d threads per
// (head, query row):
//   * rotate the query (butterflies in LDS), nu_j = ||(Hn q)_j||^2 per group of channels that shares a
//     (scale, zero-point) (one group = the whole vector for per-token quantization);
//   * pass 1: every thread scores a strided subset of the keys (cached keys from their packed
//     codes, corrected by b = scale^2 / 24 * sum_j step_j^2 nu_j; current keys from k_cur) to find
//     the row maximum;
//   * pass 2: scores again, p = exp(s - max); blocks of d weights go through LDS so that thread c
//     accumulates output channel c; the cached part is accumulated in the rotated basis and
//     rotated back before the current part is added.
// Throughput is a few TFLOP/s at best; the matrix-core kernel is the fast path.
// The same file holds the diagnostics kernel (quantized against unquantized attention per row).
#include "kvq_internal.h"

namespace kvq {
namespace {

template <int D> __device__ inline void fwht_lds(float *buf, int c)
{
    // In-place Sylvester-Hadamard transform of buf[0..D) by D threads; unnormalised.
#pragma unroll
    for (int h = 1; h < D; h <<= 1) {
        __syncthreads();
        const float a = buf[c & ~h], b = buf[c | h];
        __syncthreads();
        buf[c] = (c & h) ? a - b : a + b;
    }
    __syncthreads();
}

template <int D> __device__ inline float block_reduce(float v, float *scratch, int c, bool is_max)
{
    __syncthreads();
    scratch[c] = v;
    __syncthreads();
    for (int s = D / 2; s > 0; s >>= 1) {
        if (c < s) scratch[c] = is_max ? fmaxf(scratch[c], scratch[c + s]) : scratch[c] + scratch[c + s];
        __syncthreads();
    }
    const float r = scratch[0];
    __syncthreads();
    return r;
}

// log(sinh(x)/x), the log moment of uniform noise on one channel (Eq. 12 of the paper): a series where
// the closed form would cancel, the overflow-free closed form elsewhere.
__device__ inline float log_sinhc(float x)
{
    x = fabsf(x);
    if (x < 0.5f) {
        const float x2 = x * x;
        return x2 * (1.0f / 6.0f + x2 * (-1.0f / 180.0f + x2 * (1.0f / 2835.0f + x2 * (-1.0f / 37800.0f + x2 * (1.0f / 467775.0f)))));
    }
    return x + log1pf(-expf(-2.0f * x)) - logf(2.0f * x);
}

// State of one (query head, query row) workgroup that both kernels below share: the rotated query, the
// per-group correction factors and the decoders of cached keys and values.
template <int D, int BITS, typename T> struct SimtRow {
    static constexpr int WPL = D * BITS / 64;
    static constexpr uint32_t MASK = (1u << BITS) - 1u;
    const AttentionArgs &a;
    const float *q_rot, *q_raw, *corr_g;   // LDS: Hn (s * q); q; softmax_scale^2 / 24 * nu_j per group
    int head, group, G;
    bool fp8_meta;
    float sigma, off;
    int64_t meta0, cap_tokens;
    const uint32_t *k_head, *v_head;

    // sigma q~ . k^_t - b for the cached key at logical position t_logical
    __device__ float cached_score(int64_t t_logical) const
    {
        const CacheView &cv = a.cv;
        const int64_t t = t_logical % cap_tokens;   // position in the ring
        const uint32_t *tile = k_head + (t / kTileTokens) * tile_words(D, BITS);
        const int tt = (int)(t % kTileTokens);
        if (cv.key_axis == KVQ_KEYS_PER_CHANNEL) {
            // One (scale, zero-point) per channel, shared by the tokens of the key's block (appendix on
            // per-channel quantization): b = sigma^2/24 sum_c q~_c^2 step_c^2 is the same for every key of
            // the block; it is summed here next to the dot product, channel by channel.
            const int64_t slot = cv.k_block[t];
            const float *sc = cv.kc_scale + (slot * cv.num_heads + head) * D;
            const float *zc = cv.kc_zero + (slot * cv.num_heads + head) * D;
            const float cs = a.correction == 1 ? sigma * sigma * (1.0f / 24.0f) : 0.0f;
            float dot = 0.0f, b = 0.0f;
            for (int hh = 0; hh < 2; ++hh) {
                const uint32_t *slot_w = tile + (hh * 32 + tt) * WPL;
                for (int w = 0; w < WPL; ++w) {
                    const uint32_t word = slot_w[w];
                    for (int j = 0; j < 16 / BITS; ++j) {
                        const int slab = BITS == 2 ? 2 * w + (j >> 2) : w;
                        const int ch = 16 * slab + 8 * hh + 2 * (j & 3);
                        for (int e = 0; e < 2; ++e) {
                            const float code = (float)((word >> (BITS * j + 16 * e)) & MASK);
                            const float step = sc[ch + e], qs = q_rot[ch + e] * step;
                            dot = fmaf(qs, code - zc[ch + e], dot);
                            b = fmaf(cs * qs, qs, b);
                            if (a.correction == 2) b += log_sinhc(0.5f * sigma * qs);
                        }
                    }
                }
            }
            return sigma * dot - b;
        }
        float scale_g[4], zero_g[4], b = 0.0f;
        for (int g = 0; g < G; ++g) {
            if (fp8_meta) {
                scale_g[g] = e4m3_to_float(cv.k_scale8[(meta0 + t) * G + g]);
                zero_g[g] = bf16_to_float(cv.k_zero16[(meta0 + t) * G + g]);
            } else {
                scale_g[g] = cv.k_scale[meta0 + t];
                zero_g[g] = -cv.k_negzero[meta0 + t] - off;
            }
            b += corr_g[g] * scale_g[g] * scale_g[g];
        }
        float dot = 0.0f;
        for (int hh = 0; hh < 2; ++hh) {
            const uint32_t *slot = tile + (hh * 32 + tt) * WPL;
            for (int w = 0; w < WPL; ++w) {
                const uint32_t word = slot[w];
                for (int j = 0; j < 16 / BITS; ++j) {
                    const int slab = BITS == 2 ? 2 * w + (j >> 2) : w;
                    const int ch = 16 * slab + 8 * hh + 2 * (j & 3);
                    const float c0 = (float)((word >> (BITS * j)) & MASK);
                    const float c1 = (float)((word >> (BITS * j + 16)) & MASK);
                    const float scale = scale_g[ch / group], zero = zero_g[ch / group];   // ch, ch + 1: same group
                    dot = fmaf(q_rot[ch], (c0 - zero) * scale, dot);
                    dot = fmaf(q_rot[ch + 1], (c1 - zero) * scale, dot);
                    if (a.correction == 2)   // exact form: sum over channels of log(sinh a / a), a = sigma q~_c step / 2
                        b += log_sinhc(0.5f * sigma * q_rot[ch] * scale) + log_sinhc(0.5f * sigma * q_rot[ch + 1] * scale);
                }
            }
        }
        return sigma * dot - b;
    }
    // sigma q . k for row j of an unquantized [token][head][channel] tensor (the current keys, or the
    // cached keys before quantization)
    __device__ float plain_score(const void *k, int64_t j) const
    {
        const T *kp = static_cast<const T *>(k) + j * a.stride_token + (int64_t)head * a.stride_head;
        float dot = 0.0f;
        for (int ch = 0; ch < D; ++ch) dot = fmaf(q_raw[ch], Io<T>::load(kp + ch), dot);
        return sigma * dot;
    }
    // channel c (rotated basis) of the dequantized cached value at logical position t_logical
    __device__ float cached_value(int64_t t_logical, int c) const
    {
        const CacheView &cv = a.cv;
        const int64_t t = t_logical % cap_tokens;
        int word, shift;
        value_code_pos(D, BITS, (int)(t % kTileTokens), c, word, shift);
        const uint32_t w = v_head[(t / kTileTokens) * tile_words(D, BITS) + word];
        const float code = (float)((w >> shift) & MASK);
        float vz, vs;
        if (fp8_meta) {
            const int64_t gi = (meta0 + t) * G + c / group;
            vs = e4m3_to_float(cv.v_scale8[gi]);
            vz = bf16_to_float(cv.v_zero16[gi]);
        } else {
            vs = cv.v_scale[meta0 + t];
            vz = cv.v_zero_off[meta0 + t] - off;
        }
        return (code - vz) * vs;
    }
    __device__ float plain_value(const void *v, int64_t j, int c) const
    {
        return Io<T>::load(static_cast<const T *>(v) + j * a.stride_token + (int64_t)head * a.stride_head + c);
    }
};

// Loads and rotates the query of (qhead, row) into q_raw / q_rot, fills corr_g, and returns the row state.
// All D threads of the workgroup call it.
template <int D, int BITS, typename T>
__device__ inline SimtRow<D, BITS, T> prepare_row(const AttentionArgs &a, int qhead, int64_t row, float *q_rot,
                                                  float *q_raw, float *corr_g, float *scratch, uint32_t &sign_c)
{
    const CacheView &cv = a.cv;
    const int c = threadIdx.x;
    const int head = qhead / a.q_per_kv;        // key/value head
    const float norm = D == 64 ? 0.125f : 0.088388347648318f;
    const float sigma = a.softmax_scale;
    const T *qp = static_cast<const T *>(a.q) + row * a.q_stride_token + (int64_t)qhead * a.q_stride_head;
    const float qc = Io<T>::load(qp + c);
    q_raw[c] = qc;
    sign_c = sign_bits_from(cv, c);   // randomised rotation x -> Hn (s * x): bit 0 set means s_c = -1
    q_rot[c] = flip_sign(qc, sign_c);
    fwht_lds<D>(q_rot, c);
    q_rot[c] *= norm;
    const bool fp8_meta = cv.meta_format == KVQ_META_FP8_BF16;
    const int group = fp8_meta ? cv.group_size : D;
    const int G = D / group;
    // per-group squared norms of the rotated query (Appendix "Extension to QuaRot"); with one group
    // this is ||q||^2
    __syncthreads();
    scratch[c] = q_rot[c] * q_rot[c];
    __syncthreads();
    if (c < G) {
        float nu = 0.0f;
        for (int i = 0; i < group; ++i) nu += scratch[c * group + i];
        corr_g[c] = a.correction == 1 ? sigma * sigma * nu * (1.0f / 24.0f) : 0.0f;
    }
    __syncthreads();
    SimtRow<D, BITS, T> r{a, q_rot, q_raw, corr_g, head, group, G, fp8_meta, sigma, code_offset(BITS),
                          (int64_t)head * cv.cap_tiles * kTileTokens, cv.cap_tiles * kTileTokens,
                          cv.k_codes + (int64_t)head * cv.cap_tiles * tile_words(D, BITS),
                          cv.v_codes + (int64_t)head * cv.cap_tiles * tile_words(D, BITS)};
    return r;
}

template <int D, int BITS, typename T>
__global__ __launch_bounds__(D) void attention_simt_kernel(AttentionArgs a)
{
    __shared__ float q_rot[D];   // Hn q
    __shared__ float q_raw[D];
    __shared__ float p_blk[D];
    __shared__ float scratch[D];
    __shared__ float corr_g[4];  // softmax_scale^2 / 24 * nu_j per group (at most 4 groups)
    // Enqueued behind a matrix-core launch: there is work only if that launch has stood back (flagged cache).
    if (a.only_if_flagged && !cache_flagged(a.status)) return;
    const int c = threadIdx.x;
    const int qhead = blockIdx.y;               // query head
    // One row per workgroup in an ordinary launch (gridDim.x = m); the gated launch behind a matrix-core kernel
    // has fewer workgroups, which walk the rows (its usual fate is to return above, and a small grid does that
    // in a few microseconds where one workgroup per row took 40 at 200 000 rows).
    for (int64_t row = blockIdx.x; row < a.m; row += gridDim.x) {
    __syncthreads();   // the previous row's shared arrays are no longer read
    // current keys this row sees (all of them, or under the causal mask those up to its own position)
    int64_t n_vis = a.n_cur;
    if (a.causal) {
        const int64_t upto = row + (a.n_cur - a.m) + 1;
        n_vis = upto < n_vis ? upto : n_vis;
        n_vis = n_vis < 0 ? 0 : n_vis;
    }
    const float norm = D == 64 ? 0.125f : 0.088388347648318f;
    uint32_t sign_c;
    const SimtRow<D, BITS, T> r = prepare_row<D, BITS, T>(a, qhead, row, q_rot, q_raw, corr_g, scratch, sign_c);

    // Pass 1: row maximum.
    float mx = -INFINITY;
    for (int64_t i = c; i < a.cache_len; i += D) mx = fmaxf(mx, r.cached_score(a.cache_start + i));
    for (int64_t j = c; j < n_vis; j += D) mx = fmaxf(mx, r.plain_score(a.k_cur, j));
    mx = block_reduce<D>(mx, scratch, c, true);

    // Pass 2: weights and weighted sums.
    float sum_s = 0.0f, sum_r = 0.0f, acc = 0.0f;
    for (int64_t base = 0; base < a.cache_len; base += D) {
        const int64_t i = base + c;
        const float p = i < a.cache_len ? expf(r.cached_score(a.cache_start + i) - mx) : 0.0f;
        sum_s += p;
        __syncthreads();
        p_blk[c] = p;
        __syncthreads();
        const int cnt = (int)((a.cache_len - base) < D ? (a.cache_len - base) : D);
        for (int jj = 0; jj < cnt; ++jj) acc = fmaf(p_blk[jj], r.cached_value(a.cache_start + base + jj, c), acc);
    }
    // Rotate the cached part back: out_S = Hn^T acc (Hn symmetric).
    __syncthreads();
    scratch[c] = acc;
    fwht_lds<D>(scratch, c);
    acc = flip_sign(scratch[c] * norm, sign_c);
    __syncthreads();
    for (int64_t base = 0; base < n_vis; base += D) {
        const int64_t j = base + c;
        const float p = j < n_vis ? expf(r.plain_score(a.k_cur, j) - mx) : 0.0f;
        sum_r += p;
        __syncthreads();
        p_blk[c] = p;
        __syncthreads();
        const int cnt = (int)((n_vis - base) < D ? (n_vis - base) : D);
        for (int jj = 0; jj < cnt; ++jj) acc = fmaf(p_blk[jj], r.plain_value(a.v_cur, base + jj, c), acc);
    }
    sum_s = block_reduce<D>(sum_s, scratch, c, false);
    sum_r = block_reduce<D>(sum_r, scratch, c, false);
    const float inv = 1.0f / (sum_s + sum_r);
    T *op = static_cast<T *>(a.out) + row * a.q_stride_token + (int64_t)qhead * a.q_stride_head;
    Io<T>::store(op + c, acc * inv);
    if (a.mass_cached && c == 0) a.mass_cached[(int64_t)qhead * a.m + row] = sum_s * inv;
    }
}

// Attention-level diagnostics (attention stealing; appendices on the Jensen-Shannon divergence of the
// attention weights and on the output MSE): the quantized, optionally corrected attention of one row
// against attention over the unquantized cached keys / values k_ref, v_ref, on the same queries and current
// block.  Per (head, row) it writes
//   [0] P_S of the unquantized cache   [1] P_S of the quantized cache
//   [2] JSD(p, p^) in nats over all keys   [3] mean over channels of (o^ - o)^2.
// Pass 1 finds maximum and partition sum of both score rows (online, then combined over the
// workgroup); pass 2 scores again with the normalisers known and accumulates everything else.
template <int D, int BITS, typename T>
__global__ __launch_bounds__(D) void diagnostics_simt_kernel(AttentionArgs a, const void *k_ref, const void *v_ref,
                                                             float *diag)
{
    __shared__ float q_rot[D];
    __shared__ float q_raw[D];
    __shared__ float pq_blk[D];   // weights of the quantized side
    __shared__ float pr_blk[D];   // weights of the unquantized side
    __shared__ float scratch[D];
    __shared__ float corr_g[4];
    const int c = threadIdx.x;
    const int head = blockIdx.y;
    const int64_t row = blockIdx.x;
    const float norm = D == 64 ? 0.125f : 0.088388347648318f;
    uint32_t sign_c;
    const SimtRow<D, BITS, T> r = prepare_row<D, BITS, T>(a, head, row, q_rot, q_raw, corr_g, scratch, sign_c);

    // Pass 1.
    float mq = -INFINITY, zq = 0.0f, mr = -INFINITY, zr = 0.0f;
    auto online = [](float s, float &mx, float &z) {
        const float top = fmaxf(mx, s);
        z = z * expf(mx - top) + expf(s - top);   // first key: z = 0, expf(-inf) = 0
        mx = top;
    };
    for (int64_t i = c; i < a.cache_len; i += D) {
        online(r.cached_score(a.cache_start + i), mq, zq);
        online(r.plain_score(k_ref, i), mr, zr);
    }
    for (int64_t j = c; j < a.n_cur; j += D) {
        const float s = r.plain_score(a.k_cur, j);
        online(s, mq, zq);
        online(s, mr, zr);
    }
    const float top_q = block_reduce<D>(mq, scratch, c, true);
    const float top_r = block_reduce<D>(mr, scratch, c, true);
    const float inv_q = 1.0f / block_reduce<D>(zq > 0.0f ? zq * expf(mq - top_q) : 0.0f, scratch, c, false);
    const float inv_r = 1.0f / block_reduce<D>(zr > 0.0f ? zr * expf(mr - top_r) : 0.0f, scratch, c, false);

    // One key's share of the divergence: with x = (p^ - p) / (p^ + p) the two ratios to the mixture are
    // 1 - x and 1 + x, and log1p keeps the nearly cancelling pair accurate.
    auto jsd_term = [](float p, float ph) -> float {
        const float s = p + ph;
        if (!(s > 0.0f)) return 0.0f;
        const float x = (ph - p) / s;
        float t = 0.0f;
        if (x < 1.0f) t += (1.0f - x) * log1pf(-x);
        if (x > -1.0f) t += (1.0f + x) * log1pf(x);
        return 0.25f * s * t;
    };

    // Pass 2.
    float ps_q = 0.0f, ps_r = 0.0f, jsd = 0.0f, acc_q = 0.0f, acc_r = 0.0f;
    for (int64_t base = 0; base < a.cache_len; base += D) {
        const int64_t i = base + c;
        float pq = 0.0f, pr = 0.0f;
        if (i < a.cache_len) {
            pq = expf(r.cached_score(a.cache_start + i) - top_q) * inv_q;
            pr = expf(r.plain_score(k_ref, i) - top_r) * inv_r;
        }
        ps_q += pq;
        ps_r += pr;
        jsd += jsd_term(pr, pq);
        __syncthreads();
        pq_blk[c] = pq;
        pr_blk[c] = pr;
        __syncthreads();
        const int cnt = (int)((a.cache_len - base) < D ? (a.cache_len - base) : D);
        for (int jj = 0; jj < cnt; ++jj) {
            acc_q = fmaf(pq_blk[jj], r.cached_value(a.cache_start + base + jj, c), acc_q);
            acc_r = fmaf(pr_blk[jj], r.plain_value(v_ref, base + jj, c), acc_r);
        }
    }
    __syncthreads();
    scratch[c] = acc_q;
    fwht_lds<D>(scratch, c);
    acc_q = flip_sign(scratch[c] * norm, sign_c);
    __syncthreads();
    for (int64_t base = 0; base < a.n_cur; base += D) {
        const int64_t j = base + c;
        float pq = 0.0f, pr = 0.0f;
        if (j < a.n_cur) {
            const float s = r.plain_score(a.k_cur, j);
            pq = expf(s - top_q) * inv_q;
            pr = expf(s - top_r) * inv_r;
        }
        jsd += jsd_term(pr, pq);
        __syncthreads();
        pq_blk[c] = pq;
        pr_blk[c] = pr;
        __syncthreads();
        const int cnt = (int)((a.n_cur - base) < D ? (a.n_cur - base) : D);
        for (int jj = 0; jj < cnt; ++jj) {
            const float v = r.plain_value(a.v_cur, base + jj, c);
            acc_q = fmaf(pq_blk[jj], v, acc_q);
            acc_r = fmaf(pr_blk[jj], v, acc_r);
        }
    }
    ps_q = block_reduce<D>(ps_q, scratch, c, false);
    ps_r = block_reduce<D>(ps_r, scratch, c, false);
    jsd = block_reduce<D>(jsd, scratch, c, false);
    const float mse = block_reduce<D>((acc_q - acc_r) * (acc_q - acc_r), scratch, c, false) * (1.0f / D);
    if (c == 0) {
        float *dst = diag + ((int64_t)head * a.m + row) * 4;
        dst[0] = ps_r;
        dst[1] = ps_q;
        dst[2] = jsd;
        dst[3] = mse;
    }
}

}  // namespace

hipError_t launch_attention_simt(const AttentionArgs &a, hipStream_t stream)
{
    const dim3 grid((unsigned)(a.only_if_flagged && a.m > 256 ? 256 : a.m), (unsigned)(a.cv.num_heads * a.q_per_kv));
    const bool bf16 = a.cv.io_dtype == KVQ_BF16;
#define KVQ_A(D, B)                                                                                         \
    if (a.cv.head_dim == D && a.cv.bits == B) {                                                             \
        if (bf16) return launch_kernel(attention_simt_kernel<D, B, uint16_t>, grid, dim3(D), 0, stream, a);  \
        return launch_kernel(attention_simt_kernel<D, B, float>, grid, dim3(D), 0, stream, a);               \
    }
    KVQ_A(128, 2)
    KVQ_A(128, 4)
    KVQ_A(64, 2)
    KVQ_A(64, 4)
#undef KVQ_A
    return hipErrorInvalidValue;
}

hipError_t launch_diagnostics_simt(const AttentionArgs &a, const void *k_ref, const void *v_ref, float *diag,
                                   hipStream_t stream)
{
    const dim3 grid((unsigned)a.m, (unsigned)a.cv.num_heads);
    const bool bf16 = a.cv.io_dtype == KVQ_BF16;
#define KVQ_A(D, B)                                                                                           \
    if (a.cv.head_dim == D && a.cv.bits == B) {                                                               \
        if (bf16)                                                                                             \
            return launch_kernel(diagnostics_simt_kernel<D, B, uint16_t>, grid, dim3(D), 0, stream, a, k_ref, v_ref, diag); \
        return launch_kernel(diagnostics_simt_kernel<D, B, float>, grid, dim3(D), 0, stream, a, k_ref, v_ref, diag);        \
    }
    KVQ_A(128, 2)
    KVQ_A(128, 4)
    KVQ_A(64, 2)
    KVQ_A(64, 4)
#undef KVQ_A
    return hipErrorInvalidValue;
}

}  // namespace kvq
