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

template <int D, int BITS, typename T>
__global__ __launch_bounds__(D) void attention_simt_kernel(AttentionArgs a)
{
    constexpr int WPL = D * BITS / 64;
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    __shared__ float q_rot[D];   // Hn q
    __shared__ float q_raw[D];
    __shared__ float p_blk[D];
    __shared__ float scratch[D];
    __shared__ float corr_g[4];  // softmax_scale^2 / 24 * nu_j per group (at most 4 groups)
    const CacheView &cv = a.cv;
    const int c = threadIdx.x;
    const int qhead = blockIdx.y;               // query head
    const int head = qhead / a.q_per_kv;        // key/value head
    const int64_t row = blockIdx.x;
    // current keys this row sees (all of them, or under the causal mask those up to its own position)
    int64_t n_vis = a.n_cur;
    if (a.causal) {
        const int64_t upto = row + (a.n_cur - a.m) + 1;
        n_vis = upto < n_vis ? upto : n_vis;
        n_vis = n_vis < 0 ? 0 : n_vis;
    }
    const float norm = D == 64 ? 0.125f : 0.088388347648318f;
    const float sigma = a.softmax_scale;
    const float off = code_offset(BITS);

    const T *qp = static_cast<const T *>(a.q) + row * a.q_stride_token + (int64_t)qhead * a.q_stride_head;
    const float qc = Io<T>::load(qp + c);
    q_raw[c] = qc;
    const uint32_t sign_c = sign_bits_from(cv, c);   // randomised rotation x -> Hn (s * x): bit 0 set means s_c = -1
    q_rot[c] = flip_sign(qc, sign_c);
    fwht_lds<D>(q_rot, c);
    q_rot[c] *= norm;
    const bool fp8_meta = cv.meta_format == KVQ_META_FP8_BF16;
    const int group = fp8_meta ? cv.group_size : D;
    const int G = D / group;
    {
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
    }

    const int64_t meta0 = (int64_t)head * cv.cap_tiles * kTileTokens;
    const uint32_t *k_head = cv.k_codes + (int64_t)head * cv.cap_tiles * tile_words(D, BITS);
    const uint32_t *v_head = cv.v_codes + (int64_t)head * cv.cap_tiles * tile_words(D, BITS);

    const int64_t cap_tokens = cv.cap_tiles * kTileTokens;
    auto cached_score = [&](int64_t t_logical) -> float {
        const int64_t t = t_logical % cap_tokens;   // position in the ring
        const uint32_t *tile = k_head + (t / kTileTokens) * tile_words(D, BITS);
        const int tt = (int)(t % kTileTokens);
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
    };
    auto current_score = [&](int64_t j) -> float {
        const T *kp = static_cast<const T *>(a.k_cur) + j * a.stride_token + (int64_t)head * a.stride_head;
        float dot = 0.0f;
        for (int ch = 0; ch < D; ++ch) dot = fmaf(q_raw[ch], Io<T>::load(kp + ch), dot);
        return sigma * dot;
    };

    // Pass 1: row maximum.
    float mx = -INFINITY;
    for (int64_t i = c; i < a.cache_len; i += D) mx = fmaxf(mx, cached_score(a.cache_start + i));
    for (int64_t j = c; j < n_vis; j += D) mx = fmaxf(mx, current_score(j));
    mx = block_reduce<D>(mx, scratch, c, true);

    // Pass 2: weights and weighted sums.
    float sum_s = 0.0f, sum_r = 0.0f, acc = 0.0f;
    for (int64_t base = 0; base < a.cache_len; base += D) {
        const int64_t i = base + c;
        const float p = i < a.cache_len ? expf(cached_score(a.cache_start + i) - mx) : 0.0f;
        sum_s += p;
        __syncthreads();
        p_blk[c] = p;
        __syncthreads();
        const int cnt = (int)((a.cache_len - base) < D ? (a.cache_len - base) : D);
        for (int jj = 0; jj < cnt; ++jj) {
            const int64_t t = (a.cache_start + base + jj) % cap_tokens;
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
            acc = fmaf(p_blk[jj], (code - vz) * vs, acc);
        }
    }
    // Rotate the cached part back: out_S = Hn^T acc (Hn symmetric).
    __syncthreads();
    scratch[c] = acc;
    fwht_lds<D>(scratch, c);
    acc = flip_sign(scratch[c] * norm, sign_c);
    __syncthreads();
    for (int64_t base = 0; base < n_vis; base += D) {
        const int64_t j = base + c;
        const float p = j < n_vis ? expf(current_score(j) - mx) : 0.0f;
        sum_r += p;
        __syncthreads();
        p_blk[c] = p;
        __syncthreads();
        const int cnt = (int)((n_vis - base) < D ? (n_vis - base) : D);
        for (int jj = 0; jj < cnt; ++jj) {
            const T *vp = static_cast<const T *>(a.v_cur) + (base + jj) * a.stride_token + (int64_t)head * a.stride_head;
            acc = fmaf(p_blk[jj], Io<T>::load(vp + c), acc);
        }
    }
    sum_s = block_reduce<D>(sum_s, scratch, c, false);
    sum_r = block_reduce<D>(sum_r, scratch, c, false);
    const float inv = 1.0f / (sum_s + sum_r);
    T *op = static_cast<T *>(a.out) + row * a.q_stride_token + (int64_t)qhead * a.q_stride_head;
    Io<T>::store(op + c, acc * inv);
    if (a.mass_cached && c == 0) a.mass_cached[(int64_t)qhead * a.m + row] = sum_s * inv;
}

}  // namespace

hipError_t launch_attention_simt(const AttentionArgs &a, hipStream_t stream)
{
    const dim3 grid((unsigned)a.m, (unsigned)(a.cv.num_heads * a.q_per_kv));
    const bool bf16 = a.cv.io_dtype == KVQ_BF16;
#define KVQ_A(D, B)                                                                                         \
    if (a.cv.head_dim == D && a.cv.bits == B) {                                                             \
        if (bf16) hipLaunchKernelGGL((attention_simt_kernel<D, B, uint16_t>), grid, dim3(D), 0, stream, a); \
        else hipLaunchKernelGGL((attention_simt_kernel<D, B, float>), grid, dim3(D), 0, stream, a);         \
        return hipGetLastError();                                                                           \
    }
    KVQ_A(128, 2)
    KVQ_A(128, 4)
    KVQ_A(64, 2)
    KVQ_A(64, 4)
#undef KVQ_A
    return hipErrorInvalidValue;
}

}  // namespace kvq
