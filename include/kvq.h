/*
 * kvq.h -- C ABI of the quantized-KV chunk-attention library for AMD MI355X (gfx950).
 *
 * The library implements one hot path of "Quantized Keys Steal Attention: Bias
 * Correction for KV-Cache Compression in Video Diffusion":
 *
 *   kvq_quantize_append   rotate (Hadamard), quantize (asymmetric round-to-nearest,
 *                         per token or per group of channels of a token) and bit-pack
 *                         one chunk's keys and values into the cache
 *                         [Preliminaries: Eq. 1, "Quantization granularity",
 *                         "Hadamard rotation"; "Effective bitwidth" for the metadata]
 *   kvq_chunk_attention   current-chunk queries attend to the packed cache of earlier
 *                         chunks and to the unquantized keys/values of the current
 *                         chunk in one joint softmax, with the second-order Taylor
 *                         correction b subtracted from every cached-key score
 *                         [Alg. 1; Eq. 2-4, Eq. 13, Eq. 15; App. "Extension to QuaRot"]
 *
 * Conventions
 *   - Plain C types only.  Pointers named dev_* / q / k / v / out / mass_cached are
 *     DEVICE pointers; everything else is host memory.
 *   - The caller owns every device buffer, including the cache storage; the library
 *     never allocates or frees device memory.
 *   - Launching calls are asynchronous on the HIP stream passed as `hip_stream`
 *     (a hipStream_t cast to void*; NULL is the default stream).  They return after
 *     argument validation and enqueue.  Calls that touch the same cache must be
 *     stream-ordered by the caller.  They enqueue kernels only (no allocation, no
 *     memset, no synchronisation), so they may be recorded into a HIP graph once each
 *     kernel has been launched outside a capture; the host-side counters of the
 *     cache (length, window, blocks) change at call time, not at replay.
 *   - Errors are returned as kvq_status; nothing aborts or throws.  On any error the
 *     cache object is unchanged; nothing has been enqueued, except that an append to a
 *     KVQ_KEYS_PER_CHANNEL cache, which is four launches, may have enqueued the first ones
 *     when the runtime refuses a later one (they write work space and slots that no
 *     live token refers to).
 *   - Tensors are [token][head][channel] with element strides `stride_token`,
 *     `stride_head` (channel stride 1), in the cache's io_dtype.
 *   - The packed layout inside the cache storage is private to the library; the
 *     canonical view (one code per byte, scale, zero-point) is available through
 *     kvq_cache_export.
 */
#ifndef KVQ_H
#define KVQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kvq_cache kvq_cache; /* opaque host object */

typedef enum {
    KVQ_OK = 0,
    KVQ_ERR_INVALID_ARG = 1, /* null pointer, negative size, misaligned buffer, bad range */
    KVQ_ERR_UNSUPPORTED = 2, /* head_dim not 64/128, bits not 2/4, group_size not 32/64/head_dim, rotate != 1,
                                groups smaller than a token without KVQ_META_FP8_BF16 */
    KVQ_ERR_CAPACITY = 3,    /* append would exceed capacity_tokens */
    KVQ_ERR_HIP = 4          /* the HIP runtime refused a launch */
} kvq_status;

typedef enum { KVQ_BF16 = 0, KVQ_FP32 = 1 } kvq_dtype;

/* Storage format of the (scale, zero-point) pairs. */
typedef enum {
    KVQ_META_FP32 = 0,    /* one fp32 scale and one fp32 zero-point per token (group_size == head_dim only) */
    KVQ_META_FP8_BF16 = 1 /* one FP8 E4M3 scale and one BF16 zero-point per group: 24 bits per group, the
                             format of the paper's effective-bitwidth formula B + 24/g */
} kvq_meta_format;

/* Axis along which the keys share a (scale, zero-point). */
typedef enum {
    KVQ_KEYS_PER_TOKEN = 0,  /* one pair (or one per group of channels) per token: the paper's main setting */
    KVQ_KEYS_PER_CHANNEL = 1 /* one pair per rotated channel, shared by the tokens of one kvq_quantize_append
                                call (appendix "Per-Channel Quantization Correction").  The correction is then
                                one scalar per query and appended block.  Values stay per token.  Needs
                                KVQ_META_FP32 and group_size == head_dim.  BF16 caches with head_dim 128 run on the
                                matrix cores, one pass over the cached keys per appended block of the window
                                (windows of more than 40 blocks, fp32 I/O, head_dim 64 and the exact correction on
                                the fp32 vector kernel).  At most capacity/32 + 2 appended blocks can be live at once */
} kvq_key_axis;

typedef struct {
    int32_t num_heads;       /* >= 1 */
    int32_t head_dim;        /* 64 or 128 */
    int32_t bits;            /* 2 or 4 */
    int32_t group_size;      /* channels of a token sharing one (scale, zero-point): 32, 64 or head_dim */
    int32_t rotate;          /* must be 1: normalised Sylvester-Hadamard rotation before quantization */
    int32_t io_dtype;        /* kvq_dtype of q/k/v/out.  KVQ_BF16 with head_dim 128 runs on the matrix cores (every
                                format); fp32 I/O, head_dim 64 and the exact correction run an fp32 vector kernel */
    int32_t meta_format;     /* kvq_meta_format */
    int32_t key_axis;        /* kvq_key_axis */
    int64_t capacity_tokens; /* >= 1; storage is sized for this many tokens per head */
} kvq_cache_desc;

/* Device bytes the caller must provide for a cache of this description, with cap32 = capacity rounded
 * up to 32 tokens:
 *   KVQ_META_FP32      2 * num_heads * cap32 * (head_dim*bits/8 + 8)
 *   KVQ_META_FP8_BF16  2 * num_heads * cap32 * (head_dim*bits/8 + 3 * head_dim/group_size)
 * (codes plus the metadata, for K and for V); KVQ_KEYS_PER_CHANNEL adds
 *   (cap32/32 + 2) * num_heads * head_dim * 8 + cap32 * 4 + num_heads * head_dim * 32, rounded up to 256
 * (per-block scales and zero-points, the block of every token, work space of the append in flight).
 * Every cache ends with a status block of 256 bytes (included in the figure returned): its first word is set by
 * kvq_quantize_append when a stored zero-point reaches 65500 in magnitude, which the matrix-core attention
 * kernels cannot carry exactly (see kvq_chunk_attention).
 * Returns 0 for an invalid or unsupported description. */
size_t kvq_cache_bytes(const kvq_cache_desc *desc);

/* Creates the host object over caller-provided device storage (`dev_mem`, at least
 * kvq_cache_bytes(desc) bytes, 256-byte aligned).  The storage need not be initialised.
 * The cache starts empty. */
kvq_status kvq_cache_create(const kvq_cache_desc *desc, void *dev_mem, size_t bytes, kvq_cache **out);

/* Frees the host object only; the device storage stays with the caller. */
void kvq_cache_destroy(kvq_cache *cache);

/* Number of live tokens (host-side counter; -1 for a null cache). */
int64_t kvq_cache_len(const kvq_cache *cache);

/* Forget every token / every token from new_len on (host-side counters only; 0 <= new_len <= len). */
kvq_status kvq_cache_reset(kvq_cache *cache);
kvq_status kvq_cache_truncate(kvq_cache *cache, int64_t new_len);

/* Randomised Hadamard rotation (rotation paragraph of the method section: the rotation applied to keys and
 * queries is a Hadamard matrix combined with random signs).  negate: host array [head_dim]; a nonzero entry c
 * gives channel c the sign -1, so that vectors are mapped x -> Hn (s * x) before quantization, queries the
 * same way, and the cached part of the output is mapped back with the transpose.  Null restores the plain
 * rotation (all +1), which is also the state of a new cache.  Drawing the signs is the caller's business.
 * Allowed only while the cache holds no token (KVQ_ERR_INVALID_ARG otherwise): stored codes belong to the
 * rotation they were written with.  Exported codes are in the order of the rotated channels either way. */
kvq_status kvq_cache_set_rotation_signs(kvq_cache *cache, const uint8_t *negate);

/* Sliding window (the cached-chunk window of chunk-wise video generation): forget the n_tokens oldest
 * tokens (0 <= n_tokens <= len; host-side counters only).  The storage is a ring of 32-token tiles, so the
 * space is reused by later appends; positions in kvq_chunk_attention and kvq_cache_export count from the
 * oldest live token.  An append fails with KVQ_ERR_CAPACITY when live and new tokens together touch more
 * tiles than the storage has; with evictions and appends in multiples of 32 tokens that is exactly
 * len + n_tokens > capacity_tokens. */
kvq_status kvq_cache_evict(kvq_cache *cache, int64_t n_tokens);

/*
 * Append one chunk: for each (token, head) the key and the value vector are rotated by the
 * normalised Hadamard matrix, quantized to `bits` with one (scale, zero-point) per token
 *     step = (max - min) / (2^bits - 1),  z = -round(min/step),
 *     code = clamp(round(x/step) + z, 0, 2^bits - 1)            (round: nearest, ties to even)
 * and packed.  With KVQ_META_FP8_BF16 the same is done per group of group_size rotated channels, with
 * the stored step the smallest FP8 E4M3 value >= (max - min)/(2^bits - 1) (so that the grid still covers
 * [min, max]; steps above 448 saturate) and the stored zero-point the BF16 value nearest to z; codes are
 * taken with the stored values: where |z| > 256 the BF16 zero-point differs from z, codes that would leave
 * [0, 2^bits - 1] clamp, and the bound |x^ - x| <= step / 2 of Eq. 1 holds only for groups with |z| <= 256.
 * A constant vector (group) has its range widened to include 0; an all-zero one gets step 0.  The rotation is carried out exactly in double precision, so for inputs whose
 * nonzero magnitudes in one vector span at most 2^38 (BF16 values) the codes, scales and
 * zero-points are a bit-exact function of the input.
 *
 * k, v: device, [n_tokens][num_heads][head_dim] in io_dtype with the given element strides.
 * n_tokens == 0 is a no-op.  KVQ_ERR_CAPACITY if len + n_tokens > capacity (nothing written).
 */
kvq_status kvq_quantize_append(kvq_cache *cache, const void *k, const void *v, int64_t n_tokens,
                               int64_t stride_token, int64_t stride_head, void *hip_stream);

/*
 * kvq_quantize_append for callers that cannot allocate device memory or bring a work space along: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results.  The
 * difference is where an append to a KVQ_KEYS_PER_CHANNEL cache keeps its work space (per head and channel the
 * range of the block being appended, L / range and the zero-point: 32 bytes each): not in the cache storage but in
 * a static device array inside the library, 256 KiB per GPU, held until the process ends.  That array serves
 * num_heads * head_dim <= 8192; a larger cache gets KVQ_ERR_CAPACITY and nothing is enqueued.  The call allocates
 * and frees nothing, on the host side it only looks the array's device address up (once per device).  All calls
 * on one GPU share the array: the append overwrites what the previous one left, and two such appends that overlap
 * in time on one GPU (different streams, different caches) race -- order them on one stream or with events.
 * For per-token caches, whose append has no work space, this is kvq_quantize_append.
 */
kvq_status kvq_quantize_append_static(kvq_cache *cache, const void *k, const void *v, int64_t n_tokens,
                                      int64_t stride_token, int64_t stride_head, void *hip_stream);

/*
 * Corrected chunk attention.  For every head and query row m:
 *     cached key i in [cache_start, cache_start + cache_len), counted from the oldest live token:
 *         s_i = softmax_scale * (Hn q_m) . k^_i  -  b_mi,
 *         b_mi = correction ? softmax_scale^2 / 24 * sum_j step_ij^2 * ||(Hn q_m)_j||^2 : 0
 *         (j runs over the groups; per token this is softmax_scale^2 * step_i^2 * ||q_m||^2 / 24)
 *     current key j in [0, n_cur):   s_j = softmax_scale * q_m . k_cur_j
 *     p = softmax over all of them;  out_m = sum_i p_i v^_i (rotated back) + sum_j p_j v_cur_j
 *     mass_cached[head][m] = sum over cached keys of p      (attention mass P_S; P_R = 1 - P_S)
 * k^, v^ are the dequantized cache entries, step_i the stored key scale.  With
 * softmax_scale = 1/sqrt(head_dim) b is the paper's step^2 ||q||^2 / (24 d).
 *
 * q, out: device [m][num_heads][head_dim]; k_cur, v_cur: device [n_cur][num_heads][head_dim];
 * all in io_dtype with the same strides.  mass_cached: device float [num_heads][m] or NULL.
 * softmax_scale == 0 selects 1/sqrt(head_dim).  correction: 0 off, 1 Taylor (Eq. 13 / 15), 2 exact form
 * b_mi = sum_c log(sinh(a_c)/a_c), a_c = softmax_scale * (Hn q_m)_c * step_i,g(c) / 2 (Eq. 12; a diagnostic
 * mode that always runs the fp32 vector kernel).
 * cache_len == 0 (first chunk) and n_cur == 0 are allowed, not both; m == 0 is a no-op.
 * `out` must not alias the inputs.
 * Which kernel runs: matrix cores for BF16 caches with head_dim 128 (every format), the fp32 vector kernel
 * otherwise.  The matrix-core kernels carry a zero-point as two 16-bit pieces, exact
 * below 2^16.  A cache that has stored a larger one since it was created or last reset (vectors whose offset is
 * tens of thousands of times their range) is marked by the append; for such a cache the matrix-core launch
 * returns without writing and a vector-kernel launch enqueued behind it does the work, with the same results as
 * kvq_chunk_attention_fp32.  The mark is only cleared by kvq_cache_reset followed by an append.
 */
kvq_status kvq_chunk_attention(const kvq_cache *cache, int64_t cache_start, int64_t cache_len,
                               const void *q, const void *k_cur, const void *v_cur,
                               int64_t m, int64_t n_cur, int64_t stride_token, int64_t stride_head,
                               float softmax_scale, int correction,
                               void *out, float *mass_cached, void *hip_stream);

/*
 * kvq_chunk_attention with the options of the partial-prefill setting (the paper's cross-domain
 * experiment: a quantized cached prefix and a multi-token causal current block in one softmax).
 *   q_heads_per_kv_head  grouped-query attention: q, out and mass_cached have num_heads * this heads;
 *                        query head h attends to key/value head h / this.  1 = as kvq_chunk_attention.
 *   causal               1: current key j is visible to query row r only if j <= r + n_cur - m (the
 *                        queries are the last m positions of the current block; requires n_cur >= m).
 *                        Cached keys are always visible.
 *   q_stride_token/head  element strides of q and out (stride_token / stride_head of the call are those
 *                        of k_cur and v_cur); 0, 0 = the same strides.
 * opts == NULL is kvq_chunk_attention.  mass_cached: [num_heads * q_heads_per_kv_head][m].
 */
typedef struct {
    int32_t q_heads_per_kv_head;
    int32_t causal;
    int64_t q_stride_token, q_stride_head;
} kvq_attention_opts;

kvq_status kvq_chunk_attention_ex(const kvq_cache *cache, int64_t cache_start, int64_t cache_len,
                                  const void *q, const void *k_cur, const void *v_cur,
                                  int64_t m, int64_t n_cur, int64_t stride_token, int64_t stride_head,
                                  float softmax_scale, int correction, const kvq_attention_opts *opts,
                                  void *out, float *mass_cached, void *hip_stream);

/* Same contract as kvq_chunk_attention, but always runs the fp32 vector-ALU kernel (Alg. 1 in
 * single precision, no matrix cores): slow, for reference-precision results on any cache. */
kvq_status kvq_chunk_attention_fp32(const kvq_cache *cache, int64_t cache_start, int64_t cache_len,
                                    const void *q, const void *k_cur, const void *v_cur,
                                    int64_t m, int64_t n_cur, int64_t stride_token, int64_t stride_head,
                                    float softmax_scale, int correction,
                                    void *out, float *mass_cached, void *hip_stream);

/*
 * Attention-level diagnostics of the bias and of its repair (attention stealing, the equation that defines
 * Delta P_S; appendices "Attention JSD Distributions" and "Attention Output MSE"): the attention of
 * kvq_chunk_attention over the quantized window, with the given correction mode (0, 1, 2), compared per
 * (head, query row) with attention over the same tokens unquantized.
 * k_ref, v_ref: device [cache_len][num_heads][head_dim], io_dtype, strides of k_cur / v_cur: the keys and
 * values that were appended at window positions cache_start .. cache_start + cache_len - 1 (the caller kept
 * them; the library cannot recover them).  Other arguments as for kvq_chunk_attention.
 * diag: device float [num_heads][m][4], written with
 *   [0] P_S, the mass on the window under unquantized attention   [1] P_S under quantized attention
 *       ([1] - [0] is the attention stealing)
 *   [2] Jensen-Shannon divergence (natural logarithm, in [0, log 2]) between the two weight vectors over all
 *       cache_len + n_cur keys
 *   [3] mean over channels of the squared difference of the two attention outputs.
 * Runs on the fp32 vector kernel (two passes over the keys per row): a measuring tool, not a fast path.
 */
kvq_status kvq_attention_diagnostics(const kvq_cache *cache, int64_t cache_start, int64_t cache_len,
                                     const void *q, const void *k_ref, const void *v_ref,
                                     const void *k_cur, const void *v_cur, int64_t m, int64_t n_cur,
                                     int64_t stride_token, int64_t stride_head, float softmax_scale,
                                     int correction, float *diag, void *hip_stream);

/*
 * Canonical view of cached tokens [start, start + count), for parity checks and dump/restore.
 * which: 0 = keys, 1 = values.  codes: device uint8 [num_heads][count][head_dim], one code per
 * byte, channel order of the rotated vector.  scales, zeros: device float [num_heads][count][G],
 * G = head_dim / group_size, holding exactly the stored values (keys of a KVQ_KEYS_PER_CHANNEL cache:
 * G = head_dim, every token carries the per-channel values of its block).  Any of the three output
 * pointers may be NULL.
 */
kvq_status kvq_cache_export(const kvq_cache *cache, int which, int64_t start, int64_t count,
                            uint8_t *codes, float *scales, float *zeros, void *hip_stream);

/* Static, never-null description of a status value. */
const char *kvq_status_string(kvq_status status);

/* Library version, "major.minor". */
const char *kvq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KVQ_H */
