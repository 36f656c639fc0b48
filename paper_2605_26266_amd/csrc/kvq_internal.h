// Internal declarations shared by the host layer and the gfx950 kernels.
//
// Packed cache layout (private to the library)
// --------------------------------------------
// Per head the cache holds, for keys and for values, a sequence of 32-token tiles of packed
// codes plus four float arrays indexed by token.  A tile is 64 "lane slots" of WPL = d*bits/64
// 32-bit words each, laid out lane-major, so that one wavefront reads a whole tile with a
// single 16- or 32-byte load per lane and every lane receives exactly the codes its matrix-core
// operand registers need:
//
//  key tile   lane slot = 32*hh + token_in_tile.  The slot holds the codes of the rotated
//             channels c with bit 3 of c equal to hh, i.e. the eight contraction indices
//             8*hh..8*hh+7 of every 16-wide slab that this lane feeds to a 32x32x16 MFMA.
//  value tile lane slot = 32*hh + (channel mod 32).  The slot holds, for the channels
//             c, c+32, c+64, c+96, the codes of the 16 tokens of the tile with bit 2 of the
//             token index equal to hh -- the contraction (token) indices this lane feeds to
//             the P*V MFMA, in the order in which the score MFMA leaves its results in that lane.
//
// Inside a word codes sit in pairs (low half-word, high half-word) `bits` apart, so that one
// shift and one and-or turn a word into a register of two bf16 operands.
//
// Per-token metadata: k_scale, k_negzero = -(zero + OFFSET), v_scale, v_zero_off = zero + OFFSET,
// where OFFSET (4 for 2-bit, 16 for 4-bit codes) is the constant that the bit pattern used for
// in-register dequantization adds to every code.  Integers of that size are exact in float.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <tuple>

#include "../../include/kvq.h"

namespace kvq {

constexpr int kTileTokens = 32;

struct CacheView {
    uint32_t *k_codes;   // [H][cap_tiles][64][WPL]
    uint32_t *v_codes;   // [H][cap_tiles][64][WPL]
    float *k_scale;      // [H][cap32]
    float *k_negzero;    // [H][cap32]   -(zero + OFFSET)
    float *v_scale;      // [H][cap32]
    float *v_zero_off;   // [H][cap32]   zero + OFFSET
    int64_t cap_tiles;   // tiles per head
    int32_t num_heads, head_dim, bits, io_dtype;
    // KVQ_META_FP8_BF16 caches use these instead of the four float arrays (G = head_dim / group_size):
    int32_t group_size, meta_format;
    uint8_t *k_scale8, *v_scale8;    // [H][cap32][G]  FP8 E4M3 encodings
    uint16_t *k_zero16, *v_zero16;   // [H][cap32][G]  BF16 encodings
    // Randomised Hadamard rotation x -> Hn (s * x): bit c of the mask set means s_c = -1.  All zero is the
    // plain rotation.
    uint32_t sign_mask[4];
    // KVQ_KEYS_PER_CHANNEL: keys share one (scale, zero-point) per channel within an appended block.
    int32_t key_axis, max_blocks;
    float *kc_scale, *kc_zero;       // [max_blocks][H][d]  per block slot
    uint32_t *k_block;               // [cap32]             block slot of the token at each ring position
    unsigned long long *kc_range;    // [H][d][2]           work space of the append in flight: min, max (ordered keys)
    double *kc_inv, *kc_z;           // [H][d]              work space: L / range and the zero-point, per channel
    // Status block at the end of the storage (kStatusBytes).  Word 0: sticky, set by the quantize kernels when a stored
    // zero-point is too large for the matrix-core attention kernels (kMatrixZeroLimit), read by every attention launch.
    uint32_t *status;
};
constexpr int kStatusBytes = 256;
// The matrix-core kernels carry OFFSET + zero-point as two bf16 pieces: exact for integers below 2^16.
constexpr float kMatrixZeroLimit = 65500.0f;

// Sign bits of the channels first .. first + 31 - (first mod 32), bit 0 = channel `first`.
__device__ inline uint32_t sign_bits_from(const CacheView &cv, int first)
{
    const int w = first >> 5;
    const uint32_t m = w == 0 ? cv.sign_mask[0] : w == 1 ? cv.sign_mask[1] : w == 2 ? cv.sign_mask[2] : cv.sign_mask[3];
    return m >> (first & 31);
}
// Uniform over the grid (kernel argument): lets a kernel skip the sign flips of the plain rotation.
__device__ inline bool has_signs(const CacheView &cv)
{
    return (cv.sign_mask[0] | cv.sign_mask[1] | cv.sign_mask[2] | cv.sign_mask[3]) != 0u;
}
__device__ inline float flip_sign(float x, uint32_t bit0) { return __uint_as_float(__float_as_uint(x) ^ (bit0 << 31)); }
__device__ inline double flip_sign(double x, uint32_t bit0)
{
    return __hiloint2double(__double2hiint(x) ^ (int)(bit0 << 31), __double2loint(x));
}

// FP8 E4M3 (bias 7, 3 mantissa bits, subnormals m * 2^-9, no infinities) -> float.  Scales are never
// negative and never the NaN encoding.
__host__ __device__ inline float e4m3_to_float(uint8_t b)
{
    const int e = (b >> 3) & 15, m = b & 7;
    const float mag = e == 0 ? (float)m * 0.001953125f : (float)(8 + m) * (float)(1u << e) * 0.0009765625f;
    return (b & 0x80) ? -mag : mag;   // (8 + m) * 2^(e - 10) = (1 + m/8) * 2^(e - 7)
}

__host__ __device__ inline int words_per_lane(int d, int bits) { return d * bits / 64; }
__host__ __device__ inline int tile_words(int d, int bits) { return d * bits; }  // 64 * WPL
__host__ __device__ inline float code_offset(int bits) { return bits == 2 ? 4.0f : 16.0f; }

// Word index inside the tile and bit position of the code of (token-in-tile t, rotated channel c).
__host__ __device__ inline void key_code_pos(int d, int bits, int t, int c, int &word, int &shift)
{
    const int slab = c >> 4, hh = (c >> 3) & 1, reg = (c >> 1) & 3, e = c & 1;
    const int lane = hh * 32 + t;
    int q, j;
    if (bits == 2) { q = slab >> 1; j = 4 * (slab & 1) + reg; }
    else           { q = slab;      j = reg; }
    word = lane * words_per_lane(d, bits) + q;
    shift = bits * j + 16 * e;
}

__host__ __device__ inline void value_code_pos(int d, int bits, int t, int c, int &word, int &shift)
{
    const int blk = c >> 5, r = c & 31;
    const int s = t >> 4, g = (t >> 3) & 1, hh = (t >> 2) & 1, x = (t >> 1) & 1, e = t & 1;
    const int reg = 2 * g + x;
    const int lane = hh * 32 + r;
    int q, j;
    if (bits == 2) { q = blk;         j = 4 * s + reg; }
    else           { q = 2 * blk + s; j = reg; }
    word = lane * words_per_lane(d, bits) + q;
    shift = bits * j + 16 * e;
}

// bf16 <-> float on raw bit patterns (round to nearest even on the way down).
__device__ inline float bf16_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ inline uint16_t float_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <typename T> struct Io;
template <> struct Io<float> {
    __device__ static float load(const float *p) { return *p; }
    __device__ static void store(float *p, float v) { *p = v; }
};
template <> struct Io<uint16_t> {
    __device__ static float load(const uint16_t *p) { return bf16_to_float(*p); }
    __device__ static void store(uint16_t *p, float v) { *p = float_to_bf16(v); }
};

// Launch with the status of this launch as return value.  (hipGetLastError() after a <<< >>> launch would also
// return, and clear, an error that some earlier HIP call of the process left behind on this thread.)
template <typename... KArgs, typename... Args>
hipError_t launch_kernel(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream, Args &&...args)
{
    static_assert(sizeof...(KArgs) == sizeof...(Args), "one argument per kernel parameter");
    std::tuple<KArgs...> copy{static_cast<KArgs>(args)...};
    return std::apply(
        [&](auto &...a) {
            void *ptrs[] = {static_cast<void *>(&a)...};
            return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, lds_bytes, stream);
        },
        copy);
}

// Launchers implemented in the kernel translation units.  All return hipError_t of the launch.
// block_slot: slot of the block this append creates (KVQ_KEYS_PER_CHANNEL caches only).
// static_scratch: the per-channel work space of the append (ranges, L / range, zero-points per head and channel)
// is taken from the library's static device array instead of the cache storage.
hipError_t launch_quantize_append(const CacheView &cv, const void *k, const void *v, int64_t old_len,
                                  int64_t n_tokens, int64_t stride_token, int64_t stride_head, int block_slot,
                                  hipStream_t stream, bool static_scratch = false);
// Largest num_heads * head_dim that the static work space serves.
constexpr int kStaticScratchChannels = 8192;
hipError_t launch_export(const CacheView &cv, int which, int64_t start, int64_t count, uint8_t *codes,
                         float *scales, float *zeros, hipStream_t stream);
// Clears the status block (first append after kvq_cache_create / kvq_cache_reset).
// A kernel that needs more dynamic LDS than the default limit has to be told so once per device (the attribute belongs
// to the kernel as loaded on the current device).  `done` holds one bit per device ordinal; devices beyond 63 are
// configured on every call.
inline hipError_t configure_dynamic_lds(const void *kernel, size_t bytes, std::atomic<uint64_t> &done)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < 64;
    if (tracked && ((done.load(std::memory_order_acquire) >> dev) & 1u)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess && tracked) done.fetch_or(uint64_t(1) << dev, std::memory_order_release);
    return e;
}

hipError_t launch_status_clear(const CacheView &cv, hipStream_t stream);

// One appended block of a KVQ_KEYS_PER_CHANNEL cache inside the attended window: its parameter slot and its
// token range relative to cache_start.
struct KeyBlock {
    int32_t slot, start, end;
};
constexpr int kMaxKeyBlocks = 40;   // more blocks than this in one window: vector kernel

struct AttentionArgs {
    CacheView cv;
    int64_t cache_start, cache_len;   // logical token positions (the storage is a ring of cap_tiles tiles)
    int64_t phys_tile_first;          // physical tile that holds logical token cache_start
    const void *q, *k_cur, *v_cur;
    int64_t m, n_cur, stride_token, stride_head;   // strides of k_cur / v_cur
    int64_t q_stride_token, q_stride_head;         // strides of q / out
    int32_t q_per_kv;   // query heads per key/value head (grouped-query attention); query head h uses KV head h / q_per_kv
    int32_t causal;     // current key j visible to query row r only if j <= r + n_cur - m
    float softmax_scale;
    int correction;
    void *out;
    float *mass_cached;
    int32_t n_key_blocks;                 // matrix-core path of per-channel caches only
    KeyBlock key_blocks[kMaxKeyBlocks];
    // The cache's status word (null: nothing has been appended since the cache was created or reset, there is
    // nothing to look at).  A matrix-core launch returns at once when the word is set; the vector launch that the
    // host enqueues behind it with only_if_flagged = 1 returns at once when it is not.
    const uint32_t *status;
    int32_t only_if_flagged;
};
__device__ inline bool cache_flagged(const uint32_t *status) { return status != nullptr && *status != 0u; }
hipError_t launch_attention_simt(const AttentionArgs &a, hipStream_t stream);
hipError_t launch_attention_mfma(const AttentionArgs &a, hipStream_t stream);
// Per (head, row) [P_S unquantized, P_S quantized, JSD, output MSE] against the unquantized cached k_ref / v_ref
// ([cache_len][H][d], strides of k_cur); a.out and a.mass_cached are not used.
hipError_t launch_diagnostics_simt(const AttentionArgs &a, const void *k_ref, const void *v_ref, float *diag,
                                   hipStream_t stream);
// Matrix-core kernel for caches with several FP8/BF16 (scale, zero-point) groups per token.
bool attention_mfma_group_supported(const CacheView &cv);
hipError_t launch_attention_mfma_group(const AttentionArgs &a, hipStream_t stream);

}  // namespace kvq
