// Rotate + quantize + pack (kvq_quantize_append) and the canonical export (kvq_cache_export).
//
// One workgroup of 256 threads owns one (head, 32-token tile).  Eight lanes share a token
// vector, so the 256 threads hold the 32 key vectors of the tile in one pass and the 32 value
// vectors in a second pass.  Per vector:
//   1. load d elements (coalesced: 8 lanes x 16 elements at d = 128), widen to double;
//   2. Sylvester-Hadamard transform as log2(d) butterfly stages -- the first log2(d/8) inside
//      the lane, the last three across the 8 lanes.  Every partial sum of BF16 inputs is exact
//      in double, so the result does not depend on the order of the additions;
//   3. min / max over the vector, then the round-to-nearest rule of Eq. 1 of the paper in a
//      fixed sequence of IEEE double operations (this file is compiled with contraction off);
//   4. keys: each lane ORs its codes into the words of the tile it feeds and stores them;
//      values: codes go to LDS, then each thread assembles whole words of the token-major
//      ("transposed") value tile and stores them.  A tile that an earlier append filled partly is
//      merged word by word.
// The kernel moves d*elt bytes in and d*bits/8 + 8 bytes out per vector and no byte twice, but it is not bound by
// that traffic: the exact double-precision rotation and the rounding decisions are about 800 vector instructions
// per thread, and the vector ALU is busy for most of the kernel's time (about a third of the HBM rate is reached).
#include <mutex>

#include "kvq_internal.h"

namespace kvq {
namespace {

// Work space of kvq_quantize_append_static: per (head, channel) the range of the block being appended (two ordered
// 64-bit keys), L / range and the zero-point -- 32 bytes each, for at most kStaticScratchChannels of them (256 KiB,
// held by every GPU the library runs on until the process ends).  In host code this name is only a handle for
// hipGetSymbolAddress: the device address is looked up once per device (static_scratch_pointer) and every launch
// takes that pointer as an argument.
static __device__ __align__(256) unsigned char scratch[kStaticScratchChannels * 32];

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (each GPU holds its own copy at its own address).
hipError_t static_scratch_pointer(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

template <typename T> struct Vec;
template <> struct Vec<uint16_t> {  // bf16
    template <int N> __device__ static void load(const uint16_t *p, double (&x)[N])
    {
        static_assert(N % 8 == 0, "");
#pragma unroll
        for (int i = 0; i < N / 8; ++i) {
            const uint4 w = reinterpret_cast<const uint4 *>(p)[i];
            const uint32_t ws[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                x[8 * i + 2 * j] = (double)__uint_as_float(ws[j] << 16);
                x[8 * i + 2 * j + 1] = (double)__uint_as_float(ws[j] & 0xffff0000u);
            }
        }
    }
};
// Raw 16-element loads that are issued for K and V up front and widened to double when needed.
template <typename T> struct Raw16;
template <> struct Raw16<uint16_t> {
    uint4 w[2];
    __device__ void load(const uint16_t *p) { w[0] = reinterpret_cast<const uint4 *>(p)[0]; w[1] = reinterpret_cast<const uint4 *>(p)[1]; }
    __device__ void zero() { w[0] = make_uint4(0, 0, 0, 0); w[1] = w[0]; }
    __device__ void widen(double (&x)[16]) const
    {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint32_t ws[4] = {w[i].x, w[i].y, w[i].z, w[i].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                x[8 * i + 2 * j] = (double)__uint_as_float(ws[j] << 16);
                x[8 * i + 2 * j + 1] = (double)__uint_as_float(ws[j] & 0xffff0000u);
            }
        }
    }
};
template <> struct Raw16<float> {
    float4 w[4];
    __device__ void load(const float *p)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = reinterpret_cast<const float4 *>(p)[i];
    }
    __device__ void zero()
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    __device__ void widen(double (&x)[16]) const
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[4 * i] = (double)w[i].x; x[4 * i + 1] = (double)w[i].y;
            x[4 * i + 2] = (double)w[i].z; x[4 * i + 3] = (double)w[i].w;
        }
    }
};

template <> struct Vec<float> {
    template <int N> __device__ static void load(const float *p, double (&x)[N])
    {
        static_assert(N % 4 == 0, "");
#pragma unroll
        for (int i = 0; i < N / 4; ++i) {
            const float4 w = reinterpret_cast<const float4 *>(p)[i];
            x[4 * i] = (double)w.x;
            x[4 * i + 1] = (double)w.y;
            x[4 * i + 2] = (double)w.z;
            x[4 * i + 3] = (double)w.w;
        }
    }
};

// Smallest FP8 E4M3 value >= x for x > 0 (448 beyond the format's range) and its encoding.  Scaling by a
// power of two, ceil and scaling back are all exact in double.
__device__ inline double e4m3_ceil(double x, uint32_t &byte)
{
    x = x > 448.0 ? 448.0 : x;
    int e = (int)((__double_as_longlong(x) >> 52) & 0x7ff) - 1023;   // floor(log2 x) for normal doubles
    e = e < -6 ? -6 : e;                                              // subnormals share the lowest binade's spacing
    const double up = __longlong_as_double((long long)(1023 + 3 - e) << 52);     // 2^(3 - e)
    const double down = __longlong_as_double((long long)(1023 - 3 + e) << 52);   // 2^(e - 3)
    const double n = __builtin_ceil(x * up);   // in [1, 16]; 16 means the next binade
    const double v = n * down;
    const int ev = (int)((__double_as_longlong(v) >> 52) & 0x7ff) - 1023;
    if (ev < -6) {
        byte = (uint32_t)n;                    // subnormal: m * 2^-9 with e == -6, so n = m
    } else {
        const double m8 = v * __longlong_as_double((long long)(1023 + 3 - ev) << 52);   // 8 + m
        byte = ((uint32_t)(ev + 7) << 3) | ((uint32_t)m8 - 8u);
    }
    return v;
}

// Doubles as unsigned keys whose integer order is the numeric order (for atomic min / max).
__device__ inline unsigned long long order_key(double v)
{
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}
__device__ inline double order_value(unsigned long long k)
{
    return __longlong_as_double((long long)((k >> 63) ? (k & 0x7fffffffffffffffull) : ~k));
}

// Nearest BF16 (ties to even) of a double in one rounding: to float towards zero with a sticky last bit (24
// significant bits keep everything an 8-bit rounding looks at), then to BF16.
__device__ inline uint16_t double_to_bf16(double x)
{
    float f = __double2float_rz(x);
    if ((double)f != x) f = __uint_as_float(__float_as_uint(f) | 1u);
    return float_to_bf16(f);
}
// A stored zero-point that the matrix-core attention kernels cannot carry exactly marks the cache.
__device__ inline void flag_large_zero(const CacheView &cv, float zero)
{
    if (!(fabsf(zero) < kMatrixZeroLimit)) cv.status[0] = 1u;
}
__global__ void status_clear_kernel(CacheView cv)
{
    if (threadIdx.x < kStatusBytes / 4) cv.status[threadIdx.x] = 0u;
}

// Per-channel keys, step 0 of an append: empty ranges.
__global__ void channel_range_init_kernel(CacheView cv)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < cv.num_heads * cv.head_dim) {
        cv.kc_range[2 * i] = ~0ull;   // minimum so far
        cv.kc_range[2 * i + 1] = 0ull;   // maximum so far
    }
}

// Per-channel keys, step 2 of an append: (scale, zero-point) of every (head, channel) from the range that
// step 1 left, in the same sequence of double operations as the per-token quantizer; the block's
// metadata slot and the work space of the quantizing pass are written.
__global__ void channel_params_kernel(CacheView cv, int block_slot)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= cv.num_heads * cv.head_dim) return;
    const double L = (double)((1 << cv.bits) - 1);
    const double norm = cv.head_dim == 64 ? 0.125 : 0.08838834764831845;
    double lo = order_value(cv.kc_range[2 * i]), hi = order_value(cv.kc_range[2 * i + 1]);
    if (hi == lo) {
        lo = lo > 0.0 ? 0.0 : lo;
        hi = hi < 0.0 ? 0.0 : hi;
    }
    const bool degenerate = hi == lo;
    const double range = hi - lo;
    const double inv = degenerate ? 0.0 : L / range;
    const double step = degenerate ? 0.0 : range / L;
    const double z = degenerate ? 0.0 : -__builtin_rint(lo * inv);
    cv.kc_inv[i] = inv;
    cv.kc_z[i] = z;
    const int64_t slot = (int64_t)block_slot * cv.num_heads * cv.head_dim + i;
    cv.kc_scale[slot] = (float)(step * norm);
    cv.kc_zero[slot] = (float)z;
    flag_large_zero(cv, (float)z);
}

// GROUP == 0: one fp32 (scale, zero-point) per token.  GROUP > 0: one FP8 E4M3 scale and one BF16
// zero-point per GROUP rotated channels; codes are taken with the stored values.
// KMODE (per-channel keys, GROUP == 0 only): 0 = keys per token; 1 = range pass: the keys are rotated and
// the minimum / maximum of every channel over the appended tokens goes to cv.kc_range, nothing else is
// written; 2 = the keys take (L / range, zero-point) per channel from cv.kc_inv / cv.kc_z, the values are
// quantized per token as always, and every token records its block slot.
template <int D, int BITS, int GROUP, typename T, int KMODE = 0>
__global__ __launch_bounds__(256) void quantize_append_kernel(CacheView cv, const T *__restrict__ k,
                                                             const T *__restrict__ v, int64_t old_len,
                                                             int64_t n_tokens, int64_t stride_token,
                                                             int64_t stride_head, int block_slot)
{
    static_assert(KMODE == 0 || GROUP == 0, "per-channel keys use fp32 metadata");
    constexpr int EPL = D / 8;            // elements per lane
    constexpr int WPL = D * BITS / 64;    // words per lane slot
    constexpr int L = (1 << BITS) - 1;
    constexpr int CPW = 32 / BITS;        // codes per word
    __shared__ uint8_t v_stage[kTileTokens][D];

    const int head = blockIdx.y;
    const int64_t tile = old_len / kTileTokens + blockIdx.x;
    const int64_t tile_t0 = tile * kTileTokens;
    const int64_t lo_t = old_len > tile_t0 ? old_len : tile_t0;                    // first new token here
    const int64_t end_all = old_len + n_tokens;
    const int64_t hi_t = end_all < tile_t0 + kTileTokens ? end_all : tile_t0 + kTileTokens;
    const int row = threadIdx.x >> 3, l8 = threadIdx.x & 7;
    const int64_t t = tile_t0 + row;
    const bool valid = t >= lo_t && t < hi_t;
    // The storage is a ring of cap_tiles tiles per head: logical tile -> physical tile.
    const int64_t ptile = tile % cv.cap_tiles;
    const int64_t meta_idx = ((int64_t)head * cv.cap_tiles + ptile) * kTileTokens + row;
    uint32_t *k_tile = cv.k_codes + ((int64_t)head * cv.cap_tiles + ptile) * (64 * WPL);
    uint32_t *v_tile = cv.v_codes + ((int64_t)head * cv.cap_tiles + ptile) * (64 * WPL);
    const double norm = D == 64 ? 0.125 : 0.08838834764831845;  // 1/sqrt(d) rounded to double

#pragma unroll 1
    for (int pass = 0; pass < (KMODE == 1 ? 1 : 2); ++pass) {
        double x[EPL];
        if (valid) {
            const T *src = (pass == 0 ? k : v) + (t - old_len) * stride_token + (int64_t)head * stride_head + l8 * EPL;
            Vec<T>::template load<EPL>(src, x);
            if (has_signs(cv)) {   // signs of the randomised rotation
                const uint32_t sg = sign_bits_from(cv, l8 * EPL);
#pragma unroll
                for (int i = 0; i < EPL; ++i) x[i] = flip_sign(x[i], sg >> i);
            }
        } else {
#pragma unroll
            for (int i = 0; i < EPL; ++i) x[i] = 0.0;
        }
        // Butterflies inside the lane: channel bits 0 .. log2(EPL)-1.
#pragma unroll
        for (int h = 1; h < EPL; h <<= 1) {
#pragma unroll
            for (int i = 0; i < EPL; ++i) {
                if ((i & h) == 0) {
                    const double a = x[i], b = x[i + h];
                    x[i] = a + b;
                    x[i + h] = a - b;
                }
            }
        }
        // Butterflies across the 8 lanes of the vector: the upper lane of a pair gets a' = partner - own.
#pragma unroll
        for (int msk = 1; msk < 8; msk <<= 1) {
            const bool upper = (l8 & msk) != 0;
#pragma unroll
            for (int i = 0; i < EPL; ++i) {
                const double other = __shfl_xor(x[i], msk);
                x[i] = upper ? other - x[i] : x[i] + other;
            }
        }
        if constexpr (KMODE == 1) {
            // Minimum and maximum of every channel over the rows of this tile: across the 8 rows of a
            // wave by shuffles, across the 4 waves through LDS, then one atomic pair per channel.
            __shared__ double red[2][4][D];
            const double inf = __longlong_as_double(0x7ff0000000000000ll);
            const int wv = threadIdx.x >> 6, ln = threadIdx.x & 63;
#pragma unroll
            for (int i = 0; i < EPL; ++i) {
                double lo_i = valid ? x[i] : inf, hi_i = valid ? x[i] : -inf;
#pragma unroll
                for (int msk = 8; msk < 64; msk <<= 1) {
                    const double ol = __shfl_xor(lo_i, msk), oh = __shfl_xor(hi_i, msk);
                    lo_i = ol < lo_i ? ol : lo_i;
                    hi_i = oh > hi_i ? oh : hi_i;
                }
                if (ln < 8) {
                    red[0][wv][ln * EPL + i] = lo_i;
                    red[1][wv][ln * EPL + i] = hi_i;
                }
            }
            __syncthreads();
            if (threadIdx.x < D) {
                double lo_c = red[0][0][threadIdx.x], hi_c = red[1][0][threadIdx.x];
#pragma unroll
                for (int w2 = 1; w2 < 4; ++w2) {
                    lo_c = red[0][w2][threadIdx.x] < lo_c ? red[0][w2][threadIdx.x] : lo_c;
                    hi_c = red[1][w2][threadIdx.x] > hi_c ? red[1][w2][threadIdx.x] : hi_c;
                }
                unsigned long long *r = cv.kc_range + 2 * ((int64_t)head * D + threadIdx.x);
                if (lo_c <= hi_c) {   // the tile holds at least one appended token
                    atomicMin(r, order_key(lo_c));
                    atomicMax(r + 1, order_key(hi_c));
                }
            }
            return;
        }
        double lo = x[0], hi = x[0];
#pragma unroll
        for (int i = 1; i < EPL; ++i) {
            lo = x[i] < lo ? x[i] : lo;
            hi = x[i] > hi ? x[i] : hi;
        }
        constexpr int kGroupCh = GROUP == 0 ? D : GROUP;
        constexpr int kLanesPerGroup = kGroupCh / EPL;   // lanes that share one (scale, zero-point)
#pragma unroll
        for (int msk = 1; msk < kLanesPerGroup; msk <<= 1) {
            const double olo = __shfl_xor(lo, msk), ohi = __shfl_xor(hi, msk);
            lo = olo < lo ? olo : lo;
            hi = ohi > hi ? ohi : hi;
        }
        if (hi == lo) {  // constant vector (group): widen the range to include 0
            lo = lo > 0.0 ? 0.0 : lo;
            hi = hi < 0.0 ? 0.0 : hi;
        }
        const bool degenerate = hi == lo;  // all-zero vector (group)
        const double range = hi - lo;
        double inv, z;
        float scale, zero;
        uint32_t scale_byte = 0u;
        if constexpr (GROUP == 0) {
            inv = degenerate ? 0.0 : (double)L / range;
            const double step = degenerate ? 0.0 : range / (double)L;
            z = degenerate ? 0.0 : -__builtin_rint(lo * inv);
            scale = (float)(step * norm);
            zero = (float)z;
        } else {
            // step in the normalised domain, rounded up to the format; everything after uses the stored values
            const double step = range / (double)L * norm;
            const double s8 = degenerate ? 0.0 : e4m3_ceil(step, scale_byte);
            inv = degenerate ? 0.0 : norm / s8;
            const double zi = degenerate ? 0.0 : -__builtin_rint(lo * inv);
            zero = bf16_to_float(double_to_bf16(zi));
            z = (double)zero;
            scale = (float)s8;
        }
        int code[EPL];
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            double inv_i = inv, z_i = z;
            if (KMODE == 2 && pass == 0) {   // per-channel keys: this lane's channels are EPL * l8 + i
                inv_i = cv.kc_inv[head * D + l8 * EPL + i];
                z_i = cv.kc_z[head * D + l8 * EPL + i];
            }
            double c = __builtin_rint(x[i] * inv_i) + z_i;
            c = c < 0.0 ? 0.0 : c;
            c = c > (double)L ? (double)L : c;
            code[i] = (int)c;
        }
        // KVQ_META_FP8_BF16: the first lane of each group stores the group's pair
        const bool group_writer = GROUP != 0 && (l8 % kLanesPerGroup) == 0;
        const int64_t group_idx = GROUP != 0 ? meta_idx * (D / kGroupCh) + l8 / kLanesPerGroup : 0;

        const bool tail = t >= hi_t;  // slot of this tile that no append has reached yet: keep it finite
        if (pass == 0) {
            // The lane holds rotated channels EPL*l8 .. EPL*l8+EPL-1: one 16-wide slab (d = 128) or half
            // a slab (d = 64).  Place its codes at their final bit positions inside the word(s) they share.
            const int slab = (l8 * EPL) >> 4;
            const int lane_shift = BITS == 2 ? 8 * (slab & 1) : 0;
            const int q = BITS == 2 ? slab >> 1 : slab;
            uint32_t mine[2] = {0u, 0u};
#pragma unroll
            for (int i = 0; i < EPL; ++i) {
                const int hh_i = D == 128 ? (i >> 3) & 1 : 0;  // d = 64: all eight channels share one half
                mine[hh_i] |= (uint32_t)code[i] << (BITS * ((i >> 1) & 3) + 16 * (i & 1));
            }
            mine[0] <<= lane_shift;
            mine[1] <<= lane_shift;
            if (BITS == 2) {  // a 2-bit word spans two slabs: merge with the lane that holds the other one
                constexpr int partner = D == 128 ? 1 : 2;
                mine[0] |= __shfl_xor(mine[0], partner);
                mine[1] |= __shfl_xor(mine[1], partner);
            }
            if (valid || tail) {
                if (D == 128) {
                    if (BITS == 4) {
                        k_tile[row * WPL + q] = mine[0];
                        k_tile[(32 + row) * WPL + q] = mine[1];
                    } else {
                        const int hh = l8 & 1;
                        k_tile[(hh * 32 + row) * WPL + q] = hh ? mine[1] : mine[0];
                    }
                } else {
                    const int hh = l8 & 1;
                    if (BITS == 4 || (l8 & 2) == 0) k_tile[(hh * 32 + row) * WPL + q] = mine[0];
                }
                if constexpr (KMODE == 2) {
                    if (l8 == 2 && head == 0 && valid) cv.k_block[ptile * kTileTokens + row] = (uint32_t)block_slot;
                } else if constexpr (GROUP == 0) {
                    if (l8 == 2) cv.k_scale[meta_idx] = scale;
                    if (l8 == 3) {
                        cv.k_negzero[meta_idx] = -(zero + code_offset(BITS));
                        flag_large_zero(cv, zero);
                    }
                } else if (group_writer) {
                    cv.k_scale8[group_idx] = (uint8_t)scale_byte;
                    cv.k_zero16[group_idx] = float_to_bf16(zero);
                    flag_large_zero(cv, zero);
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < EPL; ++i) v_stage[row][l8 * EPL + i] = (uint8_t)code[i];
            if (valid || tail) {
                if constexpr (GROUP == 0) {
                    if (l8 == 2) cv.v_scale[meta_idx] = scale;
                    if (l8 == 3) {
                        cv.v_zero_off[meta_idx] = zero + code_offset(BITS);
                        flag_large_zero(cv, zero);
                    }
                } else if (group_writer) {
                    cv.v_scale8[group_idx] = (uint8_t)scale_byte;
                    cv.v_zero16[group_idx] = float_to_bf16(zero);
                    flag_large_zero(cv, zero);
                }
            }
        }
    }
    __syncthreads();
    // Assemble the value tile: word (lane slot, q) gathers CPW codes of one channel.
    const int t_keep = (int)(lo_t - tile_t0);   // tokens below this index were written by an earlier append
    const int t_new_end = (int)(hi_t - tile_t0);
    for (int w = threadIdx.x; w < 64 * WPL; w += 256) {
        const int lane = w / WPL, q = w % WPL;
        const int hh = lane >> 5, r = lane & 31;
        const int blk = BITS == 2 ? q : q >> 1;
        const int c = 32 * blk + r;
        uint32_t word = 0u, keep = 0u;
#pragma unroll
        for (int p = 0; p < CPW; ++p) {
            const int j = p % (CPW / 2), e = p / (CPW / 2);
            const int s = BITS == 2 ? (j >> 2) : (q & 1);
            const int reg = j & 3;
            const int tok = 16 * s + 8 * (reg >> 1) + 4 * hh + 2 * (reg & 1) + e;
            const int shift = BITS * j + 16 * e;
            if (tok < t_keep) keep |= (uint32_t)L << shift;
            else if (tok < t_new_end) word |= (uint32_t)v_stage[tok][c] << shift;
        }
        if (keep) word |= v_tile[w] & keep;
        v_tile[w] = word;
    }
}

// head_dim 128 variant, the shape of every benchmark config.  Same arithmetic, cheaper data movement:
// after the four butterfly stages inside the lane the 8 lanes of a vector exchange their 16 doubles
// through a padded LDS row (8 conflict-free 16-byte writes and reads per lane), after which lane l
// holds channels 16 j + 2 l + e (j = 0..7, e = 0, 1) and the last three stages run inside the lane as
// well.  In that order a lane owns exactly one register position (reg = l mod 4, half = l / 4) of every
// 16-wide slab of the key tile, so the key words are built with compile-time shifts and merged across the
// 4 lanes of a quad with DPP.
template <int CTRL> __device__ inline double dpp_f64(double v)
{
    const long long b = __double_as_longlong(v);
    const int lo = (int)b, hi = (int)(b >> 32);
    const uint32_t l2 = (uint32_t)__builtin_amdgcn_update_dpp(lo, lo, CTRL, 0xf, 0xf, false);
    const uint32_t h2 = (uint32_t)__builtin_amdgcn_update_dpp(hi, hi, CTRL, 0xf, 0xf, false);
    return __longlong_as_double((long long)(((unsigned long long)h2 << 32) | l2));
}
__device__ inline uint32_t quad_or(uint32_t v)
{
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, true);  // quad_perm [1,0,3,2]
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, true);  // quad_perm [2,3,0,1]
    return v;
}

// GROUP as in the generic kernel: 0 = one fp32 pair per token, 32 / 64 / 128 = FP8 E4M3 scale and BF16
// zero-point per GROUP rotated channels.  After the exchange a lane holds two channels of every slab, so a
// group of 32 (64, 128) channels is registers 4 g .. 4 g + 3 (8 g .. 8 g + 7, all) of all eight lanes.
template <int BITS, typename T, int GROUP = 0>
__global__ __launch_bounds__(256) void quantize_append_kernel128(CacheView cv, const T *__restrict__ k,
                                                                const T *__restrict__ v, int64_t old_len,
                                                                int64_t n_tokens, int64_t stride_token,
                                                                int64_t stride_head)
{
    constexpr int D = 128;
    constexpr int WPL = D * BITS / 64;
    constexpr int L = (1 << BITS) - 1;
    constexpr int CPW = 32 / BITS;
    constexpr int kRowDoubles = D + 16;   // each 16-channel chunk is followed by 2 doubles of padding
    __shared__ __align__(16) double xpose[kTileTokens][kRowDoubles];
    __shared__ __align__(16) uint8_t v_stage[kTileTokens][D];

    const int head = blockIdx.y;
    const int64_t tile = old_len / kTileTokens + blockIdx.x;
    const int64_t tile_t0 = tile * kTileTokens;
    const int64_t lo_t = old_len > tile_t0 ? old_len : tile_t0;
    const int64_t end_all = old_len + n_tokens;
    const int64_t hi_t = end_all < tile_t0 + kTileTokens ? end_all : tile_t0 + kTileTokens;
    const int row = threadIdx.x >> 3, l8 = threadIdx.x & 7;
    const int reg = l8 & 3, hh = l8 >> 2;
    const int64_t t = tile_t0 + row;
    const bool valid = t >= lo_t && t < hi_t;
    const bool tail = t >= hi_t;
    // The storage is a ring of cap_tiles tiles per head: logical tile -> physical tile.
    const int64_t ptile = tile % cv.cap_tiles;
    const int64_t meta_idx = ((int64_t)head * cv.cap_tiles + ptile) * kTileTokens + row;
    uint32_t *k_tile = cv.k_codes + ((int64_t)head * cv.cap_tiles + ptile) * (64 * WPL);
    uint32_t *v_tile = cv.v_codes + ((int64_t)head * cv.cap_tiles + ptile) * (64 * WPL);
    double *rowbuf = xpose[row];

    // Both loads are in flight before any arithmetic starts.
    Raw16<T> raw_k, raw_v;
    if (valid) {
        const int64_t off = (t - old_len) * stride_token + (int64_t)head * stride_head + l8 * 16;
        raw_k.load(k + off);
        raw_v.load(v + off);
    } else {
        raw_k.zero();
        raw_v.zero();
    }
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        double x[16];
        if (pass == 0) raw_k.widen(x);
        else raw_v.widen(x);
        if (has_signs(cv)) {
            const uint32_t sg = sign_bits_from(cv, l8 * 16);   // signs of the randomised rotation
#pragma unroll
            for (int i = 0; i < 16; ++i) x[i] = flip_sign(x[i], sg >> i);
        }
#pragma unroll
        for (int h = 1; h < 16; h <<= 1) {   // channel bits 0..3
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if ((i & h) == 0) {
                    const double a = x[i], b = x[i + h];
                    x[i] = a + b;
                    x[i + h] = a - b;
                }
        }
        // Exchange inside the vector's 8 lanes (same wavefront: LDS operations of a wave complete in order).
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            double2 w;
            w.x = x[2 * i];
            w.y = x[2 * i + 1];
            *reinterpret_cast<double2 *>(rowbuf + 18 * l8 + 2 * i) = w;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const double2 w = *reinterpret_cast<const double2 *>(rowbuf + 18 * j + 2 * l8);
            x[2 * j] = w.x;       // channel 16 j + 2 l8
            x[2 * j + 1] = w.y;   // channel 16 j + 2 l8 + 1
        }
#pragma unroll
        for (int h = 2; h < 16; h <<= 1) {   // channel bits 4..6 = bits 1..3 of the register index
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if ((i & h) == 0) {
                    const double a = x[i], b = x[i + h];
                    x[i] = a + b;
                    x[i + h] = a - b;
                }
        }
        // No NaNs can occur here (finite inputs, exact sums), so min/max are plain selections.
        constexpr int kG = GROUP == 0 ? 1 : D / GROUP;   // groups per vector
        constexpr int kRegs = 16 / kG;                    // registers of a lane that belong to one group
        uint32_t code[16];
        // Range of every group (all eight lanes end up with all of them); lane l then works out the
        // parameters of group l mod kG only and the lanes exchange the results.
        double lo_mine = 0.0, hi_mine = 0.0;
#pragma unroll
        for (int g = 0; g < kG; ++g) {
            double lo = __builtin_fmin(x[kRegs * g], x[kRegs * g + 1]), hi = __builtin_fmax(x[kRegs * g], x[kRegs * g + 1]);
#pragma unroll
            for (int i = 2; i < kRegs; ++i) {
                lo = __builtin_fmin(lo, x[kRegs * g + i]);
                hi = __builtin_fmax(hi, x[kRegs * g + i]);
            }
            // across the vector's 8 lanes with data-parallel moves: neighbours, pairs, then the mirror image
            // inside the 8 lanes (by then the four lanes of a quad agree, so lane l meets the other quad)
            lo = __builtin_fmin(lo, dpp_f64<0xB1>(lo)); hi = __builtin_fmax(hi, dpp_f64<0xB1>(hi));      // quad_perm [1,0,3,2]
            lo = __builtin_fmin(lo, dpp_f64<0x4E>(lo)); hi = __builtin_fmax(hi, dpp_f64<0x4E>(hi));      // quad_perm [2,3,0,1]
            lo = __builtin_fmin(lo, dpp_f64<0x141>(lo)); hi = __builtin_fmax(hi, dpp_f64<0x141>(hi));    // row_half_mirror
            if (g == 0 || (l8 & (kG - 1)) == g) { lo_mine = lo; hi_mine = hi; }
        }
        double inv_mine, z_mine;
        float my_scale, my_zero;
        uint32_t my_byte = 0u;
        {
            double lo = lo_mine, hi = hi_mine;
            if (hi == lo) {  // constant vector (group): widen the range to include 0
                lo = lo > 0.0 ? 0.0 : lo;
                hi = hi < 0.0 ? 0.0 : hi;
            }
            const bool degenerate = hi == lo;  // all-zero vector (group)
            const double range = hi - lo;
            if constexpr (GROUP == 0) {
                inv_mine = degenerate ? 0.0 : (double)L / range;
                const double step = degenerate ? 0.0 : range / (double)L;
                z_mine = degenerate ? 0.0 : -__builtin_rint(lo * inv_mine);
                my_scale = (float)(step * 0.08838834764831845);  // 1/sqrt(128) rounded to double
                my_zero = (float)z_mine;
            } else {
                // step in the normalised domain, rounded up to the format; everything after uses the stored values
                const double step = range / (double)L * 0.08838834764831845;
                const double s8 = degenerate ? 0.0 : e4m3_ceil(step, my_byte);
                inv_mine = degenerate ? 0.0 : 0.08838834764831845 / s8;
                const double zr = degenerate ? 0.0 : -__builtin_rint(lo * inv_mine);
                my_zero = bf16_to_float(double_to_bf16(zr));
                z_mine = (double)my_zero;
                my_scale = (float)s8;
            }
        }
#pragma unroll
        for (int g = 0; g < kG; ++g) {
            // lanes g, g + kG, ... of the vector hold group g's parameters; take them from lane g
            const double inv = kG == 1 ? inv_mine : __shfl(inv_mine, g, 8);
            const int zi = kG == 1 ? (int)z_mine : __shfl((int)z_mine, g, 8);
            // round(u * inv) + z and the clamp are exact in 32-bit integers (|z| + L < 2^31 by the documented
            // domain), so they give the same codes as the double-precision statement of Eq. 1.
#pragma unroll
            for (int i = kRegs * g; i < kRegs * (g + 1); ++i) {
                // 1.5 * 2^52 added to a double below 2^31 in magnitude leaves its round-to-nearest-even integer in
                // the low word of the sum (this file is compiled without contraction: product, then sum)
                const double shifted = x[i] * inv + 6755399441055744.0;
                const int c = (int)(uint32_t)__double_as_longlong(shifted) + zi;
                code[i] = (uint32_t)(c < 0 ? 0 : (c > L ? L : c));   // one v_med3_i32
            }
        }
        const float scale = my_scale, zero = my_zero;   // GROUP == 0: the same in every lane
        const int64_t group_idx = meta_idx * kG + l8;   // KVQ_META_FP8_BF16: lane g < kG stores group g's pair

        if (pass == 0) {
            // register index 2 j + e <-> slab j, element pair position `reg`, half `hh`
            if (BITS == 2) {
                uint32_t w[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t base = code[4 * q] | (code[4 * q + 1] << 16) | (code[4 * q + 2] << 8) | (code[4 * q + 3] << 24);
                    w[q] = quad_or(base << (2 * reg));
                }
                if ((valid || tail) && reg == 0) {
                    uint4 out;
                    out.x = w[0]; out.y = w[1]; out.z = w[2]; out.w = w[3];
                    *reinterpret_cast<uint4 *>(k_tile + (hh * 32 + row) * WPL) = out;
                }
            } else {
                uint32_t w[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) w[j] = quad_or((code[2 * j] | (code[2 * j + 1] << 16)) << (4 * reg));
                if ((valid || tail) && reg < 2) {
                    uint4 out;
                    out.x = reg ? w[4] : w[0]; out.y = reg ? w[5] : w[1];
                    out.z = reg ? w[6] : w[2]; out.w = reg ? w[7] : w[3];
                    *reinterpret_cast<uint4 *>(k_tile + (hh * 32 + row) * WPL + 4 * reg) = out;
                }
            }
            if (valid || tail) {
                if constexpr (GROUP == 0) {
                    if (l8 == 2) cv.k_scale[meta_idx] = scale;
                    if (l8 == 3) {
                        cv.k_negzero[meta_idx] = -(zero + code_offset(BITS));
                        flag_large_zero(cv, zero);
                    }
                } else if (l8 < kG) {
                    cv.k_scale8[group_idx] = (uint8_t)my_byte;
                    cv.k_zero16[group_idx] = float_to_bf16(my_zero);
                    flag_large_zero(cv, my_zero);
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                *reinterpret_cast<uint16_t *>(&v_stage[row][16 * j + 2 * l8]) = (uint16_t)(code[2 * j] | (code[2 * j + 1] << 8));
            if (valid || tail) {
                if constexpr (GROUP == 0) {
                    if (l8 == 2) cv.v_scale[meta_idx] = scale;
                    if (l8 == 3) {
                        cv.v_zero_off[meta_idx] = zero + code_offset(BITS);
                        flag_large_zero(cv, zero);
                    }
                } else if (l8 < kG) {
                    cv.v_scale8[group_idx] = (uint8_t)my_byte;
                    cv.v_zero16[group_idx] = float_to_bf16(my_zero);
                    flag_large_zero(cv, my_zero);
                }
            }
        }
    }
    __syncthreads();
    // Assemble the value tile: word (lane slot, q) gathers CPW codes of one channel.  Rows that this
    // append does not own staged zeros, so only a tile begun by an earlier append needs merging.
    const int t_keep = (int)(lo_t - tile_t0);
    for (int w = threadIdx.x; w < 64 * WPL; w += 256) {
        const int lane = w / WPL, q = w % WPL;
        const int vh = lane >> 5, r = lane & 31;
        const int blk = BITS == 2 ? q : q >> 1;
        const int c = 32 * blk + r;
        uint32_t word = 0u;
#pragma unroll
        for (int p = 0; p < CPW; ++p) {
            const int j = p % (CPW / 2), e = p / (CPW / 2);
            const int s = BITS == 2 ? (j >> 2) : (q & 1);
            const int rg = j & 3;
            const int tok = 16 * s + 8 * (rg >> 1) + 4 * vh + 2 * (rg & 1) + e;
            word |= (uint32_t)v_stage[tok][c] << (BITS * j + 16 * e);
        }
        if (t_keep > 0) {   // uniform over the workgroup
            uint32_t keep = 0u;
#pragma unroll
            for (int p = 0; p < CPW; ++p) {
                const int j = p % (CPW / 2), e = p / (CPW / 2);
                const int s = BITS == 2 ? (j >> 2) : (q & 1);
                const int rg = j & 3;
                const int tok = 16 * s + 8 * (rg >> 1) + 4 * vh + 2 * (rg & 1) + e;
                keep |= (tok < t_keep ? (uint32_t)L : 0u) << (BITS * j + 16 * e);
            }
            word |= v_tile[w] & keep;
        }
        v_tile[w] = word;
    }
}

template <int D, int BITS>
__global__ __launch_bounds__(D) void export_kernel(CacheView cv, int which, int64_t start, int64_t count,
                                                  uint8_t *codes, float *scales, float *zeros)
{
    const int head = blockIdx.y;
    const int c = threadIdx.x;
    for (int64_t i = blockIdx.x; i < count; i += gridDim.x) {
        const int64_t t = start + i;
        const int64_t tile = (t / kTileTokens) % cv.cap_tiles;   // physical tile of the ring
        const int tt = (int)(t % kTileTokens);
        const uint32_t *base = (which == 0 ? cv.k_codes : cv.v_codes) +
                               ((int64_t)head * cv.cap_tiles + tile) * tile_words(D, BITS);
        int word, shift;
        if (which == 0) key_code_pos(D, BITS, tt, c, word, shift);
        else value_code_pos(D, BITS, tt, c, word, shift);
        if (codes) codes[((int64_t)head * count + i) * D + c] = (uint8_t)((base[word] >> shift) & ((1u << BITS) - 1u));
        const int64_t mi = ((int64_t)head * cv.cap_tiles + tile) * kTileTokens + tt;
        if (cv.key_axis == KVQ_KEYS_PER_CHANNEL && which == 0) {   // every token carries its block's per-channel values
            const int64_t slot = cv.k_block[tile * kTileTokens + tt];
            const int64_t si = (slot * cv.num_heads + head) * D + c, oi = ((int64_t)head * count + i) * D + c;
            if (scales) scales[oi] = cv.kc_scale[si];
            if (zeros) zeros[oi] = cv.kc_zero[si];
        } else if (cv.meta_format == KVQ_META_FP32) {
            if (c == 0) {
                if (scales) scales[(int64_t)head * count + i] = which == 0 ? cv.k_scale[mi] : cv.v_scale[mi];
                if (zeros)
                    zeros[(int64_t)head * count + i] =
                        which == 0 ? -cv.k_negzero[mi] - code_offset(BITS) : cv.v_zero_off[mi] - code_offset(BITS);
            }
        } else if (c % cv.group_size == 0) {
            const int G = D / cv.group_size, g = c / cv.group_size;
            const int64_t gi = mi * G + g, oi = ((int64_t)head * count + i) * G + g;
            if (scales) scales[oi] = e4m3_to_float(which == 0 ? cv.k_scale8[gi] : cv.v_scale8[gi]);
            if (zeros) zeros[oi] = bf16_to_float(which == 0 ? cv.k_zero16[gi] : cv.v_zero16[gi]);
        }
    }
}

template <int D, int BITS, typename T>
hipError_t launch_q(const CacheView &cv, const void *k, const void *v, int64_t old_len, int64_t n, int64_t st,
                    int64_t sh, int block_slot, hipStream_t stream)
{
    const int64_t first_tile = old_len / kTileTokens;
    const int64_t last_tile = (old_len + n - 1) / kTileTokens;
    const dim3 grid((unsigned)(last_tile - first_tile + 1), (unsigned)cv.num_heads);
    const dim3 block(256);
    const T *kp = static_cast<const T *>(k), *vp = static_cast<const T *>(v);
    if (cv.key_axis == KVQ_KEYS_PER_CHANNEL) {
        // ranges of the block -> per-channel parameters -> codes (keys per channel, values per token); the sequence
        // stops at the first launch that fails (the cache's token count is only advanced when all four are enqueued)
        const dim3 nb((unsigned)((cv.num_heads * cv.head_dim + 255) / 256));
        hipError_t e = launch_kernel(channel_range_init_kernel, nb, block, 0, stream, cv);
        if (e != hipSuccess) return e;
        e = launch_kernel(quantize_append_kernel<D, BITS, 0, T, 1>, grid, block, 0, stream, cv, kp, vp, old_len, n, st, sh, block_slot);
        if (e != hipSuccess) return e;
        e = launch_kernel(channel_params_kernel, nb, block, 0, stream, cv, block_slot);
        if (e != hipSuccess) return e;
        return launch_kernel(quantize_append_kernel<D, BITS, 0, T, 2>, grid, block, 0, stream, cv, kp, vp, old_len, n, st, sh, block_slot);
    }
    if constexpr (D == 128) {
        if (cv.meta_format == KVQ_META_FP8_BF16) {
            if (cv.group_size == 32)
                return launch_kernel(quantize_append_kernel128<BITS, T, 32>, grid, block, 0, stream, cv, kp, vp, old_len, n, st, sh);
            if (cv.group_size == 64)
                return launch_kernel(quantize_append_kernel128<BITS, T, 64>, grid, block, 0, stream, cv, kp, vp, old_len, n, st, sh);
            return launch_kernel(quantize_append_kernel128<BITS, T, 128>, grid, block, 0, stream, cv, kp, vp, old_len, n, st, sh);
        }
    }
    if (cv.meta_format == KVQ_META_FP8_BF16) {
        if (cv.group_size == 32)
            return launch_kernel(quantize_append_kernel<D, BITS, 32, T, 0>, grid, block, 0, stream, cv, kp, vp, old_len, n, st, sh, 0);
        if (cv.group_size == 64)
            return launch_kernel(quantize_append_kernel<D, BITS, 64, T, 0>, grid, block, 0, stream, cv, kp, vp, old_len, n, st, sh, 0);
        if constexpr (D == 128)
            return launch_kernel(quantize_append_kernel<D, BITS, 128, T, 0>, grid, block, 0, stream, cv, kp, vp, old_len, n, st, sh, 0);
        else
            return hipErrorInvalidValue;
    } else if constexpr (D == 128) {
        return launch_kernel(quantize_append_kernel128<BITS, T, 0>, grid, block, 0, stream, cv, kp, vp, old_len, n, st, sh);
    } else {
        return launch_kernel(quantize_append_kernel<D, BITS, 0, T, 0>, grid, block, 0, stream, cv, kp, vp, old_len, n, st, sh, 0);
    }
}

}  // namespace

hipError_t launch_quantize_append(const CacheView &cv_in, const void *k, const void *v, int64_t old_len,
                                  int64_t n_tokens, int64_t stride_token, int64_t stride_head, int block_slot,
                                  hipStream_t stream, bool static_scratch)
{
    CacheView cv = cv_in;
    if (static_scratch && cv.key_axis == KVQ_KEYS_PER_CHANNEL) {
        // The three work arrays move to the static array; the first launch of the append fills the ranges with
        // their empty values, so what an earlier call left there does not matter.
        const int64_t hd = (int64_t)cv.num_heads * cv.head_dim;
        if (hd > kStaticScratchChannels) return hipErrorInvalidValue;   // (the entry point has refused this already)
        void *base = nullptr;
        const hipError_t e = static_scratch_pointer(&base);
        if (e != hipSuccess) return e;
        unsigned char *p = static_cast<unsigned char *>(base);
        cv.kc_range = reinterpret_cast<unsigned long long *>(p);
        cv.kc_inv = reinterpret_cast<double *>(p + hd * 16);
        cv.kc_z = reinterpret_cast<double *>(p + hd * 24);
    }
    const bool bf16 = cv.io_dtype == KVQ_BF16;
#define KVQ_Q(D, B)                                                                                                         \
    if (cv.head_dim == D && cv.bits == B)                                                                                   \
        return bf16 ? launch_q<D, B, uint16_t>(cv, k, v, old_len, n_tokens, stride_token, stride_head, block_slot, stream)  \
                    : launch_q<D, B, float>(cv, k, v, old_len, n_tokens, stride_token, stride_head, block_slot, stream);
    KVQ_Q(128, 2)
    KVQ_Q(128, 4)
    KVQ_Q(64, 2)
    KVQ_Q(64, 4)
#undef KVQ_Q
    return hipErrorInvalidValue;
}

hipError_t launch_status_clear(const CacheView &cv, hipStream_t stream)
{
    return launch_kernel(status_clear_kernel, dim3(1), dim3(64), 0, stream, cv);
}

hipError_t launch_export(const CacheView &cv, int which, int64_t start, int64_t count, uint8_t *codes,
                         float *scales, float *zeros, hipStream_t stream)
{
    const unsigned gx = (unsigned)(count < 4096 ? count : 4096);
    const dim3 grid(gx, (unsigned)cv.num_heads);
#define KVQ_E(D, B)                                                                                        \
    if (cv.head_dim == D && cv.bits == B)                                                                  \
        return launch_kernel(export_kernel<D, B>, grid, dim3(D), 0, stream, cv, which, start, count, codes, scales, zeros);
    KVQ_E(128, 2)
    KVQ_E(128, 4)
    KVQ_E(64, 2)
    KVQ_E(64, 4)
#undef KVQ_E
    return hipErrorInvalidValue;
}

}  // namespace kvq
