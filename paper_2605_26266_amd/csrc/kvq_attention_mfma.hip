// Matrix-core chunk attention for gfx950: BF16 I/O, head_dim 128, 2- or 4-bit cache.
//
// Work split.  One workgroup = 4 wavefronts = 256 query rows of one head; each wavefront owns
// 64 rows (two 32-row blocks) for the whole key loop, so the waves only meet at the barriers
// of the staging pipeline.  Everything is computed transposed,
//     S^T = K Q~^T           (A operand: keys,     B operand: queries)
//     O^T = V^T P^T          (A operand: channels, B operand: queries)
// with v_mfma_f32_32x32x16_bf16.  In that orientation a lane owns one query row (row = lane
// mod 32) of every result tile, so the softmax row maximum and row sum are reductions inside a
// lane plus one exchange between the two lane halves, and the probabilities the score MFMA
// leaves in a lane are exactly that lane's B operand of the P*V MFMA -- no shuffle, no LDS round
// trip for P.
//
// Cached keys/values (Alg. 1 of the paper, cached block).  Packed tiles (see kvq_internal.h) are
// staged through LDS 128 keys at a time, double buffered.  A lane pulls its 16 or 32 bytes of codes
// and turns every word into MFMA operand registers with one shift and one and-or per register: the
// code lands in the top mantissa bits of a 16-bit float whose exponent makes the value OFFSET + code
// (4 + code for 2 bits, 16 + code for 4 bits).  Key codes and the rotated query use f16 (same MFMA
// rate as bf16, three more significant bits for the query, codes exact either way); value codes and
// probabilities use bf16 (its range is needed for p * value-scale).  Per-token scale and zero-point never touch the
// operands: with one (scale, zero) per token
//     s_mi = scale_i * ( q~_m . (OFFSET + code_i)  -  (OFFSET + z_i) * sum_c q~_mc  -  scale_i * nu'_m )
// where q~ already carries softmax_scale * log2(e) / sqrt(d), and nu'_m = softmax_scale^2 *
// log2(e) * ||q_m||^2 / 24 is the Taylor correction b (Eq. 13 / Eq. 15 with one group) in units of
// scale_i^2 -- one fused multiply-add per cached score, computed from ||q_m||^2 once per row.
// On the value side the value scale is folded into the probability before it is rounded to bf16,
// and the zero-point/OFFSET term is a per-row scalar tau_m = sum_i p'_mi (OFFSET + z_i), accumulated
// from the rounded probabilities so that it cancels exactly.  The cached part of O lives in the
// rotated basis; when the cached keys are done the accumulators are rotated back in registers
// (six butterfly stages inside the lane, one between the lane halves) and the loop continues with
// the current chunk in the original basis.
//
// Current keys/values (unquantized block).  K rows are read straight into A operands; V tiles are
// transposed through LDS (token-major operands); scores get no correction.
//
// The running maximum is exact; accumulators are only rescaled on tiles where some row's maximum
// actually grows.
#include "kvq_internal.h"

namespace kvq {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int D = 128;
constexpr int kWaves = 4;
constexpr int kRowsPerWave = 64;
constexpr int kRowsPerBlock = kWaves * kRowsPerWave;  // 256
constexpr int kStageTiles = 4;
constexpr int kStageKeys = kStageTiles * kTileTokens;  // 128
constexpr int kQRowWords = 68;    // 64 words of f16 pairs + 4 words padding (bank spread)
constexpr int kVtRowWords = 18;   // 32 tokens of bf16 = 16 words + 2 words padding
constexpr float kLog2e = 1.4426950408889634f;

template <int BITS> struct Stage {
    static constexpr int WPL = D * BITS / 64;
    static constexpr int kCodeWords = kStageTiles * 64 * WPL;
    static constexpr int kWords = 2 * kCodeWords + 4 * kStageKeys;  // K codes, V codes, 4 float arrays
};

template <int BITS> constexpr size_t lds_bytes()
{
    // two stage buffers | per-wave query staging (also reused for the V^T tiles) | per-row scalars
    return sizeof(uint32_t) * (2 * Stage<BITS>::kWords + kRowsPerBlock * kQRowWords + 2 * kRowsPerBlock);
}

__device__ inline f32x16 mfma(u32x4 a, u32x4 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                   0, 0, 0);
}

// Same-rate f16 variant, used for the cached-key scores: codes are exact in f16 as well, and the
// rotated, pre-scaled query keeps 11 significant bits instead of 8.
__device__ inline f32x16 mfma_f16(u32x4 a, u32x4 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

__device__ inline uint32_t pack_f16(float lo, float hi)
{
    f32x2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, f16x2));
}

__device__ inline float f16_lo(uint32_t w) { return (float)__builtin_bit_cast(f16x2, w)[0]; }
__device__ inline float f16_hi(uint32_t w) { return (float)__builtin_bit_cast(f16x2, w)[1]; }

__device__ inline uint32_t pack_bf16(float lo, float hi)
{
    f32x2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

// Register j of a packed word: two codes -> two bf16 values OFFSET + code.
template <int BITS> __device__ inline uint32_t unpack_pair(uint32_t w, int j)
{
    if (BITS == 2) {
        const int sh = 5 - 2 * j;
        const uint32_t x = sh >= 0 ? (w << sh) : (w >> (-sh));
        return (x & 0x00600060u) | 0x40804080u;
    } else {
        const int sh = 3 - 4 * j;
        const uint32_t x = sh >= 0 ? (w << sh) : (w >> (-sh));
        return (x & 0x00780078u) | 0x41804180u;
    }
}

// Key codes become f16 values OFFSET + code: the code sits in the top mantissa bits of 4.0 / 16.0.
template <int BITS> __device__ inline uint32_t unpack_pair_f16(uint32_t w, int j)
{
    if (BITS == 2) {
        const int sh = 8 - 2 * j;
        const uint32_t x = sh >= 0 ? (w << sh) : (w >> (-sh));
        return (x & 0x03000300u) | 0x44004400u;
    } else {
        const int sh = 6 - 4 * j;
        const uint32_t x = sh >= 0 ? (w << sh) : (w >> (-sh));
        return (x & 0x03c003c0u) | 0x4c004c00u;
    }
}

// A operand (4 registers) of 16-wide slab `slab` of a key tile, from the lane's WPL code words.
template <int BITS> __device__ inline u32x4 key_operand(const uint32_t *w, int slab)
{
    u32x4 r;
    if (BITS == 2) {
        const uint32_t word = w[slab >> 1];
        const int j0 = 4 * (slab & 1);
        r.x = unpack_pair_f16<2>(word, j0); r.y = unpack_pair_f16<2>(word, j0 + 1);
        r.z = unpack_pair_f16<2>(word, j0 + 2); r.w = unpack_pair_f16<2>(word, j0 + 3);
    } else {
        const uint32_t word = w[slab];
        r.x = unpack_pair_f16<4>(word, 0); r.y = unpack_pair_f16<4>(word, 1);
        r.z = unpack_pair_f16<4>(word, 2); r.w = unpack_pair_f16<4>(word, 3);
    }
    return r;
}

// A operand of a value tile: channel block `blk` (32 channels), token slab `s` (16 tokens).
template <int BITS> __device__ inline u32x4 value_operand(const uint32_t *w, int blk, int s)
{
    u32x4 r;
    if (BITS == 2) {
        const uint32_t word = w[blk];
        const int j0 = 4 * s;
        r.x = unpack_pair<2>(word, j0); r.y = unpack_pair<2>(word, j0 + 1);
        r.z = unpack_pair<2>(word, j0 + 2); r.w = unpack_pair<2>(word, j0 + 3);
    } else {
        const uint32_t word = w[2 * blk + s];
        r.x = unpack_pair<4>(word, 0); r.y = unpack_pair<4>(word, 1);
        r.z = unpack_pair<4>(word, 2); r.w = unpack_pair<4>(word, 3);
    }
    return r;
}

__device__ inline float xhalf(float v) { return __shfl_xor(v, 32); }

struct RowState {
    float m;      // running maximum (log2 domain)
    float l_s;    // this lane's share of the cached partition sum
    float l_r;    // this lane's share of the current partition sum
    float tau;    // this lane's share of sum_i p'_i (OFFSET + z_i)
};

template <int BITS, bool CORR>
__global__ __launch_bounds__(256, 1) void attention_mfma_kernel(AttentionArgs a, int row_blocks)
{
    constexpr int WPL = Stage<BITS>::WPL;
    constexpr int kCodeWords = Stage<BITS>::kCodeWords;
    extern __shared__ __align__(16) uint32_t lds[];
    auto stage_buf = [&](int64_t i) -> uint32_t * { return lds + (i & 1) * Stage<BITS>::kWords; };
    uint32_t *q_stage = lds + 2 * Stage<BITS>::kWords;
    float *row_scal = reinterpret_cast<float *>(q_stage + kRowsPerBlock * kQRowWords);

    const CacheView &cv = a.cv;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n = lane & 31, hh = lane >> 5;

    // Workgroups are handed to the 8 XCDs round-robin; keep all row blocks of a head on one XCD so
    // that its packed cache is fetched into that XCD's L2 once.
    int head, rblk;
    {
        const int bid = blockIdx.x;
        if ((cv.num_heads & 7) == 0) {
            const int xcd = bid & 7, j = bid >> 3;
            head = (j / row_blocks) * 8 + xcd;
            rblk = j % row_blocks;
        } else {
            head = bid / row_blocks;
            rblk = bid % row_blocks;
        }
    }
    const int64_t wave_row0 = (int64_t)rblk * kRowsPerBlock + wave * kRowsPerWave;
    const int64_t head_off = (int64_t)head * a.stride_head;
    const uint16_t *q_base = static_cast<const uint16_t *>(a.q) + head_off;
    const float c_log = a.softmax_scale * kLog2e;

    // ---------------------------------------------------------------- query preparation ----
    // Lane r of the wave rotates query row wave_row0 + r: q~ = Hn q * softmax_scale * log2(e),
    // rounded to f16; nu = ||q||^2; the row sum of the rounded q~ (needed for the zero-point term).
    uint32_t *my_q = q_stage + (wave * kRowsPerWave) * kQRowWords;
    u32x4 qop[2][8];  // B operands of the score MFMA: lane (n, hh) holds channels 16*slab + 8*hh .. +7 of rows n, n + 32
    {
        int64_t row = wave_row0 + lane;
        row = row < a.m ? row : a.m - 1;
        const uint4 *src = reinterpret_cast<const uint4 *>(q_base + row * a.stride_token);
        float x[D];
#pragma unroll
        for (int i = 0; i < D / 8; ++i) {
            const uint4 w = src[i];
            const uint32_t ws[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                x[8 * i + 2 * j] = __uint_as_float(ws[j] << 16);
                x[8 * i + 2 * j + 1] = __uint_as_float(ws[j] & 0xffff0000u);
            }
        }
        float nu = 0.0f;
#pragma unroll
        for (int i = 0; i < D; ++i) nu = fmaf(x[i], x[i], nu);
#pragma unroll
        for (int h = 1; h < D; h <<= 1) {
#pragma unroll
            for (int i = 0; i < D; ++i) {
                if ((i & h) == 0) {
                    const float p = x[i], q2 = x[i + h];
                    x[i] = p + q2;
                    x[i + h] = p - q2;
                }
            }
        }
        const float cq = c_log * 0.088388347648318f;
        // q~ = high + low, both f16: the pair carries ~22 significant bits through the MFMA.
        float ssum = 0.0f;
        uint32_t whi[D / 2], wlo[D / 2];
#pragma unroll
        for (int i = 0; i < D / 2; ++i) {
            const float v0 = x[2 * i] * cq, v1 = x[2 * i + 1] * cq;
            whi[i] = pack_f16(v0, v1);
            const float h0 = f16_lo(whi[i]), h1 = f16_hi(whi[i]);
            wlo[i] = pack_f16(v0 - h0, v1 - h1);
            ssum += (h0 + f16_lo(wlo[i])) + (h1 + f16_hi(wlo[i]));
        }
        row_scal[2 * (wave * kRowsPerWave + lane)] = ssum;
        row_scal[2 * (wave * kRowsPerWave + lane) + 1] = -a.softmax_scale * a.softmax_scale * kLog2e * nu * (1.0f / 24.0f);
        // The staging rows hold the high parts first (read into registers below), then the low parts,
        // which stay in LDS for the whole cached-key loop.
        uint32_t *dst = my_q + lane * kQRowWords;
#pragma unroll
        for (int i = 0; i < D / 8; ++i) {
            u32x4 w;
            w.x = whi[4 * i]; w.y = whi[4 * i + 1]; w.z = whi[4 * i + 2]; w.w = whi[4 * i + 3];
            *reinterpret_cast<u32x4 *>(dst + 4 * i) = w;
        }
        __syncthreads();
        const uint32_t *hsrc = my_q + n * kQRowWords + 4 * hh;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int s = 0; s < 8; ++s)
                qop[rb][s] = *reinterpret_cast<const u32x4 *>(hsrc + 32 * rb * kQRowWords + 8 * s);
        __syncthreads();
#pragma unroll
        for (int i = 0; i < D / 8; ++i) {
            u32x4 w;
            w.x = wlo[4 * i]; w.y = wlo[4 * i + 1]; w.z = wlo[4 * i + 2]; w.w = wlo[4 * i + 3];
            *reinterpret_cast<u32x4 *>(dst + 4 * i) = w;
        }
    }
    __syncthreads();
    float ssum[2], nnu[2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        ssum[rb] = row_scal[2 * (wave * kRowsPerWave + 32 * rb + n)];
        nnu[rb] = row_scal[2 * (wave * kRowsPerWave + 32 * rb + n) + 1];
    }

    const uint32_t *q_lo = my_q + n * kQRowWords + 4 * hh;
    f32x16 o[4][2];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[b][rb][v] = 0.0f;
    RowState st[2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) { st[rb].m = -INFINITY; st[rb].l_s = 0.0f; st[rb].l_r = 0.0f; st[rb].tau = 0.0f; }

    // ---------------------------------------------------------------------- cached keys ----
    if (a.cache_len > 0) {
        const int64_t cs = a.cache_start, ce = a.cache_start + a.cache_len;
        const int64_t t_first = cs / kTileTokens, t_last = (ce - 1) / kTileTokens;
        const int64_t n_stages = (t_last - t_first + kStageTiles) / kStageTiles;
        const int64_t head_tile0 = (int64_t)head * cv.cap_tiles;
        const int64_t meta0 = head_tile0 * kTileTokens;

        // Loader: the stage's K codes, V codes and the four float arrays are contiguous in memory.
        constexpr int kCodeVecs = kCodeWords / 4;          // 16-byte vectors per tensor per stage
        constexpr int kCodeIters = kCodeVecs / 256;        // 1 (2 bit) or 2 (4 bit)
        u32x4 pre_k[kCodeIters], pre_v[kCodeIters];
        f32x2 pre_meta;
        auto prefetch = [&](int64_t stage) {
            const int64_t tile0 = t_first + stage * kStageTiles;
            // Never read past the cache storage: clamp the vector's tile, the data is not used then.
#pragma unroll
            for (int it = 0; it < kCodeIters; ++it) {
                const int vec = tid + 256 * it;
                int64_t tile = tile0 + vec / (16 * WPL);
                tile = tile < cv.cap_tiles ? tile : cv.cap_tiles - 1;
                const int64_t word = (head_tile0 + tile) * (64 * WPL) + (vec % (16 * WPL)) * 4;
                pre_k[it] = *reinterpret_cast<const u32x4 *>(cv.k_codes + word);
                pre_v[it] = *reinterpret_cast<const u32x4 *>(cv.v_codes + word);
            }
            const int arr = tid >> 6, pair = tid & 63;     // 4 arrays x 64 pairs of floats
            int64_t tok = tile0 * kTileTokens + 2 * pair;
            const int64_t cap = cv.cap_tiles * kTileTokens;
            tok = tok < cap ? tok : cap - 2;
            const float *src = arr == 0 ? cv.k_scale : arr == 1 ? cv.k_negzero : arr == 2 ? cv.v_scale : cv.v_zero_off;
            pre_meta = *reinterpret_cast<const f32x2 *>(src + meta0 + tok);
        };
        auto commit = [&](uint32_t *buf) {
#pragma unroll
            for (int it = 0; it < kCodeIters; ++it) {
                const int vec = tid + 256 * it;
                *reinterpret_cast<u32x4 *>(buf + 4 * vec) = pre_k[it];
                *reinterpret_cast<u32x4 *>(buf + kCodeWords + 4 * vec) = pre_v[it];
            }
            *reinterpret_cast<f32x2 *>(reinterpret_cast<float *>(buf + 2 * kCodeWords) + 2 * tid) = pre_meta;
        };

        prefetch(0);
        commit(stage_buf(0));
        __syncthreads();
        for (int64_t stage = 0; stage < n_stages; ++stage) {
            const bool more = stage + 1 < n_stages;
            if (more) prefetch(stage + 1);
            const uint32_t *buf = stage_buf(stage);
            const float *meta = reinterpret_cast<const float *>(buf + 2 * kCodeWords);
            const int64_t tile0 = t_first + stage * kStageTiles;
            const int tiles_here = (int)((t_last - tile0 + 1) < kStageTiles ? (t_last - tile0 + 1) : kStageTiles);
            for (int tl = 0; tl < tiles_here; ++tl) {
                const int64_t tile = tile0 + tl;
                // ---- scores: S^T = K q~^T on raw codes
                uint32_t kw[WPL];
                {
                    const uint32_t *src = buf + tl * 64 * WPL + lane * WPL;
#pragma unroll
                    for (int i = 0; i < WPL / 4; ++i) {
                        const u32x4 w = *reinterpret_cast<const u32x4 *>(src + 4 * i);
                        kw[4 * i] = w.x; kw[4 * i + 1] = w.y; kw[4 * i + 2] = w.z; kw[4 * i + 3] = w.w;
                    }
                }
                f32x16 s[2];
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) s[rb][v] = 0.0f;
                // Opaque copy of the address so the loads below are issued per tile instead of being
                // hoisted out of the loop into registers that do not exist.
                const uint32_t *q_lo_t = q_lo;
                asm volatile("" : "+v"(q_lo_t));
#pragma unroll
                for (int slab = 0; slab < 8; ++slab) {
                    const u32x4 kop = key_operand<BITS>(kw, slab);
                    s[0] = mfma_f16(kop, qop[0][slab], s[0]);
                    s[1] = mfma_f16(kop, qop[1][slab], s[1]);
                    // low parts of q~ stay in LDS (the register file is full): 2 x 16 bytes per slab
                    const u32x4 lo0 = *reinterpret_cast<const u32x4 *>(q_lo_t + 8 * slab);
                    const u32x4 lo1 = *reinterpret_cast<const u32x4 *>(q_lo_t + 32 * kQRowWords + 8 * slab);
                    s[0] = mfma_f16(kop, lo0, s[0]);
                    s[1] = mfma_f16(kop, lo1, s[1]);
                }
                // ---- per-key constants of the 16 keys this lane sees: keys 8g + 4hh + 0..3, g = 0..3
                float k_scale[16], k_nz[16], v_scale[16], v_zo[16];
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int key = tl * kTileTokens + 8 * g + 4 * hh;
                    const float4 c0 = *reinterpret_cast<const float4 *>(meta + key);
                    const float4 c1 = *reinterpret_cast<const float4 *>(meta + kStageKeys + key);
                    const float4 c2 = *reinterpret_cast<const float4 *>(meta + 2 * kStageKeys + key);
                    const float4 c3 = *reinterpret_cast<const float4 *>(meta + 3 * kStageKeys + key);
                    k_scale[4 * g] = c0.x; k_scale[4 * g + 1] = c0.y; k_scale[4 * g + 2] = c0.z; k_scale[4 * g + 3] = c0.w;
                    k_nz[4 * g] = c1.x; k_nz[4 * g + 1] = c1.y; k_nz[4 * g + 2] = c1.z; k_nz[4 * g + 3] = c1.w;
                    v_scale[4 * g] = c2.x; v_scale[4 * g + 1] = c2.y; v_scale[4 * g + 2] = c2.z; v_scale[4 * g + 3] = c2.w;
                    v_zo[4 * g] = c3.x; v_zo[4 * g + 1] = c3.y; v_zo[4 * g + 2] = c3.z; v_zo[4 * g + 3] = c3.w;
                }
                const int64_t key_base = tile * kTileTokens + 4 * hh;
                const bool edge = key_base - 4 * hh < cs || key_base - 4 * hh + kTileTokens > ce;
                // ---- softmax on the two 32-row blocks
                u32x4 pop[2][2];
#pragma unroll
                for (int rb = 0; rb < 2; ++rb) {
                    float t[16];
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        float x = fmaf(k_nz[v], ssum[rb], s[rb][v]);
                        if (CORR) x = fmaf(k_scale[v], nnu[rb], x);
                        t[v] = k_scale[v] * x;
                    }
                    if (edge) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int64_t key = key_base + 8 * (v >> 2) + (v & 3);
                            t[v] = (key >= cs && key < ce) ? t[v] : -INFINITY;
                        }
                    }
                    float tmax = t[0];
#pragma unroll
                    for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, t[v]);
                    tmax = fmaxf(tmax, xhalf(tmax));
                    const float m_new = fmaxf(st[rb].m, tmax);
                    const float m_use = m_new == -INFINITY ? 0.0f : m_new;
                    if (__any(m_new > st[rb].m)) {
                        const float alpha = __builtin_amdgcn_exp2f(st[rb].m - m_use);
                        st[rb].l_s *= alpha;
                        st[rb].tau *= alpha;
#pragma unroll
                        for (int b = 0; b < 4; ++b)
#pragma unroll
                            for (int v = 0; v < 16; ++v) o[b][rb][v] *= alpha;
                        st[rb].m = m_new;
                    }
                    float lsum = 0.0f, tau = 0.0f;
                    uint32_t pw[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const float p0 = __builtin_amdgcn_exp2f(t[2 * i] - m_use);
                        const float p1 = __builtin_amdgcn_exp2f(t[2 * i + 1] - m_use);
                        lsum += p0 + p1;
                        pw[i] = pack_bf16(p0 * v_scale[2 * i], p1 * v_scale[2 * i + 1]);
                        tau = fmaf(__uint_as_float(pw[i] << 16), v_zo[2 * i], tau);
                        tau = fmaf(__uint_as_float(pw[i] & 0xffff0000u), v_zo[2 * i + 1], tau);
                    }
                    st[rb].l_s += lsum;
                    st[rb].tau += tau;
                    pop[rb][0].x = pw[0]; pop[rb][0].y = pw[1]; pop[rb][0].z = pw[2]; pop[rb][0].w = pw[3];
                    pop[rb][1].x = pw[4]; pop[rb][1].y = pw[5]; pop[rb][1].z = pw[6]; pop[rb][1].w = pw[7];
                }
                // ---- O^T += V^T P^T on raw codes
                uint32_t vw[WPL];
                {
                    const uint32_t *src = buf + kCodeWords + tl * 64 * WPL + lane * WPL;
#pragma unroll
                    for (int i = 0; i < WPL / 4; ++i) {
                        const u32x4 w = *reinterpret_cast<const u32x4 *>(src + 4 * i);
                        vw[4 * i] = w.x; vw[4 * i + 1] = w.y; vw[4 * i + 2] = w.z; vw[4 * i + 3] = w.w;
                    }
                }
#pragma unroll
                for (int b = 0; b < 4; ++b) {
#pragma unroll
                    for (int sl = 0; sl < 2; ++sl) {
                        const u32x4 vop = value_operand<BITS>(vw, b, sl);
                        o[b][0] = mfma(vop, pop[0][sl], o[b][0]);
                        o[b][1] = mfma(vop, pop[1][sl], o[b][1]);
                    }
                }
            }
            if (more) commit(stage_buf(stage + 1));
            __syncthreads();
        }

        // ---- leave the rotated basis: O <- Hn^T (O_rot - tau 1).  Channel index of register
        // (b, v) in lane half hh: c = 32 b + 8 (v >> 2) + 4 hh + (v & 3).
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            // bits 0, 1 (v bits 0, 1) and bits 3, 4 (v bits 2, 3)
#pragma unroll
            for (int h = 1; h < 16; h <<= 1) {
#pragma unroll
                for (int b = 0; b < 4; ++b)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        if ((v & h) == 0) {
                            const float p = o[b][rb][v], q2 = o[b][rb][v + h];
                            o[b][rb][v] = p + q2;
                            o[b][rb][v + h] = p - q2;
                        }
            }
            // bits 5, 6 (channel block)
#pragma unroll
            for (int h = 1; h < 4; h <<= 1) {
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    if ((b & h) == 0) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const float p = o[b][rb][v], q2 = o[b + h][rb][v];
                            o[b][rb][v] = p + q2;
                            o[b + h][rb][v] = p - q2;
                        }
                    }
            }
            // bit 2 lives in the lane half
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float own = o[b][rb][v], other = xhalf(own);
                    o[b][rb][v] = (hh ? other - own : own + other) * 0.088388347648318f;
                }
            // Hn^T (tau 1) = tau sqrt(d) e_0: only channel 0 (lane half 0, block 0, register 0) sees it.
            const float tau_all = st[rb].tau + xhalf(st[rb].tau);
            if (hh == 0) o[0][rb][0] -= tau_all * 11.313708498984761f;
        }
    }

    // --------------------------------------------------------------------- current keys ----
    if (a.n_cur > 0) {
        const uint16_t *k_base = static_cast<const uint16_t *>(a.k_cur) + head_off;
        const uint16_t *v_base = static_cast<const uint16_t *>(a.v_cur) + head_off;
        // B operands: the raw (unrotated, unscaled) bf16 queries.
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            int64_t row = wave_row0 + 32 * rb + n;
            row = row < a.m ? row : a.m - 1;
            const uint16_t *src = q_base + row * a.stride_token + 8 * hh;
#pragma unroll
            for (int s = 0; s < 8; ++s) qop[rb][s] = *reinterpret_cast<const u32x4 *>(src + 16 * s);
        }
        // V^T staging: two buffers of 128 channel rows x 32 tokens (bf16), reusing the query staging area.
        __syncthreads();
        auto vt = [&](int64_t i) -> uint16_t * { return reinterpret_cast<uint16_t *>(q_stage + (i & 1) * D * kVtRowWords); };
        const int64_t n_tiles = (a.n_cur + kTileTokens - 1) / kTileTokens;
        u32x4 pre_vt[2];
        const int ld_key = tid & 31, ld_oct = tid >> 5;  // octets ld_oct and ld_oct + 8
        auto prefetch_v = [&](int64_t tile) {
            int64_t key = tile * kTileTokens + ld_key;
            key = key < a.n_cur ? key : a.n_cur - 1;
            const uint16_t *src = v_base + key * a.stride_token;
            pre_vt[0] = *reinterpret_cast<const u32x4 *>(src + 8 * ld_oct);
            pre_vt[1] = *reinterpret_cast<const u32x4 *>(src + 8 * (ld_oct + 8));
        };
        auto commit_v = [&](uint16_t *buf) {
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const uint32_t ws[4] = {pre_vt[it].x, pre_vt[it].y, pre_vt[it].z, pre_vt[it].w};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int ch = 8 * (ld_oct + 8 * it) + e;
                    const uint16_t val = (uint16_t)(e & 1 ? ws[e >> 1] >> 16 : ws[e >> 1] & 0xffffu);
                    buf[ch * (2 * kVtRowWords) + ld_key] = val;
                }
            }
        };
        prefetch_v(0);
        commit_v(vt(0));
        __syncthreads();
        for (int64_t tile = 0; tile < n_tiles; ++tile) {
            const bool more = tile + 1 < n_tiles;
            if (more) prefetch_v(tile + 1);
            // ---- scores S^T = K q^T, K rows straight from memory
            f32x16 s[2];
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int v = 0; v < 16; ++v) s[rb][v] = 0.0f;
            {
                int64_t key = tile * kTileTokens + n;
                key = key < a.n_cur ? key : a.n_cur - 1;
                const uint16_t *src = k_base + key * a.stride_token + 8 * hh;
                u32x4 kop[8];
#pragma unroll
                for (int slab = 0; slab < 8; ++slab) kop[slab] = *reinterpret_cast<const u32x4 *>(src + 16 * slab);
#pragma unroll
                for (int slab = 0; slab < 8; ++slab) {
                    s[0] = mfma(kop[slab], qop[0][slab], s[0]);
                    s[1] = mfma(kop[slab], qop[1][slab], s[1]);
                }
            }
            const int64_t key_base = tile * kTileTokens + 4 * hh;
            const bool edge = (tile + 1) * kTileTokens > a.n_cur;
            u32x4 pop[2][2];
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                float t[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) t[v] = s[rb][v] * c_log;
                if (edge) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int64_t key = key_base + 8 * (v >> 2) + (v & 3);
                        t[v] = key < a.n_cur ? t[v] : -INFINITY;
                    }
                }
                float tmax = t[0];
#pragma unroll
                for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, t[v]);
                tmax = fmaxf(tmax, xhalf(tmax));
                const float m_new = fmaxf(st[rb].m, tmax);
                const float m_use = m_new == -INFINITY ? 0.0f : m_new;
                if (__any(m_new > st[rb].m)) {
                    const float alpha = __builtin_amdgcn_exp2f(st[rb].m - m_use);
                    st[rb].l_s *= alpha;
                    st[rb].l_r *= alpha;
#pragma unroll
                    for (int b = 0; b < 4; ++b)
#pragma unroll
                        for (int v = 0; v < 16; ++v) o[b][rb][v] *= alpha;
                    st[rb].m = m_new;
                }
                float lsum = 0.0f;
                uint32_t pw[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float p0 = __builtin_amdgcn_exp2f(t[2 * i] - m_use);
                    const float p1 = __builtin_amdgcn_exp2f(t[2 * i + 1] - m_use);
                    lsum += p0 + p1;
                    pw[i] = pack_bf16(p0, p1);
                }
                st[rb].l_r += lsum;
                pop[rb][0].x = pw[0]; pop[rb][0].y = pw[1]; pop[rb][0].z = pw[2]; pop[rb][0].w = pw[3];
                pop[rb][1].x = pw[4]; pop[rb][1].y = pw[5]; pop[rb][1].z = pw[6]; pop[rb][1].w = pw[7];
            }
            // ---- O^T += V^T P^T, V^T from LDS: tokens 16 sl + 4 hh + 0..3 and 16 sl + 8 + 4 hh + 0..3
            const uint32_t *vsrc = reinterpret_cast<const uint32_t *>(vt(tile));
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const uint32_t *rowp = vsrc + (32 * b + n) * kVtRowWords + 2 * hh;
#pragma unroll
                for (int sl = 0; sl < 2; ++sl) {
                    const u32x2 lo = *reinterpret_cast<const u32x2 *>(rowp + 8 * sl);
                    const u32x2 hi = *reinterpret_cast<const u32x2 *>(rowp + 8 * sl + 4);
                    u32x4 vop;
                    vop.x = lo.x; vop.y = lo.y; vop.z = hi.x; vop.w = hi.y;
                    o[b][0] = mfma(vop, pop[0][sl], o[b][0]);
                    o[b][1] = mfma(vop, pop[1][sl], o[b][1]);
                }
            }
            if (more) commit_v(vt(tile + 1));
            __syncthreads();
        }
    }

    // ------------------------------------------------------------------------- epilogue ----
    uint16_t *out_base = static_cast<uint16_t *>(a.out) + head_off;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        const float l_s = st[rb].l_s + xhalf(st[rb].l_s);
        const float l_r = st[rb].l_r + xhalf(st[rb].l_r);
        const float inv = 1.0f / (l_s + l_r);
        const int64_t row = wave_row0 + 32 * rb + n;
        if (row < a.m) {
            uint16_t *dst = out_base + row * a.stride_token + 4 * hh;
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    u32x2 w;
                    w.x = pack_bf16(o[b][rb][4 * g] * inv, o[b][rb][4 * g + 1] * inv);
                    w.y = pack_bf16(o[b][rb][4 * g + 2] * inv, o[b][rb][4 * g + 3] * inv);
                    *reinterpret_cast<u32x2 *>(dst + 32 * b + 8 * g) = w;
                }
            if (a.mass_cached && hh == 0) a.mass_cached[(int64_t)head * a.m + row] = l_s * inv;
        }
    }
}

template <int BITS, bool CORR> hipError_t launch(const AttentionArgs &a, hipStream_t stream)
{
    static bool configured = false;  // per instantiation; the attribute is a property of the kernel
    const void *fn = reinterpret_cast<const void *>(&attention_mfma_kernel<BITS, CORR>);
    if (!configured) {
        const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes<BITS>());
        if (e != hipSuccess) return e;
        configured = true;
    }
    const int row_blocks = (int)((a.m + kRowsPerBlock - 1) / kRowsPerBlock);
    const int64_t blocks = (int64_t)row_blocks * a.cv.num_heads;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL((attention_mfma_kernel<BITS, CORR>), dim3((unsigned)blocks), dim3(256), lds_bytes<BITS>(), stream,
                       a, row_blocks);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attention_mfma(const AttentionArgs &a, hipStream_t stream)
{
    if (a.cv.head_dim != D || a.cv.io_dtype != KVQ_BF16) return hipErrorInvalidValue;
    if (a.cv.bits == 2) return a.correction ? launch<2, true>(a, stream) : launch<2, false>(a, stream);
    if (a.cv.bits == 4) return a.correction ? launch<4, true>(a, stream) : launch<4, false>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace kvq
