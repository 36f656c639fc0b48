// Matrix-core chunk attention for gfx950: BF16 I/O, head_dim 128, 2- or 4-bit cache with one (scale, zero-point)
// per token (fp32 or FP8/BF16 metadata) or with per-channel keys (see PERCH below).
//
// Work split.  One workgroup = 4 wavefronts = 256 query rows of one head; each wavefront owns
// 64 rows (two 32-row blocks) for the whole key loop, so the waves only meet at one barrier per
// 128 staged keys.  Everything is computed transposed,
//     S^T = K Q~^T           (A operand: keys,     B operand: queries)
//     O^T = V^T P^T          (A operand: channels, B operand: queries)
// with v_mfma_f32_32x32x16.  In that orientation a lane owns one query row (row = lane mod 32) of
// every result tile, so the softmax row maximum and row sum are reductions inside a lane plus one
// exchange between the two lane halves, and the probabilities the score MFMA leaves in a lane are
// exactly that lane's B operand of the P*V MFMA -- no shuffle, no LDS round trip for P.
//
// Cached keys/values (Alg. 1 of the paper, cached block).  Packed tiles (see kvq_internal.h) are
// staged through LDS 128 keys at a time (four buffers, one barrier per stage).  A lane pulls its 16
// or 32 bytes of codes and turns every word into MFMA operand registers with an and-or per register
// and a shift per one to three registers: the code lands in mantissa bits of a 16-bit float whose
// exponent makes the value BASE + weight * code (see "Unpacking" below).  Key codes and the rotated
// query use f16 (same MFMA rate as bf16, three more significant bits; codes are exact either way) and
// the query is carried as an f16 high part plus a low part (f16, or FP8 where the switches below say so);
// value codes and probabilities use bf16 (its range is needed for p * value-scale).  The 2-bit keys of
// per-token caches take a shorter way (KVQ_KEYS_FP4 below): the codes are FP4 values as they stand and the query
// is four FP6 pieces, multiplied by the block-scaled 64-channel MFMA at twice the FP8 rate.  Per-token scale and zero-point never touch the operands: with one
// (scale, zero) per token
//     s_mi = scale_i * ( q~_m . (BASE + code_i)  -  z_i * sum_c q~_mc  -  BASE * W_m  -  scale_i * nu'_m )
// where q~ already carries softmax_scale * log2(e) / sqrt(d), W_m is the sum of the operand values of
// the row, and nu'_m = softmax_scale^2 * log2(e) * ||q_m||^2 / 24 is the Taylor correction b (Eq. 13 /
// Eq. 15 with one group) in units of scale_i^2, from ||q_m||^2 computed once per row.  The rank-one
// terms ride on the matrix cores as well: the loader turns (zero, scale, window mask) of each key into
// one more 16-wide A operand, the row constants form its B operand, split into bf16 pieces that add up
// to fp32 accuracy.  The correction therefore costs no vector instruction at all; what is left per
// score is one fused multiply-add (scale, minus the reference maximum), the exponential and the P*V
// bookkeeping.  On the value side the value scale is folded into the probability before it is rounded
// to bf16 -- as log2(value scale) / scale_i in two spare slots of that same constant-term operand, so
// that 2^e already is p' = p * value scale and the row sum takes p back as p' / value scale in one fused
// multiply-add -- and the zero-point/BASE term is a per-row scalar tau_m = sum_i p'_mi (BASE + z_i),
// accumulated from the rounded probabilities (dot2 on bf16 pairs) so that it cancels exactly.  The
// cached part of O lives in the rotated basis; when the cached keys are done the accumulators are
// rotated back in registers (six butterfly stages inside the lane, one between the lane halves) and
// the loop continues with the current chunk in the original basis.
//
// Software pipeline.  One iteration issues the score MFMAs of tile t+1 next to the exponentials of
// tile t, then the P*V MFMAs of tile t next to the scaling of the scores of tile t+1, so that a single
// wave per SIMD keeps the matrix pipe and the vector ALU busy at the same time.
//
// Online softmax.  Each row keeps a reference maximum m and the partial sums l_S, l_R.  The reference
// only moves when a tile's maximum exceeds it by more than 2^8 (results stay exact: a stale reference
// just scales numerator and denominator alike); that rare case leaves the fast loop, rescales, and
// re-enters, which keeps the accumulators pinned in their registers inside the loop.
//
// Current keys/values (unquantized block, kvq_mfma_current_phase.inc).  K rows are staged through LDS one tile
// ahead, V tiles are transposed through LDS (token-major operands); scores get no correction.
#include "kvq_internal.h"

// 1: the rotated query enters the score MFMAs as an f16 high part plus an f16 low part (two MFMAs per
// slab and row block); 0: high part only.
#ifndef KVQ_Q_LOW_PART
#define KVQ_Q_LOW_PART 1
#endif
// Number of 16-channel slabs whose low query parts stay in accumulation registers instead of being read
// from LDS for every key tile (4 registers per slab and 32-row block).  With 4 the 4-bit kernel spills, and
// a spill reload lands in the loader behind the prefetch loads, where it waits for them on every stage;
// with 2 nothing spills (9.60 -> 9.31 ms at 4 bits on the benchmark shape).
#ifndef KVQ_Q_LOW_RESIDENT_SLABS
#define KVQ_Q_LOW_RESIDENT_SLABS 2
#endif
// 1 (2-bit caches only): the low query part is an FP8 E4M3 operand with one power-of-two scale per row and
// meets the key codes in v_mfma_scale_f32_32x32x64_f8f6f4 (64 channels per instruction at twice the
// 16-bit rate): 4 MFMAs per key tile instead of 16, the whole low part resident in 32 accumulation
// registers.  0: f16 low part as for 4-bit caches.
// 1 (2-bit caches, not the per-channel path): the key codes are the MFMA operand.  E2M1 encodes 0, 0.5, 1, 1.5 as
// 0..3, so a packed word is two FP4 operand registers (w & 0x33333333, (w >> 2) & 0x33333333); the query is four
// FP6 (E2M3) pieces n_k / 2 with one power-of-two scale per row and piece, n_k integers of at most four bits plus
// sign, each piece four bits finer than the one before.  16 v_mfma_scale_f32_32x32x64_f8f6f4 (FP4 x FP6) per key
// tile replace 16 f16 and 4 FP8 MFMAs, 12 unpacking instructions replace 64, the BASE term vanishes (W = 0), and
// the 96 piece registers live where the 64 + 32 registers of the high and low parts lived.  0: high + low pair.
#ifndef KVQ_KEYS_FP4
#define KVQ_KEYS_FP4 1
#endif
#ifndef KVQ_Q_LOW_FP8
#define KVQ_Q_LOW_FP8 1
#endif
// 1 (kernels with FP4 key operands): the score MFMAs are written out with vector-register destinations, so that no
// score has to be copied out of an accumulation register before the vector ALU can scale it (32 copies per key tile).
#ifndef KVQ_SCORES_IN_VGPRS
#define KVQ_SCORES_IN_VGPRS 1
#endif
// 1 (same kernels): the fast loop is unrolled over the four tiles of a stage, which turns a tile's place inside its
// stage buffer into immediate offsets and the stage opening into straight-line code.
#ifndef KVQ_UNROLL_STAGE
#define KVQ_UNROLL_STAGE 1
#endif

namespace kvq {
namespace {

#define KVQ_INT4_KEY_SHARE 1   // 4-bit key pairs share their shifts two by two (kvq_mfma_common.h)
#include "kvq_mfma_common.h"

constexpr int kBuffers = 4;    // power of two: buffer index = stage & 3

// Word offsets inside one stage buffer.
template <int BITS> struct Stage {
    static constexpr int WPL = D * BITS / 64;
    static constexpr int kCodeWords = kStageTiles * 64 * WPL;   // per tensor
    static constexpr int kK = 0;
    static constexpr int kV = kCodeWords;
    static constexpr int kCop = 2 * kCodeWords;                 // [tile][lane][4]  constant-term A operand
    static constexpr int kKScale = kCop + kStageTiles * 64 * 4; // [tile][hh][16]   float
    static constexpr int kVScale = kKScale + kStageKeys;        // [tile][hh][16]   float: 1 / (value scale * 4^g)
    static constexpr int kVzHi = kVScale + kStageKeys;          // [tile][hh][8]    bf16 pairs
    static constexpr int kVzLo = kVzHi + kStageKeys / 2;
    static constexpr int kFlags = kVzLo + kStageKeys / 2;       // 2 words: "some low zero-point part is nonzero"
    static constexpr int kWords = kFlags + 4;
};

template <int BITS> constexpr size_t lds_bytes()
{
    // stage buffers | per-wave low parts of q~ (also staging for the query prep and the V^T tiles) | row scalars
    return sizeof(uint32_t) * (kBuffers * Stage<BITS>::kWords + kRowsPerBlock * kQRowWords + 4 * kRowsPerBlock);
}


// FP8META: the cache holds one FP8 E4M3 scale and one BF16 zero-point per token instead of two floats.
// PERCH: keys quantized per channel and appended block (appendix on per-channel quantization).  Inside a block
// the channel steps go into the query operand, q'_c = q~_c * step_c, after which the block looks like a
// per-token cache with step 1 and zero-point 0 whose rows carry two constants: Z = sum_c q'_c z_c and the
// block's correction sigma^2 / 24 * sum_c (q^_c step_c)^2.  The cached keys are therefore processed block by
// block, the query operands prepared anew for each.
template <int BITS, bool CORR, bool FP8META, bool PERCH = false>
__global__ __launch_bounds__(kThreads, 1) void attention_mfma_kernel(AttentionArgs a, int row_blocks)
{
    if (cache_flagged(a.status)) return;   // the vector kernel enqueued behind this launch serves such a cache
    using St = Stage<BITS>;
    constexpr int WPL = St::WPL;
    extern __shared__ __align__(16) uint32_t lds[];
    uint32_t *q_stage = lds + kBuffers * St::kWords;
    float *row_scal = reinterpret_cast<float *>(q_stage + kRowsPerBlock * kQRowWords);

    const CacheView &cv = a.cv;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n = lane & 31, hh = lane >> 5;

    // Workgroups are handed to the 8 XCDs round-robin; keep all row blocks of all query heads of a
    // key/value head on one XCD so that its packed cache is fetched into that XCD's L2 once.
    int head, qhead, rblk;   // key/value head, query head, 256-row block
    {
        const int bid = blockIdx.x;
        const int per_head = row_blocks * a.q_per_kv;
        int j;
        if ((cv.num_heads & 7) == 0) {
            const int xcd = bid & 7;
            j = bid >> 3;
            head = (j / per_head) * 8 + xcd;
        } else {
            j = bid;
            head = j / per_head;
        }
        const int local = j % per_head;
        qhead = head * a.q_per_kv + local / row_blocks;
        rblk = local % row_blocks;
    }
    const int64_t wave_row0 = (int64_t)rblk * kRowsPerBlock + wave * kRowsPerWave;
    const int64_t head_off = (int64_t)head * a.stride_head;          // k_cur / v_cur
    const int64_t qhead_off = (int64_t)qhead * a.q_stride_head;      // q / out
    const uint16_t *q_base = static_cast<const uint16_t *>(a.q) + qhead_off;
    const float c_log = a.softmax_scale * kLog2e;
    const UnpackConsts uc = make_unpack_consts<BITS>();

    // ---------------------------------------------------------------- query preparation ----
    // kPrepLanes adjacent lanes rotate one query row of the block: q~ = Hn q * softmax_scale * log2(e),
    // split into an f16 high and low part; nu = ||q||^2; the row sum of the (high + low) parts.
    constexpr bool kFp4 = KVQ_KEYS_FP4 && BITS == 2 && !PERCH;
    constexpr bool kVs = KVQ_SCORES_IN_VGPRS && kFp4;   // score tile in vector registers (written-out MFMAs)
    constexpr bool kLoFp8 = KVQ_Q_LOW_PART && KVQ_Q_LOW_FP8 && BITS == 2 && !kFp4;
    constexpr bool kLoF16 = KVQ_Q_LOW_PART && !kLoFp8 && !kFp4;
    constexpr int kPrepLanes = kThreads / kRowsPerBlock;   // 1 or 2
    constexpr int kPrepCh = D / kPrepLanes;                 // channels per lane
    // FP4 keys: the query as four FP6 (E2M3) pieces, B operands of the 64-channel MFMAs: [row block][piece][MFMA]
    i32x6 qp[kRB][4][2];
    u32x4 qop[kRB][8];  // B operands of the score MFMA: lane (n, hh) holds channels 16*slab + 8*hh .. +7 of rows n + 32 rb
    {
        const int prow = tid / kPrepLanes, ppart = tid % kPrepLanes;
        int64_t row = (int64_t)rblk * kRowsPerBlock + prow;
        row = row < a.m ? row : a.m - 1;
        const uint4 *src = reinterpret_cast<const uint4 *>(q_base + row * a.q_stride_token + ppart * kPrepCh);
        float x[kPrepCh];
#pragma unroll
        for (int i = 0; i < kPrepCh / 8; ++i) {
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
        for (int i = 0; i < kPrepCh; ++i) nu = fmaf(x[i], x[i], nu);
        // Randomised rotation: the channel signs come before the Hadamard matrix.
        if (has_signs(a.cv))
#pragma unroll
        for (int w = 0; w < kPrepCh / 32; ++w) {
            const uint32_t sg = sign_bits_from(a.cv, ppart * kPrepCh + 32 * w);
#pragma unroll
            for (int i = 0; i < 32; ++i) x[32 * w + i] = flip_sign(x[32 * w + i], sg >> i);
        }
#pragma unroll
        for (int h = 1; h < kPrepCh; h <<= 1) {
#pragma unroll
            for (int i = 0; i < kPrepCh; ++i) {
                if ((i & h) == 0) {
                    const float p = x[i], q2 = x[i + h];
                    x[i] = p + q2;
                    x[i + h] = p - q2;
                }
            }
        }
        if constexpr (kPrepLanes == 2) {   // last butterfly stage: between the two lanes of the row
            nu += __shfl_xor(nu, 1);
#pragma unroll
            for (int i = 0; i < kPrepCh; ++i) {
                const float other = __shfl_xor(x[i], 1);
                x[i] = ppart ? other - x[i] : x[i] + other;
            }
        }
        // Channel c of the operand carries 4^g(c) (the inverse of the weight its key codes are unpacked with).
        const float cq = c_log * 0.088388347648318f;
#pragma unroll
        for (int i = 0; i < kPrepCh; ++i) x[i] *= cq * (kFp4 ? 1.0f : (float)(1 << (Unpack<BITS>::kClassBits * key_channel_class<BITS>(i))));
        // The staging rows hold the high parts first (read into registers below), then the low parts,
        // which stay in LDS for the whole cached-key loop.
        uint32_t *dst = q_stage + prow * kQRowWords + ppart * (kPrepCh / 2);
        if constexpr (!kFp4) {
#pragma unroll
        for (int i = 0; i < kPrepCh / 8; ++i) {
            u32x4 w;
            w.x = pack_f16(x[8 * i], x[8 * i + 1]); w.y = pack_f16(x[8 * i + 2], x[8 * i + 3]);
            w.z = pack_f16(x[8 * i + 4], x[8 * i + 5]); w.w = pack_f16(x[8 * i + 6], x[8 * i + 7]);
            *reinterpret_cast<u32x4 *>(dst + 4 * i) = w;
        }
        __syncthreads();
        const uint32_t *hsrc = q_stage + (wave * kRowsPerWave + n) * kQRowWords + 4 * hh;
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
            for (int s = 0; s < 8; ++s)
                qop[rb][s] = *reinterpret_cast<const u32x4 *>(hsrc + 32 * rb * kQRowWords + 8 * s);
        __syncthreads();
        }
        float ssum = 0.0f, ssum_w = 0.0f;   // sum of q~ (true scale), sum of the weighted operand values
        if constexpr (kFp4) {
            static_assert(!kFp4 || kPrepLanes == 1, "one lane prepares a whole row");
            // q~ = sum of four pieces n_k / 2 * 2^e_k, n_k integers of magnitude up to 15 (n / 2 is an E2M3 value),
            // e_0 = e0 with the row maximum in (3.75, 7.5] * 2^e0, e_k = e0 - 4 k - 1 after that.  What piece 0
            // leaves is at most a quarter of its scale, i.e. 16 half-steps of piece 1: five bits finer, and the one
            // value in 33 that does not fit (16) is clamped to 15, which leaves the next piece a whole step of its
            // predecessor instead of half a step -- again 16 of its own half-steps, clamped likewise.  The last
            // step is 2^(e0 - 14); the error is a quarter of it, half of it after a clamp.
            float mx = 0.0f;
#pragma unroll
            for (int c = 0; c < kPrepCh; ++c) {
                mx = fmaxf(mx, fabsf(x[c]));
                ssum += x[c];
            }
            int e0 = (int)((__float_as_uint(mx * (1.0f / 7.5f)) >> 23) & 0xffu) - 126;
            e0 = e0 < -100 ? -100 : e0 > 110 ? 110 : e0;
            uint32_t scale_word = 0u;
#pragma unroll
            for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    const int ek = e0 - 4 * (2 * pass + kk) - (2 * pass + kk > 0 ? 1 : 0);
                    const float half = __uint_as_float((uint32_t)(127 + ek - 1) << 23);
                    const float inv = __uint_as_float((uint32_t)(127 - ek + 1) << 23);
                    // the key operand holds code / 2: one more factor of two in the scale byte
                    scale_word |= (uint32_t)(127 + ek + 1) << (8 * (2 * pass + kk));
#pragma unroll
                    for (int op = 0; op < 4; ++op) {       // MFMA jm = op >> 1, lane half hw = op & 1
                        const int jm = op >> 1, hw = op & 1;
                        uint32_t d[6] = {0u, 0u, 0u, 0u, 0u, 0u};
#pragma unroll
                        for (int j = 0; j < 32; ++j) {
                            // element j of the lane's FP4 key operand: word 2 jm + (j >> 4), 2-bit field
                            // 2 (j & 7) + ((j >> 3) & 1) of it; the channel that field holds (see key_pair)
                            const int wd = 2 * jm + (j >> 4), f = 2 * (j & 7) + ((j >> 3) & 1);
                            const int pr = f & 7, slab = 2 * wd + (pr >> 2);
                            const int c = 16 * slab + 8 * hw + 2 * (pr & 3) + (f >> 3);
                            const float nn = fminf(fmaxf(rintf(x[c] * inv), -15.0f), 15.0f);
                            x[c] = fmaf(-nn, half, x[c]);
                            // E2M3 code of |n| / 2: 4 n below 4, 2 n + 8 below 8, n + 16 from there on
                            const float an = fabsf(nn);
                            const uint32_t mag = (uint32_t)fminf(fminf(4.0f * an, fmaf(2.0f, an, 8.0f)), an + 16.0f);
                            const uint32_t code = mag | ((__float_as_uint(nn) >> 26) & 32u);
                            const int bit = 6 * j;
                            d[bit >> 5] |= code << (bit & 31);
                            if ((bit & 31) > 26) d[(bit >> 5) + 1] |= code >> (32 - (bit & 31));
                        }
                        uint32_t *pd = q_stage + prow * kQRowWords + (2 * kk + jm) * 12 + hw * 6;
#pragma unroll
                        for (int i = 0; i < 6; i += 2) *reinterpret_cast<u32x2 *>(pd + i) = u32x2{d[i], d[i + 1]};
                    }
                }
                __syncthreads();
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                        for (int jm = 0; jm < 2; ++jm) {
                            const uint32_t *ps = q_stage + (wave * kRowsPerWave + 32 * rb + n) * kQRowWords + (2 * kk + jm) * 12 + hh * 6;
                            const u32x2 p0 = *reinterpret_cast<const u32x2 *>(ps), p1 = *reinterpret_cast<const u32x2 *>(ps + 2),
                                        p2 = *reinterpret_cast<const u32x2 *>(ps + 4);
                            qp[rb][2 * pass + kk][jm] = i32x6{(int)p0.x, (int)p0.y, (int)p1.x, (int)p1.y, (int)p2.x, (int)p2.y};
                        }
                __syncthreads();
            }
            // the row sum of what the pieces hold: the sum of q~ minus the sum of what is left of it
#pragma unroll
            for (int c = 0; c < kPrepCh; ++c) ssum -= x[c];
            row_scal[4 * prow + 3] = __uint_as_float(scale_word);
        } else if constexpr (kLoFp8) {
            static_assert(!kLoFp8 || kPrepLanes == 1, "one lane prepares a whole row");
            // Low parts at true scale (the weight 4^g of the high operand taken out again: exact), their
            // largest magnitude, and from it the row's power-of-two scale: the largest low part lands in
            // [128, 256), inside the E4M3 range.
            float lo_t[kPrepCh], mx = 0.0f;
#pragma unroll
            for (int c = 0; c < kPrepCh; c += 2) {
                const uint32_t hi = pack_f16(x[c], x[c + 1]);
                const float wgt = 1.0f / (float)(1 << (Unpack<BITS>::kClassBits * key_channel_class<BITS>(c)));   // both channels share a class
                lo_t[c] = (x[c] - f16_lo(hi)) * wgt;
                lo_t[c + 1] = (x[c + 1] - f16_hi(hi)) * wgt;
                mx = fmaxf(mx, fmaxf(fabsf(lo_t[c]), fabsf(lo_t[c + 1])));
                ssum_w += f16_lo(hi) + f16_hi(hi);
                ssum += (f16_lo(hi) + f16_hi(hi)) * wgt;
            }
            const int ex = mx > 0.0f ? (int)((__float_as_uint(mx) >> 23) & 0xffu) - 127 - 7 : 0;   // floor(log2 mx) - 7
            const float down = __uint_as_float((uint32_t)(127 - ex) << 23), up = __uint_as_float((uint32_t)(127 + ex) << 23);
            // Operand order: MFMA j (channels of key words 2 j, 2 j + 1), lane half hh, register r8, byte b hold
            // the channel whose code the key unpacking puts into the same byte.
#pragma unroll
            for (int w = 0; w < 32; ++w) {
                const int j = w >> 4, hw = (w >> 3) & 1, r8 = w & 7;
                float v[4];
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int slab = 2 * (2 * j + (r8 >> 2)) + (b & 1);
                    v[b] = lo_t[16 * slab + 8 * hw + 2 * (r8 & 3) + (b >> 1)] * down;
                }
                int word = __builtin_amdgcn_cvt_pk_fp8_f32(v[0], v[1], 0, false);
                word = __builtin_amdgcn_cvt_pk_fp8_f32(v[2], v[3], word, true);
                dst[w] = (uint32_t)word;
                float dec = 0.0f;
#pragma unroll
                for (int b = 0; b < 4; ++b) dec += e4m3_to_float((uint8_t)((uint32_t)word >> (8 * b)));
                ssum += dec * up;      // the sums follow the operands the MFMAs will see
                ssum_w += 2.0f * (dec * up);   // FP8 key values are 8 + code, twice the BASE the constant term takes off
            }
            row_scal[4 * prow + 3] = __int_as_float(127 + ex);
        } else {
#pragma unroll
        for (int i = 0; i < kPrepCh / 8; ++i) {
            uint32_t lo[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float v0 = x[8 * i + 2 * j], v1 = x[8 * i + 2 * j + 1];
                const uint32_t hi = pack_f16(v0, v1);
                const float h0 = f16_lo(hi), h1 = f16_hi(hi);
                lo[j] = pack_f16(v0 - h0, v1 - h1);
#if KVQ_Q_LOW_PART
                const float pair = (h0 + f16_lo(lo[j])) + (h1 + f16_hi(lo[j]));   // both channels share a class
#else
                const float pair = h0 + h1;
#endif
                ssum_w += pair;
                ssum += pair * (1.0f / (float)(1 << (Unpack<BITS>::kClassBits * key_channel_class<BITS>(8 * i + 2 * j))));
            }
            u32x4 w;
            w.x = lo[0]; w.y = lo[1]; w.z = lo[2]; w.w = lo[3];
            *reinterpret_cast<u32x4 *>(dst + 4 * i) = w;
        }
        }
        if constexpr (kPrepLanes == 2) {
            ssum += __shfl_xor(ssum, 1);
            ssum_w += __shfl_xor(ssum_w, 1);
        }
        if (ppart == 0) {
            row_scal[4 * prow] = ssum;
            row_scal[4 * prow + 1] = ssum_w;
            row_scal[4 * prow + 2] = CORR ? -a.softmax_scale * a.softmax_scale * kLog2e * nu * (1.0f / 24.0f) : 0.0f;
        }
    }
    __syncthreads();
    // B operand of the constant-term MFMA, per 32-row block.  The raw score is sum_c (q~_c 4^g) (BASE +
    // 4^-g code_c) = q~ . code + BASE * W with W the sum of the weighted operand values, so what has to
    // come off is z * S + BASE * W (S = sum_c q~_c).  Lane half 0 multiplies the key's -z pieces and the
    // mask bias, lane half 1 the key's scale pieces and the constant -BASE:
    //   hh = 0: [S_h, S_m, S_l, S_h, S_m, S_l, 1, 0]     S in three bf16 pieces
    //   hh = 1: [N_h, N_l, N_h, N_l, W_h, W_m, W_l, 0]   N = -nu' in two pieces, W in three
    u32x4 rowop[kRB];
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) {
        const float *rs = row_scal + 4 * (wave * kRowsPerWave + 32 * rb + n);
        const float ssum = rs[0], wsum = rs[1], nnu = rs[2];
        const uint16_t s_h = bf16_bits(ssum);
        const float r1 = ssum - bf16_val(s_h);
        const uint16_t s_m = bf16_bits(r1);
        const uint16_t s_l = bf16_bits(r1 - bf16_val(s_m));
        const uint16_t w_h = bf16_bits(wsum);
        const float r2 = wsum - bf16_val(w_h);
        const uint16_t w_m = bf16_bits(r2);
        const uint16_t w_l = bf16_bits(r2 - bf16_val(w_m));
        const uint16_t n_h = bf16_bits(nnu);
        const uint16_t n_l = bf16_bits(nnu - bf16_val(n_h));
        const uint32_t one = 0x3f80u;
        u32x4 w0, w1;
        w0.x = s_h | ((uint32_t)s_m << 16); w0.y = s_l | ((uint32_t)s_h << 16);
        w0.z = s_m | ((uint32_t)s_l << 16); w0.w = one | (one << 16);
        w1.x = n_h | ((uint32_t)n_l << 16); w1.y = w1.x;
        w1.z = w_h | ((uint32_t)w_m << 16); w1.w = w_l | (one << 16);
        rowop[rb] = hh ? w1 : w0;
    }
    const uint32_t lo_off = (uint32_t)((wave * kRowsPerWave + n) * kQRowWords + 4 * hh);  // words into q_stage
    // The 64 registers of query operands live in accumulation registers (MFMA reads them from there
    // directly), which leaves the vector registers to the score tile in flight.
    if constexpr (!kFp4) {
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
        for (int s = 0; s < 8; ++s) asm volatile("" : "+a"(qop[rb][s]));
    }
    // FP4 keys: the 96 registers of query pieces likewise, and the four scale bytes of each row
    int qp_scale[kRB] = {};
    if constexpr (kFp4) {
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    if (kVs && k == 3 && j == 1) asm volatile("" : "+v"(qp[rb][k][j]));
                    else asm volatile("" : "+a"(qp[rb][k][j]));
                }
            qp_scale[rb] = __float_as_int(row_scal[4 * (wave * kRowsPerWave + 32 * rb + n) + 3]);
        }
    }
    // 2-bit codes are FP4 (E2M1) values as they stand, 0, 0.5, 1, 1.5: a packed word is two operand registers, the
    // even and the odd fields, each in the low half of a nibble.  Four pieces x two 64-channel MFMAs per row block,
    // FP4 x FP6 at twice the FP8 rate; opsel picks the piece's byte of the row's scale word.
    uint32_t f4_mask = 0x33333333u;
    asm volatile("" : "+s"(f4_mask));
    auto fp4_operand = [&](auto j_, const uint32_t (&kw)[WPL]) {   // key words 2 J, 2 J + 1
        constexpr int J = decltype(j_)::value;
        const uint32_t w0 = kw[(2 * J) % WPL], w1 = kw[(2 * J + 1) % WPL];
        return i32x8{(int)(w0 & f4_mask), (int)((w0 >> 2) & f4_mask), (int)(w1 & f4_mask), (int)((w1 >> 2) & f4_mask), 0, 0, 0, 0};
    };
    auto fp4_mfma = [&](auto j_, auto k_, const i32x8 &a4, f32x16 (&sn)[kRB]) {   // piece K against key words 2 J, 2 J + 1
        constexpr int J = decltype(j_)::value, K = decltype(k_)::value;
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) {
            const i32x6 b6 = qp[rb][K][J];
            const i32x8 b8 = {b6[0], b6[1], b6[2], b6[3], b6[4], b6[5], 0, 0};
            sn[rb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a4, b8, sn[rb], 4, 2, 0, 0x7f, K, qp_scale[rb]);
        }
    };
    auto score_fp4 = [&](auto j_, const uint32_t (&kw)[WPL], f32x16 (&sn)[kRB]) {
        const i32x8 a4 = fp4_operand(j_, kw);
        static_for<4>([&](auto k_) { fp4_mfma(j_, k_, a4, sn); });
    };
    // The same MFMAs with the score tile in vector registers (kVs).  The compiler keeps every MFMA result of this
    // kernel in accumulation registers, from where each score would have to be copied before the vector ALU can
    // touch it; written out, the instruction takes a vector-register tuple as C and D.  What the compiler no longer
    // sees it no longer guards, so the wait states the hardware asks for are placed here, as the compiler places them
    // for MFMAs of its own: two between a vector write of an operand and the MFMA that reads it (`fresh`: the A
    // operand has just been made), and twelve between the last MFMA of a chain and the first vector instruction
    // that reads the tile (KVQ_SCORE_TILE_READY).  Dependent MFMAs on one tile need none.
    int f4_scale_one = 0x7f;
    asm volatile("" : "+v"(f4_scale_one));
    auto fp4_operand4 = [&](auto j_, const uint32_t (&kw)[WPL]) {
        constexpr int J = decltype(j_)::value;
        const uint32_t w0 = kw[(2 * J) % WPL], w1 = kw[(2 * J + 1) % WPL];
        return i32x4{(int)(w0 & f4_mask), (int)((w0 >> 2) & f4_mask), (int)(w1 & f4_mask), (int)((w1 >> 2) & f4_mask)};
    };
    auto fp4_mfma_v = [&](auto j_, auto k_, auto fresh_, const i32x4 &a4, f32x16 &s, int rb) {
        constexpr int J = decltype(j_)::value, K = decltype(k_)::value;
        constexpr bool FRESH = decltype(fresh_)::value != 0;
        const i32x6 b6 = qp[rb][K][J];
        const int sb = qp_scale[rb];
        // (the accumulation registers hold the output tile and all but two of the sixteen piece operands; those two
        // stay in vector registers, which leaves the register allocator a few accumulation registers)
#define KVQ_FP4_MFMA_V(NOP, SEL)                                                                                      \
        {                                                                                                             \
            if constexpr (K == 3 && J == 1)                                                                           \
                asm(NOP "v_mfma_scale_f32_32x32x64_f8f6f4 %0, %1, %2, %0, %3, %4 " SEL " cbsz:4 blgp:2"           \
                    : "+v"(s) : "v"(a4), "v"(b6), "v"(f4_scale_one), "v"(sb));                                        \
            else                                                                                                      \
                asm(NOP "v_mfma_scale_f32_32x32x64_f8f6f4 %0, %1, %2, %0, %3, %4 " SEL " cbsz:4 blgp:2"           \
                    : "+v"(s) : "v"(a4), "a"(b6), "v"(f4_scale_one), "v"(sb));                                        \
        }
        if constexpr (K == 0 && FRESH) KVQ_FP4_MFMA_V("s_nop 1\n\t", "op_sel_hi:[0,0,0]")
        if constexpr (K == 0 && !FRESH) KVQ_FP4_MFMA_V("", "op_sel_hi:[0,0,0]")
        if constexpr (K == 1) KVQ_FP4_MFMA_V("", "op_sel:[0,1,0] op_sel_hi:[0,0,0]")
        if constexpr (K == 2) KVQ_FP4_MFMA_V("", "op_sel_hi:[0,1,0]")
        if constexpr (K == 3) KVQ_FP4_MFMA_V("", "op_sel:[0,1,0] op_sel_hi:[0,1,0]")
#undef KVQ_FP4_MFMA_V
    };
    // first MFMA of a score tile: the constant terms, C = 0
    auto const_mfma_v = [&](f32x16 &s, const u32x4 &cop, const u32x4 &rop) {
        asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(s) : "v"(cop), "v"(rop));
    };
    // every vector read of the tile goes through here: NOP completes the twelve wait states after the last MFMA
#define KVQ_SCORE_TILE_READY(NOP, S) asm volatile(NOP : "+v"((S)[0]), "+v"((S)[kRB - 1]))

    // FP8 low part: B operands of the two 64-channel MFMAs per 32-row block, and the rows' scale bytes
    i32x8 lo8[kRB][2];
    int lo_scale[kRB];
    if constexpr (kLoFp8) {
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) {
            const uint32_t *src = q_stage + (wave * kRowsPerWave + 32 * rb + n) * kQRowWords + 8 * hh;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const u32x4 w0 = *reinterpret_cast<const u32x4 *>(src + 16 * j);
                const u32x4 w1 = *reinterpret_cast<const u32x4 *>(src + 16 * j + 4);
                lo8[rb][j] = i32x8{(int)w0.x, (int)w0.y, (int)w0.z, (int)w0.w, (int)w1.x, (int)w1.y, (int)w1.z, (int)w1.w};
                asm volatile("" : "+a"(lo8[rb][j]));
            }
            lo_scale[rb] = __float_as_int(row_scal[4 * (wave * kRowsPerWave + 32 * rb + n) + 3]);
        }
    }
    // Low-part MFMAs of 64 channels (key words 2 J and 2 J + 1): the codes become FP8 values 8 + code, four to
    // a register, in the byte order the low operand was written in.
    // (mask in a scalar, base in a vector register: the form v_and_or_b32 can encode)
    uint32_t f8_mask = 0x03030303u, f8_base = 0x50505050u;
    asm volatile("" : "+s"(f8_mask));
    asm volatile("" : "+v"(f8_base));
    auto low_part_fp8 = [&](auto j_, const uint32_t (&kw)[WPL], f32x16 (&sn)[kRB]) {
        constexpr int J = decltype(j_)::value;
        i32x8 a8;
#pragma unroll
        for (int r8 = 0; r8 < 8; ++r8) {
            const uint32_t w = kw[(2 * J + (r8 >> 2)) % WPL];
            const uint32_t sh = w >> (2 * (r8 & 3));   // no shift for the first code; w >> 2 is shared with the f16 unpacking
            a8[r8] = (int)((sh & f8_mask) | f8_base);
        }
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb)
            sn[rb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, lo8[rb][J], sn[rb], 0, 0, 0, 0x7f, 0, lo_scale[rb]);
    };
    constexpr int kLoRes = kLoF16 ? KVQ_Q_LOW_RESIDENT_SLABS : 0;
    u32x4 lo_res[kRB][kLoRes > 0 ? kLoRes : 1];
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
        for (int s = 0; s < kLoRes; ++s) {
            lo_res[rb][s] = *reinterpret_cast<const u32x4 *>(q_stage + lo_off + 32 * rb * kQRowWords + 8 * s);
            asm volatile("" : "+a"(lo_res[rb][s]));
        }

    f32x16 o[4][kRB];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[b][rb][v] = 0.0f;
    // Keeps the 128 output accumulators in accumulation registers at the points where the fast loops
    // are entered, so that the loops carry them there instead of copying them around.
    auto pin_accumulators = [&]() {
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) asm volatile("" : "+a"(o[b][rb]));
    };
    float m_ref[kRB] = {};              // reference maximum (log2 domain); set by the first tile
    float l_s[kRB] = {}, l_r[kRB] = {}, tau[kRB] = {};
    bool first = true;                  // no tile has set the reference yet

    // Leaves the fast loops: move the reference of the rows whose pending tile maximum `tmax` (relative
    // to the old reference) is too large, and rescale what has been accumulated so far.
    auto move_reference = [&](float (&e)[kRB][16], const float (&tmax)[kRB]) {
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) {
            const bool mv = first || tmax[rb] > kRescaleThreshold;
            const float delta = mv ? tmax[rb] : 0.0f;
            const float alpha = first ? 1.0f : __builtin_amdgcn_exp2f(-delta);
            m_ref[rb] += delta;
#pragma unroll
            for (int v = 0; v < 16; ++v) e[rb][v] -= delta;
            l_s[rb] *= alpha;
            l_r[rb] *= alpha;
            tau[rb] *= alpha;
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[b][rb][v] *= alpha;
        }
        first = false;
        pin_accumulators();
    };

    auto over_threshold = [&](const float (&tmax)[kRB]) {
        bool over = false;
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) over = over || tmax[rb] > kRescaleThreshold;
        return over;
    };

    // The query preparation once more, for one block of a per-channel cache (the operands above are replaced):
    // ch_step, ch_zero are the steps and zero-points of the rotated channels of that block.
    auto reprepare = [&](const float *ch_step, const float *ch_zero) {
    if constexpr (PERCH) {
    {
        const int prow = tid / kPrepLanes, ppart = tid % kPrepLanes;
        int64_t row = (int64_t)rblk * kRowsPerBlock + prow;
        row = row < a.m ? row : a.m - 1;
        const uint4 *src = reinterpret_cast<const uint4 *>(q_base + row * a.q_stride_token + ppart * kPrepCh);
        float x[kPrepCh];
#pragma unroll
        for (int i = 0; i < kPrepCh / 8; ++i) {
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
        for (int i = 0; i < kPrepCh; ++i) nu = fmaf(x[i], x[i], nu);
        // Randomised rotation: the channel signs come before the Hadamard matrix.
        if (has_signs(a.cv))
#pragma unroll
        for (int w = 0; w < kPrepCh / 32; ++w) {
            const uint32_t sg = sign_bits_from(a.cv, ppart * kPrepCh + 32 * w);
#pragma unroll
            for (int i = 0; i < 32; ++i) x[32 * w + i] = flip_sign(x[32 * w + i], sg >> i);
        }
#pragma unroll
        for (int h = 1; h < kPrepCh; h <<= 1) {
#pragma unroll
            for (int i = 0; i < kPrepCh; ++i) {
                if ((i & h) == 0) {
                    const float p = x[i], q2 = x[i + h];
                    x[i] = p + q2;
                    x[i + h] = p - q2;
                }
            }
        }
        if constexpr (kPrepLanes == 2) {   // last butterfly stage: between the two lanes of the row
            nu += __shfl_xor(nu, 1);
#pragma unroll
            for (int i = 0; i < kPrepCh; ++i) {
                const float other = __shfl_xor(x[i], 1);
                x[i] = ppart ? other - x[i] : x[i] + other;
            }
        }
        if constexpr (PERCH) {   // q^_c step_c: the block's correction, then the operand
            nu = 0.0f;
#pragma unroll
            for (int i = 0; i < kPrepCh; ++i) {
                x[i] *= ch_step[i];
                const float t = x[i] * 0.088388347648318f;
                nu = fmaf(t, t, nu);
            }
        }
        // Channel c of the operand carries 4^g(c) (the inverse of the weight its key codes are unpacked with).
        const float cq = c_log * 0.088388347648318f;
#pragma unroll
        for (int i = 0; i < kPrepCh; ++i) x[i] *= cq * (float)(1 << (Unpack<BITS>::kClassBits * key_channel_class<BITS>(i)));
        // The staging rows hold the high parts first (read into registers below), then the low parts,
        // which stay in LDS for the whole cached-key loop.
        uint32_t *dst = q_stage + prow * kQRowWords + ppart * (kPrepCh / 2);
#pragma unroll
        for (int i = 0; i < kPrepCh / 8; ++i) {
            u32x4 w;
            w.x = pack_f16(x[8 * i], x[8 * i + 1]); w.y = pack_f16(x[8 * i + 2], x[8 * i + 3]);
            w.z = pack_f16(x[8 * i + 4], x[8 * i + 5]); w.w = pack_f16(x[8 * i + 6], x[8 * i + 7]);
            *reinterpret_cast<u32x4 *>(dst + 4 * i) = w;
        }
        __syncthreads();
        const uint32_t *hsrc = q_stage + (wave * kRowsPerWave + n) * kQRowWords + 4 * hh;
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
            for (int s = 0; s < 8; ++s)
                qop[rb][s] = *reinterpret_cast<const u32x4 *>(hsrc + 32 * rb * kQRowWords + 8 * s);
        __syncthreads();
        float ssum = 0.0f, ssum_w = 0.0f;   // sum of q~ (true scale), sum of the weighted operand values
        if constexpr (kLoFp8) {
            static_assert(!kLoFp8 || kPrepLanes == 1, "one lane prepares a whole row");
            // Low parts at true scale (the weight 4^g of the high operand taken out again: exact), their
            // largest magnitude, and from it the row's power-of-two scale: the largest low part lands in
            // [128, 256), inside the E4M3 range.
            float lo_t[kPrepCh], mx = 0.0f;
#pragma unroll
            for (int c = 0; c < kPrepCh; c += 2) {
                const uint32_t hi = pack_f16(x[c], x[c + 1]);
                const float wgt = 1.0f / (float)(1 << (Unpack<BITS>::kClassBits * key_channel_class<BITS>(c)));   // both channels share a class
                lo_t[c] = (x[c] - f16_lo(hi)) * wgt;
                lo_t[c + 1] = (x[c + 1] - f16_hi(hi)) * wgt;
                mx = fmaxf(mx, fmaxf(fabsf(lo_t[c]), fabsf(lo_t[c + 1])));
                ssum_w += f16_lo(hi) + f16_hi(hi);
                if constexpr (PERCH) ssum += (f16_lo(hi) * ch_zero[c] + f16_hi(hi) * ch_zero[c + 1]) * wgt;
                else ssum += (f16_lo(hi) + f16_hi(hi)) * wgt;
            }
            const int ex = mx > 0.0f ? (int)((__float_as_uint(mx) >> 23) & 0xffu) - 127 - 7 : 0;   // floor(log2 mx) - 7
            const float down = __uint_as_float((uint32_t)(127 - ex) << 23), up = __uint_as_float((uint32_t)(127 + ex) << 23);
            // Operand order: MFMA j (channels of key words 2 j, 2 j + 1), lane half hh, register r8, byte b hold
            // the channel whose code the key unpacking puts into the same byte.
#pragma unroll
            for (int w = 0; w < 32; ++w) {
                const int j = w >> 4, hw = (w >> 3) & 1, r8 = w & 7;
                float v[4];
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int slab = 2 * (2 * j + (r8 >> 2)) + (b & 1);
                    v[b] = lo_t[16 * slab + 8 * hw + 2 * (r8 & 3) + (b >> 1)] * down;
                }
                int word = __builtin_amdgcn_cvt_pk_fp8_f32(v[0], v[1], 0, false);
                word = __builtin_amdgcn_cvt_pk_fp8_f32(v[2], v[3], word, true);
                dst[w] = (uint32_t)word;
                float dec = 0.0f, dec_z = 0.0f;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const float d8 = e4m3_to_float((uint8_t)((uint32_t)word >> (8 * b)));
                    dec += d8;
                    if constexpr (PERCH) {
                        const int slab = 2 * (2 * j + (r8 >> 2)) + (b & 1);
                        dec_z = fmaf(d8, ch_zero[16 * slab + 8 * hw + 2 * (r8 & 3) + (b >> 1)], dec_z);
                    }
                }
                ssum += (PERCH ? dec_z : dec) * up;      // the sums follow the operands the MFMAs will see
                ssum_w += 2.0f * (dec * up);   // FP8 key values are 8 + code, twice the BASE the constant term takes off
            }
            row_scal[4 * prow + 3] = __int_as_float(127 + ex);
        } else {
#pragma unroll
        for (int i = 0; i < kPrepCh / 8; ++i) {
            uint32_t lo[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float v0 = x[8 * i + 2 * j], v1 = x[8 * i + 2 * j + 1];
                const uint32_t hi = pack_f16(v0, v1);
                const float h0 = f16_lo(hi), h1 = f16_hi(hi);
                lo[j] = pack_f16(v0 - h0, v1 - h1);
#if KVQ_Q_LOW_PART
                const float pair = (h0 + f16_lo(lo[j])) + (h1 + f16_hi(lo[j]));   // both channels share a class
#else
                const float pair = h0 + h1;
#endif
                ssum_w += pair;
                const float wgt = 1.0f / (float)(1 << (Unpack<BITS>::kClassBits * key_channel_class<BITS>(8 * i + 2 * j)));
#if KVQ_Q_LOW_PART
                if constexpr (PERCH)
                    ssum += ((h0 + f16_lo(lo[j])) * ch_zero[8 * i + 2 * j] + (h1 + f16_hi(lo[j])) * ch_zero[8 * i + 2 * j + 1]) * wgt;
                else
#endif
                ssum += pair * wgt;
            }
            u32x4 w;
            w.x = lo[0]; w.y = lo[1]; w.z = lo[2]; w.w = lo[3];
            *reinterpret_cast<u32x4 *>(dst + 4 * i) = w;
        }
        }
        if constexpr (kPrepLanes == 2) {
            ssum += __shfl_xor(ssum, 1);
            ssum_w += __shfl_xor(ssum_w, 1);
        }
        if (ppart == 0) {
            row_scal[4 * prow] = ssum;
            row_scal[4 * prow + 1] = ssum_w;
            row_scal[4 * prow + 2] = CORR ? -a.softmax_scale * a.softmax_scale * kLog2e * nu * (1.0f / 24.0f) : 0.0f;
        }
    }
    __syncthreads();
    // B operand of the constant-term MFMA, per 32-row block.  The raw score is sum_c (q~_c 4^g) (BASE +
    // 4^-g code_c) = q~ . code + BASE * W with W the sum of the weighted operand values, so what has to
    // come off is z * S + BASE * W (S = sum_c q~_c).  Lane half 0 multiplies the key's -z pieces and the
    // mask bias, lane half 1 the key's scale pieces and the constant -BASE:
    //   hh = 0: [S_h, S_m, S_l, S_h, S_m, S_l, 1, 0]     S in three bf16 pieces
    //   hh = 1: [N_h, N_l, N_h, N_l, W_h, W_m, W_l, 0]   N = -nu' in two pieces, W in three
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) {
        const float *rs = row_scal + 4 * (wave * kRowsPerWave + 32 * rb + n);
        const float ssum = rs[0], wsum = rs[1], nnu = rs[2];
        const uint16_t s_h = bf16_bits(ssum);
        const float r1 = ssum - bf16_val(s_h);
        const uint16_t s_m = bf16_bits(r1);
        const uint16_t s_l = bf16_bits(r1 - bf16_val(s_m));
        const uint16_t w_h = bf16_bits(wsum);
        const float r2 = wsum - bf16_val(w_h);
        const uint16_t w_m = bf16_bits(r2);
        const uint16_t w_l = bf16_bits(r2 - bf16_val(w_m));
        const uint16_t n_h = bf16_bits(nnu);
        const uint16_t n_l = bf16_bits(nnu - bf16_val(n_h));
        const uint32_t one = 0x3f80u;
        u32x4 w0, w1;
        w0.x = s_h | ((uint32_t)s_m << 16); w0.y = s_l | ((uint32_t)s_h << 16);
        w0.z = s_m | ((uint32_t)s_l << 16); w0.w = one | (one << 16);
        w1.x = n_h | ((uint32_t)n_l << 16); w1.y = w1.x;
        w1.z = w_h | ((uint32_t)w_m << 16); w1.w = w_l | (one << 16);
        rowop[rb] = hh ? w1 : w0;
    }
    // The 64 registers of query operands live in accumulation registers (MFMA reads them from there
    // directly), which leaves the vector registers to the score tile in flight.
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
        for (int s = 0; s < 8; ++s) asm volatile("" : "+a"(qop[rb][s]));

    if constexpr (kLoFp8) {
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) {
            const uint32_t *src = q_stage + (wave * kRowsPerWave + 32 * rb + n) * kQRowWords + 8 * hh;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const u32x4 w0 = *reinterpret_cast<const u32x4 *>(src + 16 * j);
                const u32x4 w1 = *reinterpret_cast<const u32x4 *>(src + 16 * j + 4);
                lo8[rb][j] = i32x8{(int)w0.x, (int)w0.y, (int)w0.z, (int)w0.w, (int)w1.x, (int)w1.y, (int)w1.z, (int)w1.w};
                asm volatile("" : "+a"(lo8[rb][j]));
            }
            lo_scale[rb] = __float_as_int(row_scal[4 * (wave * kRowsPerWave + 32 * rb + n) + 3]);
        }
    }
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
        for (int s = 0; s < kLoRes; ++s) {
            lo_res[rb][s] = *reinterpret_cast<const u32x4 *>(q_stage + lo_off + 32 * rb * kQRowWords + 8 * s);
            asm volatile("" : "+a"(lo_res[rb][s]));
        }
    }
    };

    // ---------------------------------------------------------------------- cached keys ----
    if (a.cache_len > 0) {
        // Per-channel caches: one pass per key block of the window, each with its own query operands.
        for (int bi = 0; bi < (PERCH ? a.n_key_blocks : 1); ++bi) {
        int64_t cs = a.cache_start, ce = a.cache_start + a.cache_len;
        int phys_first = (int)a.phys_tile_first;
        if constexpr (PERCH) {
            const KeyBlock kb = a.key_blocks[bi];
            cs = a.cache_start + kb.start;
            ce = a.cache_start + kb.end;
            phys_first = (int)((a.phys_tile_first + (cs / kTileTokens - a.cache_start / kTileTokens)) % cv.cap_tiles);
            __syncthreads();   // every wave has left the previous block's tiles and staging rows
            reprepare(cv.kc_scale + ((int64_t)kb.slot * cv.num_heads + head) * D,
                      cv.kc_zero + ((int64_t)kb.slot * cv.num_heads + head) * D);
        }
        const int64_t t_first = cs / kTileTokens, t_last = (ce - 1) / kTileTokens;
        const int n_tiles = (int)(t_last - t_first + 1);
        const int n_stages = (n_tiles + kStageTiles - 1) / kStageTiles;
        const int64_t head_tile0 = (int64_t)head * cv.cap_tiles;
        const int64_t meta0 = head_tile0 * kTileTokens;

        // ---- loader: global -> registers (prefetch), registers -> LDS (commit, builds the constants)
        constexpr int kCodeVecs = St::kCodeWords / 4;               // 16-byte vectors per tensor and stage
        constexpr int kCodeIters = 2 * kCodeVecs / kThreads;        // vectors per thread (keys, then values)
        u32x4 pre_kv[kCodeIters];
        float pre_a = 0.0f, pre_b = 0.0f, pre_c = 0.0f;
        uint32_t pre_in_window = 0u;   // a vector register, not a lane mask: it lives across the loop's branches
        const int ld_key = tid & 127, ld_half = (tid >> 7) & 1; // one (key, operand half) per thread below 256
        const bool ld_meta = tid < 2 * kStageKeys;
        // Ring arithmetic in 32 bits (the launcher sends caches of 2^20 tiles or more per head elsewhere): the
        // stage's first physical tile is uniform, a thread adds its tile inside the stage and wraps once more.
        const int cap = (int)cv.cap_tiles;
        const int first_off = (int)(cs - t_first * kTileTokens);   // position of cache_start inside its tile
        const int win_len = (int)(ce - cs);
        // Addresses are a uniform 64-bit base (head) plus a 32-bit offset per thread, the form a global load
        // takes with its base in scalar registers: no 64-bit address per thread is kept across the loop.
        const uint32_t *k_head = cv.k_codes + head_tile0 * (64 * WPL), *v_head = cv.v_codes + head_tile0 * (64 * WPL);
        const float *m_kscale = cv.k_scale + meta0, *m_knegzero = cv.k_negzero + meta0;
        const float *m_vscale = cv.v_scale + meta0, *m_vzero = cv.v_zero_off + meta0;
        const uint8_t *m_kscale8 = cv.k_scale8 + meta0, *m_vscale8 = cv.v_scale8 + meta0;
        const uint16_t *m_kzero16 = cv.k_zero16 + meta0, *m_vzero16 = cv.v_zero16 + meta0;
        auto prefetch = [&](int stage) {
            if (stage >= n_stages) return;
            int ring0 = phys_first + stage * kStageTiles;   // < 2 cap + 4: n_tiles <= cap + 1
            ring0 -= ring0 >= cap ? cap : 0;
            ring0 -= ring0 >= cap ? cap : 0;
#pragma unroll
            for (int it = 0; it < kCodeIters; ++it) {
                const int vec = (tid + kThreads * it) % kCodeVecs;   // it < kCodeIters / 2: keys, else values
                int tile = ring0 + vec / (16 * WPL);
                tile -= tile >= cap ? cap : 0;    // tiles past the window wrap onto tiles of the storage: masked later
                tile = tile < cap ? tile : cap - 1;   // (a ring of fewer than four tiles)
                const uint32_t word = (uint32_t)tile * (64 * WPL) + (uint32_t)(vec % (16 * WPL)) * 4u;
                pre_kv[it] = *reinterpret_cast<const u32x4 *>((it < kCodeIters / 2 ? k_head : v_head) + word);
            }
            if (!ld_meta) return;
            const int rel = stage * kStageKeys + ld_key - first_off;    // position inside the window
            pre_in_window = (rel >= 0 && rel < win_len) ? 1u : 0u;
            int mt = ring0 + (ld_key >> 5);
            mt -= mt >= cap ? cap : 0;
            mt = mt < cap ? mt : cap - 1;
            const uint32_t tok = (uint32_t)mt * kTileTokens + (uint32_t)(ld_key & 31);
            if constexpr (PERCH) {   // keys: step 1, the row constant Z meets -1 where a zero-point would stand
                if (ld_half == 0) {
                    pre_a = -1.0f - Unpack<BITS>::kStoredOffset;
                    pre_b = 1.0f;
                    pre_c = m_vscale[tok];
                } else {
                    pre_a = 1.0f;
                    pre_b = m_vscale[tok];
                    pre_c = m_vzero[tok];
                }
            } else if constexpr (!FP8META) {
                if (ld_half == 0) {
                    pre_a = m_knegzero[tok];
                    pre_b = m_kscale[tok];
                    pre_c = m_vscale[tok];
                } else {
                    pre_a = m_kscale[tok];
                    pre_b = m_vscale[tok];
                    pre_c = m_vzero[tok];
                }
            } else {   // FP8 E4M3 scale, BF16 zero-point, one pair per token: the raw encodings, decoded at the commit
                       // (decoding here would make the wave wait for the loads it has just issued)
                // (the aligned words that hold the token's byte / half-word: plain dword loads, like the fp32 format)
                const float *w_ks = reinterpret_cast<const float *>(m_kscale8), *w_vs = reinterpret_cast<const float *>(m_vscale8);
                const float *w_kz = reinterpret_cast<const float *>(m_kzero16), *w_vz = reinterpret_cast<const float *>(m_vzero16);
                if (ld_half == 0) {
                    pre_a = w_kz[tok >> 1];
                    pre_b = w_ks[tok >> 2];
                    pre_c = w_vs[tok >> 2];
                } else {
                    pre_a = w_ks[tok >> 2];
                    pre_b = w_vs[tok >> 2];
                    pre_c = w_vz[tok >> 1];
                }
            }
        };
        auto commit = [&](int stage) {
            if (stage >= n_stages) return;
            uint32_t *buf = lds + ((uint32_t)stage % kBuffers) * St::kWords;
#pragma unroll
            for (int it = 0; it < kCodeIters; ++it) {
                const int g = tid + kThreads * it;   // kV == kK + 4 * kCodeVecs: keys then values, contiguous
                *reinterpret_cast<u32x4 *>(buf + St::kK + 4 * g) = pre_kv[it];
            }
            if (!ld_meta) return;
            const bool pre_valid = pre_in_window != 0u;
            // Position of this key in the per-lane order of the score tile: [tile][hh][4 g + r].
            const int tl = ld_key >> 5, r = ld_key & 31;
            const int slot = tl * 32 + ((r >> 2) & 1) * 16 + 4 * (r >> 3) + (r & 3);
            // The value scale (times the weight 4^g its key's probability carries, see below) is not multiplied
            // into the probability: its logarithm is added to the score, as lambda / key scale in the two free
            // slots of the constant-term operand (two bf16 pieces against ones), so that 2^e already is
            // p * value scale; the row sum gets p back through the reciprocal kept in the kVScale array.
            // Scales are clamped away from zero (an all-zero row has scale 0): such a key scores 0 and its
            // value contributes 2^-64 p, as good as the exact 0.
            const int g2 = 2 * value_register_class<BITS>(slot & 15);
            // What this loader half has: the key scale, the value scale, and one zero-point term (half 0: minus the
            // key's stored zero-point, half 1: the value's).  Picked with selects, the same instructions in both halves.
            float m_ks = ld_half == 0 ? pre_b : pre_a;
            float m_vs = ld_half == 0 ? pre_c : pre_b;
            float m_z = ld_half == 0 ? pre_a : pre_c;
            if constexpr (FP8META) {   // decode what the prefetch brought
                const int sb = 8 * (ld_key & 3), sh = 16 * (ld_key & 1);   // the token's byte / half-word inside its word
                const float zs = bf16_val((uint16_t)(__float_as_uint(m_z) >> sh)) + Unpack<BITS>::kStoredOffset;
                m_ks = e4m3_low_byte(__float_as_uint(m_ks) >> sb);
                m_vs = e4m3_low_byte(__float_as_uint(m_vs) >> sb);
                m_z = ld_half == 0 ? -zs : zs;
            }
            const float vs_eff = ldexpf(fmaxf(m_vs, 0x1p-64f), g2);
            const float ks_eff = fmaxf(m_ks, 0x1p-40f);
            // (v_rcp_f32: one unit in the last place, far inside what lambda and the row sums need; both loader
            // halves run the same instructions on the same inputs, so their pieces belong to one value)
            const float lam = pre_valid ? __log2f(vs_eff) * __builtin_amdgcn_rcpf(ks_eff) : 0.0f;
            const uint16_t lam_h = bf16_bits(lam);
            const uint16_t lam_l = bf16_bits(lam - bf16_val(lam_h));
            u32x4 cop;
            if (ld_half == 0) {
                // -zero in two bf16 pieces (exact for |.| < 2^16), and the window mask.
                const float nz = pre_valid ? m_z + Unpack<BITS>::kStoredOffset : 0.0f;
                const uint16_t z_h = bf16_bits(nz);
                const uint16_t z_l = bf16_bits(nz - bf16_val(z_h));
                cop.x = z_h | ((uint32_t)z_h << 16); cop.y = z_h | ((uint32_t)z_l << 16);
                cop.z = z_l | ((uint32_t)z_l << 16);
                cop.w = (pre_valid ? 0u : (uint32_t)bf16_bits(kMaskBias)) | ((uint32_t)lam_h << 16);
                reinterpret_cast<float *>(buf + St::kKScale)[slot] = pre_valid ? ks_eff : 1.0f;
            } else {
                const float ks = pre_valid ? ks_eff : 0.0f;
                const uint16_t k_h = bf16_bits(ks);
                const uint16_t k_l = bf16_bits(ks - bf16_val(k_h));
                const uint32_t nb = pre_valid ? (uint32_t)bf16_bits(-Unpack<BITS>::kKeyBase) : 0u;   // exact
                cop.x = k_h | ((uint32_t)k_h << 16); cop.y = k_l | ((uint32_t)k_l << 16);
                cop.z = nb | (nb << 16); cop.w = nb | ((uint32_t)lam_l << 16);
                // Tokens outside the window: the mask bias makes their probability exactly 0, and nothing
                // derived from what the storage holds there (it need not be initialised) enters the tile.
                // The probability of this key meets value codes unpacked with weight 4^-g: it carries 4^g
                // (through the value scale), and tau's multiplier is BASE + 4^-g z.
                const float vz = pre_valid ? Unpack<BITS>::kValueBase + ldexpf(m_z - Unpack<BITS>::kStoredOffset, -g2) : 0.0f;
                reinterpret_cast<float *>(buf + St::kVScale)[slot] = pre_valid ? __builtin_amdgcn_rcpf(vs_eff) : 0.0f;
                const uint16_t v_h = bf16_bits(vz);
                const uint16_t v_l = bf16_bits(vz - bf16_val(v_h));
                reinterpret_cast<uint16_t *>(buf + St::kVzHi)[slot] = v_h;
                reinterpret_cast<uint16_t *>(buf + St::kVzLo)[slot] = v_l;
                // this half of the loader threads is two whole waves: one flag word each
                const bool lo_any = __any(v_l != 0);
                if (lane == 0) buf[St::kFlags + (wave & 1)] = lo_any ? 1u : 0u;
            }
            *reinterpret_cast<u32x4 *>(buf + St::kCop + (tl * 64 + ld_half * 32 + r) * 4) = cop;
        };

        // ---- pieces of one pipeline iteration
        // Scores of tile t (raw accumulators): constant-term MFMA, then high and low query parts.
        auto score_tile = [&](int t, f32x16 (&sn)[kRB]) {
            const uint32_t *buf = lds + ((uint32_t)(t >> 2) % kBuffers) * St::kWords;
            const int tl = t & 3;
            uint32_t kw[WPL];
            {
                const uint32_t *src = buf + St::kK + tl * 64 * WPL + lane * WPL;
#pragma unroll
                for (int i = 0; i < WPL / 4; ++i) {
                    const u32x4 w = *reinterpret_cast<const u32x4 *>(src + 4 * i);
                    kw[4 * i] = w.x; kw[4 * i + 1] = w.y; kw[4 * i + 2] = w.z; kw[4 * i + 3] = w.w;
                }
            }
            const u32x4 cop = *reinterpret_cast<const u32x4 *>(buf + St::kCop + (tl * 64 + lane) * 4);
            if constexpr (kVs) {
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) const_mfma_v(sn[rb], cop, rowop[rb]);
                static_for<2>([&](auto j_) {
                    const i32x4 a4 = fp4_operand4(j_, kw);
                    static_for<4>([&](auto k_) {
#pragma unroll
                        for (int rb = 0; rb < kRB; ++rb) fp4_mfma_v(j_, k_, IntC<1>{}, a4, sn[rb], rb);
                    });
                });
                KVQ_SCORE_TILE_READY("s_nop 11", sn);
                return;
            }
            f32x16 zero;
#pragma unroll
            for (int v = 0; v < 16; ++v) zero[v] = 0.0f;
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) sn[rb] = mfma_bf16(cop, rowop[rb], zero);
            // The low parts of q~ stay in LDS: the offset is made opaque so that the loads are issued per
            // tile instead of being hoisted into registers that do not exist.
            uint32_t off = lo_off;
            asm volatile("" : "+v"(off));
            const uint32_t *qlo = q_stage + off;
            if constexpr (kFp4) {
                score_fp4(IntC<0>{}, kw, sn);
                score_fp4(IntC<1>{}, kw, sn);
            } else
            static_for<8>([&](auto s_) {
                constexpr int SLAB = decltype(s_)::value;
                const u32x4 kop = key_operand<BITS, SLAB>(kw, uc);
                u32x4 lo[kRB];
                if constexpr (kLoF16 && SLAB >= kLoRes) {
#pragma unroll
                    for (int rb = 0; rb < kRB; ++rb) lo[rb] = *reinterpret_cast<const u32x4 *>(qlo + 32 * rb * kQRowWords + 8 * SLAB);
                }
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) sn[rb] = mfma_f16(kop, qop[rb][SLAB], sn[rb]);
                if constexpr (kLoF16) {
#pragma unroll
                    for (int rb = 0; rb < kRB; ++rb) {
                        if constexpr (SLAB < kLoRes) sn[rb] = mfma_f16(kop, lo_res[rb][SLAB], sn[rb]);
                        else sn[rb] = mfma_f16(kop, lo[rb], sn[rb]);
                    }
                }
            });
            if constexpr (kLoFp8) {
                low_part_fp8(IntC<0>{}, kw, sn);
                low_part_fp8(IntC<1>{}, kw, sn);
            }
        };
        // e = scale_i * raw - reference; returns the tile maximum of e per row block.
        auto finalize_tile = [&](int t, const f32x16 (&sn)[kRB], float (&e)[kRB][16], float (&tmax)[kRB]) {
            const uint32_t *buf = lds + ((uint32_t)(t >> 2) % kBuffers) * St::kWords;
            const float *ks = reinterpret_cast<const float *>(buf + St::kKScale) + (t & 3) * 32 + hh * 16;
            float k_scale[16];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 c = *reinterpret_cast<const float4 *>(ks + 4 * g);
                k_scale[4 * g] = c.x; k_scale[4 * g + 1] = c.y; k_scale[4 * g + 2] = c.z; k_scale[4 * g + 3] = c.w;
            }
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) {
#pragma unroll
                for (int v = 0; v < 16; ++v) e[rb][v] = fmaf(k_scale[v], sn[rb][v], -m_ref[rb]);
                float mx = fmaxf(e[rb][0], e[rb][1]);
#pragma unroll
                for (int v = 2; v < 16; v += 2) mx = fmaxf(mx, fmaxf(e[rb][v], e[rb][v + 1]));
                tmax[rb] = max_halves(mx);
            }
        };
        // p' = 2^e (the value scale is in e), partial sums of p' / value-scale, p' rounded to bf16 (B operands), tau.
        auto exp_tile = [&](int t, const float (&e)[kRB][16], u32x4 (&pop)[kRB][2]) {
            const uint32_t *buf = lds + ((uint32_t)(t >> 2) % kBuffers) * St::kWords;
            const int pos = (t & 3) * 32 + hh * 16;
            const float *vsp = reinterpret_cast<const float *>(buf + St::kVScale) + pos;
            float v_inv[16];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 c = *reinterpret_cast<const float4 *>(vsp + 4 * g);
                v_inv[4 * g] = c.x; v_inv[4 * g + 1] = c.y; v_inv[4 * g + 2] = c.z; v_inv[4 * g + 3] = c.w;
            }
            uint32_t zh[8], zl[8];
            {
                const u32x4 h0 = *reinterpret_cast<const u32x4 *>(buf + St::kVzHi + pos / 2);
                const u32x4 h1 = *reinterpret_cast<const u32x4 *>(buf + St::kVzHi + pos / 2 + 4);
                const u32x4 l0 = *reinterpret_cast<const u32x4 *>(buf + St::kVzLo + pos / 2);
                const u32x4 l1 = *reinterpret_cast<const u32x4 *>(buf + St::kVzLo + pos / 2 + 4);
                zh[0] = h0.x; zh[1] = h0.y; zh[2] = h0.z; zh[3] = h0.w; zh[4] = h1.x; zh[5] = h1.y; zh[6] = h1.z; zh[7] = h1.w;
                zl[0] = l0.x; zl[1] = l0.y; zl[2] = l0.z; zl[3] = l0.w; zl[4] = l1.x; zl[5] = l1.y; zl[6] = l1.z; zl[7] = l1.w;
            }
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) {
                float lsum = 0.0f, tacc = 0.0f;
                uint32_t pw[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float p0 = __builtin_amdgcn_exp2f(e[rb][2 * i]);
                    const float p1 = __builtin_amdgcn_exp2f(e[rb][2 * i + 1]);
                    lsum = fmaf(p1, v_inv[2 * i + 1], fmaf(p0, v_inv[2 * i], lsum));
                    pw[i] = pack_bf16(p0, p1);
                    tacc = dot2_bf16(pw[i], zh[i], tacc);
                    tacc = dot2_bf16(pw[i], zl[i], tacc);
                }
                l_s[rb] += lsum;
                tau[rb] += tacc;
                pop[rb][0].x = pw[0]; pop[rb][0].y = pw[1]; pop[rb][0].z = pw[2]; pop[rb][0].w = pw[3];
                pop[rb][1].x = pw[4]; pop[rb][1].y = pw[5]; pop[rb][1].z = pw[6]; pop[rb][1].w = pw[7];
            }
        };
        // O^T += V^T P^T on raw codes.
        auto pv_tile = [&](int t, const u32x4 (&pop)[kRB][2]) {
            const uint32_t *buf = lds + ((uint32_t)(t >> 2) % kBuffers) * St::kWords;
            uint32_t vw[WPL];
            {
                const uint32_t *src = buf + St::kV + (t & 3) * 64 * WPL + lane * WPL;
#pragma unroll
                for (int i = 0; i < WPL / 4; ++i) {
                    const u32x4 w = *reinterpret_cast<const u32x4 *>(src + 4 * i);
                    vw[4 * i] = w.x; vw[4 * i + 1] = w.y; vw[4 * i + 2] = w.z; vw[4 * i + 3] = w.w;
                }
            }
            static_for<4>([&](auto b_) {
                constexpr int B = decltype(b_)::value;
                const u32x4 v0 = value_operand<BITS, B, 0>(vw, uc);
                const u32x4 v1 = value_operand<BITS, B, 1>(vw, uc);
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) o[B][rb] = mfma_bf16(v0, pop[rb][0], o[B][rb]);
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) o[B][rb] = mfma_bf16(v1, pop[rb][1], o[B][rb]);
            });
        };
        // One steady-state iteration, interleaved by hand: the score MFMAs of tile t+1 (4 per key slab)
        // next to one eighth of the exponential work of tile t, then the P*V MFMAs of tile t (4 per channel
        // block) next to one quarter of the score scaling of tile t+1.  Nothing crosses a chunk boundary,
        // so every group of four MFMAs has about as much independent vector work beside it, and every LDS
        // operand is requested one chunk (or one iteration) before the instruction that consumes it.
        struct Prefetched {
            uint32_t kw[WPL];   // packed key codes of the tile scored next
            u32x4 cop;          // its constant-term operand
        };
        auto prefetch_keys_at = [&](const uint32_t *buf, int tl, Prefetched &pf) {
            const uint32_t *src = buf + St::kK + tl * 64 * WPL + lane * WPL;
#pragma unroll
            for (int i = 0; i < WPL / 4; ++i) {
                const u32x4 w = *reinterpret_cast<const u32x4 *>(src + 4 * i);
                pf.kw[4 * i] = w.x; pf.kw[4 * i + 1] = w.y; pf.kw[4 * i + 2] = w.z; pf.kw[4 * i + 3] = w.w;
            }
            pf.cop = *reinterpret_cast<const u32x4 *>(buf + St::kCop + (tl * 64 + lane) * 4);
        };
        auto prefetch_keys = [&](int t, Prefetched &pf) {
            const uint32_t *buf = lds + ((uint32_t)(t >> 2) % kBuffers) * St::kWords;
            const int tl = t & 3;
            const uint32_t *src = buf + St::kK + tl * 64 * WPL + lane * WPL;
#pragma unroll
            for (int i = 0; i < WPL / 4; ++i) {
                const u32x4 w = *reinterpret_cast<const u32x4 *>(src + 4 * i);
                pf.kw[4 * i] = w.x; pf.kw[4 * i + 1] = w.y; pf.kw[4 * i + 2] = w.z; pf.kw[4 * i + 3] = w.w;
            }
            pf.cop = *reinterpret_cast<const u32x4 *>(buf + St::kCop + (tl * 64 + lane) * 4);
        };
        uint32_t stage_lo_flag = 0u;   // "some low zero-point part is nonzero" of the stage that holds the tile in hand
        // tl_: IntC<t mod 4> where the caller knows it at compile time (the unrolled fast loop), IntC<-1> otherwise.
        auto fused_iteration = [&](auto tl_, int t, Prefetched &pf, f32x16 (&sn)[kRB], float (&e)[kRB][16], float (&tmax)[kRB],
                                   u32x4 (&pop)[kRB][2], uint32_t &lo_flag) {
            constexpr int TL = decltype(tl_)::value;
            const uint32_t *bufc = lds + ((uint32_t)(t >> 2) % kBuffers) * St::kWords;         // holds tile t
            const uint32_t *bufx = lds + ((uint32_t)((t >> 2) + 1) % kBuffers) * St::kWords;   // the stage after
            const uint32_t *bufn = TL < 0 ? lds + ((uint32_t)((t + 1) >> 2) % kBuffers) * St::kWords : TL == 3 ? bufx : bufc;   // holds tile t+1
            const int tln = TL < 0 ? (t + 1) & 3 : (TL + 1) & 3, tlc = TL < 0 ? t & 3 : TL;
            const int pos = tlc * 32 + hh * 16;
            // requests for this iteration's exponential work
            float v_inv[16];
            {
                const float *vsp = reinterpret_cast<const float *>(bufc + St::kVScale) + pos;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 c = *reinterpret_cast<const float4 *>(vsp + 4 * g);
                    v_inv[4 * g] = c.x; v_inv[4 * g + 1] = c.y; v_inv[4 * g + 2] = c.z; v_inv[4 * g + 3] = c.w;
                }
            }
            uint32_t zh[8];
            {
                const u32x4 h0 = *reinterpret_cast<const u32x4 *>(bufc + St::kVzHi + pos / 2);
                const u32x4 h1 = *reinterpret_cast<const u32x4 *>(bufc + St::kVzHi + pos / 2 + 4);
                zh[0] = h0.x; zh[1] = h0.y; zh[2] = h0.z; zh[3] = h0.w; zh[4] = h1.x; zh[5] = h1.y; zh[6] = h1.z; zh[7] = h1.w;
            }
            // The flags belong to the stage: the unrolled loop reads them with the stage's first tile only.
            if constexpr (TL <= 0) {
                const u32x2 lo_flags = *reinterpret_cast<const u32x2 *>(bufc + St::kFlags);
                stage_lo_flag = lo_flags.x | lo_flags.y;
            }
            uint32_t off = lo_off;
            asm volatile("" : "+v"(off));
            const uint32_t *qlo = q_stage + off;
            u32x4 lo_cur[kRB], lo_nxt[kRB], kop_prev;
            f32x16 zero;
#pragma unroll
            for (int v = 0; v < 16; ++v) zero[v] = 0.0f;
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) {
                if constexpr (kVs) const_mfma_v(sn[rb], pf.cop, rowop[rb]);
                else sn[rb] = mfma_bf16(pf.cop, rowop[rb], zero);
            }
            float lsum[kRB] = {}, tacc[kRB] = {};
            uint32_t pw[kRB][8];
            uint32_t vw[WPL];
            float k_scale[16];
            auto exp_chunk = [&](auto c_) {
                constexpr int C = decltype(c_)::value;   // one eighth of the tile: kRB probability words
                constexpr int RB = (C * kRB) / 8, I0 = (C * kRB) % 8;
#pragma unroll
                for (int i = I0; i < I0 + kRB; ++i) {
                    const float p0 = __builtin_amdgcn_exp2f(e[RB][2 * i]);
                    const float p1 = __builtin_amdgcn_exp2f(e[RB][2 * i + 1]);
                    lsum[RB] = fmaf(p1, v_inv[2 * i + 1], fmaf(p0, v_inv[2 * i], lsum[RB]));
                    pw[RB][i] = pack_bf16(p0, p1);
                    tacc[RB] = dot2_bf16(pw[RB][i], zh[i], tacc[RB]);
                }
            };
            i32x8 a4 = {};
            i32x4 a4v = {};
            KVQ_CHUNK_FENCE();
            static_for<8>([&](auto s_) {
                constexpr int SLAB = decltype(s_)::value;
                // This slab's low query parts are requested now and multiplied one chunk later, so that no
                // MFMA of the iteration waits for LDS: the high parts and the key codes are in registers.
                if constexpr (kLoF16 && SLAB >= kLoRes) {
#pragma unroll
                    for (int rb = 0; rb < kRB; ++rb)
                        lo_nxt[rb] = *reinterpret_cast<const u32x4 *>(qlo + 32 * rb * kQRowWords + 8 * SLAB);
                }
                if constexpr (SLAB == 5) {  // value codes and key scales for the second half of the iteration
                    const uint32_t *src = bufc + St::kV + tlc * 64 * WPL + lane * WPL;
#pragma unroll
                    for (int i = 0; i < WPL / 4; ++i) {
                        const u32x4 w = *reinterpret_cast<const u32x4 *>(src + 4 * i);
                        vw[4 * i] = w.x; vw[4 * i + 1] = w.y; vw[4 * i + 2] = w.z; vw[4 * i + 3] = w.w;
                    }
                    const float *ks = reinterpret_cast<const float *>(bufn + St::kKScale) + tln * 32 + hh * 16;
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const float4 c = *reinterpret_cast<const float4 *>(ks + 4 * g);
                        k_scale[4 * g] = c.x; k_scale[4 * g + 1] = c.y; k_scale[4 * g + 2] = c.z; k_scale[4 * g + 3] = c.w;
                    }
                }
                u32x4 kop;
                if constexpr (kVs) {    // chunk SLAB: piece SLAB % 4 against key words 2 (SLAB / 4), + 1
                    if constexpr (SLAB % 4 == 0) a4v = fp4_operand4(IntC<SLAB / 4>{}, pf.kw);
                    fp4_mfma_v(IntC<SLAB / 4>{}, IntC<SLAB % 4>{}, IntC<1>{}, a4v, sn[0], 0);
#pragma unroll
                    for (int rb = 1; rb < kRB; ++rb) fp4_mfma_v(IntC<SLAB / 4>{}, IntC<SLAB % 4>{}, IntC<0>{}, a4v, sn[rb], rb);
                } else if constexpr (kFp4) {
                    if constexpr (SLAB % 4 == 0) a4 = fp4_operand(IntC<SLAB / 4>{}, pf.kw);
                    fp4_mfma(IntC<SLAB / 4>{}, IntC<SLAB % 4>{}, a4, sn);
                } else {
                    kop = key_operand<BITS, SLAB>(pf.kw, uc);
#pragma unroll
                    for (int rb = 0; rb < kRB; ++rb) sn[rb] = mfma_f16(kop, qop[rb][SLAB], sn[rb]);
                }
                if constexpr (SLAB >= 1) {
                    if constexpr (kLoF16) {
#pragma unroll
                        for (int rb = 0; rb < kRB; ++rb) {
                            if constexpr (SLAB - 1 < kLoRes) sn[rb] = mfma_f16(kop_prev, lo_res[rb][SLAB - 1], sn[rb]);
                            else sn[rb] = mfma_f16(kop_prev, lo_cur[rb], sn[rb]);
                        }
                    }
                    if constexpr (kLoFp8 && SLAB == 4) low_part_fp8(IntC<0>{}, pf.kw, sn);   // key words 0, 1: slabs 0..3
                    exp_chunk(IntC<SLAB - 1>{});
                }
                if constexpr (kLoF16) {
                    kop_prev = kop;
                    if constexpr (SLAB >= kLoRes) {
#pragma unroll
                        for (int rb = 0; rb < kRB; ++rb) lo_cur[rb] = lo_nxt[rb];
                    }
                }
                KVQ_CHUNK_FENCE();
            });
            if constexpr (kLoF16) {
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) {
                    if constexpr (7 < kLoRes) sn[rb] = mfma_f16(kop_prev, lo_res[rb][7], sn[rb]);
                    else sn[rb] = mfma_f16(kop_prev, lo_cur[rb], sn[rb]);
                }
            }
            if constexpr (kLoFp8) low_part_fp8(IntC<1>{}, pf.kw, sn);
            exp_chunk(IntC<7>{});
            // Four exponentials and two conversions have been issued since the last score MFMA: six more wait
            // states make the twelve that a vector read of its result needs.
            if constexpr (kVs) asm volatile("s_nop 5" : "+v"(sn[0]), "+v"(sn[kRB - 1]), "+v"(pw[kRB - 1][6]), "+v"(pw[kRB - 1][7]));
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) {
                l_s[rb] += lsum[rb];
                tau[rb] += tacc[rb];
                pop[rb][0].x = pw[rb][0]; pop[rb][0].y = pw[rb][1]; pop[rb][0].z = pw[rb][2]; pop[rb][0].w = pw[rb][3];
                pop[rb][1].x = pw[rb][4]; pop[rb][1].y = pw[rb][5]; pop[rb][1].z = pw[rb][6]; pop[rb][1].w = pw[rb][7];
            }
            lo_flag = stage_lo_flag;
            // key codes of the tile after next (its stage has been opened at the top of this iteration)
            if constexpr (TL < 0) prefetch_keys(t + 2, pf);
            else prefetch_keys_at(TL >= 2 ? bufx : bufc, (TL + 2) & 3, pf);
            KVQ_CHUNK_FENCE();   // the score accumulators are read after all of the above, not before
            float mx[kRB];
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) mx[rb] = -INFINITY;
            static_for<4>([&](auto b_) {
                constexpr int B = decltype(b_)::value;
                const u32x4 v0 = value_operand<BITS, B, 0>(vw, uc);
                const u32x4 v1 = value_operand<BITS, B, 1>(vw, uc);
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) o[B][rb] = mfma_bf16(v0, pop[rb][0], o[B][rb]);
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) o[B][rb] = mfma_bf16(v1, pop[rb][1], o[B][rb]);
                constexpr int RB = (B * 4 * kRB) / 16, V0 = (B * 4 * kRB) % 16;   // one quarter of the tile
#pragma unroll
                for (int v = V0; v < V0 + 4 * kRB; ++v) e[RB][v] = fmaf(k_scale[v], sn[RB][v], -m_ref[RB]);
#pragma unroll
                for (int v = V0; v < V0 + 4 * kRB; v += 2) mx[RB] = __builtin_fmaxf(__builtin_fmaxf(mx[RB], e[RB][v]), e[RB][v + 1]);
                KVQ_CHUNK_FENCE();
            });
            // tmax: the maximum over this lane's 16 keys of each row block.  The loop only asks whether any lane is
            // over the threshold; the other half of the row is brought in (max_halves) when the loop has been left.
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) tmax[rb] = mx[rb];
        };
        // Zero-points whose OFFSET + z needs a second bf16 piece (magnitude above 256) are rare.  The loader
        // flags the stages that hold one; the fast loop only carries the flag and is left after such a tile,
        // whose probabilities (still in pop) then meet the low parts here.
        auto add_low_zero_points = [&](int t, const u32x4 (&pop)[kRB][2]) {
            const uint32_t *buf = lds + ((uint32_t)(t >> 2) % kBuffers) * St::kWords;
            const int pos = (t & 3) * 32 + hh * 16;
            const u32x4 l0 = *reinterpret_cast<const u32x4 *>(buf + St::kVzLo + pos / 2);
            const u32x4 l1 = *reinterpret_cast<const u32x4 *>(buf + St::kVzLo + pos / 2 + 4);
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) {
                float tl = 0.0f;
                tl = dot2_bf16(pop[rb][0].x, l0.x, tl); tl = dot2_bf16(pop[rb][0].y, l0.y, tl);
                tl = dot2_bf16(pop[rb][0].z, l0.z, tl); tl = dot2_bf16(pop[rb][0].w, l0.w, tl);
                tl = dot2_bf16(pop[rb][1].x, l1.x, tl); tl = dot2_bf16(pop[rb][1].y, l1.y, tl);
                tl = dot2_bf16(pop[rb][1].z, l1.z, tl); tl = dot2_bf16(pop[rb][1].w, l1.w, tl);
                tau[rb] += tl;
            }
        };
        // A stage becomes visible one tile before its first tile is scored.
        auto open_stage = [&](int stage) {
            commit(stage);
            prefetch(stage + 1);
            __syncthreads();
        };

        prefetch(0);
        open_stage(0);
        f32x16 sn[kRB];
        float e[kRB][16], tmax[kRB];
        u32x4 pop[kRB][2];
        score_tile(0, sn);
        finalize_tile(0, sn, e, tmax);
        if (n_tiles > 4) open_stage(1);   // stages are opened two tiles before their first tile is scored
        Prefetched pf;
        prefetch_keys(1, pf);
        int t = 0;
        int t_open = 6;      // stage s (tiles 4 s ..) is opened while tile 4 s - 2 is being scored: s = 2 at t = 6
        bool done = false;
        uint32_t lo_flag = 0u;   // nonzero: tile t-1 still owes tau its low zero-point parts
        while (!done) {
            if (__builtin_amdgcn_readfirstlane(lo_flag) != 0u) {
                add_low_zero_points(t - 1, pop);
                lo_flag = 0u;
            }
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) tmax[rb] = max_halves(tmax[rb]);   // (a fused iteration leaves per-lane maxima)
            move_reference(e, tmax);
            // fast loop: nothing in here touches the accumulators except the MFMAs
            if constexpr (KVQ_UNROLL_STAGE && kVs) {
                // Up to the next stage boundary one tile at a time (the loop is left and re-entered at any tile when
                // a reference maximum has to move), then four tiles per trip.  Stage s is opened while tile 4 s - 2
                // is being scored; stages 0 and 1 are open when the loop is entered for the first time.
                bool leave = false;
#define KVQ_STEP(TLV)                                                                                                 \
                {                                                                                                     \
                    if (__builtin_expect(t + 1 >= n_tiles, 0)) {                                                      \
                        done = true;                                                                                  \
                        leave = true;                                                                                 \
                        break;                                                                                        \
                    }                                                                                                 \
                    if (((TLV) == 2 || ((TLV) < 0 && (t & 3) == 2)) && t >= 6) open_stage((t + 2) >> 2);              \
                    fused_iteration(IntC<(TLV)>{}, t, pf, sn, e, tmax, pop, lo_flag);                                 \
                    ++t;                                                                                              \
                    if (__builtin_expect(__any(over_threshold(tmax) || lo_flag != 0u), 0)) {                          \
                        leave = true;                                                                                 \
                        break;                                                                                        \
                    }                                                                                                 \
                }
                while ((t & 3) != 0) KVQ_STEP(-1)
                if (!leave)
                    for (;;) {
                        KVQ_STEP(0)
                        KVQ_STEP(1)
                        KVQ_STEP(2)
                        KVQ_STEP(3)
                    }
#undef KVQ_STEP
                if (done) {   // the last tile has no successor to score
                    exp_tile(t, e, pop);
                    pv_tile(t, pop);
                }
            } else
            for (;;) {
                if (__builtin_expect(t + 1 >= n_tiles, 0)) {
                    exp_tile(t, e, pop);
                    pv_tile(t, pop);
                    done = true;
                    break;
                }
                if (__builtin_expect(t == t_open, 0)) {
                    open_stage((t + 2) >> 2);
                    t_open += 4;
                }
                fused_iteration(IntC<-1>{}, t, pf, sn, e, tmax, pop, lo_flag);
                ++t;
                if (__builtin_expect(__any(over_threshold(tmax) || lo_flag != 0u), 0)) break;
            }
        }

        }   // key blocks

        // ---- leave the rotated basis: O <- Hn^T (O_rot - tau 1).  Channel index of register
        // (b, v) in lane half hh: c = 32 b + 8 (v >> 2) + 4 hh + (v & 3).
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) {
#pragma unroll
            for (int h = 1; h < 16; h <<= 1) {   // channel bits 0, 1 (v bits 0, 1) and 3, 4 (v bits 2, 3)
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
#pragma unroll
            for (int h = 1; h < 4; h <<= 1) {    // channel bits 5, 6 (block)
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
#pragma unroll
            for (int b = 0; b < 4; ++b)          // channel bit 2 lives in the lane half
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float own = o[b][rb][v], other = xhalf(own);
                    o[b][rb][v] = (hh ? other - own : own + other) * 0.088388347648318f;
                }
            // Hn^T (tau 1) = tau sqrt(d) e_0: only channel 0 (lane half 0, block 0, register 0) sees it.
            const float tau_all = tau[rb] + xhalf(tau[rb]);
            if (hh == 0) o[0][rb][0] -= tau_all * 11.313708498984761f;
            // The transpose of the randomised rotation ends with the channel signs.
            if (has_signs(a.cv))
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const uint32_t sg = a.cv.sign_mask[b] >> (4 * hh);
#pragma unroll
                for (int v = 0; v < 16; ++v) o[b][rb][v] = flip_sign(o[b][rb][v], sg >> (8 * (v >> 2) + (v & 3)));
            }
        }
    }

#include "kvq_mfma_current_phase.inc"

    // ------------------------------------------------------------------------- epilogue ----
    uint16_t *out_base = static_cast<uint16_t *>(a.out) + qhead_off;
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) {
        const float ls = l_s[rb] + xhalf(l_s[rb]);
        const float lr = l_r[rb] + xhalf(l_r[rb]);
        const float inv = 1.0f / (ls + lr);
        const int64_t row = wave_row0 + 32 * rb + n;
        if (row < a.m) {
            uint16_t *dst = out_base + row * a.q_stride_token + 4 * hh;
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    u32x2 w;
                    w.x = pack_bf16(o[b][rb][4 * g] * inv, o[b][rb][4 * g + 1] * inv);
                    w.y = pack_bf16(o[b][rb][4 * g + 2] * inv, o[b][rb][4 * g + 3] * inv);
                    *reinterpret_cast<u32x2 *>(dst + 32 * b + 8 * g) = w;
                }
            if (a.mass_cached && hh == 0) a.mass_cached[(int64_t)qhead * a.m + row] = ls * inv;
        }
    }
}

template <int BITS, bool CORR, bool FP8META, bool PERCH = false> hipError_t launch(const AttentionArgs &a, hipStream_t stream)
{
    static std::atomic<uint64_t> configured{0};  // per instantiation and device
    const void *fn = reinterpret_cast<const void *>(&attention_mfma_kernel<BITS, CORR, FP8META, PERCH>);
    const hipError_t ce = configure_dynamic_lds(fn, lds_bytes<BITS>(), configured);
    if (ce != hipSuccess) return ce;
    const int row_blocks = (int)((a.m + kRowsPerBlock - 1) / kRowsPerBlock);
    const int64_t blocks = (int64_t)row_blocks * a.cv.num_heads * a.q_per_kv;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    return launch_kernel(attention_mfma_kernel<BITS, CORR, FP8META, PERCH>, dim3((unsigned)blocks), dim3(kThreads), lds_bytes<BITS>(),
                         stream, a, row_blocks);
}

}  // namespace

hipError_t launch_attention_mfma(const AttentionArgs &a, hipStream_t stream)
{
    if (a.cv.head_dim != D || a.cv.io_dtype != KVQ_BF16) return hipErrorInvalidValue;
    if (a.cv.meta_format != KVQ_META_FP32 && a.cv.group_size != D) return hipErrorInvalidValue;
    if (a.cache_len > (int64_t)0x3fffffff * kTileTokens) return hipErrorInvalidValue;
    const bool fp8 = a.cv.meta_format == KVQ_META_FP8_BF16;
    if (a.cv.key_axis == KVQ_KEYS_PER_CHANNEL) {   // the caller has listed the key blocks of the window
        if (fp8 || a.n_key_blocks < 1 || a.n_key_blocks > kMaxKeyBlocks || a.cache_len < 1) return hipErrorInvalidValue;
        if (a.cv.bits == 2) return a.correction ? launch<2, true, false, true>(a, stream) : launch<2, false, false, true>(a, stream);
        return a.correction ? launch<4, true, false, true>(a, stream) : launch<4, false, false, true>(a, stream);
    }
    if (a.cv.bits == 2 && !fp8) return a.correction ? launch<2, true, false>(a, stream) : launch<2, false, false>(a, stream);
    if (a.cv.bits == 4 && !fp8) return a.correction ? launch<4, true, false>(a, stream) : launch<4, false, false>(a, stream);
    if (a.cv.bits == 2 && fp8) return a.correction ? launch<2, true, true>(a, stream) : launch<2, false, true>(a, stream);
    if (a.cv.bits == 4 && fp8) return a.correction ? launch<4, true, true>(a, stream) : launch<4, false, true>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace kvq
