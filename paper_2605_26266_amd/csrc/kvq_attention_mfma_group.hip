// Matrix-core chunk attention for caches with several (scale, zero-point) groups per token:
// BF16 I/O, head_dim 128, FP8-E4M3 scales and BF16 zero-points per group of 32 or 64 rotated channels
// (the storage format of the paper's "Effective bitwidth" formula, B + 24/g); 2- or 4-bit codes.
//
// The structure is that of the per-token kernel (kvq_attention_mfma.hip: transposed products, one wave
// per 64 query rows, lazy reference maximum, hand-interleaved pipeline); what changes is where the
// scales go.  A step with an FP8 scale has four significant bits, and an unpacked code value
// BASE + 4^-g code at most seven, so their product is exact in f16.  Hence:
//   * keys: every operand register is multiplied by its group's step (one v_pk_mul_f16), the score MFMA
//     accumulates sum_j step_ij (q~_j . code_ij) + BASE sum_j step_ij W_mj directly in log2 units, and
//     nothing is left to scale afterwards;
//   * the constant terms  sum_j step_ij (z_ij S_mj + BASE W_mj) + step_ij^2 nu'_mj  (zero-points, operand
//     offset, and the per-group Taylor correction of Alg. 1 / App. "Extension to QuaRot") are 11 G + 1
//     rank-one products, i.e. three (G = 4) or two (G = 2) extra 16-wide MFMAs whose A operands the
//     loader builds per key and whose B operands are built per query row in the prologue;
//   * values: a 32-channel block of the output lies inside one group, so the value operand registers
//     are multiplied by per-token steps as well (f16 operands; probabilities are f16 with the reference
//     maximum shifted by 2^7 to keep small weights out of the denormals), and the zero-point term of
//     each group is one more row of a small A operand, so tau_j comes out of two MFMAs per tile
//     instead of vector dot products.
#include "kvq_internal.h"

#include <type_traits>

namespace kvq {
namespace {

#include "kvq_mfma_common.h"

#ifndef KVQ_FREE_LAST_ROWOP
#define KVQ_FREE_LAST_ROWOP 1
#endif
constexpr int kGBuffers = 3;         // a stage is overwritten three stages after it was opened
constexpr float kPShift = 7.0f;      // f16 probabilities: the row maximum sits at 2^7, overflow at 2^16

__device__ inline uint32_t pk_mul_f16(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(f16x2, a) * __builtin_bit_cast(f16x2, b));
}
__device__ inline uint16_t f16_bits(float f) { return (uint16_t)(pack_f16(f, 0.0f) & 0xffffu); }
__device__ inline float f16_val(uint16_t b) { return f16_lo((uint32_t)b); }

// Constant-term slots.  Slot s = 11 j + t belongs to group j; slot 11 G is the window mask; slots 11 G + 1
// and 11 G + 2 carry minus the row's reference maximum (two bf16 pieces on the row side against ones on the
// key side), so that the accumulators come out relative to the reference and no vector instruction has to
// subtract it.  The reference is kept equal to the sum of its two pieces.
//   t = 0..2   key side step_j             x row side -BASE W_j      in three bf16 pieces
//   t = 3..8   key side (z step)_j, 2 pcs  x row side -S_j           in three pieces (each key piece meets all)
//   t = 9..10  key side step_j^2           x row side -nu'_j         in two pieces
template <int G> struct Slots {
    static constexpr int kCount = 11 * G + 3;
    static constexpr int kOperands = (kCount + 15) / 16;   // 16-wide MFMAs
};
struct Split3 {
    uint16_t h, m, l;
};
__device__ inline Split3 split3(float x)
{
    Split3 r;
    r.h = bf16_bits(x);
    const float r1 = x - bf16_val(r.h);
    r.m = bf16_bits(r1);
    r.l = bf16_bits(r1 - bf16_val(r.m));
    return r;
}
struct RowGroup {      // per query row and group
    Split3 s, w;       // -S_j, -BASE W_j
    uint16_t n_h, n_l; // -nu'_j
};
struct KeyGroup {      // per key and group
    uint16_t step, step2, zs_h, zs_l;   // bf16: step, step^2 (both exact), z * step in two pieces
};
template <int G> __device__ inline uint16_t row_slot(const RowGroup (&r)[G], int s)
{
    if (s == 11 * G) return 0x3f80u;   // 1.0
    if (s > 11 * G) return 0u;
    const int j = s / 11, t = s % 11;
    const RowGroup &g = r[j];
    switch (t) {
        case 0: return g.w.h; case 1: return g.w.m; case 2: return g.w.l;
        case 3: case 6: return g.s.h; case 4: case 7: return g.s.m; case 5: case 8: return g.s.l;
        case 9: return g.n_h; default: return g.n_l;
    }
}
template <int G> __device__ inline uint16_t key_slot(const KeyGroup (&k)[G], uint16_t bias, int s)
{
    if (s == 11 * G) return bias;
    if (s == 11 * G + 1 || s == 11 * G + 2) return 0x3f80u;   // 1.0 against the reference pieces
    if (s > 11 * G) return 0u;
    const int j = s / 11, t = s % 11;
    const KeyGroup &g = k[j];
    if (t < 3) return g.step;
    if (t < 6) return g.zs_h;
    if (t < 9) return g.zs_l;
    return g.step2;
}

// Word offsets inside one stage buffer (128 keys).
template <int BITS, int G> struct GStage {
    static constexpr int WPL = D * BITS / 64;
    static constexpr int NC = Slots<G>::kOperands;
    static constexpr int kCodeWords = kStageTiles * 64 * WPL;   // per tensor
    static constexpr int kK = 0;
    static constexpr int kV = kCodeWords;
    static constexpr int kCop = 2 * kCodeWords;                       // [tile][NC][lane][4]   constant-term A operands
    static constexpr int kKs = kCop + kStageTiles * NC * 64 * 4;      // [tile][key][G]        f16 pair (step, step)
    static constexpr int kVs = kKs + kStageKeys * G;                  // [tile][blk][hh][8]    f16 pairs of value steps
    static constexpr int kTau = kVs + kStageTiles * 4 * 2 * 8;        // [tile][slab][hh][8 rows][4]  f16 A operand of tau
    static constexpr int kWords = kTau + kStageTiles * 2 * 2 * 8 * 4;
};

// Low query parts.  Those of the first kLoResident 16-channel slabs stay in accumulation registers, the others in
// LDS, rows kLoRowWords apart.  4-bit codes with groups of 32 have the largest stage buffers (three of 33 KB); with
// all eight slabs in LDS (70 KB) the workgroup would need more than the 160 KB a compute unit has, with six (53 KB)
// it fits.  In that variant the high parts are staged through the (still unused) stage buffers in the prologue.
template <int BITS, int G> struct LoLayout {
    static constexpr int kResident = (BITS == 4 && G == 4) ? 2 : 0;
    static constexpr int kRowWords = kResident ? (8 - kResident) * 8 + 4 : kQRowWords;
};

template <int BITS, int G> constexpr size_t group_lds_bytes()
{
    // stage buffers (the prologue's row constants live in them before the first stage is committed) |
    // low parts of q~ (also staging for the query prep and the V^T tiles)
    return sizeof(uint32_t) * (kGBuffers * GStage<BITS, G>::kWords + kRowsPerBlock * LoLayout<BITS, G>::kRowWords);
}

template <int BITS, bool CORR, int G>
__global__ __launch_bounds__(kThreads, 1) void attention_mfma_group_kernel(AttentionArgs a, int row_blocks)
{
    static_assert(kRB == 2, "64 rows per wave");
    if (cache_flagged(a.status)) return;   // the vector kernel enqueued behind this launch serves such a cache
    using St = GStage<BITS, G>;
    constexpr int WPL = St::WPL;
    constexpr int NC = St::NC;
    constexpr int kSlabsPerGroup = 8 / G;      // key slabs (16 channels) per group
    constexpr int kBlocksPerGroup = 4 / G;     // value blocks (32 channels) per group
    constexpr float kBase = Unpack<BITS>::kKeyBase;   // f16 unpacking on both sides
    extern __shared__ __align__(16) uint32_t lds[];
    uint32_t *q_stage = lds + kGBuffers * St::kWords;
    float *row_scal = reinterpret_cast<float *>(lds);   // [row][G][4]: S_j, W_j, -nu'_j; prologue only
    constexpr int kLoRes = LoLayout<BITS, G>::kResident, kLoRowWords = LoLayout<BITS, G>::kRowWords;
    // staging of the high parts (and of the resident low parts) in the prologue: rows kQRowWords apart
    uint32_t *hi_stage = kLoRes ? lds + kRowsPerBlock * G * 4 : q_stage;
    static_assert(!kLoRes || kRowsPerBlock * G * 4 + kRowsPerBlock * kQRowWords <= kGBuffers * St::kWords, "staging fits the stage buffers");
    static_assert(kRowsPerBlock * kLoRowWords >= 2 * D * 20 + 2 * kTileTokens * kQRowWords, "the current-chunk phase stages V^T and K tiles here");

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
    // Lane r of the block rotates query row r: q~ = Hn q * softmax_scale * log2(e) (times 4^g per channel,
    // the inverse of the weight its key codes are unpacked with), split into an f16 high and low part,
    // and per group the sums S_j (true scale), W_j (operand values) and nu_j = ||(Hn q)_j||^2.
    u32x4 qop[kRB][8];
    {
        const int prow = tid;
        int64_t row = (int64_t)rblk * kRowsPerBlock + prow;
        row = row < a.m ? row : a.m - 1;
        const uint4 *src = reinterpret_cast<const uint4 *>(q_base + row * a.q_stride_token);
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
        // Randomised rotation: the channel signs come before the Hadamard matrix.
        if (has_signs(a.cv))
#pragma unroll
        for (int i = 0; i < D; ++i) x[i] = flip_sign(x[i], a.cv.sign_mask[i >> 5] >> (i & 31));
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
        float nu[G];
#pragma unroll
        for (int j = 0; j < G; ++j) {
            nu[j] = 0.0f;
#pragma unroll
            for (int i = 0; i < D / G; ++i) nu[j] = fmaf(x[j * (D / G) + i], x[j * (D / G) + i], nu[j]);
        }
        const float cq = c_log * 0.088388347648318f;
#pragma unroll
        for (int i = 0; i < D; ++i) x[i] *= cq * (float)(1 << (2 * key_channel_class<BITS>(i)));
        uint32_t *dst = hi_stage + prow * kQRowWords;
        uint32_t *dst_lo = q_stage + prow * kLoRowWords;
#pragma unroll
        for (int i = 0; i < D / 8; ++i) {
            u32x4 w;
            w.x = pack_f16(x[8 * i], x[8 * i + 1]); w.y = pack_f16(x[8 * i + 2], x[8 * i + 3]);
            w.z = pack_f16(x[8 * i + 4], x[8 * i + 5]); w.w = pack_f16(x[8 * i + 6], x[8 * i + 7]);
            *reinterpret_cast<u32x4 *>(dst + 4 * i) = w;
        }
        __syncthreads();
        const uint32_t *hsrc = hi_stage + (wave * kRowsPerWave + n) * kQRowWords + 4 * hh;
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
            for (int s = 0; s < 8; ++s)
                qop[rb][s] = *reinterpret_cast<const u32x4 *>(hsrc + 32 * rb * kQRowWords + 8 * s);
        __syncthreads();
        float ssum[G], wsum[G];
#pragma unroll
        for (int j = 0; j < G; ++j) ssum[j] = wsum[j] = 0.0f;
#pragma unroll
        for (int i = 0; i < D / 8; ++i) {
            uint32_t lo[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float v0 = x[8 * i + 2 * j], v1 = x[8 * i + 2 * j + 1];
                const uint32_t hi = pack_f16(v0, v1);
                const float h0 = f16_lo(hi), h1 = f16_hi(hi);
                lo[j] = pack_f16(v0 - h0, v1 - h1);
                const float pair = (h0 + f16_lo(lo[j])) + (h1 + f16_hi(lo[j]));   // both channels share a class and a group
                const int c = 8 * i + 2 * j;
                wsum[c / (D / G)] += pair;
                ssum[c / (D / G)] += pair * (1.0f / (float)(1 << (2 * key_channel_class<BITS>(c))));
            }
            u32x4 w;
            w.x = lo[0]; w.y = lo[1]; w.z = lo[2]; w.w = lo[3];
            // eight channels = half a slab: the resident slabs go back through the staging rows, the others to their place
            if (i < 2 * kLoRes) *reinterpret_cast<u32x4 *>(dst + 4 * i) = w;
            else *reinterpret_cast<u32x4 *>(dst_lo + 4 * (i - 2 * kLoRes)) = w;
        }
#pragma unroll
        for (int j = 0; j < G; ++j) {
            float *rs = row_scal + (prow * G + j) * 4;
            rs[0] = ssum[j];
            rs[1] = wsum[j];
            // ||(Hn q)_j||^2 = nu_j / d on the unnormalised transform
            rs[2] = CORR ? -a.softmax_scale * a.softmax_scale * kLog2e * nu[j] * (1.0f / (24.0f * D)) : 0.0f;
        }
    }
    __syncthreads();
    // B operands of the constant-term MFMAs, per 32-row block: lane (row n, half hh) holds slots
    // 16 c + 8 hh .. + 7 of operand c.
    u32x4 rowop[NC][kRB];
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) {
        RowGroup rg[G];
#pragma unroll
        for (int j = 0; j < G; ++j) {
            const float *rs = row_scal + ((wave * kRowsPerWave + 32 * rb + n) * G + j) * 4;
            rg[j].s = split3(-rs[0]);
            rg[j].w = split3(-kBase * rs[1]);
            rg[j].n_h = bf16_bits(rs[2]);
            rg[j].n_l = bf16_bits(rs[2] - bf16_val(rg[j].n_h));
        }
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            uint32_t w[2][4];
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    w[h2][k] = (uint32_t)row_slot<G>(rg, 16 * c + 8 * h2 + 2 * k) |
                               ((uint32_t)row_slot<G>(rg, 16 * c + 8 * h2 + 2 * k + 1) << 16);
            rowop[c][rb].x = hh ? w[1][0] : w[0][0]; rowop[c][rb].y = hh ? w[1][1] : w[0][1];
            rowop[c][rb].z = hh ? w[1][2] : w[0][2]; rowop[c][rb].w = hh ? w[1][3] : w[0][3];
        }
    }
    u32x4 lo_res[kRB][kLoRes > 0 ? kLoRes : 1];
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
        for (int s = 0; s < kLoRes; ++s) {
            lo_res[rb][s] = *reinterpret_cast<const u32x4 *>(hi_stage + (wave * kRowsPerWave + 32 * rb + n) * kQRowWords + 4 * hh + 8 * s);
            asm volatile("" : "+a"(lo_res[rb][s]));
        }
    __syncthreads();   // the row constants and the staging rows are dead: the loader may now write the stage buffers
    const uint32_t lo_off = (uint32_t)((wave * kRowsPerWave + n) * kLoRowWords + 4 * hh);  // words into q_stage
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
        for (int s = 0; s < 8; ++s) asm volatile("" : "+a"(qop[rb][s]));
#pragma unroll
    for (int c = 0; c < NC - KVQ_FREE_LAST_ROWOP; ++c)   // the last operand holds the reference slots and changes with them
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) asm volatile("" : "+a"(rowop[c][rb]));

    f32x16 o[4][kRB];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[b][rb][v] = 0.0f;
    auto pin_accumulators = [&]() {
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) asm volatile("" : "+a"(o[b][rb]));
    };
    float m_ref[kRB] = {};              // reference (log2 domain): row maximum minus kPShift
    float l_s[kRB] = {}, l_r[kRB] = {};
    // tau[rb][i]: lanes of half hh hold, for query row n, row 4 hh + i of the tau operand = piece (i & 1)
    // of group 2 hh + (i >> 1)
    float tau[kRB][4] = {};
    bool first = true;

    // Writes the pieces of minus the reference into slots 11 G + 1, 11 G + 2 of the row operands of block rb.
    auto set_reference_slots = [&](int rb, uint16_t neg_h, uint16_t neg_l) {
        static_for<2>([&](auto p_) {
            constexpr int P2 = decltype(p_)::value;
            constexpr int SL = 11 * G + 1 + P2, C = SL / 16, K = SL % 16, R = (K % 8) / 2;
            const uint32_t val = P2 == 0 ? neg_h : neg_l;
            if (hh == K / 8) {
                const uint32_t old = rowop[C][rb][R];
                rowop[C][rb][R] = (K % 2) ? ((old & 0x0000ffffu) | (val << 16)) : ((old & 0xffff0000u) | val);
            }
        });
    };
    auto move_reference = [&](float (&e)[kRB][16], const float (&tmax)[kRB]) {
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) {
            const bool mv = first || tmax[rb] > kRescaleThreshold + kPShift;
            // the new reference is the sum of two bf16 pieces: the operand slots hold exactly what is subtracted
            const float want = m_ref[rb] + (mv ? tmax[rb] - kPShift : 0.0f);
            const uint16_t r_h = bf16_bits(want);
            const uint16_t r_l = bf16_bits(want - bf16_val(r_h));
            const float delta = mv ? (bf16_val(r_h) + bf16_val(r_l)) - m_ref[rb] : 0.0f;
            const float alpha = first ? 1.0f : __builtin_amdgcn_exp2f(-delta);
            m_ref[rb] += delta;
            if (mv) set_reference_slots(rb, (uint16_t)(r_h ^ 0x8000u), (uint16_t)(r_l ^ 0x8000u));
#pragma unroll
            for (int v = 0; v < 16; ++v) e[rb][v] -= delta;
            l_s[rb] *= alpha;
            l_r[rb] *= alpha;
#pragma unroll
            for (int i = 0; i < 4; ++i) tau[rb][i] *= alpha;
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
        for (int rb = 0; rb < kRB; ++rb) over = over || tmax[rb] > kRescaleThreshold + kPShift;
        return over;
    };

    // ---------------------------------------------------------------------- cached keys ----
    if (a.cache_len > 0) {
        const int64_t cs = a.cache_start, ce = a.cache_start + a.cache_len;
        const int64_t t_first = cs / kTileTokens, t_last = (ce - 1) / kTileTokens;
        const int n_tiles = (int)(t_last - t_first + 1);
        const int n_stages = (n_tiles + kStageTiles - 1) / kStageTiles;
        const int64_t head_tile0 = (int64_t)head * cv.cap_tiles;
        const int64_t meta0 = head_tile0 * kTileTokens;

        // ---- loader: global -> registers (prefetch), registers -> LDS (commit, builds every per-key operand)
        constexpr int kCodeVecs = St::kCodeWords / 4;
        constexpr int kCodeIters = 2 * kCodeVecs / kThreads;
        u32x4 pre_kv[kCodeIters];
        // The G E4M3 scales and G BF16 zero-points of a token are fetched as whole words and only taken apart when
        // the stage is committed: unpacking them here would make the wave wait for the loads it has just issued.
        using ScaleWord = typename std::conditional<G == 4, uint32_t, uint16_t>::type;   // G bytes
        using ZeroWord = typename std::conditional<G == 4, uint64_t, uint32_t>::type;    // G half-words
        ScaleWord raw_ks = 0, raw_vs = 0;
        ZeroWord raw_kz = 0, raw_vz = 0;
        uint32_t pre_in_window = 0u;   // a vector register, not a lane mask: it lives across the loop's branches
        const int ld_key = tid & 127, ld_half = (tid >> 7) & 1;
        // Ring arithmetic in 32 bits (the launcher sends caches of 2^20 tiles or more per head elsewhere): the
        // stage's first physical tile is uniform, a thread adds its tile inside the stage and wraps once more.
        const int cap = (int)cv.cap_tiles;
        const int first_off = (int)(cs - t_first * kTileTokens);   // position of cache_start inside its tile
        const int win_len = (int)a.cache_len;
        const uint32_t *code_src[kCodeIters];
        int code_tile[kCodeIters];
#pragma unroll
        for (int it = 0; it < kCodeIters; ++it) {
            const int g = tid + kThreads * it, vec = g % kCodeVecs;
            code_tile[it] = vec / (16 * WPL);
            code_src[it] = (g < kCodeVecs ? cv.k_codes : cv.v_codes) + head_tile0 * (64 * WPL) + (vec % (16 * WPL)) * 4;
        }
        auto prefetch = [&](int stage) {
            if (stage >= n_stages) return;
            int ring0 = (int)a.phys_tile_first + stage * kStageTiles;   // < 2 cap + 4: n_tiles <= cap + 1
            ring0 -= ring0 >= cap ? cap : 0;
            ring0 -= ring0 >= cap ? cap : 0;
#pragma unroll
            for (int it = 0; it < kCodeIters; ++it) {
                int tile = ring0 + code_tile[it];
                tile -= tile >= cap ? cap : 0;    // tiles past the window wrap onto tiles of the storage: masked later
                tile = tile < cap ? tile : cap - 1;   // (a ring of fewer than four tiles)
                pre_kv[it] = *reinterpret_cast<const u32x4 *>(code_src[it] + (int64_t)tile * (64 * WPL));
            }
            const int rel = stage * kStageKeys + ld_key - first_off;    // position inside the window
            pre_in_window = (rel >= 0 && rel < win_len) ? 1u : 0u;
            int mt = ring0 + (ld_key >> 5);
            mt -= mt >= cap ? cap : 0;
            mt = mt < cap ? mt : cap - 1;
            const int64_t tok = (int64_t)mt * kTileTokens + (ld_key & 31);
            const int64_t gi = (meta0 + tok) * G;
            raw_ks = *reinterpret_cast<const ScaleWord *>(cv.k_scale8 + gi);   // gi is a multiple of G: aligned
            raw_kz = *reinterpret_cast<const ZeroWord *>(cv.k_zero16 + gi);
            if (ld_half == 1) {
                raw_vs = *reinterpret_cast<const ScaleWord *>(cv.v_scale8 + gi);
                raw_vz = *reinterpret_cast<const ZeroWord *>(cv.v_zero16 + gi);
            }
        };
        auto commit = [&](int stage) {
            if (stage >= n_stages) return;
            uint32_t *buf = lds + ((uint32_t)stage % kGBuffers) * St::kWords;
#pragma unroll
            for (int it = 0; it < kCodeIters; ++it) {
                const int g = tid + kThreads * it;
                *reinterpret_cast<u32x4 *>(buf + St::kK + 4 * g) = pre_kv[it];
            }
            const bool pre_valid = pre_in_window != 0u;
            const int tl = ld_key >> 5, r = ld_key & 31;
            // Keys outside the window: every key-side factor is 0, the mask slot carries the bias.
            KeyGroup kg[G];
            uint32_t ks_pair[G];
#pragma unroll
            for (int j = 0; j < G; ++j) {
                const float step = pre_valid ? e4m3_low_byte((uint32_t)(raw_ks >> (8 * j))) : 0.0f;
                const float zs = step * bf16_val((uint16_t)(raw_kz >> (16 * j)));   // 4 x 8 significant bits: exact
                kg[j].step = bf16_bits(step);
                kg[j].step2 = bf16_bits(step * step);
                kg[j].zs_h = bf16_bits(zs);
                kg[j].zs_l = bf16_bits(zs - bf16_val(kg[j].zs_h));
                const uint32_t sf = f16_bits(step);
                ks_pair[j] = sf | (sf << 16);
            }
            const uint16_t bias = pre_valid ? (uint16_t)0 : bf16_bits(kMaskBias);
            // ld_half is uniform over a wave: each half builds only its own eight slots of every operand
            auto build_cops = [&](auto h_) {
                constexpr int H2 = decltype(h_)::value;
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    u32x4 cop;
                    cop.x = (uint32_t)key_slot<G>(kg, bias, 16 * c + 8 * H2 + 0) | ((uint32_t)key_slot<G>(kg, bias, 16 * c + 8 * H2 + 1) << 16);
                    cop.y = (uint32_t)key_slot<G>(kg, bias, 16 * c + 8 * H2 + 2) | ((uint32_t)key_slot<G>(kg, bias, 16 * c + 8 * H2 + 3) << 16);
                    cop.z = (uint32_t)key_slot<G>(kg, bias, 16 * c + 8 * H2 + 4) | ((uint32_t)key_slot<G>(kg, bias, 16 * c + 8 * H2 + 5) << 16);
                    cop.w = (uint32_t)key_slot<G>(kg, bias, 16 * c + 8 * H2 + 6) | ((uint32_t)key_slot<G>(kg, bias, 16 * c + 8 * H2 + 7) << 16);
                    *reinterpret_cast<u32x4 *>(buf + St::kCop + ((tl * NC + c) * 64 + H2 * 32 + r) * 4) = cop;
                }
            };
            if (ld_half == 0) build_cops(IntC<0>{});
            else build_cops(IntC<1>{});
            if (ld_half == 0) {
#pragma unroll
                for (int j = 0; j < G; ++j) buf[St::kKs + (tl * 32 + r) * G + j] = ks_pair[j];
            } else {
                // Value side of token r of the tile.  In the order in which the score MFMA leaves the tile in
                // a lane, the token is element v of lane half th: register v >> 1 of the P operand.
                const int th = (r >> 2) & 1, v = 4 * (r >> 3) + (r & 3);
                const int g2 = 2 * value_register_class<BITS>(v);
                uint16_t *vs16 = reinterpret_cast<uint16_t *>(buf + St::kVs);
                uint16_t *tau16 = reinterpret_cast<uint16_t *>(buf + St::kTau);
#pragma unroll
                for (int j = 0; j < G; ++j) {
                    const float step = pre_valid ? e4m3_low_byte((uint32_t)(raw_vs >> (8 * j))) : 0.0f;
                    const uint16_t sw = f16_bits(ldexpf(step, g2));   // step * 4^g, the inverse weight of the codes
#pragma unroll
                    for (int b = j * kBlocksPerGroup; b < (j + 1) * kBlocksPerGroup; ++b)
                        vs16[(((tl * 4 + b) * 2 + th) * 8 + (v >> 1)) * 2 + (v & 1)] = sw;
                    // tau multiplier: what the operand holds for code = z, i.e. step * (BASE 4^g + z)
                    const float zz = step * (ldexpf(kBase, g2) + bf16_val((uint16_t)(raw_vz >> (16 * j))));
                    const uint16_t z_h = f16_bits(zz);
                    const uint16_t z_l = f16_bits(zz - f16_val(z_h));
                    const int sl = v >> 3, i = v & 7;
                    const int base = ((((tl * 2 + sl) * 2 + th) * 8 + 2 * j) * 4 + (i >> 1)) * 2 + (i & 1);
                    tau16[base] = z_h;
                    tau16[base + 8] = z_l;   // next row: 4 words = 8 half-words further
                }
            }
        };

        // ---- pieces of one pipeline iteration
        struct Prefetched {
            uint32_t kw[WPL];
            u32x4 cop[NC];
        };
        auto prefetch_keys = [&](int t, Prefetched &pf) {
            const uint32_t *buf = lds + ((uint32_t)(t >> 2) % kGBuffers) * St::kWords;
            const int tl = t & 3;
            const uint32_t *src = buf + St::kK + tl * 64 * WPL + lane * WPL;
#pragma unroll
            for (int i = 0; i < WPL / 4; ++i) {
                const u32x4 w = *reinterpret_cast<const u32x4 *>(src + 4 * i);
                pf.kw[4 * i] = w.x; pf.kw[4 * i + 1] = w.y; pf.kw[4 * i + 2] = w.z; pf.kw[4 * i + 3] = w.w;
            }
#pragma unroll
            for (int c = 0; c < NC; ++c)
                pf.cop[c] = *reinterpret_cast<const u32x4 *>(buf + St::kCop + ((tl * NC + c) * 64 + lane) * 4);
        };
        // Steps of the lane's key for tile t, one f16 pair per group.
        auto load_key_steps = [&](int t, uint32_t (&ks)[G]) {
            const uint32_t *buf = lds + ((uint32_t)(t >> 2) % kGBuffers) * St::kWords;
            const uint32_t *src = buf + St::kKs + ((t & 3) * 32 + n) * G;
            if constexpr (G == 4) {
                const u32x4 w = *reinterpret_cast<const u32x4 *>(src);
                ks[0] = w.x; ks[1] = w.y; ks[2] = w.z; ks[3] = w.w;
            } else {
                const u32x2 w = *reinterpret_cast<const u32x2 *>(src);
                ks[0] = w.x; ks[1] = w.y;
            }
        };
        auto scaled_key_operand = [&](auto s_, const uint32_t (&kw)[WPL], const uint32_t (&ks)[G]) {
            constexpr int SLAB = decltype(s_)::value;
            u32x4 kop = key_operand<BITS, SLAB>(kw, uc);
            const uint32_t s2 = ks[SLAB / kSlabsPerGroup];
            kop.x = pk_mul_f16(kop.x, s2); kop.y = pk_mul_f16(kop.y, s2);
            kop.z = pk_mul_f16(kop.z, s2); kop.w = pk_mul_f16(kop.w, s2);
            return kop;
        };
        // Value operand of block BLK, token slab S, from the lane's value words and the tile's step pairs.
        auto scaled_value_operand = [&](auto b_, auto sl_, const uint32_t (&vw)[WPL], const uint32_t (&vs)[8]) {
            constexpr int BLK = decltype(b_)::value, S = decltype(sl_)::value;
            u32x4 r;
            if constexpr (BITS == 2) {
                const uint32_t word = vw[BLK];
                r.x = key_pair<2, 4 * S>(word, uc); r.y = key_pair<2, 4 * S + 1>(word, uc);
                r.z = key_pair<2, 4 * S + 2>(word, uc); r.w = key_pair<2, 4 * S + 3>(word, uc);
            } else {
                const uint32_t word = vw[2 * BLK + S];
                r.x = key_pair<4, 0>(word, uc); r.y = key_pair<4, 1>(word, uc);
                r.z = key_pair<4, 2>(word, uc); r.w = key_pair<4, 3>(word, uc);
            }
            r.x = pk_mul_f16(r.x, vs[4 * S]); r.y = pk_mul_f16(r.y, vs[4 * S + 1]);
            r.z = pk_mul_f16(r.z, vs[4 * S + 2]); r.w = pk_mul_f16(r.w, vs[4 * S + 3]);
            return r;
        };
        auto load_value_steps = [&](const uint32_t *buf, int tl, int blk, uint32_t (&vs)[8]) {
            const uint32_t *src = buf + St::kVs + ((tl * 4 + blk) * 2 + hh) * 8;
            const u32x4 w0 = *reinterpret_cast<const u32x4 *>(src), w1 = *reinterpret_cast<const u32x4 *>(src + 4);
            vs[0] = w0.x; vs[1] = w0.y; vs[2] = w0.z; vs[3] = w0.w; vs[4] = w1.x; vs[5] = w1.y; vs[6] = w1.z; vs[7] = w1.w;
        };
        auto zero16 = [&]() {
            f32x16 z;
#pragma unroll
            for (int v = 0; v < 16; ++v) z[v] = 0.0f;
            return z;
        };
        // tau of tile t from its probabilities: rows 4 hh .. 4 hh + 3 of the result belong to this lane half.
        // Row 8 of the operand is all ones, so that the same two MFMAs also leave the tile's row sum (of the
        // rounded probabilities, the ones the output is made of) in register 4 of the lanes of half 0; row 12,
        // which lands in register 4 of half 1, is zero.  (Rows 8 .. 31 otherwise repeat rows 0 .. 7 and are
        // not read.)
        const uint32_t tau_keep = (n == 8 || n == 12) ? 0u : 0xffffffffu;
        const uint32_t tau_ones = n == 8 ? 0x3c003c00u : 0u;   // f16 1.0 pairs
        auto load_tau_operand = [&](int t, u32x4 (&top)[2]) {
            const uint32_t *buf = lds + ((uint32_t)(t >> 2) % kGBuffers) * St::kWords;
            const uint32_t *src = buf + St::kTau + ((((t & 3) * 2) * 2 + hh) * 8 + (n & 7)) * 4;
            top[0] = *reinterpret_cast<const u32x4 *>(src);
            top[1] = *reinterpret_cast<const u32x4 *>(src + 2 * 8 * 4);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) top[i][j] = (top[i][j] & tau_keep) | tau_ones;
        };
        auto add_tau = [&](const u32x4 (&top)[2], const u32x4 (&pop)[kRB][2]) {
            const u32x4 t0 = top[0], t1 = top[1];
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) {
                f32x16 tt = mfma_f16(t0, pop[rb][0], zero16());
                tt = mfma_f16(t1, pop[rb][1], tt);
#pragma unroll
                for (int i = 0; i < 4; ++i) tau[rb][i] += tt[i];
                l_s[rb] += tt[4];   // half 0: the row sum of the tile; half 1: zero
            }
        };
        // Scores of tile t in log2 units (everything but the reference): constant terms, then high and low
        // query parts against the scaled key operands.
        auto score_tile = [&](int t, f32x16 (&sn)[kRB]) {
            Prefetched pf;
            prefetch_keys(t, pf);
            uint32_t ks[G];
            load_key_steps(t, ks);
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) {
                sn[rb] = mfma_bf16(pf.cop[0], rowop[0][rb], zero16());
#pragma unroll
                for (int c = 1; c < NC; ++c) sn[rb] = mfma_bf16(pf.cop[c], rowop[c][rb], sn[rb]);
            }
            uint32_t off = lo_off;
            asm volatile("" : "+v"(off));
            const uint32_t *qlo = q_stage + off;
            static_for<8>([&](auto s_) {
                constexpr int SLAB = decltype(s_)::value;
                const u32x4 kop = scaled_key_operand(s_, pf.kw, ks);
                u32x4 lo[kRB];
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) {
                    if constexpr (SLAB < kLoRes) lo[rb] = lo_res[rb][SLAB];
                    else lo[rb] = *reinterpret_cast<const u32x4 *>(qlo + 32 * rb * kLoRowWords + 8 * (SLAB - kLoRes));
                }
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) sn[rb] = mfma_f16(kop, qop[rb][SLAB], sn[rb]);
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) sn[rb] = mfma_f16(kop, lo[rb], sn[rb]);
            });
        };
        auto finalize_tile = [&](const f32x16 (&sn)[kRB], float (&e)[kRB][16], float (&tmax)[kRB]) {
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) {
#pragma unroll
                for (int v = 0; v < 16; ++v) e[rb][v] = sn[rb][v];   // already relative to the reference
                float mx = fmaxf(e[rb][0], e[rb][1]);
#pragma unroll
                for (int v = 2; v < 16; v += 2) mx = fmaxf(mx, fmaxf(e[rb][v], e[rb][v + 1]));
                tmax[rb] = max_halves(mx);
            }
        };
        // p = 2^e as f16 B operands (the row sums come out of the tau MFMAs).
        auto exp_tile = [&](const float (&e)[kRB][16], u32x4 (&pop)[kRB][2]) {
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) {
                uint32_t pw[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float p0 = __builtin_amdgcn_exp2f(e[rb][2 * i]);
                    const float p1 = __builtin_amdgcn_exp2f(e[rb][2 * i + 1]);
                    pw[i] = pack_f16(p0, p1);
                }
                pop[rb][0].x = pw[0]; pop[rb][0].y = pw[1]; pop[rb][0].z = pw[2]; pop[rb][0].w = pw[3];
                pop[rb][1].x = pw[4]; pop[rb][1].y = pw[5]; pop[rb][1].z = pw[6]; pop[rb][1].w = pw[7];
            }
        };
        auto load_value_words = [&](int t, uint32_t (&vw)[WPL]) {
            const uint32_t *buf = lds + ((uint32_t)(t >> 2) % kGBuffers) * St::kWords;
            const uint32_t *src = buf + St::kV + (t & 3) * 64 * WPL + lane * WPL;
#pragma unroll
            for (int i = 0; i < WPL / 4; ++i) {
                const u32x4 w = *reinterpret_cast<const u32x4 *>(src + 4 * i);
                vw[4 * i] = w.x; vw[4 * i + 1] = w.y; vw[4 * i + 2] = w.z; vw[4 * i + 3] = w.w;
            }
        };
        // O^T += V^T P^T with the steps folded into the value operand; tau from the same probabilities.
        auto pv_tile = [&](int t, const u32x4 (&pop)[kRB][2]) {
            const uint32_t *buf = lds + ((uint32_t)(t >> 2) % kGBuffers) * St::kWords;
            uint32_t vw[WPL];
            load_value_words(t, vw);
            static_for<4>([&](auto b_) {
                constexpr int B = decltype(b_)::value;
                uint32_t vs[8];
                load_value_steps(buf, t & 3, B, vs);
                const u32x4 v0 = scaled_value_operand(b_, IntC<0>{}, vw, vs);
                const u32x4 v1 = scaled_value_operand(b_, IntC<1>{}, vw, vs);
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) o[B][rb] = mfma_f16(v0, pop[rb][0], o[B][rb]);
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) o[B][rb] = mfma_f16(v1, pop[rb][1], o[B][rb]);
            });
            u32x4 top[2];
            load_tau_operand(t, top);
            add_tau(top, pop);
        };
        // One steady-state iteration: score MFMAs of tile t+1 next to the exponentials of tile t, then the
        // P*V MFMAs of tile t next to the reference subtraction of tile t+1, then tau of tile t.
        auto fused_iteration = [&](int t, Prefetched &pf, f32x16 (&sn)[kRB], float (&e)[kRB][16], float (&tmax)[kRB],
                                   u32x4 (&pop)[kRB][2]) {
            const uint32_t *bufc = lds + ((uint32_t)(t >> 2) % kGBuffers) * St::kWords;
            uint32_t ks[G];
            load_key_steps(t + 1, ks);
            uint32_t off = lo_off;
            asm volatile("" : "+v"(off));
            const uint32_t *qlo = q_stage + off;
            u32x4 lo_cur[kRB], lo_nxt[kRB], kop_prev;
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) {
                sn[rb] = mfma_bf16(pf.cop[0], rowop[0][rb], zero16());
#pragma unroll
                for (int c = 1; c < NC; ++c) sn[rb] = mfma_bf16(pf.cop[c], rowop[c][rb], sn[rb]);
            }
            uint32_t pw[kRB][8];
            uint32_t vw[WPL];
            uint32_t vs_cur[8], vs_nxt[8];
            u32x4 top[2];
            auto exp_chunk = [&](auto c_) {
                constexpr int C = decltype(c_)::value;
                constexpr int RB = (C * kRB) / 8, I0 = (C * kRB) % 8;
#pragma unroll
                for (int i = I0; i < I0 + kRB; ++i) {
                    const float p0 = __builtin_amdgcn_exp2f(e[RB][2 * i]);
                    const float p1 = __builtin_amdgcn_exp2f(e[RB][2 * i + 1]);
                    pw[RB][i] = pack_f16(p0, p1);
                }
            };
            KVQ_CHUNK_FENCE();
            static_for<8>([&](auto s_) {
                constexpr int SLAB = decltype(s_)::value;
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) {
                    if constexpr (SLAB < kLoRes) lo_nxt[rb] = lo_res[rb][SLAB];
                    else lo_nxt[rb] = *reinterpret_cast<const u32x4 *>(qlo + 32 * rb * kLoRowWords + 8 * (SLAB - kLoRes));
                }
                if constexpr (SLAB == 5) load_value_words(t, vw);
                if constexpr (SLAB == 7) load_value_steps(bufc, t & 3, 0, vs_cur);
                const u32x4 kop = scaled_key_operand(s_, pf.kw, ks);
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) sn[rb] = mfma_f16(kop, qop[rb][SLAB], sn[rb]);
                if constexpr (SLAB >= 1) {
#pragma unroll
                    for (int rb = 0; rb < kRB; ++rb) sn[rb] = mfma_f16(kop_prev, lo_cur[rb], sn[rb]);
                    exp_chunk(IntC<SLAB - 1>{});
                }
                kop_prev = kop;
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) lo_cur[rb] = lo_nxt[rb];
                KVQ_CHUNK_FENCE();
            });
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) sn[rb] = mfma_f16(kop_prev, lo_cur[rb], sn[rb]);
            exp_chunk(IntC<7>{});
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) {
                pop[rb][0].x = pw[rb][0]; pop[rb][0].y = pw[rb][1]; pop[rb][0].z = pw[rb][2]; pop[rb][0].w = pw[rb][3];
                pop[rb][1].x = pw[rb][4]; pop[rb][1].y = pw[rb][5]; pop[rb][1].z = pw[rb][6]; pop[rb][1].w = pw[rb][7];
            }
            prefetch_keys(t + 2, pf);
            KVQ_CHUNK_FENCE();
            float mx[kRB];
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) mx[rb] = -INFINITY;
            static_for<4>([&](auto b_) {
                constexpr int B = decltype(b_)::value;
                if constexpr (B < 3) load_value_steps(bufc, t & 3, B + 1, vs_nxt);   // next block's steps
                if constexpr (B == 0) load_tau_operand(t, top);
                const u32x4 v0 = scaled_value_operand(b_, IntC<0>{}, vw, vs_cur);
                const u32x4 v1 = scaled_value_operand(b_, IntC<1>{}, vw, vs_cur);
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) o[B][rb] = mfma_f16(v0, pop[rb][0], o[B][rb]);
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) o[B][rb] = mfma_f16(v1, pop[rb][1], o[B][rb]);
#pragma unroll
                for (int i = 0; i < 8; ++i) vs_cur[i] = vs_nxt[i];
                constexpr int RB = (B * 4 * kRB) / 16, V0 = (B * 4 * kRB) % 16;
#pragma unroll
                for (int v = V0; v < V0 + 4 * kRB; ++v) {
                    e[RB][v] = sn[RB][v];                  // already relative to the reference
                    asm volatile("" : "+v"(e[RB][v]));     // copied out of the accumulation register here, not later
                }
#pragma unroll
                for (int v = V0; v < V0 + 4 * kRB; v += 2) mx[RB] = __builtin_fmaxf(__builtin_fmaxf(mx[RB], e[RB][v]), e[RB][v + 1]);
                KVQ_CHUNK_FENCE();
            });
            add_tau(top, pop);
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) tmax[rb] = max_halves(mx[rb]);
        };
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
        finalize_tile(sn, e, tmax);
        if (n_tiles > 4) open_stage(1);
        Prefetched pf;
        prefetch_keys(1, pf);
        int t = 0;
        int t_open = 6;      // stage s (tiles 4 s ..) is opened while tile 4 s - 2 is being scored: s = 2 at t = 6
        bool done = false;
        while (!done) {
            move_reference(e, tmax);
            for (;;) {
                if (__builtin_expect(t + 1 >= n_tiles, 0)) {
                    exp_tile(e, pop);
                    pv_tile(t, pop);
                    done = true;
                    break;
                }
                if (__builtin_expect(t == t_open, 0)) {
                    open_stage((t + 2) >> 2);
                    t_open += 4;
                }
                fused_iteration(t, pf, sn, e, tmax, pop);
                ++t;
                if (__builtin_expect(__any(over_threshold(tmax)), 0)) break;
            }
        }

        // ---- leave the rotated basis: O <- Hn^T (O_rot - tau_j 1_j).  tau_j = high + low row of group j, held
        // by the lanes of half j >> 1; block b of the accumulators belongs to group b / kBlocksPerGroup.
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) {
            float tj[2] = {tau[rb][0] + tau[rb][1], tau[rb][2] + tau[rb][3]};   // groups 2 hh, 2 hh + 1
            float tg[4];   // by group index 0..3 (G = 2: groups 0, 1 live in half 0)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float own = tj[j & 1], other = xhalf(own);
                tg[j] = (hh == (j >> 1)) ? own : other;
            }
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[b][rb][v] -= tg[b / kBlocksPerGroup];
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
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float own = o[b][rb][v], other = xhalf(own);
                    o[b][rb][v] = (hh ? other - own : own + other) * 0.088388347648318f;
                }
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

template <int BITS, bool CORR, int G> hipError_t launch_group(const AttentionArgs &a, hipStream_t stream)
{
    static std::atomic<uint64_t> configured{0};  // per instantiation and device
    const void *fn = reinterpret_cast<const void *>(&attention_mfma_group_kernel<BITS, CORR, G>);
    const hipError_t ce = configure_dynamic_lds(fn, group_lds_bytes<BITS, G>(), configured);
    if (ce != hipSuccess) return ce;
    const int row_blocks = (int)((a.m + kRowsPerBlock - 1) / kRowsPerBlock);
    const int64_t blocks = (int64_t)row_blocks * a.cv.num_heads * a.q_per_kv;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    const size_t lds_size = group_lds_bytes<BITS, G>();
    return launch_kernel(attention_mfma_group_kernel<BITS, CORR, G>, dim3((unsigned)blocks), dim3(kThreads), lds_size, stream, a,
                         row_blocks);
}

}  // namespace

bool attention_mfma_group_supported(const CacheView &cv)
{
    return cv.head_dim == D && cv.io_dtype == KVQ_BF16 && cv.meta_format == KVQ_META_FP8_BF16 &&
           (cv.bits == 2 || cv.bits == 4) && (cv.group_size == 32 || cv.group_size == 64);
}

hipError_t launch_attention_mfma_group(const AttentionArgs &a, hipStream_t stream)
{
    if (!attention_mfma_group_supported(a.cv)) return hipErrorInvalidValue;
    if (a.cache_len > (int64_t)0x3fffffff * kTileTokens) return hipErrorInvalidValue;
    if (a.cv.bits == 4 && a.cv.group_size == 32) return a.correction ? launch_group<4, true, 4>(a, stream) : launch_group<4, false, 4>(a, stream);
    if (a.cv.bits == 4) return a.correction ? launch_group<4, true, 2>(a, stream) : launch_group<4, false, 2>(a, stream);
    if (a.cv.group_size == 32) return a.correction ? launch_group<2, true, 4>(a, stream) : launch_group<2, false, 4>(a, stream);
    return a.correction ? launch_group<2, true, 2>(a, stream) : launch_group<2, false, 2>(a, stream);
}

}  // namespace kvq
