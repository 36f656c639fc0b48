// Device helpers shared by the matrix-core attention kernels (per-token and group-wise): vector types,
// MFMA wrappers, 16-bit packing, the in-register unpacking of code words into MFMA operands, and
// small wave-level utilities.  Included inside namespace kvq { namespace { ... } } of each kernel file.
#pragma once

typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(6))) int i32x6;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

#ifndef KVQ_CHUNK_FENCE
#define KVQ_CHUNK_FENCE() __builtin_amdgcn_sched_barrier(0)
#endif

constexpr int D = 128;
#ifndef KVQ_ROW_BLOCKS_PER_WAVE
#define KVQ_ROW_BLOCKS_PER_WAVE 2
#endif
constexpr int kRB = KVQ_ROW_BLOCKS_PER_WAVE;          // 32-row blocks owned by one wavefront
constexpr int kRowsPerWave = 32 * kRB;
constexpr int kRowsPerBlock = 256;
constexpr int kWaves = kRowsPerBlock / kRowsPerWave;  // 8 (two per SIMD) or 4
constexpr int kThreads = 64 * kWaves;
constexpr int kStageTiles = 4;
constexpr int kStageKeys = kStageTiles * kTileTokens;  // 128
constexpr int kQRowWords = 68;    // 64 words of f16 pairs + 4 words padding (bank spread)
constexpr int kVtRowWords = 18;   // 32 tokens of bf16 = 16 words + 2 words padding
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kRescaleThreshold = 8.0f;   // log2 units a tile may exceed the reference by
constexpr float kMaskBias = -1.0e30f;

__device__ inline f32x16 mfma_bf16(u32x4 a, u32x4 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
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
__device__ inline uint16_t bf16_bits(float f) { return (uint16_t)(pack_bf16(f, 0.0f) & 0xffffu); }
__device__ inline float bf16_val(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// OCP E4M3 in the low byte of w -> float, by the hardware conversion (exact, subnormals included; the stored
// scales are finite).
__device__ inline float e4m3_low_byte(uint32_t w) { return __builtin_amdgcn_cvt_f32_fp8((int)w, 0); }

__device__ inline float dot2_bf16(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}

// Unpacking.  A packed word holds 16 (2-bit) or 8 (4-bit) codes, in pairs `bits` apart in the low and
// the high half-word; register J of the word is the pair at bit 2J (4J) of each half.  An operand
// register is made as (shifted word & mask) | base: the code lands in mantissa bits of a 16-bit float
// whose exponent is the base, i.e. the value is BASE + weight * code.
//
// 2-bit codes: three adjacent pairs are cut out of the same shifted word, at mantissa positions two bits
// apart, so their weights are 1, 1/4 and 1/16 (class g = 0, 1, 2 of register J is 2 - J mod 3).  The
// other operand of the MFMA carries the inverse weight, which is exact: for keys the query channel is
// multiplied by 4^g, for values the probability (through the value scale) is.  This saves the shift of
// five registers in eight.  Key values are 4 + code * 4^-g (f16), value values 8 + code * 4^-g (bf16).
// 4-bit codes: value values are 16 + code (bf16), one pair per shift.  Key values are 16 + code * 16^-g (f16): with
// KVQ_INT4_KEY_SHARE two adjacent pairs are cut out of one shifted word, four mantissa bits apart (class g = 1 for even
// J, 0 for odd J), and the query channel carries 16^g; without it every pair has its own shift and g = 0 (the
// group-wise kernel multiplies the key operand by an E4M3 step, and only 16 + code keeps that product exact in f16).
//
// The constants are passed through an empty asm once per kernel so that the compiler keeps them in
// registers (masks in scalars, bases in vector registers) and selects v_and_or_b32; the instruction
// itself is emitted by the compiler, which matters because it must know about the vector write in
// front of the matrix instruction that reads the register.
#ifndef KVQ_INT4_KEY_SHARE
#define KVQ_INT4_KEY_SHARE 0
#endif
struct UnpackConsts {
    uint32_t kmask[3], kbase, vmask[3], vbase;
};
template <int BITS> __device__ inline UnpackConsts make_unpack_consts()
{
    UnpackConsts c;
    if constexpr (BITS == 2) {
        c.kmask[0] = 0x03000300u; c.kmask[1] = 0x00c000c0u; c.kmask[2] = 0x00300030u;
        c.kbase = 0x44004400u;   // f16 4.0
        c.vmask[0] = 0x00300030u; c.vmask[1] = 0x000c000cu; c.vmask[2] = 0x00030003u;
        c.vbase = 0x41004100u;   // bf16 8.0
    } else {
        c.kmask[0] = c.kmask[2] = 0x03c003c0u;
        c.kmask[1] = KVQ_INT4_KEY_SHARE ? 0x003c003cu : 0x03c003c0u;
        c.kbase = 0x4c004c00u;   // f16 16.0
        c.vmask[0] = c.vmask[1] = c.vmask[2] = 0x00780078u;
        c.vbase = 0x41804180u;   // bf16 16.0
    }
#pragma unroll
    for (int g = 0; g < 3; ++g) asm volatile("" : "+s"(c.kmask[g]), "+s"(c.vmask[g]));
    asm volatile("" : "+v"(c.kbase), "+v"(c.vbase));
    return c;
}
// Offsets of the operand values and weight class of register J (see above).
template <int BITS> struct Unpack {
    static constexpr float kKeyBase = BITS == 2 ? 4.0f : 16.0f;
    static constexpr float kValueBase = BITS == 2 ? 8.0f : 16.0f;
    static constexpr float kStoredOffset = BITS == 2 ? 4.0f : 16.0f;   // the cache stores zero + this
    // register J of a key word; the weight of class g is 2^-(kClassBits g)
    __host__ __device__ static constexpr int weight_class(int j) { return BITS == 2 ? 2 - j % 3 : KVQ_INT4_KEY_SHARE ? 1 - (j & 1) : 0; }
    static constexpr int kClassBits = BITS == 2 ? 2 : 4;
};

template <int SH> __device__ inline uint32_t shift(uint32_t w)
{
    if constexpr (SH >= 0) return w << SH;
    else return w >> (-SH);
}

// Register J of a packed word -> two f16 key values.
template <int BITS, int J> __device__ inline uint32_t key_pair(uint32_t w, const UnpackConsts &c)
{
    if constexpr (BITS == 2) {
        constexpr int G = Unpack<2>::weight_class(J);          // pair lands at mantissa bits 9:8, 7:6 or 5:4
        constexpr int SH = J < 3 ? 4 : J < 6 ? -2 : -8;        // shared by the registers of one group
        static_assert(2 * J + SH == 8 - 2 * G, "key pair position");
        return (shift<SH>(w) & c.kmask[G]) | c.kbase;
    } else if constexpr (KVQ_INT4_KEY_SHARE) {
        constexpr int G = Unpack<4>::weight_class(J);          // pair lands at mantissa bits 9:6 or 5:2
        constexpr int SH = J < 2 ? 2 : -6;                      // shared by two registers
        static_assert(4 * J + SH == 6 - 4 * G, "key pair position");
        return (shift<SH>(w) & c.kmask[G]) | c.kbase;
    } else {
        return (shift<6 - 4 * J>(w) & c.kmask[0]) | c.kbase;
    }
}
// Register J of a packed word -> two bf16 value values.
template <int BITS, int J> __device__ inline uint32_t value_pair(uint32_t w, const UnpackConsts &c)
{
    if constexpr (BITS == 2) {
        constexpr int G = Unpack<2>::weight_class(J);          // pair lands at mantissa bits 5:4, 3:2 or 1:0
        constexpr int SH = J < 3 ? 0 : J < 6 ? -6 : -12;
        static_assert(2 * J + SH == 4 - 2 * G, "value pair position");
        return (shift<SH>(w) & c.vmask[G]) | c.vbase;
    } else {
        return (shift<3 - 4 * J>(w) & c.vmask[0]) | c.vbase;
    }
}

// A operand of 16-wide slab SLAB of a key tile, from the lane's WPL code words.
template <int BITS, int SLAB> __device__ inline u32x4 key_operand(const uint32_t *w, const UnpackConsts &c)
{
    u32x4 r;
    if constexpr (BITS == 2) {
        const uint32_t word = w[SLAB >> 1];
        constexpr int J0 = 4 * (SLAB & 1);
        r.x = key_pair<2, J0>(word, c); r.y = key_pair<2, J0 + 1>(word, c);
        r.z = key_pair<2, J0 + 2>(word, c); r.w = key_pair<2, J0 + 3>(word, c);
    } else {
        const uint32_t word = w[SLAB];
        r.x = key_pair<4, 0>(word, c); r.y = key_pair<4, 1>(word, c);
        r.z = key_pair<4, 2>(word, c); r.w = key_pair<4, 3>(word, c);
    }
    return r;
}
// A operand of a value tile: channel block BLK (32 channels), token slab S (16 tokens).
template <int BITS, int BLK, int S> __device__ inline u32x4 value_operand(const uint32_t *w, const UnpackConsts &c)
{
    u32x4 r;
    if constexpr (BITS == 2) {
        const uint32_t word = w[BLK];
        constexpr int J0 = 4 * S;
        r.x = value_pair<2, J0>(word, c); r.y = value_pair<2, J0 + 1>(word, c);
        r.z = value_pair<2, J0 + 2>(word, c); r.w = value_pair<2, J0 + 3>(word, c);
    } else {
        const uint32_t word = w[2 * BLK + S];
        r.x = value_pair<4, 0>(word, c); r.y = value_pair<4, 1>(word, c);
        r.z = value_pair<4, 2>(word, c); r.w = value_pair<4, 3>(word, c);
    }
    return r;
}
// Weight class of query channel c (keys) and of the key held in score register v (values).
template <int BITS> __host__ __device__ constexpr int key_channel_class(int c)
{
    return Unpack<BITS>::weight_class(BITS == 2 ? 4 * ((c >> 4) & 1) + ((c >> 1) & 3) : (c >> 1) & 3);
}
template <int BITS> __host__ __device__ constexpr int value_register_class(int v)
{
    return BITS == 2 ? Unpack<BITS>::weight_class(v >> 1) : 0;
}

__device__ inline float xhalf(float v) { return __shfl_xor(v, 32); }
// max(v, value held by the same lane of the other half-wave)
__device__ inline float max_halves(float v)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    // the instruction itself: fmaxf would first quiet both inputs (two more instructions per call)
    float m;
    asm("v_max_f32 %0, %1, %2" : "=v"(m) : "v"(__uint_as_float(r[0])), "v"(__uint_as_float(r[1])));
    return m;
}

template <int I> struct IntC { static constexpr int value = I; };
template <int N, typename F> __device__ inline void static_for(F &&f)
{
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(IntC<N - 1>{});
    }
}
