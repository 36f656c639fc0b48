// Issue-rate microbenchmarks for gfx950, the yardsticks the attention and quantize kernels are read
// against: sustained MFMA rate, what vector instructions cost next to MFMAs in one in-order wave (and
// with two waves per SIMD), LDS read rate by access width, the rate of the block-scaled 32x32x64 MFMA by
// operand format (with a check of the FP4 / FP6 operand layout against a host product), and a plain HBM
// copy of the size one quantize-append call moves.  Stand-alone program; every loop has a fixed trip count.
//
//   kvq_microbench            prints one table per experiment
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cmath>
#include <vector>

typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;

#define CHECK(x)                                                                        \
    do {                                                                                \
        hipError_t e_ = (x);                                                            \
        if (e_ != hipSuccess) {                                                         \
            fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, hipGetErrorString(e_));  \
            exit(1);                                                                    \
        }                                                                               \
    } while (0)

constexpr int kBlocks = 256;   // one workgroup per compute unit
constexpr int kIters = 5000;    // x kSteps steps per kernel: several milliseconds, so that clocks have settled
constexpr int kSteps = 32;      // steps per loop iteration

enum Op { kFma, kMul, kAndOr, kShift, kCvtPk, kDot2, kExp2, kMax3 };

// W waves per SIMD; each wave runs kIters x kSteps steps of (one 32x32x16 MFMA on one of CH accumulators,
// then NV independent vector instructions of kind OP).
// CH = -1: the MFMA takes the constant 0 as its C operand (nothing accumulated, no accumulator read).
// The loop body starts on a 64-byte boundary plus 4 * HEAD bytes: where the instructions fall relative to
// the 64-byte instruction lines changes the time of a dense stream of 8-byte instructions by up to
// 30 % (line_crossing_kernel below measures what one crossing costs), so the alignment is fixed rather than left to
// chance (the padding is at most 15 one-cycle no-ops
// per kSteps steps).
template <int W, int CH, int NV, Op OP, int HEAD = 0>
__global__ __launch_bounds__(256 * W, 1) void mix_kernel(float *out, uint32_t mask, uint32_t base)
{
    f16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = (_Float16)(threadIdx.x * 0.001f + i);
        b[i] = (_Float16)(i * 0.5f);
    }
    f32x16 c[8];
    for (int j = 0; j < 8; ++j)
        for (int v = 0; v < 16; ++v) c[j][v] = 0.0f;
    float x[16], y[16];
    uint32_t u[16];
    for (int i = 0; i < 16; ++i) {
        x[i] = threadIdx.x * 0.01f + i;
        y[i] = 0.5f + 0.001f * i + threadIdx.x * 1.0e-6f;
        u[i] = threadIdx.x * 7 + i;
    }
    const uint32_t bs = base + threadIdx.x;
    for (int it = 0; it < kIters; ++it) {
        asm volatile(".p2align 6");
#pragma unroll
        for (int p = 0; p < HEAD; ++p) asm volatile("s_nop 0");
#pragma unroll
        for (int j = 0; j < kSteps; ++j) {
            if (CH > 0) c[j % (CH > 0 ? CH : 1)] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c[j % (CH > 0 ? CH : 1)], 0, 0, 0);
            if (CH < 0) {
                f32x16 zero;
                for (int v = 0; v < 16; ++v) zero[v] = 0.0f;
                c[j & 7] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, zero, 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const int k = (j * NV + v) & 15, k1 = (k + 1) & 15;
                if (OP == kFma) x[k] = __builtin_fmaf(x[k], y[k], y[k1]);
                else if (OP == kMul) x[k] = x[k] * y[k];
                else if (OP == kAndOr) { asm("" : "+v"(u[k]));  u[k] = (u[k] & mask) | bs; }   // opaque source: cannot be folded
                else if (OP == kShift) { asm("" : "+v"(u[k]));  u[k] = u[k] >> 1; }
                else if (OP == kCvtPk) {
                    f32x2 f = {x[k], y[k]};
                    u[k] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
                    x[k] = __uint_as_float(u[k]);
                } else if (OP == kDot2)
                    x[k] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, u[k]), __builtin_bit_cast(bf16x2, u[k1]), x[k], false);
                else if (OP == kExp2) x[k] = __builtin_amdgcn_exp2f(x[k]);
                else if (OP == kMax3) y[k] = __builtin_fmaxf(__builtin_fmaxf(y[k], x[k]), x[k1]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    float s = 0.0f;
    for (int j = 0; j < 8; ++j)
        for (int v = 0; v < 16; ++v) s += c[j][v];
    for (int i = 0; i < 16; ++i) s += x[i] + y[i] + (float)u[i];
    out[blockIdx.x * 256 * W + threadIdx.x] = s;
}

template <typename F> float time_ms(F &&launch)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    launch();   // warm-up
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    launch();
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms = 0.0f;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    CHECK(hipGetLastError());
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
    return ms;
}

// ns per step (one MFMA + NV instructions) and per SIMD: with W waves a SIMD completes W steps in that time.
template <int W, int CH, int NV, Op OP, int HEAD = 0> double step_ns(float *out)
{
    const float ms = time_ms([&] { mix_kernel<W, CH, NV, OP, HEAD><<<kBlocks, 256 * W>>>(out, 0x03000300u, 0x44004400u); });
    return ms * 1e6 / ((double)kIters * kSteps) / W;
}

template <Op OP> void op_row(float *out, const char *name)
{
    const double a = step_ns<1, 4, 8, OP>(out), b = step_ns<1, 4, 16, OP>(out);
    const double c = step_ns<2, 4, 8, OP>(out), d = step_ns<2, 4, 16, OP>(out);
    printf("| %-12s | %6.2f | %6.2f | %5.2f | %6.2f | %6.2f | %5.2f |\n", name, a, b, (b - a) / 8, c, d, (d - c) / 8);
}

template <typename T> __global__ __launch_bounds__(512, 1) void lds_kernel(uint32_t *out, int iters)
{
    extern __shared__ u32x4 lds[];
    for (int i = threadIdx.x; i < 8192; i += 512) lds[i] = u32x4{(uint32_t)i, 1u, 2u, 3u};
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const T *base = reinterpret_cast<const T *>(lds + (wave & 3) * 1024) + lane;
    for (int it = 0; it < iters; ++it) {
        T r[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) r[j] = base[64 * j];
#pragma unroll
        for (int j = 0; j < 16; ++j) asm volatile("" ::"v"(r[j]));
        asm volatile("" : "+v"(base));
    }
    out[blockIdx.x * 512 + threadIdx.x] = 0u;
}

template <typename T> void lds_row(uint32_t *out, const char *name)
{
    const int iters = 4000;
    CHECK(hipFuncSetAttribute((const void *)lds_kernel<T>, hipFuncAttributeMaxDynamicSharedMemorySize, 8192 * 16));
    const float ms = time_ms([&] { lds_kernel<T><<<kBlocks, 512, 8192 * 16>>>(out, iters); });
    const double instr = (double)iters * 16 * 8;   // wave-instructions per compute unit
    printf("| %-13s | %6.2f | %7.1f |\n", name, ms * 1e6 / instr, instr * 64 * sizeof(T) / (ms * 1e6));
}

// v_mfma_scale_f32_32x32x64_f8f6f4 by operand format (FA, FB: 0 = FP8 E4M3, 2 = FP6 E2M3, 4 = FP4 E2M1), one
// wave per SIMD, four accumulator chains, all scales 1.
template <int FA, int FB> __global__ __launch_bounds__(256, 1) void scaled_mfma_kernel(float *out, int iters)
{
    i32x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = 0x22222222;
        b[i] = 0x08208208 + (int)threadIdx.x;
    }
    f32x16 c[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) c[k] = {};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 4; ++k) c[k] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c[k], FA, FB, 0, 0x7f, 0, 0x7f);
    }
    float s = 0.0f;
#pragma unroll
    for (int k = 0; k < 4; ++k) s += c[k][0] + c[k][9];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}
template <int FA, int FB> double scaled_mfma_ns(float *out)
{
    const int iters = kIters * 4;
    const float ms = time_ms([&] { scaled_mfma_kernel<FA, FB><<<kBlocks, 256>>>(out, iters); });
    return ms * 1e6 / (4.0 * iters);
}

// One FP4 (A) x FP6 (B) instruction on operands laid out as: lane l holds row (column) l mod 32 and the K
// indices 32 (l div 32) + j, j = 0..31, element j in bits 4j.. of A's first four registers and bits 6j.. of B's
// first six; B carries a power-of-two scale per column (E8M0 byte in the scale register's low byte).
__global__ __launch_bounds__(64, 1) void fp4_fp6_once(const i32x8 *a, const i32x8 *b, const int *scale_b, float *out)
{
    const int l = threadIdx.x;
    f32x16 c = {};
    c = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[l], b[l], c, 4, 2, 0, 0x7f, 0, scale_b[l]);
#pragma unroll
    for (int v = 0; v < 16; ++v) out[l * 16 + v] = c[v];
}
int check_fp4_fp6_layout(float *out)
{
    auto fp4 = [](int n) {
        const float t[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};
        return (n & 8) ? -t[n & 7] : t[n & 7];
    };
    auto fp6 = [](int n) {   // E2M3, bias 1
        const int e = (n >> 3) & 3, m = n & 7;
        const float mag = e == 0 ? m / 8.0f : (float)(1 << (e - 1)) * (1.0f + m / 8.0f);
        return (n & 32) ? -mag : mag;
    };
    std::vector<int> A(32 * 64), B(64 * 32), hs(64);
    uint32_t seed = 12345u;
    auto next = [&]() { seed = seed * 1664525u + 1013904223u; return (int)(seed >> 16); };
    for (auto &x : A) x = next() % 16;
    for (auto &x : B) x = next() % 64;
    std::vector<i32x8> ha(64), hb(64);
    for (int l = 0; l < 64; ++l) {
        uint32_t ra[8] = {}, rb[8] = {};
        for (int j = 0; j < 32; ++j) {
            const int k = 32 * (l / 32) + j, bit = 6 * j;
            ra[j / 8] |= (uint32_t)A[(l % 32) * 64 + k] << (4 * (j % 8));
            const uint64_t v = (uint64_t)B[k * 32 + (l % 32)] << (bit % 32);
            rb[bit / 32] |= (uint32_t)v;
            if (bit / 32 + 1 < 8) rb[bit / 32 + 1] |= (uint32_t)(v >> 32);
        }
        for (int i = 0; i < 8; ++i) {
            ha[l][i] = (int)ra[i];
            hb[l][i] = (int)rb[i];
        }
        hs[l] = 0x7f - (l % 32) % 5;
    }
    i32x8 *da, *db;
    int *ds;
    CHECK(hipMalloc(&da, 64 * sizeof(i32x8)));
    CHECK(hipMalloc(&db, 64 * sizeof(i32x8)));
    CHECK(hipMalloc(&ds, 64 * sizeof(int)));
    CHECK(hipMemcpy(da, ha.data(), 64 * sizeof(i32x8), hipMemcpyHostToDevice));
    CHECK(hipMemcpy(db, hb.data(), 64 * sizeof(i32x8), hipMemcpyHostToDevice));
    CHECK(hipMemcpy(ds, hs.data(), 64 * sizeof(int), hipMemcpyHostToDevice));
    fp4_fp6_once<<<1, 64>>>(da, db, ds, out);
    CHECK(hipDeviceSynchronize());
    std::vector<float> ho(64 * 16);
    CHECK(hipMemcpy(ho.data(), out, ho.size() * sizeof(float), hipMemcpyDeviceToHost));
    int bad = 0;
    for (int l = 0; l < 64; ++l)
        for (int v = 0; v < 16; ++v) {
            const int n = l % 32, i = 8 * (v / 4) + 4 * (l / 32) + v % 4;   // accumulator register v of lane l
            double want = 0.0;
            for (int k = 0; k < 64; ++k) want += (double)fp4(A[i * 64 + k]) * fp6(B[k * 32 + n]);
            want = std::ldexp(want, -(n % 5));
            if (std::fabs(want - ho[l * 16 + v]) > 1e-5 * (1.0 + std::fabs(want))) ++bad;
        }
    CHECK(hipFree(da)); CHECK(hipFree(db)); CHECK(hipFree(ds));
    return bad;
}

// What an instruction that crosses a 64-byte line costs.  The whole loop, branch included, is one asm statement that
// starts on a 64-byte boundary, so the placement of every instruction is known: v_fma_f32 (VOP3) is 8 bytes, s_nop 4.
//   VAR 0: 200 FMAs, aligned                       VAR 1: the same behind one s_nop (every eighth FMA crosses a line)
//   VAR 2: 24 lines of [7 FMAs, 2 s_nop], aligned   VAR 3: the same behind one s_nop: every FMA is misaligned by 4
//          bytes (some cross a 32-byte boundary), none crosses a 64-byte line
#define KVQ_F1(i) "v_fma_f32 %" #i ", %" #i ", %9, 1.0\n"
#define KVQ_F8 KVQ_F1(0) KVQ_F1(1) KVQ_F1(2) KVQ_F1(3) KVQ_F1(4) KVQ_F1(5) KVQ_F1(6) KVQ_F1(7)
#define KVQ_F25 KVQ_F8 KVQ_F8 KVQ_F8 KVQ_F1(0)
#define KVQ_F200 KVQ_F25 KVQ_F25 KVQ_F25 KVQ_F25 KVQ_F25 KVQ_F25 KVQ_F25 KVQ_F25
#define KVQ_L64 KVQ_F1(0) KVQ_F1(1) KVQ_F1(2) KVQ_F1(3) KVQ_F1(4) KVQ_F1(5) KVQ_F1(6) "s_nop 0\n s_nop 0\n"
#define KVQ_L64X8 KVQ_L64 KVQ_L64 KVQ_L64 KVQ_L64 KVQ_L64 KVQ_L64 KVQ_L64 KVQ_L64
#define KVQ_LOOP(BODY)                                                                                          \
    asm volatile(".p2align 6\n 1:\n" BODY "s_sub_u32 %8, %8, 1\n s_cmp_lg_u32 %8, 0\n s_cbranch_scc1 1b\n"       \
                 : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]), "+s"(n) \
                 : "s"(s)                                                                                       \
                 : "scc")
template <int VAR> __global__ __launch_bounds__(256, 1) void line_crossing_kernel(float *out, int iters, float s)
{
    float x[8];
    for (int i = 0; i < 8; ++i) x[i] = s * (float)(threadIdx.x + i);
    int n = iters;   // > 0: the loop counts down to 0
    if constexpr (VAR == 0) KVQ_LOOP(KVQ_F200);
    if constexpr (VAR == 1) KVQ_LOOP("s_nop 0\n" KVQ_F200);
    if constexpr (VAR == 2) KVQ_LOOP(KVQ_L64X8 KVQ_L64X8 KVQ_L64X8);
    if constexpr (VAR == 3) KVQ_LOOP("s_nop 0\n" KVQ_L64X8 KVQ_L64X8 KVQ_L64X8);
    float r = (float)n;
    for (int i = 0; i < 8; ++i) r += x[i];
    out[blockIdx.x * 256 + threadIdx.x] = r;
}
template <int VAR> double line_crossing_ns(float *out)
{
    const int iters = 40000;
    line_crossing_kernel<VAR><<<kBlocks, 256>>>(out, 2000, 0.001f);
    CHECK(hipDeviceSynchronize());
    const float ms = time_ms([&] { line_crossing_kernel<VAR><<<kBlocks, 256>>>(out, iters, 0.001f); });
    return ms * 1e6 / iters;   // ns per loop iteration
}

__global__ void copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, size_t n)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

int main()
{
    float *out;
    CHECK(hipMalloc(&out, (size_t)kBlocks * 512 * sizeof(float)));

    for (int r = 0; r < 8; ++r) step_ns<1, 4, 8, kFma>(out);   // bring the clocks up before the first figure

    printf("## MFMA only: ns per v_mfma_f32_32x32x16_f16 per SIMD (32768 flop each, 1024 SIMDs)\n\n");
    printf("| waves/SIMD | accumulator chains | ns per MFMA | chip TFLOP/s |\n|---|---|---|---|\n");
    {
        const double r[5] = {step_ns<1, 1, 0, kFma>(out), step_ns<1, 2, 0, kFma>(out), step_ns<1, 4, 0, kFma>(out),
                             step_ns<1, 8, 0, kFma>(out), step_ns<2, 4, 0, kFma>(out)};
        const int w[5] = {1, 1, 1, 1, 2}, ch[5] = {1, 2, 4, 8, 4};
        for (int i = 0; i < 5; ++i) printf("| %d | %d | %.2f | %.0f |\n", w[i], ch[i], r[i], 32768.0 / r[i] * 1024 / 1e3);
    }

    printf("\n## One MFMA followed by N independent v_fma_f32: ns per step per SIMD\n\n");
    printf("| N | 1 wave/SIMD | 2 waves/SIMD |\n|---|---|---|\n");
    printf("| 0 | %.2f | %.2f |\n", step_ns<1, 4, 0, kFma>(out), step_ns<2, 4, 0, kFma>(out));
    printf("| 4 | %.2f | %.2f |\n", step_ns<1, 4, 4, kFma>(out), step_ns<2, 4, 4, kFma>(out));
    printf("| 8 | %.2f | %.2f |\n", step_ns<1, 4, 8, kFma>(out), step_ns<2, 4, 8, kFma>(out));
    printf("| 12 | %.2f | %.2f |\n", step_ns<1, 4, 12, kFma>(out), step_ns<2, 4, 12, kFma>(out));
    printf("| 16 | %.2f | %.2f |\n", step_ns<1, 4, 16, kFma>(out), step_ns<2, 4, 16, kFma>(out));
    printf("| 16, no MFMA | %.2f | %.2f |\n", step_ns<1, 0, 16, kFma>(out), step_ns<2, 0, 16, kFma>(out));
    printf("| 12, MFMA with C = 0 | %.2f | %.2f |\n", step_ns<1, -1, 12, kFma>(out), step_ns<2, -1, 12, kFma>(out));
    printf("| 16, MFMA with C = 0 | %.2f | %.2f |\n", step_ns<1, -1, 16, kFma>(out), step_ns<2, -1, 16, kFma>(out));

    printf("\n## The same step (1 MFMA + 8 v_fma_f32, 1 wave/SIMD) with the loop body 0, 4, 8, 28 bytes past a 64-byte boundary\n\n");
    printf("| offset | ns per step |\n|---|---|\n");
    printf("| 0 | %.2f |\n| 4 | %.2f |\n| 8 | %.2f |\n| 12 | %.2f |\n| 28 | %.2f |\n", step_ns<1, 4, 8, kFma, 0>(out),
           step_ns<1, 4, 8, kFma, 1>(out), step_ns<1, 4, 8, kFma, 2>(out), step_ns<1, 4, 8, kFma, 3>(out),
           step_ns<1, 4, 8, kFma, 7>(out));

    printf("\n## Marginal cost of one vector instruction next to MFMAs (step = 1 MFMA + N instr; ns per SIMD)\n\n");
    printf("| instruction | 1w N=8 | 1w N=16 | 1w ns/instr | 2w N=8 | 2w N=16 | 2w ns/instr |\n|---|---|---|---|---|---|---|\n");
    op_row<kFma>(out, "v_fma_f32");
    op_row<kMul>(out, "v_mul_f32");
    op_row<kAndOr>(out, "v_and_or_b32");
    op_row<kShift>(out, "v_lshrrev_b32");
    op_row<kCvtPk>(out, "v_cvt_pk_bf16");
    op_row<kDot2>(out, "v_dot2_bf16");
    op_row<kExp2>(out, "v_exp_f32");
    op_row<kMax3>(out, "v_max3_f32");

    printf("\n## Instructions that cross a 64-byte line (one wave per SIMD, the loop written out in asm)\n\n");
    {
        const double a = line_crossing_ns<0>(out), b = line_crossing_ns<1>(out), c = line_crossing_ns<2>(out), d = line_crossing_ns<3>(out);
        printf("| loop body | ns per iteration | |\n|---|---|---|\n");
        printf("| 200 v_fma_f32 (8 bytes each), aligned | %.1f | %.3f ns per instruction |\n", a, a / 200);
        printf("| the same behind one 4-byte s_nop: 25 FMAs cross a line | %.1f | %.2f ns per crossing |\n", b, (b - a) / 25);
        printf("| 24 x [7 v_fma_f32, 2 s_nop], aligned | %.1f | %.2f ns per s_nop |\n", c, (c - 168 * a / 200) / 48);
        printf("| the same behind one s_nop: misaligned by 4 bytes, no crossing | %.1f | |\n", d);
    }

    printf("\n## LDS reads, 8 waves per compute unit, conflict-free: per wave-instruction and compute unit\n\n");
    printf("| instruction | ns | bytes per ns |\n|---|---|---|\n");
    lds_row<uint32_t>(reinterpret_cast<uint32_t *>(out), "ds_read_b32");
    lds_row<u32x2>(reinterpret_cast<uint32_t *>(out), "ds_read_b64");
    lds_row<u32x4>(reinterpret_cast<uint32_t *>(out), "ds_read_b128");

    printf("\n## v_mfma_scale_f32_32x32x64_f8f6f4 by operand format: ns per instruction per SIMD (131072 flop each)\n\n");
    printf("| A | B | ns per MFMA | chip TFLOP/s |\n|---|---|---|---|\n");
    {
        const double r[5] = {scaled_mfma_ns<0, 0>(out), scaled_mfma_ns<4, 0>(out), scaled_mfma_ns<4, 2>(out),
                             scaled_mfma_ns<2, 2>(out), scaled_mfma_ns<4, 4>(out)};
        const char *fa[5] = {"FP8", "FP4", "FP4", "FP6", "FP4"}, *fb[5] = {"FP8", "FP8", "FP6", "FP6", "FP4"};
        for (int i = 0; i < 5; ++i) printf("| %s | %s | %.2f | %.0f |\n", fa[i], fb[i], r[i], 131072.0 / r[i] * 1024 / 1e3);
    }
    printf("\nFP4 x FP6 with a per-column power-of-two scale against a host product of the same operands "
           "(2-bit codes 0..3 are the FP4 values 0, 0.5, 1, 1.5): %d mismatches of 1024\n", check_fp4_fp6_layout(out));

    printf("\n## HBM copy of the bytes one quantize-append call moves at the large shape\n\n");
    {
        // 100.7 MB read + 15.7 MB written by the quantizer; a copy reads and writes n bytes each: n = 58.2 MB
        const size_t bytes = 58200000 / 16 * 16, n = bytes / 16;
        u32x4 *src, *dst;
        CHECK(hipMalloc(&src, bytes));
        CHECK(hipMalloc(&dst, bytes));
        CHECK(hipMemset(src, 1, bytes));
        float best = 1e30f;
        for (int r = 0; r < 5; ++r) {
            const float ms = time_ms([&] { copy_kernel<<<kBlocks * 16, 256>>>(src, dst, n); });
            best = ms < best ? ms : best;
        }
        printf("copy of 2 x %.1f MB: %.1f us, %.2f TB/s\n", bytes / 1e6, best * 1e3, 2.0 * bytes / (best * 1e-3) / 1e12);
        const size_t big = (size_t)1 << 30;
        u32x4 *s2, *d2;
        CHECK(hipMalloc(&s2, big));
        CHECK(hipMalloc(&d2, big));
        CHECK(hipMemset(s2, 1, big));
        best = 1e30f;
        for (int r = 0; r < 3; ++r) {
            const float ms = time_ms([&] { copy_kernel<<<kBlocks * 16, 256>>>(s2, d2, big / 16); });
            best = ms < best ? ms : best;
        }
        printf("copy of 2 x 1 GiB: %.1f us, %.2f TB/s\n", best * 1e3, 2.0 * big / (best * 1e-3) / 1e12);
        CHECK(hipFree(src)); CHECK(hipFree(dst)); CHECK(hipFree(s2)); CHECK(hipFree(d2));
    }
    CHECK(hipFree(out));
    return 0;
}
