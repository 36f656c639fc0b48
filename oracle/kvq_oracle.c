/*
 * kvq_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, double-precision CPU statement of what the quantized-KV chunk
 * attention path computes, written from the paper.  Only tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it.  It shares no code, header,
 * table or constant generator with the HIP library.
 *
 * Every function is the definition written out: dense +-1 sums for the
 * Hadamard rotation, the literal round-to-nearest quantizer, a full score row
 * per query followed by one softmax over [cached | current] keys.  No blocking,
 * no online softmax, no fast transform.  OpenMP is used only to run independent
 * rows on several cores.
 *
 * Pins (tests/test_oracle_*.py): closed forms for the exponential moment of
 * uniform noise, Monte-Carlo on the scalar case, orthogonality of the rotation,
 * the |error| <= step/2 bound, hand-worked rows, textbook softmax attention via
 * an independent numpy formula, permutation invariance, and special cases
 * (step 0, no cache, per-channel steps).  The paper prints no worked numeric
 * example, so nothing here is pinned to printed numbers.
 *
 * Build: gcc -O2 -std=c99 -fopenmp -ffp-contract=off -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Entry (r, c) of the Sylvester Hadamard matrix of any power-of-two order:
 * +1 when r and c share an even number of set bits, else -1. */
static double hadamard_sign(unsigned r, unsigned c)
{
    unsigned x = r & c, parity = 0;
    while (x) { parity ^= (x & 1u); x >>= 1; }
    return parity ? -1.0 : 1.0;
}

static int is_pow2(int d) { return d > 0 && (d & (d - 1)) == 0; }

/* 1/sqrt(d) rounded once to double; written out for the two supported sizes so
 * the value does not depend on a library sqrt. */
static double inv_sqrt_d(int d)
{
    if (d == 64) return 0.125;
    if (d == 128) return 0.08838834764831845; /* sqrt(2)/16 */
    return 1.0 / sqrt((double)d);
}

int kvqo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* u = H_d x, the unnormalised rotation (Preliminaries, "Hadamard rotation").
 * Each output is one left-to-right sum of +-x_c. */
int kvqo_hadamard(int d, const double *x, double *u)
{
    if (!is_pow2(d)) return 1;
    for (int r = 0; r < d; ++r) {
        double s = 0.0;
        for (int c = 0; c < d; ++c) s += hadamard_sign((unsigned)r, (unsigned)c) * x[c];
        u[r] = s;
    }
    return 0;
}

/*
 * Asymmetric round-to-nearest quantization of `rows` vectors (Eq. 1 and the
 * sentence after it: scale and zero-point cover the [min, max] range), per
 * group of `group` consecutive channels, after an optional Hadamard rotation.
 *
 *   u      = H_d x                      (rotate != 0; otherwise u = x)
 *   lo, hi = min, max of u over the group; a constant group has its range
 *            widened to include 0 (all-zero group: step 0, codes 0)
 *   inv    = L / (hi - lo),  L = 2^bits - 1
 *   z      = -rint(lo * inv)            (integer, any sign)
 *   code   = clamp(rint(u * inv) + z, 0, L)
 *   scale  = float((hi - lo) / L * n)   n = 1/sqrt(d) with rotation, 1 without
 *   zero   = float(z)
 * so that (code - zero) * scale reconstructs the normalised rotated vector.
 * rint rounds ties to even.  Decisions are taken on the unnormalised u; the
 * positive factor n only enters the stored scale.
 *
 * x: [rows][d] doubles.  codes: [rows][d] bytes.  scale, zero: [rows][d/group].
 */
int kvqo_quantize_rows(int64_t rows, int d, int bits, int group, int rotate,
                       const double *x, uint8_t *codes, float *scale, float *zero)
{
    if (rows < 0 || d <= 0 || group <= 0 || d % group != 0) return 1;
    if (bits < 1 || bits > 8) return 1;
    if (rotate && !is_pow2(d)) return 1;
    const double L = (double)((1 << bits) - 1);
    const double norm = rotate ? inv_sqrt_d(d) : 1.0;
    const int G = d / group;
    int failed = 0;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < rows; ++t) {
        double *u = (double *)malloc(sizeof(double) * (size_t)d);
        if (!u) { failed = 1; continue; }
        const double *xr = x + t * d;
        if (rotate) kvqo_hadamard(d, xr, u);
        else memcpy(u, xr, sizeof(double) * (size_t)d);
        for (int j = 0; j < G; ++j) {
            const double *ug = u + j * group;
            uint8_t *cg = codes + t * d + j * group;
            double lo = ug[0], hi = ug[0];
            for (int c = 1; c < group; ++c) {
                if (ug[c] < lo) lo = ug[c];
                if (ug[c] > hi) hi = ug[c];
            }
            if (hi == lo) {
                if (lo > 0.0) lo = 0.0;
                if (hi < 0.0) hi = 0.0;
            }
            if (hi == lo) {
                for (int c = 0; c < group; ++c) cg[c] = 0;
                scale[t * G + j] = 0.0f;
                zero[t * G + j] = 0.0f;
                continue;
            }
            const double range = hi - lo;
            const double inv = L / range;
            const double step = range / L;
            const double z = -rint(lo * inv);
            for (int c = 0; c < group; ++c) {
                double k = rint(ug[c] * inv) + z;
                if (k < 0.0) k = 0.0;
                if (k > L) k = L;
                cg[c] = (uint8_t)k;
            }
            scale[t * G + j] = (float)(step * norm);
            zero[t * G + j] = (float)z;
        }
        free(u);
    }
    return failed;
}

/*
 * Per-channel quantization (appendix "Per-Channel Quantization Correction": the
 * step depends on the channel and is shared by all tokens of the block).  The
 * same quantizer as kvqo_quantize_rows with the roles of tokens and channels
 * exchanged: for every channel c of the (optionally rotated) vectors,
 *
 *   lo, hi = min, max over the `rows` tokens of the block; a constant channel
 *            has its range widened to include 0 (all-zero: step 0, codes 0)
 *   inv    = L / (hi - lo),   z = -rint(lo * inv)
 *   code   = clamp(rint(u[t][c] * inv) + z, 0, L)      for every token t
 *   scale[c] = float((hi - lo) / L * n),  zero[c] = float(z)
 *
 * x: [rows][d] doubles.  codes: [rows][d] bytes.  scale, zero: [d].
 */
int kvqo_quantize_cols(int64_t rows, int d, int bits, int rotate,
                       const double *x, uint8_t *codes, float *scale, float *zero)
{
    if (rows <= 0 || d <= 0) return 1;
    if (bits < 1 || bits > 8) return 1;
    if (rotate && !is_pow2(d)) return 1;
    const double L = (double)((1 << bits) - 1);
    const double norm = rotate ? inv_sqrt_d(d) : 1.0;
    double *u = (double *)malloc(sizeof(double) * (size_t)rows * (size_t)d);
    if (!u) return 1;
    for (int64_t t = 0; t < rows; ++t) {
        if (rotate) kvqo_hadamard(d, x + t * d, u + t * d);
        else memcpy(u + t * d, x + t * d, sizeof(double) * (size_t)d);
    }
    for (int c = 0; c < d; ++c) {
        double lo = u[c], hi = u[c];
        for (int64_t t = 1; t < rows; ++t) {
            if (u[t * d + c] < lo) lo = u[t * d + c];
            if (u[t * d + c] > hi) hi = u[t * d + c];
        }
        if (hi == lo) {
            if (lo > 0.0) lo = 0.0;
            if (hi < 0.0) hi = 0.0;
        }
        if (hi == lo) {
            for (int64_t t = 0; t < rows; ++t) codes[t * d + c] = 0;
            scale[c] = 0.0f;
            zero[c] = 0.0f;
            continue;
        }
        const double range = hi - lo;
        const double inv = L / range;
        const double step = range / L;
        const double z = -rint(lo * inv);
        for (int64_t t = 0; t < rows; ++t) {
            double k = rint(u[t * d + c] * inv) + z;
            if (k < 0.0) k = 0.0;
            if (k > L) k = L;
            codes[t * d + c] = (uint8_t)k;
        }
        scale[c] = (float)(step * norm);
        zero[c] = (float)z;
    }
    free(u);
    return 0;
}

/*
 * FP8 E4M3 (the 8-bit format with 4 exponent bits, bias 7, 3 mantissa bits, no
 * infinities, largest finite value 448, subnormals m * 2^-9): the smallest
 * representable value that is >= x, for x > 0.  Values above 448 saturate at
 * 448 (the range is then not covered; callers see the clamp in the codes).
 * Returns the value; *byte receives its encoding.
 */
double kvqo_e4m3_ceil(double x, uint8_t *byte)
{
    if (!(x > 0.0)) { if (byte) *byte = 0; return 0.0; }
    if (x > 448.0) x = 448.0;
    int e;                      /* x = f * 2^e, f in [0.5, 1)  =>  x in [2^(e-1), 2^e) */
    (void)frexp(x, &e);
    int E = e - 1;              /* floor(log2 x) */
    if (E < -6) E = -6;         /* subnormals share the spacing of the lowest binade */
    const double ulp = ldexp(1.0, E - 3);
    const double v = ceil(x / ulp) * ulp;   /* x / ulp is exact (power of two) */
    if (byte) {
        int ev;
        (void)frexp(v, &ev);
        int Ev = ev - 1;
        unsigned bits;
        if (Ev < -6) {
            bits = (unsigned)(v / ldexp(1.0, -9));                 /* subnormal: exponent field 0 */
        } else {
            const unsigned m = (unsigned)(v / ldexp(1.0, Ev - 3)) - 8u;
            bits = ((unsigned)(Ev + 7) << 3) | m;
        }
        *byte = (uint8_t)bits;
    }
    return v;
}

/* Nearest BF16 value (8 significant bits, ties to even) of a double that is an
 * integer or any value well inside the float range. */
double kvqo_bf16_round(double x)
{
    if (x == 0.0 || x != x) return x;
    int e;
    (void)frexp(x, &e);                 /* |x| in [2^(e-1), 2^e) */
    const double ulp = ldexp(1.0, e - 8);
    return rint(x / ulp) * ulp;         /* rint: ties to even */
}

/*
 * Group-wise asymmetric round-to-nearest quantization with the metadata format
 * of "Effective bitwidth" / the storage note of the cost appendix: per group one
 * FP8 E4M3 scale and one BF16 zero-point (24 bits per group).  The paper fixes
 * the formats, not the rounding; the reading taken here keeps Eq. 1's promise
 * that scale and zero-point cover [min, max]:
 *
 *   u      = H_d x  (rotate)            lo, hi over the group as in kvqo_quantize_rows
 *   step   = (hi - lo) / L * n          n = 1/sqrt(d) with rotation, 1 without
 *   s8     = smallest E4M3 value >= step            (the stored scale)
 *   inv    = n / s8
 *   z      = -rint(lo * inv),  zb = BF16(z)         (the stored zero-point)
 *   code   = clamp(rint(u * inv) + zb, 0, L)
 * Every operation is one IEEE double operation in this order.
 * scale, zero: [rows][d/group] floats holding exactly the stored values;
 * scale_bytes (nullable): the E4M3 encodings.
 */
int kvqo_quantize_rows_fp8meta(int64_t rows, int d, int bits, int group, int rotate,
                               const double *x, uint8_t *codes, float *scale, float *zero,
                               uint8_t *scale_bytes)
{
    if (rows < 0 || d <= 0 || group <= 0 || d % group != 0) return 1;
    if (bits < 1 || bits > 8) return 1;
    if (rotate && !is_pow2(d)) return 1;
    const double L = (double)((1 << bits) - 1);
    const double norm = rotate ? inv_sqrt_d(d) : 1.0;
    const int G = d / group;
    int failed = 0;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < rows; ++t) {
        double *u = (double *)malloc(sizeof(double) * (size_t)d);
        if (!u) { failed = 1; continue; }
        const double *xr = x + t * d;
        if (rotate) kvqo_hadamard(d, xr, u);
        else memcpy(u, xr, sizeof(double) * (size_t)d);
        for (int j = 0; j < G; ++j) {
            const double *ug = u + j * group;
            uint8_t *cg = codes + t * d + j * group;
            double lo = ug[0], hi = ug[0];
            for (int c = 1; c < group; ++c) {
                if (ug[c] < lo) lo = ug[c];
                if (ug[c] > hi) hi = ug[c];
            }
            if (hi == lo) {
                if (lo > 0.0) lo = 0.0;
                if (hi < 0.0) hi = 0.0;
            }
            if (hi == lo) {
                for (int c = 0; c < group; ++c) cg[c] = 0;
                scale[t * G + j] = 0.0f;
                zero[t * G + j] = 0.0f;
                if (scale_bytes) scale_bytes[t * G + j] = 0;
                continue;
            }
            const double range = hi - lo;
            const double step = range / L * norm;
            uint8_t sb;
            const double s8 = kvqo_e4m3_ceil(step, &sb);
            const double inv = norm / s8;
            const double z = -rint(lo * inv);
            const double zb = kvqo_bf16_round(z);
            for (int c = 0; c < group; ++c) {
                double k = rint(ug[c] * inv) + zb;
                if (k < 0.0) k = 0.0;
                if (k > L) k = L;
                cg[c] = (uint8_t)k;
            }
            scale[t * G + j] = (float)s8;
            zero[t * G + j] = (float)zb;
            if (scale_bytes) scale_bytes[t * G + j] = sb;
        }
        free(u);
    }
    return failed;
}

/* Reconstruction x^ = (x_q - z) * step (sentence after Eq. 1), in the basis the
 * codes were taken in.  out: [rows][d] doubles. */
int kvqo_dequantize_rows(int64_t rows, int d, int group, const uint8_t *codes,
                         const float *scale, const float *zero, double *out)
{
    if (rows < 0 || d <= 0 || group <= 0 || d % group != 0) return 1;
    const int G = d / group;
    for (int64_t t = 0; t < rows; ++t)
        for (int c = 0; c < d; ++c) {
            const int64_t g = t * G + c / group;
            out[t * d + c] = ((double)codes[t * d + c] - (double)zero[g]) * (double)scale[g];
        }
    return 0;
}

/* log(sinh(a)/a), the per-channel log moment of uniform noise (Eq. 12), in a
 * form that neither overflows for large |a| nor cancels for small |a|. */
double kvqo_log_sinhc(double a)
{
    a = fabs(a);
    if (a < 1e-3) {
        const double a2 = a * a;
        return a2 / 6.0 - a2 * a2 / 180.0 + a2 * a2 * a2 / 2835.0;
    }
    /* sinh(a)/a = e^a (1 - e^{-2a}) / (2a) */
    return a + log1p(-exp(-2.0 * a)) - log(2.0 * a);
}

/*
 * Correction b for one (query, key) pair.
 *   qv    : the query in the basis the key was quantized in (rotated query
 *           under rotation; Appendix "Extension to QuaRot"), d values
 *   step  : the key's step size per group, G = d/group values
 *   sigma : softmax scale (1/sqrt(d) in the paper)
 *   mode 1: second-order Taylor form  sigma^2/24 * sum_j step_j^2 * ||qv_j||^2
 *           (Eq. 13 / Eq. 15; sigma^2 = 1/d gives the paper's 1/(24 d))
 *   mode 2: exact form  sum_c log(sinh(a_c)/a_c),  a_c = sigma*qv_c*step/2 (Eq. 12)
 *   mode 0: 0
 */
double kvqo_correction(int d, int group, const double *qv, const double *step,
                       double sigma, int mode)
{
    if (mode == 0) return 0.0;
    const int G = d / group;
    double b = 0.0;
    if (mode == 1) {
        for (int j = 0; j < G; ++j) {
            double nu = 0.0;
            for (int c = j * group; c < (j + 1) * group; ++c) nu += qv[c] * qv[c];
            b += step[j] * step[j] * nu;
        }
        return b * sigma * sigma / 24.0;
    }
    for (int c = 0; c < d; ++c) b += kvqo_log_sinhc(0.5 * sigma * qv[c] * step[c / group]);
    return b;
}

/*
 * Chunk attention for one head (Alg. 1 with Eq. 2-4), every step in order:
 *
 *   qv        = Hn q          (rotate != 0; Hn = H_d / sqrt(d))   else qv = q
 *   s^_i      = sigma * qv . k^_i          i in S  (cached, dequantized keys)
 *   s_j       = sigma * q  . k_j           j in R  (current keys)
 *   b_i       = correction(qv, step_i)     subtracted from cached scores only
 *   p         = softmax(concat(s^ - b, s)) with the row maximum subtracted
 *   P_S       = sum_{i in S} p_i
 *   o         = Hn^T (sum_{i in S} p_i v^_i) + sum_{j in R} p_j v_j
 *
 * k^, v^ [ns][d]: dequantized cached keys / values in the basis they were
 * quantized in (rotated and normalised when rotate != 0).  kstep [ns][d/group]:
 * the stored step of each cached key group.  Current keys / values kr, vr
 * [nr][d] and queries q [m][d] are in the original basis, as is out [m][d].
 * mass_cached [m] (nullable) receives P_S.  ns == 0 or nr == 0 are allowed,
 * not both.
 * causal != 0 (the partial-prefill setting of the cross-domain experiment: the
 * current block is the last nr positions of a causal sequence and the queries
 * are its last m positions): current key j is visible to query r only if
 * j <= r + nr - m; cached keys are always visible.
 * signs (nullable, [d], entries +1 / -1; used only with rotate != 0): the
 * randomised Hadamard rotation of the rotation paragraph of the method section,
 * x -> Hn (signs * x).  The cache was quantized in that basis, so the query is
 * mapped the same way and the cached part of the output is mapped back with
 * the transpose, o_S = signs * (Hn^T acc).
 */
int kvqo_attention_masked(int d, int group, int64_t m, int64_t ns, int64_t nr,
                          const double *q, const double *khat, const double *kstep,
                          const double *vhat, const double *kr, const double *vr,
                          double sigma, int correction, int rotate, int causal, const double *signs,
                          double *out, double *mass_cached);

int kvqo_attention(int d, int group, int64_t m, int64_t ns, int64_t nr,
                   const double *q, const double *khat, const double *kstep,
                   const double *vhat, const double *kr, const double *vr,
                   double sigma, int correction, int rotate,
                   double *out, double *mass_cached)
{
    return kvqo_attention_masked(d, group, m, ns, nr, q, khat, kstep, vhat, kr, vr, sigma, correction, rotate, 0, NULL,
                                 out, mass_cached);
}

int kvqo_attention_masked(int d, int group, int64_t m, int64_t ns, int64_t nr,
                          const double *q, const double *khat, const double *kstep,
                          const double *vhat, const double *kr, const double *vr,
                          double sigma, int correction, int rotate, int causal, const double *signs,
                          double *out, double *mass_cached)
{
    if (d <= 0 || group <= 0 || d % group != 0 || m < 0 || ns < 0 || nr < 0) return 1;
    if (ns + nr == 0) return 1;
    if (rotate && !is_pow2(d)) return 1;
    if (correction < 0 || correction > 2) return 1;
    if (causal && ns == 0 && nr < m) return 1;   /* some query would see no key at all */
    const int G = d / group;
    const double norm = inv_sqrt_d(d);
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < m; ++r) {
        double *qv = (double *)malloc(sizeof(double) * (size_t)d * 3);
        double *s = (double *)malloc(sizeof(double) * (size_t)(ns + nr));
        if (!qv || !s) { failed = 1; free(qv); free(s); continue; }
        double *acc = qv + d, *tmp = acc + d;
        const double *qr = q + r * d;
        if (rotate) {
            /* randomised rotation: channel signs first, then the Hadamard matrix */
            if (signs) { for (int c = 0; c < d; ++c) tmp[c] = signs[c] * qr[c]; }
            kvqo_hadamard(d, signs ? tmp : qr, qv);
            for (int c = 0; c < d; ++c) qv[c] *= norm;
        } else {
            memcpy(qv, qr, sizeof(double) * (size_t)d);
        }
        for (int64_t i = 0; i < ns; ++i) {
            double dot = 0.0;
            for (int c = 0; c < d; ++c) dot += qv[c] * khat[i * d + c];
            s[i] = sigma * dot - kvqo_correction(d, group, qv, kstep + i * G, sigma, correction);
        }
        /* number of current keys this query sees */
        int64_t nvis = nr;
        if (causal) {
            nvis = r + nr - m + 1;
            if (nvis < 0) nvis = 0;
            if (nvis > nr) nvis = nr;
        }
        for (int64_t j = 0; j < nr; ++j) {
            double dot = 0.0;
            for (int c = 0; c < d; ++c) dot += qr[c] * kr[j * d + c];
            s[ns + j] = sigma * dot;
        }
        double top = ns > 0 ? s[0] : s[ns];
        for (int64_t i = 0; i < ns + nvis; ++i) if (s[i] > top) top = s[i];
        double zs = 0.0, zr = 0.0;
        for (int64_t i = 0; i < ns; ++i) { s[i] = exp(s[i] - top); zs += s[i]; }
        for (int64_t j = ns; j < ns + nr; ++j) {
            s[j] = j < ns + nvis ? exp(s[j] - top) : 0.0;   /* masked keys get weight 0 */
            zr += s[j];
        }
        const double z = zs + zr;
        for (int c = 0; c < d; ++c) acc[c] = 0.0;
        for (int64_t i = 0; i < ns; ++i) {
            const double p = s[i] / z;
            for (int c = 0; c < d; ++c) acc[c] += p * vhat[i * d + c];
        }
        if (rotate) {
            /* Hn is symmetric, so Hn^T acc is the same dense product. */
            kvqo_hadamard(d, acc, tmp);
            for (int c = 0; c < d; ++c) acc[c] = tmp[c] * norm * (signs ? signs[c] : 1.0);
        }
        for (int64_t j = 0; j < nr; ++j) {
            const double p = s[ns + j] / z;
            for (int c = 0; c < d; ++c) acc[c] += p * vr[j * d + c];
        }
        for (int c = 0; c < d; ++c) out[r * d + c] = acc[c];
        if (mass_cached) mass_cached[r] = zs / z;
        free(qv);
        free(s);
    }
    return failed;
}

/*
 * Attention-level diagnostics of the bias and of its repair (attention stealing,
 * Eq. "attn_stealing"; appendices "Attention JSD Distributions" and "Attention
 * Output MSE"): the quantized (optionally corrected) attention of one head
 * against attention over the unquantized cache, on the same queries and keys.
 *
 *   p   = softmax([sigma q.kref_i | sigma q.kr_j])          unquantized cache
 *   p^  = softmax([sigma q~.k^_i - b_i | sigma q.kr_j])      quantized cache
 *   diag[r][0] = P_S   = sum_{i in S} p_i
 *   diag[r][1] = P^_S  = sum_{i in S} p^_i      (the stealing is diag[1] - diag[0])
 *   diag[r][2] = JSD(p, p^) = KL(p || mix)/2 + KL(p^ || mix)/2, mix = (p + p^)/2,
 *                natural logarithm, over all ns + nr keys; terms with a zero
 *                probability contribute 0
 *   diag[r][3] = (1/d) sum_c (o^_c - o_c)^2,  o = sum_i p_i vref_i + sum_j p_j vr_j,
 *                o^ as kvqo_attention_masked computes it
 *
 * kref, vref [ns][d]: the cached keys / values before quantization, in the
 * original basis.  The other arguments are those of kvqo_attention_masked.
 */
int kvqo_diagnostics(int d, int group, int64_t m, int64_t ns, int64_t nr,
                     const double *q, const double *khat, const double *kstep, const double *vhat,
                     const double *kref, const double *vref, const double *kr, const double *vr,
                     double sigma, int correction, int rotate, const double *signs, double *diag)
{
    if (d <= 0 || group <= 0 || d % group != 0 || m < 0 || ns < 0 || nr < 0 || ns + nr == 0) return 1;
    if (rotate && !is_pow2(d)) return 1;
    if (correction < 0 || correction > 2) return 1;
    const int G = d / group;
    const int64_t n = ns + nr;
    const double norm = inv_sqrt_d(d);
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < m; ++r) {
        double *buf = (double *)malloc(sizeof(double) * ((size_t)d * 5 + (size_t)n * 2));
        if (!buf) { failed = 1; continue; }
        double *qv = buf, *tmp = qv + d, *acc = tmp + d, *oq = acc + d, *oref = oq + d;
        double *p = oref + d, *ph = p + n;
        const double *qr = q + r * d;
        if (rotate) {
            if (signs) { for (int c = 0; c < d; ++c) tmp[c] = signs[c] * qr[c]; }
            kvqo_hadamard(d, signs ? tmp : qr, qv);
            for (int c = 0; c < d; ++c) qv[c] *= norm;
        } else {
            memcpy(qv, qr, sizeof(double) * (size_t)d);
        }
        /* the two score rows */
        for (int64_t i = 0; i < ns; ++i) {
            double dref = 0.0, dq = 0.0;
            for (int c = 0; c < d; ++c) { dref += qr[c] * kref[i * d + c]; dq += qv[c] * khat[i * d + c]; }
            p[i] = sigma * dref;
            ph[i] = sigma * dq - kvqo_correction(d, group, qv, kstep + i * G, sigma, correction);
        }
        for (int64_t j = 0; j < nr; ++j) {
            double dot = 0.0;
            for (int c = 0; c < d; ++c) dot += qr[c] * kr[j * d + c];
            p[ns + j] = ph[ns + j] = sigma * dot;
        }
        /* two softmaxes */
        double top = p[0], toph = ph[0], z = 0.0, zh = 0.0;
        for (int64_t i = 1; i < n; ++i) { if (p[i] > top) top = p[i]; if (ph[i] > toph) toph = ph[i]; }
        for (int64_t i = 0; i < n; ++i) { p[i] = exp(p[i] - top); z += p[i]; ph[i] = exp(ph[i] - toph); zh += ph[i]; }
        for (int64_t i = 0; i < n; ++i) { p[i] /= z; ph[i] /= zh; }
        double ps = 0.0, psh = 0.0, jsd = 0.0;
        for (int64_t i = 0; i < ns; ++i) { ps += p[i]; psh += ph[i]; }
        for (int64_t i = 0; i < n; ++i) {
            const double mix = 0.5 * (p[i] + ph[i]);
            if (p[i] > 0.0) jsd += 0.5 * p[i] * log(p[i] / mix);
            if (ph[i] > 0.0) jsd += 0.5 * ph[i] * log(ph[i] / mix);
        }
        /* the two outputs */
        for (int c = 0; c < d; ++c) { acc[c] = 0.0; oref[c] = 0.0; }
        for (int64_t i = 0; i < ns; ++i)
            for (int c = 0; c < d; ++c) { acc[c] += ph[i] * vhat[i * d + c]; oref[c] += p[i] * vref[i * d + c]; }
        if (rotate) {
            kvqo_hadamard(d, acc, tmp);
            for (int c = 0; c < d; ++c) oq[c] = tmp[c] * norm * (signs ? signs[c] : 1.0);
        } else {
            memcpy(oq, acc, sizeof(double) * (size_t)d);
        }
        for (int64_t j = 0; j < nr; ++j)
            for (int c = 0; c < d; ++c) { oq[c] += ph[ns + j] * vr[j * d + c]; oref[c] += p[ns + j] * vr[j * d + c]; }
        double mse = 0.0;
        for (int c = 0; c < d; ++c) mse += (oq[c] - oref[c]) * (oq[c] - oref[c]);
        diag[r * 4 + 0] = ps;
        diag[r * 4 + 1] = psh;
        diag[r * 4 + 2] = jsd;
        diag[r * 4 + 3] = mse / d;
        free(buf);
    }
    return failed;
}
