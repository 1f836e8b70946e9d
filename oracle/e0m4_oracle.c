/*
 * CPU oracle for the E0M4 weight-only quantised matrix multiplication.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path and must never be linked into, imported by or called from
 * the product; only the tests, the smoke check and the benchmark's CPU
 * baseline leg use it.
 *
 * What is computed follows the paper's section "E0M4 FP4 quantization"
 * (quantization paragraph and dequantization formula).  fp16 means IEEE
 * binary16.  The binade is fixed at n = 1, i.e. [2, 4): the constant
 * sign+exponent pattern is 0x4000 and a 4-bit code is shifted left by
 * 10 - 4 = 6 to sit in the four highest fraction bits.
 *
 * Readings taken where the paper does not fix a detail (each one is listed in
 * the design document as well):
 *   - eps is one fp16 ulp of the binade (2^-9), so the top of the range is
 *     0x43FF = 3.998046875.
 *   - the stored "scale" is the dequantisation multiplier (w units per unit of
 *     the binade) and the stored "bias" is the image of 0 inside the binade;
 *     the forward map divides by the *stored* fp16 scale so that encoder and
 *     decoder agree.
 *   - the bias keeps only its four highest fraction bits (truncation), which
 *     makes an exact zero weight decode to exactly zero.
 *   - the group range always includes 0; the mapped value is clamped into
 *     the binade; a degenerate (tiny or zero) range takes the smallest normal
 *     fp16 as scale, an overflowing one the largest finite fp16.
 *   - the forward map is done in fp32, one IEEE operation per step, then
 *     rounded once to fp16 (the code is read from the fp16 bit pattern, as in
 *     the paper's Figure 2); since this arithmetic decides an integer code,
 *     the oracle uses the same precision as the kernel here.  Everything else
 *     is fp64.
 *   - rounding of the code: add the fifth fraction bit to the four kept bits
 *     and saturate at 15, exactly as the paper writes it.
 *
 * The file also holds the INT4 format the paper compares E0M4 with in its
 * section "Evaluation of FP4 quantization" (Tables 1 and 2).  The paper does not
 * define that quantiser; the reading taken is written above the functions, and
 * its pins tie it to that stated definition, to the E0M4 decoder (of which an
 * integer-zero-point INT4 group is a special case) and to Table 2's ratio.
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -fno-fast-math -shared -fPIC
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* binary16 <-> wider types, written out (no compiler half support).   */
/* ------------------------------------------------------------------ */

/* Exact widening of a binary16 bit pattern. */
double oracle_half_bits_to_double(uint16_t h)
{
    const int sign = (h >> 15) & 1;
    const int e = (h >> 10) & 0x1F;
    const int f = h & 0x3FF;
    double v;
    if (e == 0) {
        v = ldexp((double)f, -24);                  /* subnormal or zero */
    } else if (e == 31) {
        v = f ? NAN : INFINITY;
    } else {
        v = ldexp((double)(1024 + f), e - 25);      /* (1 + f/1024) * 2^(e-15) */
    }
    return sign ? -v : v;
}

/* Round-to-nearest-even narrowing of a double to a binary16 bit pattern.
 * One rounding, done with nearbyint() on an exactly scaled value. */
uint16_t oracle_double_to_half_bits(double d)
{
    uint16_t sign = (uint16_t)(signbit(d) ? 0x8000u : 0u);
    double a = fabs(d);
    if (isnan(d)) return (uint16_t)(sign | 0x7E00u);
    if (isinf(d)) return (uint16_t)(sign | 0x7C00u);
    if (a == 0.0) return sign;
    if (a < ldexp(1.0, -14)) {
        /* subnormal range: spacing 2^-24; a result of 1024 is the smallest
         * normal number and has exactly the right bit pattern 0x0400. */
        double q = nearbyint(ldexp(a, 24));
        return (uint16_t)(sign | (uint16_t)q);
    }
    int ex;
    (void)frexp(a, &ex);                            /* a = m * 2^ex, m in [0.5,1) */
    int e = ex - 1;                                 /* a in [2^e, 2^(e+1)) */
    double q = nearbyint(ldexp(a, 10 - e));         /* in [1024, 2048] */
    if (q >= 2048.0) { q = 1024.0; e += 1; }
    if (e > 15) return (uint16_t)(sign | 0x7C00u);  /* overflow to infinity */
    return (uint16_t)(sign | (uint16_t)((e + 15) << 10) | (uint16_t)((int)q - 1024));
}

static inline float h2f(uint16_t h) { return (float)oracle_half_bits_to_double(h); }   /* exact */
static inline uint16_t f2h(float f) { return oracle_double_to_half_bits((double)f); } /* one rounding */

/* ------------------------------------------------------------------ */
/* Dequantisation (paper: dequantization formula, two bitwise ops).    */
/* ------------------------------------------------------------------ */

#define E0M4_EXP_BITS  0x4000u   /* sign 0, exponent field 16: the binade [2,4) */
#define E0M4_SHIFT     6         /* 10 fraction bits - 4 code bits */

/* w1 bit pattern of a code: constant exponent OR (code << shift). */
uint16_t oracle_e0m4_w1_bits(int c)
{
    return (uint16_t)(E0M4_EXP_BITS | ((unsigned)(c & 15) << E0M4_SHIFT));
}

/* Inverse of the group's affine map: w = (w1 - bias) * scale, rounded once
 * to fp16.  The difference and the product are exact in fp64. */
uint16_t oracle_e0m4_decode_one(int c, uint16_t scale_bits, uint16_t bias_bits)
{
    double w1 = oracle_half_bits_to_double(oracle_e0m4_w1_bits(c));
    double b = oracle_half_bits_to_double(bias_bits);
    double s = oracle_half_bits_to_double(scale_bits);
    return oracle_double_to_half_bits((w1 - b) * s);
}

/* ------------------------------------------------------------------ */
/* Quantisation (paper: quantization paragraph).                       */
/* ------------------------------------------------------------------ */

static const float LO = 2.0f;                 /* 2^n, n = 1 */
static const float HI = 3.998046875f;         /* 2^(n+1) - eps, eps = 2^-9 (fp16 0x43FF) */

/* Scale and bias of one group of G weights. */
void oracle_e0m4_fit_group(const uint16_t* w0, int64_t G, uint16_t* scale_bits, uint16_t* bias_bits)
{
    float mn = 0.0f, mx = 0.0f;               /* the range always contains 0 */
    for (int64_t k = 0; k < G; ++k) {
        float v = h2f(w0[k]);
        if (v < mn) mn = v;
        if (v > mx) mx = v;
    }
    const float span = HI - LO;               /* 1.998046875, exact */
    float range = mx - mn;
    float s = range / span;
    if (s < 6.103515625e-05f) s = 6.103515625e-05f;   /* 2^-14, smallest normal fp16 */
    if (s > 65504.0f) s = 65504.0f;                   /* largest finite fp16 */
    uint16_t sb = f2h(s);
    float sf = h2f(sb);                       /* the stored scale, as the decoder sees it */
    float q = mn / sf;
    float b = LO - q;
    if (b < LO) b = LO;
    if (b > HI) b = HI;
    uint16_t bb = (uint16_t)(f2h(b) & 0xFFC0u);   /* keep the four highest fraction bits */
    *scale_bits = sb;
    *bias_bits = bb;
}

/* Code of one weight under given (stored) scale and bias. */
int oracle_e0m4_encode_one(uint16_t w0_bits, uint16_t scale_bits, uint16_t bias_bits)
{
    float w0 = h2f(w0_bits);
    float sf = h2f(scale_bits);
    float bf = h2f(bias_bits);
    float q = w0 / sf;
    float t = q + bf;
    if (t < LO) t = LO;
    if (t > HI) t = HI;
    uint16_t bits = f2h(t);                   /* now sign 0, exponent field 16 */
    int y1 = (bits >> 6) & 15;                /* four highest fraction bits */
    int y2 = (bits >> 5) & 1;                 /* the next bit, used for rounding */
    int c = y1 + y2;
    return c > 15 ? 15 : c;
}

/* fp16 bit pattern of the mapped value w1 before the code is cut out of it
 * (exposed so that the "same sign and exponent" invariant can be tested). */
uint16_t oracle_e0m4_forward_bits(uint16_t w0_bits, uint16_t scale_bits, uint16_t bias_bits)
{
    float t = h2f(w0_bits) / h2f(scale_bits) + h2f(bias_bits);
    if (t < LO) t = LO;
    if (t > HI) t = HI;
    return f2h(t);
}

/* W [N,K] fp16 bits, groups of G consecutive k.  codes: [N,K] one code per
 * byte; scales, bias: [N, K/G] fp16 bits. */
void oracle_e0m4_quantize(const uint16_t* W, int64_t N, int64_t K, int64_t G,
                          uint8_t* codes, uint16_t* scales, uint16_t* bias)
{
    const int64_t ng = K / G;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t g = 0; g < ng; ++g) {
            const uint16_t* w0 = W + n * K + g * G;
            uint16_t sb, bb;
            oracle_e0m4_fit_group(w0, G, &sb, &bb);
            scales[n * ng + g] = sb;
            bias[n * ng + g] = bb;
            for (int64_t k = 0; k < G; ++k)
                codes[n * K + g * G + k] = (uint8_t)oracle_e0m4_encode_one(w0[k], sb, bb);
        }
    }
}

/* Encode with caller-supplied parameters (no fitting). */
void oracle_e0m4_encode(const uint16_t* W, int64_t N, int64_t K, int64_t G,
                        const uint16_t* scales, const uint16_t* bias, uint8_t* codes)
{
    const int64_t ng = K / G;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            codes[n * K + k] = (uint8_t)oracle_e0m4_encode_one(W[n * K + k], scales[n * ng + k / G],
                                                               bias[n * ng + k / G]);
}

void oracle_e0m4_dequant(const uint8_t* codes, const uint16_t* scales, const uint16_t* bias,
                         int64_t N, int64_t K, int64_t G, uint16_t* W_out)
{
    const int64_t ng = K / G;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            W_out[n * K + k] = oracle_e0m4_decode_one(codes[n * K + k], scales[n * ng + k / G],
                                                      bias[n * ng + k / G]);
}

/* ------------------------------------------------------------------ */
/* Other code widths (paper: end of the section "E0M4 FP4              */
/* quantization": the approach carries over to other bit widths).      */
/* ------------------------------------------------------------------ */
/* E0Mk keeps the k highest fraction bits of the mapped fp16 value, 1 <= k <= 8,
 * and one more bit for rounding.  Everything is the E0M4 definition above with 4
 * replaced by k: the code is shifted left by 10 - k, it saturates at 2^k - 1,
 * the bias keeps its k highest fraction bits.  Written out again on purpose (not
 * by calling the E0M4 functions), so that k = 4 can be pinned against them. */

uint16_t oracle_e0mk_w1_bits(int c, int k)
{
    return (uint16_t)(E0M4_EXP_BITS | ((unsigned)(c & ((1 << k) - 1)) << (10 - k)));
}

uint16_t oracle_e0mk_decode_one(int c, uint16_t scale_bits, uint16_t bias_bits, int k)
{
    double w1 = oracle_half_bits_to_double(oracle_e0mk_w1_bits(c, k));
    double b = oracle_half_bits_to_double(bias_bits);
    double s = oracle_half_bits_to_double(scale_bits);
    return oracle_double_to_half_bits((w1 - b) * s);
}

void oracle_e0mk_fit_group(const uint16_t* w0, int64_t G, int k, uint16_t* scale_bits, uint16_t* bias_bits)
{
    float mn = 0.0f, mx = 0.0f;
    for (int64_t i = 0; i < G; ++i) {
        float v = h2f(w0[i]);
        if (v < mn) mn = v;
        if (v > mx) mx = v;
    }
    const float span = HI - LO;
    float range = mx - mn;
    float s = range / span;
    if (s < 6.103515625e-05f) s = 6.103515625e-05f;
    if (s > 65504.0f) s = 65504.0f;
    uint16_t sb = f2h(s);
    float sf = h2f(sb);
    float q = mn / sf;
    float b = LO - q;
    if (b < LO) b = LO;
    if (b > HI) b = HI;
    const uint16_t keep = (uint16_t)(0xFFFFu << (10 - k));     /* sign, exponent, k highest fraction bits */
    *scale_bits = sb;
    *bias_bits = (uint16_t)(f2h(b) & keep);
}

int oracle_e0mk_encode_one(uint16_t w0_bits, uint16_t scale_bits, uint16_t bias_bits, int k)
{
    float q = h2f(w0_bits) / h2f(scale_bits);
    float t = q + h2f(bias_bits);
    if (t < LO) t = LO;
    if (t > HI) t = HI;
    uint16_t bits = f2h(t);
    const int top = (1 << k) - 1;
    int y1 = (bits >> (10 - k)) & top;         /* the k highest fraction bits */
    int y2 = (bits >> (9 - k)) & 1;            /* the next one */
    int c = y1 + y2;
    return c > top ? top : c;
}

void oracle_e0mk_quantize(const uint16_t* W, int64_t N, int64_t K, int64_t G, int k,
                          uint8_t* codes, uint16_t* scales, uint16_t* bias)
{
    const int64_t ng = K / G;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t g = 0; g < ng; ++g) {
            const uint16_t* w0 = W + n * K + g * G;
            uint16_t sb, bb;
            oracle_e0mk_fit_group(w0, G, k, &sb, &bb);
            scales[n * ng + g] = sb;
            bias[n * ng + g] = bb;
            for (int64_t i = 0; i < G; ++i)
                codes[n * K + g * G + i] = (uint8_t)oracle_e0mk_encode_one(w0[i], sb, bb, k);
        }
    }
}

void oracle_e0mk_dequant(const uint8_t* codes, const uint16_t* scales, const uint16_t* bias,
                         int64_t N, int64_t K, int64_t G, int k, uint16_t* W_out)
{
    const int64_t ng = K / G;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t i = 0; i < K; ++i)
            W_out[n * K + i] = oracle_e0mk_decode_one(codes[n * K + i], scales[n * ng + i / G],
                                                      bias[n * ng + i / G], k);
}

/* ------------------------------------------------------------------ */
/* INT4 comparison format (paper: section "Evaluation of FP4           */
/* quantization", Tables 1 and 2).                                     */
/* ------------------------------------------------------------------ */
/* The paper compares E0M4 with "INT4 quantization" but does not define the
 * INT4 quantiser.  Reading taken (stated in the design document): group-wise
 * asymmetric min/max quantisation with 15 steps, an integer zero point and
 * round-to-nearest,
 *     scale = fp16((max - min) / 15), range extended to contain 0,
 *     zero  = clamp(rne(-min / scale), 0, 15),
 *     q     = clamp(rne(w / scale) + zero, 0, 15),
 *     w^    = fp16((q - zero) * scale),
 * fp32 arithmetic, one IEEE operation per step, rne = round half to even.
 * The scale is floored at the smallest normal fp16 and capped at the largest
 * finite one, like the E0M4 scale.  zero is stored as the fp16 number 0..15. */

void oracle_int4_fit_group(const uint16_t* w0, int64_t G, uint16_t* scale_bits, uint16_t* zero_bits)
{
    float mn = 0.0f, mx = 0.0f;
    for (int64_t k = 0; k < G; ++k) {
        float v = h2f(w0[k]);
        if (v < mn) mn = v;
        if (v > mx) mx = v;
    }
    float range = mx - mn;
    float s = range / 15.0f;
    if (s < 6.103515625e-05f) s = 6.103515625e-05f;
    if (s > 65504.0f) s = 65504.0f;
    uint16_t sb = f2h(s);
    float sf = h2f(sb);
    float q = mn / sf;
    float z = rintf(-q);                      /* default rounding mode: half to even */
    if (z < 0.0f) z = 0.0f;
    if (z > 15.0f) z = 15.0f;
    *scale_bits = sb;
    *zero_bits = f2h(z);                      /* exact */
}

int oracle_int4_encode_one(uint16_t w0_bits, uint16_t scale_bits, uint16_t zero_bits)
{
    float q = h2f(w0_bits) / h2f(scale_bits);
    float t = rintf(q) + h2f(zero_bits);
    if (t < 0.0f) t = 0.0f;
    if (t > 15.0f) t = 15.0f;
    return (int)t;
}

/* w^ = (q - zero) * scale: the difference is an exact small integer, the
 * product is rounded once to fp16. */
uint16_t oracle_int4_decode_one(int q, uint16_t scale_bits, uint16_t zero_bits)
{
    double d = (double)q - oracle_half_bits_to_double(zero_bits);
    return oracle_double_to_half_bits(d * oracle_half_bits_to_double(scale_bits));
}

void oracle_int4_quantize(const uint16_t* W, int64_t N, int64_t K, int64_t G,
                          uint8_t* codes, uint16_t* scales, uint16_t* zeros)
{
    const int64_t ng = K / G;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t g = 0; g < ng; ++g) {
            const uint16_t* w0 = W + n * K + g * G;
            uint16_t sb, zb;
            oracle_int4_fit_group(w0, G, &sb, &zb);
            scales[n * ng + g] = sb;
            zeros[n * ng + g] = zb;
            for (int64_t k = 0; k < G; ++k)
                codes[n * K + g * G + k] = (uint8_t)oracle_int4_encode_one(w0[k], sb, zb);
        }
    }
}

void oracle_int4_dequant(const uint8_t* codes, const uint16_t* scales, const uint16_t* zeros,
                         int64_t N, int64_t K, int64_t G, uint16_t* W_out)
{
    const int64_t ng = K / G;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            W_out[n * K + k] = oracle_int4_decode_one(codes[n * K + k], scales[n * ng + k / G],
                                                      zeros[n * ng + k / G]);
}

/* ------------------------------------------------------------------ */
/* Matrix multiplication over dequantised weights: the plain sum.      */
/* ------------------------------------------------------------------ */

/* Y[m,n] = fp16( sum_k X[m,k] * What[n,k] ), fp64 accumulation in k order.
 * absdot (may be NULL) receives sum_k |X[m,k] * What[n,k]|, the quantity the
 * acceptance tolerance is stated in. */
void oracle_e0m4_matmul(const uint16_t* X, int64_t M, const uint16_t* What, int64_t N, int64_t K,
                        uint16_t* Y, double* absdot)
{
    /* widen both operands once (exact), then the textbook triple loop */
    double* xd = (double*)malloc(sizeof(double) * (size_t)(M * K > 0 ? M * K : 1));
    for (int64_t i = 0; i < M * K; ++i) xd[i] = oracle_half_bits_to_double(X[i]);
#pragma omp parallel
    {
        double* wd = (double*)malloc(sizeof(double) * (size_t)(K > 0 ? K : 1));
#pragma omp for schedule(static)
        for (int64_t n = 0; n < N; ++n) {
            for (int64_t k = 0; k < K; ++k) wd[k] = oracle_half_bits_to_double(What[n * K + k]);
            for (int64_t m = 0; m < M; ++m) {
                double acc = 0.0, aacc = 0.0;
                for (int64_t k = 0; k < K; ++k) {
                    double p = xd[m * K + k] * wd[k];
                    acc += p;
                    aacc += fabs(p);
                }
                Y[m * N + n] = oracle_double_to_half_bits(acc);
                if (absdot) absdot[m * N + n] = aacc;
            }
        }
        free(wd);
    }
    free(xd);
}

/* ------------------------------------------------------------------ */
/* The same construction on bfloat16 (paper: closing remark of the     */
/* section "E0M4 FP4 quantization": the approach carries over to other  */
/* formats and bit widths).                                            */
/* ------------------------------------------------------------------ */
/* bfloat16 has 1 sign, 8 exponent and 7 fraction bits (the upper half of a
 * binary32).  The paper works the method out for FP16 only; the reading taken
 * for bfloat16 is the E0M4 definition with the format's own numbers:
 *   - binade [2,4): CONST_EXP_BIN_PART = 0x4000 (bfloat16 2.0),
 *     CONST_BIT_SHIFT_NUM = 7 - 4 = 3, so w1(c) = as_bf16(0x4000 | c << 3)
 *     = 2 + c/8, the same sixteen values as for FP16;
 *   - eps = one unit in the last place of the binade, 2^-6: the top of the range
 *     is 4 - 2^-6 = 3.984375 (bits 0x407F);
 *   - code = min(y1 + y2, 15) with y1 = fraction bits 6..3 and y2 = bit 2 of the
 *     mapped bfloat16 value; the bias keeps fraction bits 6..3 (& 0xFFF8);
 *   - scale is floored at the smallest normal bfloat16 (2^-126) and capped at the
 *     largest finite one; weights, scale, bias, activations and outputs are
 *     bfloat16, the arithmetic fp32 single operations as for FP16;
 *   - w = bf16((w1 - bias) * scale): difference exact, product exact in fp32
 *     (5-bit by 8-bit significands), one rounding. */

/* Exact widening of a bfloat16 bit pattern. */
double oracle_bf16_bits_to_double(uint16_t h)
{
    const int sign = (h >> 15) & 1;
    const int e = (h >> 7) & 0xFF;
    const int f = h & 0x7F;
    double v;
    if (e == 0) {
        v = ldexp((double)f, -133);                 /* subnormal or zero: f/128 * 2^-126 */
    } else if (e == 255) {
        v = f ? NAN : INFINITY;
    } else {
        v = ldexp((double)(128 + f), e - 134);      /* (1 + f/128) * 2^(e-127) */
    }
    return sign ? -v : v;
}

/* Round-to-nearest-even narrowing of a double to a bfloat16 bit pattern. */
uint16_t oracle_double_to_bf16_bits(double d)
{
    uint16_t sign = (uint16_t)(signbit(d) ? 0x8000u : 0u);
    double a = fabs(d);
    if (isnan(d)) return (uint16_t)(sign | 0x7FC0u);
    if (isinf(d)) return (uint16_t)(sign | 0x7F80u);
    if (a == 0.0) return sign;
    if (a < ldexp(1.0, -126)) {
        double q = nearbyint(ldexp(a, 133));        /* subnormal spacing 2^-133; 128 is the smallest normal */
        return (uint16_t)(sign | (uint16_t)q);
    }
    int ex;
    (void)frexp(a, &ex);
    int e = ex - 1;                                 /* a in [2^e, 2^(e+1)) */
    double q = nearbyint(ldexp(a, 7 - e));          /* in [128, 256] */
    if (q >= 256.0) { q = 128.0; e += 1; }
    if (e > 127) return (uint16_t)(sign | 0x7F80u); /* overflow to infinity */
    return (uint16_t)(sign | (uint16_t)((e + 127) << 7) | (uint16_t)((int)q - 128));
}

static inline float b2f(uint16_t h) { return (float)oracle_bf16_bits_to_double(h); }   /* exact */
static inline uint16_t f2b(float f) { return oracle_double_to_bf16_bits((double)f); } /* one rounding */

#define BF16_EXP_BITS 0x4000u
#define BF16_SHIFT    3
static const float BF_LO = 2.0f;
static const float BF_HI = 3.984375f;         /* 4 - 2^-6, bits 0x407F */

uint16_t oracle_bf16_w1_bits(int c)
{
    return (uint16_t)(BF16_EXP_BITS | ((unsigned)(c & 15) << BF16_SHIFT));
}

uint16_t oracle_bf16_decode_one(int c, uint16_t scale_bits, uint16_t bias_bits)
{
    double w1 = oracle_bf16_bits_to_double(oracle_bf16_w1_bits(c));
    double b = oracle_bf16_bits_to_double(bias_bits);
    double s = oracle_bf16_bits_to_double(scale_bits);
    return oracle_double_to_bf16_bits((w1 - b) * s);
}

void oracle_bf16_fit_group(const uint16_t* w0, int64_t G, uint16_t* scale_bits, uint16_t* bias_bits)
{
    float mn = 0.0f, mx = 0.0f;
    for (int64_t k = 0; k < G; ++k) {
        float v = b2f(w0[k]);
        if (v < mn) mn = v;
        if (v > mx) mx = v;
    }
    const float span = BF_HI - BF_LO;         /* 1.984375, exact */
    float range = mx - mn;
    float s = range / span;
    if (s < 1.17549435e-38f) s = 1.17549435e-38f;       /* 2^-126, smallest normal */
    if (s > 3.3895313892515355e38f) s = 3.3895313892515355e38f;   /* largest finite bfloat16, bits 0x7F7F */
    uint16_t sb = f2b(s);
    float sf = b2f(sb);
    float q = mn / sf;
    float b = BF_LO - q;
    if (b < BF_LO) b = BF_LO;
    if (b > BF_HI) b = BF_HI;
    uint16_t bb = (uint16_t)(f2b(b) & 0xFFF8u);
    *scale_bits = sb;
    *bias_bits = bb;
}

/* bfloat16 bit pattern of the mapped value before the code is cut out of it. */
uint16_t oracle_bf16_forward_bits(uint16_t w0_bits, uint16_t scale_bits, uint16_t bias_bits)
{
    float q = b2f(w0_bits) / b2f(scale_bits);
    float t = q + b2f(bias_bits);
    if (t < BF_LO) t = BF_LO;
    if (t > BF_HI) t = BF_HI;
    return f2b(t);
}

int oracle_bf16_encode_one(uint16_t w0_bits, uint16_t scale_bits, uint16_t bias_bits)
{
    uint16_t bits = oracle_bf16_forward_bits(w0_bits, scale_bits, bias_bits);
    int y1 = (bits >> 3) & 15;                /* four highest fraction bits */
    int y2 = (bits >> 2) & 1;                 /* the next bit, used for rounding */
    int c = y1 + y2;
    return c > 15 ? 15 : c;
}

void oracle_bf16_quantize(const uint16_t* W, int64_t N, int64_t K, int64_t G,
                          uint8_t* codes, uint16_t* scales, uint16_t* bias)
{
    const int64_t ng = K / G;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t g = 0; g < ng; ++g) {
            const uint16_t* w0 = W + n * K + g * G;
            uint16_t sb, bb;
            oracle_bf16_fit_group(w0, G, &sb, &bb);
            scales[n * ng + g] = sb;
            bias[n * ng + g] = bb;
            for (int64_t k = 0; k < G; ++k)
                codes[n * K + g * G + k] = (uint8_t)oracle_bf16_encode_one(w0[k], sb, bb);
        }
    }
}

/* Encode with caller-supplied parameters (no fitting). */
void oracle_bf16_encode(const uint16_t* W, int64_t N, int64_t K, int64_t G,
                        const uint16_t* scales, const uint16_t* bias, uint8_t* codes)
{
    const int64_t ng = K / G;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            codes[n * K + k] = (uint8_t)oracle_bf16_encode_one(W[n * K + k], scales[n * ng + k / G],
                                                               bias[n * ng + k / G]);
}

void oracle_bf16_dequant(const uint8_t* codes, const uint16_t* scales, const uint16_t* bias,
                         int64_t N, int64_t K, int64_t G, uint16_t* W_out)
{
    const int64_t ng = K / G;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            W_out[n * K + k] = oracle_bf16_decode_one(codes[n * K + k], scales[n * ng + k / G],
                                                      bias[n * ng + k / G]);
}

/* Y[m,n] = bf16( sum_k X[m,k] * What[n,k] ), all bfloat16 bit patterns, fp64 accumulation in k order. */
void oracle_bf16_matmul(const uint16_t* X, int64_t M, const uint16_t* What, int64_t N, int64_t K,
                        uint16_t* Y, double* absdot)
{
    double* xd = (double*)malloc(sizeof(double) * (size_t)(M * K > 0 ? M * K : 1));
    for (int64_t i = 0; i < M * K; ++i) xd[i] = oracle_bf16_bits_to_double(X[i]);
#pragma omp parallel
    {
        double* wd = (double*)malloc(sizeof(double) * (size_t)(K > 0 ? K : 1));
#pragma omp for schedule(static)
        for (int64_t n = 0; n < N; ++n) {
            for (int64_t k = 0; k < K; ++k) wd[k] = oracle_bf16_bits_to_double(What[n * K + k]);
            for (int64_t m = 0; m < M; ++m) {
                double acc = 0.0, aacc = 0.0;
                for (int64_t k = 0; k < K; ++k) {
                    double p = xd[m * K + k] * wd[k];
                    acc += p;
                    aacc += fabs(p);
                }
                Y[m * N + n] = oracle_double_to_bf16_bits(acc);
                if (absdot) absdot[m * N + n] = aacc;
            }
        }
        free(wd);
    }
    free(xd);
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Number of threads the parallel loops use from now on (timing the oracle on one thread); 0 if built
 * without OpenMP.  Changes no arithmetic. */
int oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n < 1) n = 1;
    omp_set_num_threads(n);
    return 1;
#else
    (void)n;
    return 0;
#endif
}
