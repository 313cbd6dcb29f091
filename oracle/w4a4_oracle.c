/*
 * CPU oracle for the W4A4 quantized linear layer (arxiv 2301.12017).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path and must never be called from it.  Only tests, the smoke
 * check and the benchmark's cpu_baseline leg may load it.
 *
 * Everything is scalar, single threaded, one loop per mathematical index.
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC (see build.py);
 * every fp32 operation below is therefore one IEEE-754 binary32 operation,
 * rounded to nearest even, in the order written.
 *
 * What follows the paper, and where:
 *   - symmetric / asymmetric uniform mapping ........ Sec. 3.1, the two displayed equations
 *   - token-wise dynamic activation ranges ........... App. A, "Activation Quantization"
 *   - group-wise weight quantization ................. App. A, "Weight Quantization"
 *   - two INT4 codes stored per INT8 element ......... Sec. 4.2 (packing paragraph)
 *   - GEMM shapes (bs*seq) x {3h,h,4h,h} x {h,h,h,4h} . Sec. 4.1
 *   - dequantize fused behind the GEMM, quantize fused
 *     behind bias-add / GELU ......................... Sec. 4.2
 *   - asymmetric needs extra "bias term" work ........ Sec. 4.3
 *
 * Readings taken where the text is silent or garbled (each is pinned by a test):
 *   - b = 4.  Signed codes live in [-8, 7], unsigned in [0, 15].
 *   - The scale divides the range by the number of steps: S = absmax/7 (symmetric),
 *     S = (max-min)/15 (asymmetric).  The equations' "S = max|x|" example would
 *     leave only codes {-1,0,1}.
 *   - The rounding operator is round-to-nearest, ties to even.
 *   - x_zero is the real-valued minimum, kept as a float (not an integer zero point).
 *   - One weight scale per output channel; "group-wise" = contiguous runs of G
 *     elements along the input (K) axis inside one output channel.
 *   - Packing is along K: element 2j in bits 0..3, element 2j+1 in bits 4..7,
 *     two's complement nibbles for signed codes.
 *   - GELU is the erf form.
 *   - A constant vector (absmax == 0, or max == min) gets S = 1 and all codes 0.
 *   - The quantizer multiplies by a per-vector reciprocal: inv = 7/absmax or
 *     15/(max-min) (one fp32 divide), code = rne(x * inv).  This sequence is part
 *     of the definition: other faithful fp32 routes differ on exact ties.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py
 * (brute force, closed forms, error bound, invariants, fp64 truth, library
 * special cases).  No function is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_SYM 0
#define ORC_ASYM 1
#define ORC_ACT_NONE 0
#define ORC_ACT_GELU 1

/* ---------------------------------------------------------------- fp16 <-> fp32 */

/* Exact widening of an IEEE binary16 bit pattern to binary32. */
float orc_h2f(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    int32_t  e    = (h >> 10) & 0x1F;
    uint32_t m    = h & 0x3FFu;
    float v;
    if (e == 0) {
        v = ldexpf((float)m, -24);                 /* subnormal or zero: m * 2^-24 */
    } else if (e == 31) {
        v = m ? NAN : INFINITY;
    } else {
        v = ldexpf((float)(m | 0x400u), e - 25);   /* (1024+m) * 2^(e-15-10) */
    }
    return sign ? -v : v;
}

/* Round an fp32 value to binary16, nearest-even; overflow gives infinity. */
uint16_t orc_f2h(float f)
{
    uint16_t sign = signbit(f) ? 0x8000u : 0u;
    float a = fabsf(f);
    if (isnan(a)) return (uint16_t)(sign | 0x7E00u);
    if (a >= 65520.0f) return (uint16_t)(sign | 0x7C00u);   /* >= max + half ulp -> inf */
    if (a < ldexpf(1.0f, -14)) {
        /* subnormal target: spacing 2^-24; a * 2^24 is exact in fp32 */
        float r = nearbyintf(ldexpf(a, 24));
        return (uint16_t)(sign | (uint16_t)r);               /* r may be 1024 = smallest normal */
    }
    int e;
    float fr = frexpf(a, &e);                                /* a = fr * 2^e, fr in [0.5,1) */
    float r = nearbyintf(ldexpf(fr, 11));                    /* 11-bit significand, in [1024,2048] */
    if (r == 2048.0f) { r = 1024.0f; e += 1; }
    int be = e - 1 + 15;                                     /* biased exponent */
    if (be >= 31) return (uint16_t)(sign | 0x7C00u);
    return (uint16_t)(sign | (uint16_t)(be << 10) | ((uint16_t)r & 0x3FFu));
}

/* ---------------------------------------------------------------- quantizers */

static float clampf(float x, float lo, float hi)
{
    return x < lo ? lo : (x > hi ? hi : x);
}

/* Sec. 3.1, symmetric mapping with b = 4.  Returns the scale S; q[k] in [-8,7]. */
void orc_quant_sym(const float *v, int n, int8_t *q, float *S)
{
    float amax = 0.0f;
    for (int k = 0; k < n; ++k) {
        float a = fabsf(v[k]);
        if (a > amax) amax = a;
    }
    if (amax == 0.0f) {
        *S = 1.0f;
        for (int k = 0; k < n; ++k) q[k] = 0;
        return;
    }
    *S = amax / 7.0f;
    float inv = 7.0f / amax;
    for (int k = 0; k < n; ++k) {
        float t = v[k] * inv;
        float r = nearbyintf(clampf(t, -8.0f, 7.0f));
        q[k] = (int8_t)r;
    }
}

/* Sec. 3.1, asymmetric mapping with b = 4.  zero = min(v); q[k] in [0,15]. */
void orc_quant_asym(const float *v, int n, uint8_t *q, float *S, float *zero)
{
    float lo = v[0], hi = v[0];
    for (int k = 1; k < n; ++k) {
        if (v[k] < lo) lo = v[k];
        if (v[k] > hi) hi = v[k];
    }
    *zero = lo;
    if (hi == lo) {
        *S = 1.0f;
        for (int k = 0; k < n; ++k) q[k] = 0;
        return;
    }
    float range = hi - lo;
    *S = range / 15.0f;
    float inv = 15.0f / range;
    for (int k = 0; k < n; ++k) {
        float d = v[k] - lo;
        float t = d * inv;
        float r = nearbyintf(clampf(t, 0.0f, 15.0f));
        q[k] = (uint8_t)r;
    }
}

/* ---------------------------------------------------------------- nibble packing */

/* n codes (n even) -> n/2 bytes.  Works for signed and unsigned codes: only
 * the low four bits of each code are kept. */
void orc_pack(const int8_t *q, int n, uint8_t *bytes)
{
    for (int j = 0; j < n / 2; ++j) {
        uint8_t lo = (uint8_t)q[2 * j] & 0xF;
        uint8_t hi = (uint8_t)q[2 * j + 1] & 0xF;
        bytes[j] = (uint8_t)(lo | (hi << 4));
    }
}

static int nib_signed(unsigned nib) { return nib >= 8 ? (int)nib - 16 : (int)nib; }

void orc_unpack_signed(const uint8_t *bytes, int n, int8_t *q)
{
    for (int j = 0; j < n / 2; ++j) {
        q[2 * j]     = (int8_t)nib_signed(bytes[j] & 0xFu);
        q[2 * j + 1] = (int8_t)nib_signed((bytes[j] >> 4) & 0xFu);
    }
}

void orc_unpack_unsigned(const uint8_t *bytes, int n, uint8_t *q)
{
    for (int j = 0; j < n / 2; ++j) {
        q[2 * j]     = bytes[j] & 0xFu;
        q[2 * j + 1] = (bytes[j] >> 4) & 0xFu;
    }
}

static int code_at(const uint8_t *row, int k, int mode)
{
    unsigned nib = (k & 1) ? ((row[k >> 1] >> 4) & 0xFu) : (row[k >> 1] & 0xFu);
    return mode == ORC_SYM ? nib_signed(nib) : (int)nib;
}

/* ---------------------------------------------------------------- step a1: activations */

/* Per-row (token-wise) quantization of an fp32 matrix Y[M, ld] (first K columns).
 * mode SYM: q int4, s[m];  mode ASYM: q uint4, s[m], z[m] = row minimum.
 * gsum (may be NULL): RA[m, g] = sum of the codes of row m inside K-group g,
 * groups of `group` columns (group == 0: one group = the whole row).
 * Returns 0, or -1 on bad arguments. */
int orc_quantize_rows_f32(const float *Y, int M, int K, int ld, int mode, int group,
                          uint8_t *q, float *s, float *z, int32_t *gsum)
{
    if (M < 0 || K <= 0 || (K & 1) || ld < K) return -1;
    int G = group == 0 ? K : group;
    if (G <= 0 || K % G) return -1;
    int ng = K / G;
    int8_t *codes = (int8_t *)malloc((size_t)K);
    if (!codes) return -1;
    for (int m = 0; m < M; ++m) {
        const float *row = Y + (size_t)m * ld;
        if (mode == ORC_SYM) {
            orc_quant_sym(row, K, codes, &s[m]);
            if (z) z[m] = 0.0f;
        } else {
            orc_quant_asym(row, K, (uint8_t *)codes, &s[m], &z[m]);
        }
        orc_pack(codes, K, q + (size_t)m * (K / 2));
        if (gsum) {
            for (int g = 0; g < ng; ++g) {
                int32_t acc = 0;
                for (int k = g * G; k < (g + 1) * G; ++k)
                    acc += mode == ORC_SYM ? (int32_t)codes[k] : (int32_t)(uint8_t)codes[k];
                gsum[(size_t)m * ng + g] = acc;
            }
        }
    }
    free(codes);
    return 0;
}

/* Same, from fp16 bit patterns X[M, ldx] (App. A, activation quantization:
 * one dynamic range per token). */
int orc_quantize_act(const uint16_t *X, int M, int K, int ldx, int mode, int group,
                     uint8_t *q, float *s, float *z, int32_t *gsum)
{
    if (M < 0 || K <= 0 || ldx < K) return -1;
    float *row = (float *)malloc(sizeof(float) * (size_t)K);
    if (!row) return -1;
    int G = group == 0 ? K : group;
    int ng = (G > 0 && K % G == 0) ? K / G : 0;
    int rc = ng ? 0 : -1;
    for (int m = 0; m < M && rc == 0; ++m) {
        for (int k = 0; k < K; ++k) row[k] = orc_h2f(X[(size_t)m * ldx + k]);
        rc = orc_quantize_rows_f32(row, 1, K, K, mode, group, q + (size_t)m * (K / 2), s + m,
                                   z ? z + m : NULL, gsum ? gsum + (size_t)m * ng : NULL);
    }
    free(row);
    return rc;
}

/* ------------------------------------------- producer fusion: LayerNorm, then step a1 */

/* LayerNorm over the K features of every token of x (+ residual), Sec. 4.2: the quantize of
 * an activation is fused with the LayerNorm (or bias-add, or GELU) that produces it.
 *     v    = x + r                         (r may be NULL)
 *     mean = sum(v) / K,   var = sum((v - mean)^2) / K          (biased, two passes)
 *     y    = (v - mean) / sqrt(var + eps) * gamma + beta
 * evaluated in double from the fp16 inputs.  y32 = (float)y is the fused kernel's value: it
 * is stored as fp16 in Y16 (the residual stream, may be NULL), as fp32 in Y32 (may be NULL;
 * for tests) and handed to orc_quantize_rows_f32, i.e. the codes come from the fp32 value,
 * never from its fp16 rounding.  Returns 0, or -1 on bad arguments. */
int orc_layernorm_quantize(const uint16_t *X, const uint16_t *R, int M, int K, int ldx,
                           const uint16_t *gamma, const uint16_t *beta, double eps,
                           int mode, int group, uint16_t *Y16, float *Y32,
                           uint8_t *q, float *s, float *z, int32_t *gsum)
{
    if (M < 0 || K <= 0 || ldx < K || !gamma || !beta || eps < 0.0) return -1;
    int G = group == 0 ? K : group;
    if (G <= 0 || K % G) return -1;
    int ng = K / G;
    double *v = (double *)malloc(sizeof(double) * (size_t)K);
    float *y = (float *)malloc(sizeof(float) * (size_t)K);
    if (!v || !y) { free(v); free(y); return -1; }
    int rc = 0;
    for (int m = 0; m < M && rc == 0; ++m) {
        double sum = 0.0;
        for (int k = 0; k < K; ++k) {
            v[k] = (double)orc_h2f(X[(size_t)m * ldx + k]);
            if (R) v[k] += (double)orc_h2f(R[(size_t)m * ldx + k]);
            sum += v[k];
        }
        const double mean = sum / (double)K;
        double sq = 0.0;
        for (int k = 0; k < K; ++k) sq += (v[k] - mean) * (v[k] - mean);
        const double rstd = 1.0 / sqrt(sq / (double)K + eps);
        for (int k = 0; k < K; ++k) {
            const double yy = (v[k] - mean) * rstd * (double)orc_h2f(gamma[k]) + (double)orc_h2f(beta[k]);
            y[k] = (float)yy;
            if (Y16) Y16[(size_t)m * K + k] = orc_f2h(y[k]);
            if (Y32) Y32[(size_t)m * K + k] = y[k];
        }
        rc = orc_quantize_rows_f32(y, 1, K, K, mode, group, q + (size_t)m * (K / 2), s + m,
                                   z ? z + m : NULL, gsum ? gsum + (size_t)m * ng : NULL);
    }
    free(v); free(y);
    return rc;
}

/* ---------------------------------------------------------------- step a0: weights */

/* App. A weight quantization of W[N, K] (fp16 bits, row n = output channel n).
 * group == 0: one group per output channel; else contiguous runs of `group`
 * along K.  Outputs: q[N, K/2]; scale[N, ng]; zero[N, ng] (ASYM; written as 0
 * for SYM when non-NULL); gsum RW[N, ng] = code sums; rowsum_deq c[N] =
 * sum over k of the dequantized weight, accumulated group by group in fp32:
 *     c = c + (scale*RW + G*zero). */
int orc_quantize_weight(const uint16_t *W, int N, int K, int mode, int group,
                        uint8_t *q, float *scale, float *zero, int32_t *gsum, float *rowsum_deq)
{
    if (N < 0 || K <= 0 || (K & 1)) return -1;
    int G = group == 0 ? K : group;
    if (G <= 0 || K % G || (G & 1)) return -1;
    int ng = K / G;
    float *v = (float *)malloc(sizeof(float) * (size_t)G);
    int8_t *codes = (int8_t *)malloc((size_t)G);
    if (!v || !codes) { free(v); free(codes); return -1; }
    for (int n = 0; n < N; ++n) {
        float c = 0.0f;
        for (int g = 0; g < ng; ++g) {
            for (int k = 0; k < G; ++k) v[k] = orc_h2f(W[(size_t)n * K + (size_t)g * G + k]);
            float S, Z = 0.0f;
            if (mode == ORC_SYM) orc_quant_sym(v, G, codes, &S);
            else orc_quant_asym(v, G, (uint8_t *)codes, &S, &Z);
            orc_pack(codes, G, q + (size_t)n * (K / 2) + (size_t)g * (G / 2));
            int32_t r = 0;
            for (int k = 0; k < G; ++k)
                r += mode == ORC_SYM ? (int32_t)codes[k] : (int32_t)(uint8_t)codes[k];
            scale[(size_t)n * ng + g] = S;
            if (zero) zero[(size_t)n * ng + g] = Z;
            if (gsum) gsum[(size_t)n * ng + g] = r;
            float t = S * (float)r;
            float u = (float)G * Z;
            float w = t + u;
            c = c + w;
        }
        if (rowsum_deq) rowsum_deq[n] = c;
    }
    free(v);
    free(codes);
    return 0;
}

/* ---------------------------------------------------------------- step a2: GEMM */

/* P[g, m, n] = sum over k in group g of qa[m,k] * qw[n,k], read from the PACKED
 * operands (Sec. 4.1 shapes: activations [M,K], weights [N,K], both K-contiguous).
 * lda = row stride of Aq in bytes.  64-bit accumulation; returns -2 if a sum does
 * not fit int32 (cannot happen for K <= 2^23), -1 on bad arguments. */
int orc_gemm_i32(const uint8_t *Aq, int lda, const uint8_t *Wq, int M, int N, int K,
                 int mode, int group, int32_t *P)
{
    if (M < 0 || N < 0 || K <= 0 || (K & 1) || lda < K / 2) return -1;
    int G = group == 0 ? K : group;
    if (G <= 0 || K % G) return -1;
    int ng = K / G;
    for (int g = 0; g < ng; ++g)
        for (int m = 0; m < M; ++m)
            for (int n = 0; n < N; ++n) {
                int64_t acc = 0;
                for (int k = g * G; k < (g + 1) * G; ++k)
                    acc += (int64_t)code_at(Aq + (size_t)m * lda, k, mode) *
                           (int64_t)code_at(Wq + (size_t)n * (K / 2), k, mode);
                if (acc > INT32_MAX || acc < INT32_MIN) return -2;
                P[((size_t)g * M + m) * N + n] = (int32_t)acc;
            }
    return 0;
}

/* ------------------------------------------------ the INT8 sibling of the path (W8A8) */

/* Sec. 3.1 symmetric mapping with b = 8 (the INT8 pipeline the paper measures INT4 against,
 * Sec. 4.1 / 4.3): S = absmax / 127, q = clamp(rne(v * (127 / absmax)), -128, 127); a zero
 * vector gets S = 1 and zero codes.  One code per byte, no packing. */
void orc_quant_sym8(const float *v, int n, int8_t *q, float *S)
{
    float amax = 0.0f;
    for (int k = 0; k < n; ++k) {
        float a = fabsf(v[k]);
        if (a > amax) amax = a;
    }
    if (amax == 0.0f) {
        *S = 1.0f;
        for (int k = 0; k < n; ++k) q[k] = 0;
        return;
    }
    *S = amax / 127.0f;
    float inv = 127.0f / amax;
    for (int k = 0; k < n; ++k) {
        float t = v[k] * inv;
        float r = nearbyintf(clampf(t, -128.0f, 127.0f));
        q[k] = (int8_t)r;
    }
}

/* Row-wise INT8 quantization of fp16 rows X[M, ldx] (first K columns): token-wise for
 * activations, per output channel for weights (App. A with b = 8).  q[M, K], s[M]. */
int orc_quantize_rows8(const uint16_t *X, int M, int K, int ldx, int8_t *q, float *s)
{
    if (M < 0 || K <= 0 || ldx < K) return -1;
    float *row = (float *)malloc(sizeof(float) * (size_t)K);
    if (!row) return -1;
    for (int m = 0; m < M; ++m) {
        for (int k = 0; k < K; ++k) row[k] = orc_h2f(X[(size_t)m * ldx + k]);
        orc_quant_sym8(row, K, q + (size_t)m * K, s + m);
    }
    free(row);
    return 0;
}

/* P[m, n] = sum_k qa[m,k] * qw[n,k] on INT8 codes, 64-bit accumulation. */
int orc_gemm8_i32(const int8_t *A, int lda, const int8_t *W, int M, int N, int K, int32_t *P)
{
    if (M < 0 || N < 0 || K <= 0 || lda < K) return -1;
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            int64_t acc = 0;
            for (int k = 0; k < K; ++k)
                acc += (int64_t)A[(size_t)m * lda + k] * (int64_t)W[(size_t)n * K + k];
            if (acc > INT32_MAX || acc < INT32_MIN) return -2;
            P[(size_t)m * N + n] = (int32_t)acc;
        }
    return 0;
}

/* ---------------------------------------------------------------- step a3: epilogue */

/* erf-form GELU of an fp32 value, evaluated in double and rounded once. */
float orc_gelu(float y)
{
    double x = (double)y;
    return (float)(0.5 * x * (1.0 + erf(x / sqrt(2.0))));
}

/* Dequantize P[ng, M, N] into fp32 Y[M, N].
 *   SYM  (zero points absent):
 *         ng == 1:  y = ((float)P * sa[m]) * sw[n];
 *         ng  > 1:  t1 = sum_g sw[n,g]*(float)P_g (g ascending),  y = sa[m] * t1.
 *   ASYM: with x^ = sa*qa + za and w^ = sw_g*qw + zw_g,
 *         sum_k x^ w^ = sa*sum_g sw_g P_g + sa*sum_g zw_g RA_g + za*c[n]:
 *         t1 = sum_g sw[n,g]*(float)P_g, t2 = sum_g zw[n,g]*(float)RA[m,g],
 *         y = sa*t1 + sa*t2 + za*c[n]   (left to right).
 * Then + bias[n] (fp16 bits, may be NULL), then GELU if act == ORC_ACT_GELU.
 * Every operation is a separately rounded fp32 operation (Sec. 4.2: dequantize
 * follows the INT4 GEMM; bias-add / GELU precede the next quantize). */
int orc_dequant(const int32_t *P, int M, int N, int ng, int mode,
                const float *sa, const float *za, const int32_t *RA,
                const float *sw, const float *zw, const float *c,
                const uint16_t *bias, int act, float *Y)
{
    if (M < 0 || N < 0 || ng <= 0) return -1;
    if (mode == ORC_ASYM && (!za || !RA || !zw || !c)) return -1;
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            float y;
            if (mode == ORC_SYM && ng == 1) {
                float p = (float)P[(size_t)m * N + n];
                float t = p * sa[m];
                y = t * sw[n];
            } else {
                float t1 = 0.0f;
                for (int g = 0; g < ng; ++g) {
                    float p = (float)P[((size_t)g * M + m) * N + n];
                    float u = sw[(size_t)n * ng + g] * p;
                    t1 = t1 + u;
                }
                y = sa[m] * t1;
                if (mode == ORC_ASYM) {
                    float t2 = 0.0f;
                    for (int g = 0; g < ng; ++g) {
                        float u = zw[(size_t)n * ng + g] * (float)RA[(size_t)m * ng + g];
                        t2 = t2 + u;
                    }
                    float a = sa[m] * t2;
                    float b = za[m] * c[n];
                    y = y + a;
                    y = y + b;
                }
            }
            if (bias) y = y + orc_h2f(bias[n]);
            if (act == ORC_ACT_GELU) y = orc_gelu(y);
            Y[(size_t)m * N + n] = y;
        }
    return 0;
}

/* fp32 -> fp16 bits, elementwise. */
void orc_store_f16(const float *Y, size_t count, uint16_t *out)
{
    for (size_t i = 0; i < count; ++i) out[i] = orc_f2h(Y[i]);
}

/* ---------------------------------------------------------------- the whole layer */

/* One W4A4 linear on already-quantized operands: GEMM, dequantize, bias, GELU,
 * then either fp16 store (requant == 0: out_f16[M,N]) or per-token requantization
 * of the fp32 rows (requant == 1: out_q[M,N/2], out_s[M], out_z[M] if
 * requant_mode is ASYM, out_gsum[M, N/requant_group] if non-NULL).
 * y_f32 (may be NULL) receives the fp32 pre-store values.  Returns 0 or <0. */
int orc_linear(const uint8_t *Aq, int lda, const float *sa, const float *za, const int32_t *RA,
               const uint8_t *Wq, const float *sw, const float *zw, const float *c,
               int M, int N, int K, int mode, int group,
               const uint16_t *bias, int act,
               int requant, int requant_mode, int requant_group,
               uint16_t *out_f16, uint8_t *out_q, float *out_s, float *out_z, int32_t *out_gsum,
               float *y_f32)
{
    int G = group == 0 ? K : group;
    if (G <= 0 || K % G) return -1;
    int ng = K / G;
    int32_t *P = (int32_t *)malloc(sizeof(int32_t) * (size_t)ng * M * N);
    float *Y = (float *)malloc(sizeof(float) * (size_t)M * N);
    int rc = (P && Y) ? 0 : -1;
    if (!rc) rc = orc_gemm_i32(Aq, lda, Wq, M, N, K, mode, group, P);
    if (!rc) rc = orc_dequant(P, M, N, ng, mode, sa, za, RA, sw, zw, c, bias, act, Y);
    if (!rc) {
        if (requant)
            rc = orc_quantize_rows_f32(Y, M, N, N, requant_mode, requant_group, out_q, out_s, out_z, out_gsum);
        else
            orc_store_f16(Y, (size_t)M * N, out_f16);
    }
    if (!rc && y_f32) memcpy(y_f32, Y, sizeof(float) * (size_t)M * N);
    free(P);
    free(Y);
    return rc;
}
