/* Test infrastructure: runs every entry point of the C oracle over small, awkward shapes with every buffer
 * allocated at exactly its documented size, so that a build with -fsanitize=address,undefined turns an
 * out-of-bounds access, a signed overflow or a misaligned access anywhere in the oracle into a non-zero exit.
 * Built and run by tests/test_oracle_sanitize.py (oracle/build.py: build_sanitize_check); checks no values. */
#include "w4a4_oracle.c"

#include <stdio.h>

static uint32_t rng_state = 12345u;
static uint32_t rnd(void) { rng_state = rng_state * 1664525u + 1013904223u; return rng_state >> 8; }
static uint16_t rnd_half(float spread)
{
    float v = ((float)(rnd() % 2001) - 1000.0f) * 0.001f * spread;
    return orc_f2h(v);
}
#define NEW(type, count) ((type *)malloc(sizeof(type) * (size_t)((count) > 0 ? (count) : 1)))
#define CHECK(expr) do { int rc_ = (expr); if (rc_ != 0) { fprintf(stderr, "%s -> %d (M=%d N=%d K=%d mode=%d group=%d)\n", #expr, rc_, M, N, K, mode, group); return 1; } } while (0)

static int one_case(int M, int N, int K, int mode, int group, int requant_mode, int requant_group)
{
    const int G = group == 0 ? K : group, ng = K / G;
    uint16_t *X = NEW(uint16_t, M * K), *W = NEW(uint16_t, N * K), *bias = NEW(uint16_t, N);
    for (int i = 0; i < M * K; ++i) X[i] = rnd_half(3.0f);
    for (int i = 0; i < N * K; ++i) W[i] = rnd_half(0.1f);
    for (int i = 0; i < N; ++i) bias[i] = rnd_half(0.05f);
    if (M > 1) for (int k = 0; k < K; ++k) X[K + k] = 0;                 /* an all-zero token */
    uint8_t *qa = NEW(uint8_t, M * (K / 2)), *qw = NEW(uint8_t, N * (K / 2));
    float *sa = NEW(float, M), *za = NEW(float, M), *sw = NEW(float, N * ng), *zw = NEW(float, N * ng), *c = NEW(float, N);
    int32_t *RA = NEW(int32_t, M * ng), *RW = NEW(int32_t, N * ng);
    CHECK(orc_quantize_act(X, M, K, K, mode, group, qa, sa, za, RA));
    CHECK(orc_quantize_weight(W, N, K, mode, group, qw, sw, zw, RW, c));
    int32_t *P = NEW(int32_t, ng * M * N);
    CHECK(orc_gemm_i32(qa, K / 2, qw, M, N, K, mode, group, P));
    float *Y = NEW(float, M * N);
    CHECK(orc_dequant(P, M, N, ng, mode, sa, za, RA, sw, zw, c, bias, ORC_ACT_GELU, Y));
    uint16_t *out16 = NEW(uint16_t, M * N);
    CHECK(orc_linear(qa, K / 2, sa, za, RA, qw, sw, zw, c, M, N, K, mode, group, bias, ORC_ACT_NONE,
                     0, 0, 0, out16, NULL, NULL, NULL, NULL, Y));
    if (N % 2 == 0) {
        const int RG = requant_group == 0 ? N : requant_group;
        if (N % RG == 0) {
            uint8_t *oq = NEW(uint8_t, M * (N / 2));
            float *os = NEW(float, M), *oz = NEW(float, M);
            int32_t *og = NEW(int32_t, M * (N / RG));
            CHECK(orc_linear(qa, K / 2, sa, za, RA, qw, sw, zw, c, M, N, K, mode, group, NULL, ORC_ACT_GELU,
                             1, requant_mode, requant_group, NULL, oq, os, oz, og, NULL));
            free(oq); free(os); free(oz); free(og);
        }
    }
    /* producer fusion and the INT8 sibling on the same inputs */
    uint16_t *gamma = NEW(uint16_t, K), *beta = NEW(uint16_t, K), *Y16 = NEW(uint16_t, M * K);
    float *Y32 = NEW(float, M * K);
    for (int k = 0; k < K; ++k) { gamma[k] = rnd_half(1.0f); beta[k] = rnd_half(0.1f); }
    CHECK(orc_layernorm_quantize(X, M > 0 ? X : NULL, M, K, K, gamma, beta, 1e-5, mode, group, Y16, Y32, qa, sa, za, RA));
    int8_t *a8 = NEW(int8_t, M * K), *w8 = NEW(int8_t, N * K);
    float *s8a = NEW(float, M), *s8w = NEW(float, N);
    CHECK(orc_quantize_rows8(X, M, K, K, a8, s8a));
    CHECK(orc_quantize_rows8(W, N, K, K, w8, s8w));
    CHECK(orc_gemm8_i32(a8, K, w8, M, N, K, P));
    free(X); free(W); free(bias); free(qa); free(qw); free(sa); free(za); free(sw); free(zw); free(c); free(RA); free(RW);
    free(P); free(Y); free(out16); free(gamma); free(beta); free(Y16); free(Y32); free(a8); free(w8); free(s8a); free(s8w);
    return 0;
}

int main(void)
{
    static const int shapes[][3] = {{0, 2, 2}, {1, 1, 2}, {1, 2, 2}, {3, 5, 6}, {2, 8, 32}, {5, 6, 64}, {4, 10, 256}, {7, 12, 384}};
    int cases = 0;
    for (unsigned i = 0; i < sizeof(shapes) / sizeof(shapes[0]); ++i)
        for (int mode = 0; mode <= 1; ++mode) {
            const int M = shapes[i][0], N = shapes[i][1], K = shapes[i][2];
            const int groups[] = {0, 2, 32, 128};
            for (unsigned gi = 0; gi < 4; ++gi) {
                const int group = groups[gi];
                if (group != 0 && K % group) continue;
                for (int rm = 0; rm <= 1; ++rm) {
                    if (one_case(M, N, K, mode, group, rm, rm ? 2 : 0)) return 1;
                    ++cases;
                }
            }
        }
    /* the fp16 conversions over every bit pattern, and the extremes of the code packers */
    for (uint32_t h = 0; h < 65536u; ++h) {
        const float f = orc_h2f((uint16_t)h);
        if (f == f && orc_f2h(f) != (uint16_t)h) { fprintf(stderr, "fp16 round trip %u\n", h); return 1; }
    }
    (void)orc_f2h(1e30f); (void)orc_f2h(-1e-30f); (void)orc_gelu(-40.0f); (void)orc_gelu(40.0f);
    printf("sanitize_check: %d cases clean\n", cases);
    return 0;
}
