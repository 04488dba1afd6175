/*
 * Drives every entry point of oracle/msgemm_oracle.c over small ragged problems with exactly sized heap
 * buffers, so that AddressSanitizer / UndefinedBehaviorSanitizer (see test_oracle_sanitizers.py) see any
 * access past an operand or any undefined arithmetic.  Results are cross-checked only lightly here (the
 * table formulation against the direct sum); the numerical pins live in test_oracle_pins.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int msgemm_oracle_decode(unsigned nibble);
unsigned msgemm_oracle_encode(int value);
int msgemm_oracle_gemm_f64_values(int64_t m, int64_t k, int64_t b, const uint8_t* codes, const double* values16,
                                  const double* scales, int64_t scale_group, const double* X, int64_t ldx,
                                  double* Y, int64_t ldy);
int msgemm_oracle_gemm_f64_codes8(int64_t m, int64_t k, int64_t b, const uint8_t* codes8, const double* values256,
                                  const double* scales, int64_t scale_group, const double* X, int64_t ldx,
                                  double* Y, int64_t ldy);
int msgemm_oracle_gemm_f64(int64_t m, int64_t k, int64_t b, const uint8_t* codes, const double* scales,
                           int64_t scale_group, const double* X, int64_t ldx, double* Y, int64_t ldy);
int msgemm_oracle_gemm_i32(int64_t m, int64_t k, int64_t b, const uint8_t* codes, const int8_t* X, int64_t ldx,
                           int32_t* Y, int64_t ldy);
int64_t msgemm_oracle_lut_groups(int64_t k, int d, int64_t scale_group);
int msgemm_oracle_lut_build_f64_values(int64_t k, int64_t b, int d, int64_t scale_group, const double* values16,
                                       const double* X, int64_t ldx, double* L);
int msgemm_oracle_lut_build_f64(int64_t k, int64_t b, int d, int64_t scale_group, const double* X, int64_t ldx,
                                double* L);
int msgemm_oracle_lut_build_i32(int64_t k, int64_t b, int d, const int8_t* X, int64_t ldx, int32_t* L);
int msgemm_oracle_lut_consume_f64(int64_t m, int64_t k, int64_t b, int d, const uint8_t* codes, const double* scales,
                                  int64_t scale_group, const double* L, double* Y, int64_t ldy);
int msgemm_oracle_lut_consume_i32(int64_t m, int64_t k, int64_t b, int d, const uint8_t* codes, const int32_t* L,
                                  int32_t* Y, int64_t ldy);
uint16_t msgemm_oracle_f64_to_f16_bits(double x);
uint16_t msgemm_oracle_f64_to_bf16_bits(double x);
void msgemm_oracle_round_f16(const double* src, uint16_t* dst, int64_t n);
void msgemm_oracle_round_bf16(const double* src, uint16_t* dst, int64_t n);
void msgemm_oracle_round_f32(const double* src, float* dst, int64_t n);

static uint32_t rng_state = 12345u;
static uint32_t rnd(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return rng_state >> 8;
}

#define REQUIRE(c) do { if (!(c)) { printf("driver: check failed at line %d: %s\n", __LINE__, #c); exit(1); } } while (0)

static void one_float_case(int64_t m, int64_t k, int64_t b, int64_t sg, int d)
{
    const int64_t nblk = sg ? k / sg : 1;
    uint8_t* codes = malloc((size_t)(m * (k / 2)));
    double* X = malloc(sizeof(double) * (size_t)(b * k));
    double* S = sg ? malloc(sizeof(double) * (size_t)(m * nblk)) : NULL;
    double* Y = malloc(sizeof(double) * (size_t)(b * m));
    double* Y2 = malloc(sizeof(double) * (size_t)(b * m));
    double values[16];
    for (int64_t i = 0; i < m * (k / 2); ++i) codes[i] = (uint8_t)rnd();
    for (int64_t i = 0; i < b * k; ++i) X[i] = (double)((int)(rnd() % 17) - 8) / 4.0;
    for (int64_t i = 0; S && i < m * nblk; ++i) S[i] = ldexp(1.0, (int)(rnd() % 5) - 2);
    for (int i = 0; i < 16; ++i) values[i] = (double)i * 0.5 - 3.0;
    REQUIRE(msgemm_oracle_gemm_f64(m, k, b, codes, S, sg, X, k, Y, m) == 0);
    const int64_t G = msgemm_oracle_lut_groups(k, d, sg);
    REQUIRE(G > 0);
    size_t entries = 1;
    for (int r = 0; r < d; ++r) entries *= 16;
    double* L = malloc(sizeof(double) * (size_t)G * entries * (size_t)b);
    REQUIRE(msgemm_oracle_lut_build_f64(k, b, d, sg, X, k, L) == 0);
    REQUIRE(msgemm_oracle_lut_consume_f64(m, k, b, d, codes, S, sg, L, Y2, m) == 0);
    for (int64_t i = 0; i < b * m; ++i) REQUIRE(Y[i] == Y2[i]);  /* dyadic inputs: both sums are exact */
    REQUIRE(msgemm_oracle_gemm_f64_values(m, k, b, codes, values, S, sg, X, k, Y, m) == 0);
    REQUIRE(msgemm_oracle_lut_build_f64_values(k, b, d, sg, values, X, k, L) == 0);
    REQUIRE(msgemm_oracle_lut_consume_f64(m, k, b, d, codes, S, sg, L, Y2, m) == 0);
    for (int64_t i = 0; i < b * m; ++i) REQUIRE(Y[i] == Y2[i]);
    uint16_t* h = malloc(sizeof(uint16_t) * (size_t)(b * m));
    float* f = malloc(sizeof(float) * (size_t)(b * m));
    msgemm_oracle_round_f16(Y, h, b * m);
    msgemm_oracle_round_bf16(Y, h, b * m);
    msgemm_oracle_round_f32(Y, f, b * m);
    free(f); free(h); free(L); free(Y2); free(Y); free(S); free(X); free(codes);
}

static void one_int_case(int64_t m, int64_t k, int64_t b, int d)
{
    uint8_t* codes = malloc((size_t)(m * (k / 2)));
    int8_t* X = malloc((size_t)(b * k));
    int32_t* Y = malloc(sizeof(int32_t) * (size_t)(b * m));
    int32_t* Y2 = malloc(sizeof(int32_t) * (size_t)(b * m));
    for (int64_t i = 0; i < m * (k / 2); ++i) codes[i] = (uint8_t)rnd();
    for (int64_t i = 0; i < b * k; ++i) X[i] = (int8_t)(rnd() & 0xff);
    /* the extremes: -8 * -128 in every position of row 0 */
    for (int64_t t = 0; t < k / 2; ++t) codes[t] = 0x88;
    for (int64_t j = 0; j < k; ++j) X[j] = -128;
    REQUIRE(msgemm_oracle_gemm_i32(m, k, b, codes, X, k, Y, m) == 0);
    REQUIRE(Y[0] == (int32_t)(1024 * k));
    const int64_t G = msgemm_oracle_lut_groups(k, d, 0);
    size_t entries = 1;
    for (int r = 0; r < d; ++r) entries *= 16;
    int32_t* L = malloc(sizeof(int32_t) * (size_t)G * entries * (size_t)b);
    REQUIRE(msgemm_oracle_lut_build_i32(k, b, d, X, k, L) == 0);
    REQUIRE(msgemm_oracle_lut_consume_i32(m, k, b, d, codes, L, Y2, m) == 0);
    for (int64_t i = 0; i < b * m; ++i) REQUIRE(Y[i] == Y2[i]);
    free(L); free(Y2); free(Y); free(X); free(codes);
}

int main(void)
{
    for (unsigned n = 0; n < 16; ++n) REQUIRE(msgemm_oracle_encode(msgemm_oracle_decode(n)) == n);
    REQUIRE(msgemm_oracle_encode(8) > 15 && msgemm_oracle_encode(-9) > 15);
    for (int d = 1; d <= 4; ++d) {
        one_float_case(1, 2, 1, 0, d);
        one_float_case(7, 10, 1, 0, d);      /* k not a multiple of d = 3, 4 */
        one_float_case(19, 48, 3, 16, d);    /* blocks of 16: short last group for d = 3 */
        one_float_case(33, 64, 2, 32, d);
        one_int_case(1, 2, 1, d);
        one_int_case(21, 26, 3, d);
    }
    /* 8-bit weights */
    {
        const int64_t m = 13, k = 24, b = 2, sg = 8;
        uint8_t* c8 = malloc((size_t)(m * k));
        double* X = malloc(sizeof(double) * (size_t)(b * k));
        double* S = malloc(sizeof(double) * (size_t)(m * (k / sg)));
        double* Y = malloc(sizeof(double) * (size_t)(b * m));
        double v[256];
        for (int i = 0; i < 256; ++i) v[i] = (double)(i - 128) / 32.0;
        for (int64_t i = 0; i < m * k; ++i) c8[i] = (uint8_t)rnd();
        for (int64_t i = 0; i < b * k; ++i) X[i] = (double)(rnd() % 9) - 4.0;
        for (int64_t i = 0; i < m * (k / sg); ++i) S[i] = 0.5;
        REQUIRE(msgemm_oracle_gemm_f64_codes8(m, k, b, c8, v, S, sg, X, k, Y, m) == 0);
        free(Y); free(S); free(X); free(c8);
    }
    /* argument checks return an error and touch nothing */
    REQUIRE(msgemm_oracle_gemm_f64(0, 2, 1, NULL, NULL, 0, NULL, 2, NULL, 1) != 0);
    REQUIRE(msgemm_oracle_lut_groups(3, 2, 0) < 0 || msgemm_oracle_lut_groups(3, 2, 0) == 2);
    /* roundings at the edges of the formats */
    const double edge[] = {0.0, -0.0, 65504.0, 65520.0, 1e-8, 5.96e-8, 2.98e-8, 1e39, -1e39, 3.4e38, 1e-45, 0.1};
    for (unsigned i = 0; i < sizeof(edge) / sizeof(edge[0]); ++i) {
        (void)msgemm_oracle_f64_to_f16_bits(edge[i]);
        (void)msgemm_oracle_f64_to_bf16_bits(edge[i]);
    }
    printf("oracle sanitizer driver: ok\n");
    return 0;
}
