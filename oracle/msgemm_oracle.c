/*
 * msGeMM CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct host implementation of what the msGeMM hot
 * path computes (arxiv 2310.06178).  Only the test-suite, the smoke check and
 * the CPU-baseline leg of the benchmark may call it; the product path (the HIP
 * library) shares no code with this file and never links or loads it.
 *
 * Two independent pieces live here:
 *
 *  1. msgemm_oracle_gemm_f64 / msgemm_oracle_gemm_i32
 *     The method reaches exactly the plain GeMM result (Section 3.2, first
 *     line of the y(i) equation: "the naive way"), so the oracle is that
 *     definition written out: decode every 4-bit code with b(.) (Section 3.1),
 *     multiply by the activation, accumulate -- fp64 for floating-point
 *     activations, int32 for int8 activations -- and, for shared-scale
 *     weights (Section 3.3), multiply each block's partial sum by its scale
 *     q(i,g).  No table is built.
 *
 *  2. msgemm_oracle_lut_build_* / msgemm_oracle_lut_consume_*
 *     A literal evaluation of the two phases: the look-up table L of
 *     Section 3.1 (equation for L(i_0..i_{d-1}, j)) and its consumption in
 *     Section 3.2 (second line of the y(i) equation).  Used only to check the
 *     invariant "LUT formulation == direct sum" and the device LUT builder.
 *
 * Parity pins (tests marked "not gpu"): the b(.) values the paper prints, the
 * 12x4x1 worked example (Sections 2, 3.1, 3.2), one-hot activation probes,
 * brute-force enumeration of all 16^d codes, closed forms for constant code
 * matrices, a library int64/fp64 matmul on independently decoded weights,
 * linearity, scale invariants, the printed MLP1/MLP2 speed-up closed forms
 * (Section 5).  The bf16 output tolerance is a reading, not fixed by the
 * paper: "parity unpinned" for that tolerance only.
 *
 * Data layout (the paper is silent on storage order; these are the readings
 * this build takes):
 *   codes : uint8 [m][k/2] row-major; byte t of row i holds column 2t in bits
 *           3:0 and column 2t+1 in bits 7:4 (d adjacent codes of a row are
 *           adjacent bits, Section 4 "int4d").  k must be even.
 *   X     : [b][ldx], column c of the paper's k x b matrix X is contiguous:
 *           X(j,c) = X[c*ldx + j].
 *   Y     : [b][ldy], Y(i,c) = Y[c*ldy + i].
 *   scales: [m][k/scale_group]; scale_group = 0 means no scales.
 *   L     : [groups][16^d][b]; the index of (i_0..i_{d-1}) is
 *           sum_r i_r << (4r), i.e. i_0 is least significant, so a packed
 *           code byte is directly the d=2 index.
 *   Groups restart at every scale-block boundary (Section 3.3 needs the d
 *   codes of a group to share a scale); a group that runs past the end of its
 *   block (k or scale_group not a multiple of d; the paper assumes
 *   divisibility, footnote in Section 3.1) is short: missing positions
 *   contribute zero whatever their index digit is.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* b(.) of Section 3.1: b(0000)=0 ... b(0111)=7, b(1000)=-8 ... b(1111)=-1. */
int msgemm_oracle_decode(unsigned nibble)
{
    static const int table[16] = {0, 1, 2, 3, 4, 5, 6, 7,
                                  -8, -7, -6, -5, -4, -3, -2, -1};
    return table[nibble & 15u];
}

/* b-hat(.) of Section 3.2: the 4-bit pattern of a value in [-8,7]; -1 -> 1111. */
unsigned msgemm_oracle_encode(int value)
{
    for (unsigned n = 0; n < 16; ++n)
        if (msgemm_oracle_decode(n) == value) return n;
    return 0xFFFFFFFFu; /* not an int4 value */
}

int msgemm_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void msgemm_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

static unsigned code_at(const uint8_t* codes, int64_t k, int64_t i, int64_t j)
{
    uint8_t byte = codes[i * (k / 2) + j / 2];
    return (j & 1) ? (unsigned)(byte >> 4) : (unsigned)(byte & 15u);
}

static int check_shape(int64_t m, int64_t k, int64_t b, int64_t scale_group)
{
    if (m <= 0 || k <= 0 || b <= 0 || (k & 1)) return -1;
    if (scale_group < 0) return -1;
    if (scale_group > 0 && (k % scale_group) != 0) return -1;
    return 0;
}

/*
 * y(i,c) = sum_g q(i,g) * sum_{j in block g} value(code(i,j)) * X(j,c)
 * (Section 3.2 first line; Section 3.3 for q).  fp64 throughout.
 * value(.) is b(.) of Section 3.1 (values16 == NULL), or an arbitrary map from
 * the 16 bit patterns to values (Section 2: the exact datatype of the weights
 * is irrelevant to the method; b(.) is the only place where the encoding
 * enters).
 */
int msgemm_oracle_gemm_f64_values(int64_t m, int64_t k, int64_t b,
                                  const uint8_t* codes, const double* values16,
                                  const double* scales, int64_t scale_group,
                                  const double* X, int64_t ldx,
                                  double* Y, int64_t ldy)
{
    if (check_shape(m, k, b, scale_group) || !codes || !X || !Y) return -1;
    if (ldx < k || ldy < m) return -1;
    if (scale_group > 0 && !scales) return -1;
    const int64_t block = scale_group > 0 ? scale_group : k;
    const int64_t nblocks = k / block;

#pragma omp parallel
    {
        double* w = (double*)malloc((size_t)k * sizeof(double));
#pragma omp for schedule(static)
        for (int64_t i = 0; i < m; ++i) {
            for (int64_t j = 0; j < k; ++j)
                w[j] = values16 ? values16[code_at(codes, k, i, j)]
                                : (double)msgemm_oracle_decode(code_at(codes, k, i, j));
            for (int64_t c = 0; c < b; ++c) {
                const double* x = X + c * ldx;
                double y = 0.0;
                for (int64_t g = 0; g < nblocks; ++g) {
                    double s = 0.0;
                    for (int64_t j = g * block; j < (g + 1) * block; ++j)
                        s += w[j] * x[j];
                    double q = scale_group > 0 ? scales[i * nblocks + g] : 1.0;
                    y += q * s;
                }
                Y[c * ldy + i] = y;
            }
        }
        free(w);
    }
    return 0;
}

/*
 * The same sum for weights of 8 bits: one code byte per element, values256
 * maps each of the 256 bit patterns to its value (Section 2: an 8-bit floating
 * point weight matrix is named as one such datatype).  codes8 is [m][k].
 *   y(i,c) = sum_g q(i,g) * sum_{j in block g} values256[code(i,j)] * X(j,c)
 */
int msgemm_oracle_gemm_f64_codes8(int64_t m, int64_t k, int64_t b,
                                  const uint8_t* codes8, const double* values256,
                                  const double* scales, int64_t scale_group,
                                  const double* X, int64_t ldx,
                                  double* Y, int64_t ldy)
{
    if (m <= 0 || k <= 0 || b <= 0 || scale_group < 0 || !codes8 || !values256 || !X || !Y) return -1;
    if (scale_group > 0 && ((k % scale_group) != 0 || !scales)) return -1;
    if (ldx < k || ldy < m) return -1;
    const int64_t block = scale_group > 0 ? scale_group : k;
    const int64_t nblocks = k / block;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        for (int64_t c = 0; c < b; ++c) {
            const double* x = X + c * ldx;
            double y = 0.0;
            for (int64_t g = 0; g < nblocks; ++g) {
                double s = 0.0;
                for (int64_t j = g * block; j < (g + 1) * block; ++j)
                    s += values256[codes8[i * k + j]] * x[j];
                double q = scale_group > 0 ? scales[i * nblocks + g] : 1.0;
                y += q * s;
            }
            Y[c * ldy + i] = y;
        }
    }
    return 0;
}

int msgemm_oracle_gemm_f64(int64_t m, int64_t k, int64_t b,
                           const uint8_t* codes,
                           const double* scales, int64_t scale_group,
                           const double* X, int64_t ldx,
                           double* Y, int64_t ldy)
{
    return msgemm_oracle_gemm_f64_values(m, k, b, codes, NULL, scales, scale_group, X, ldx, Y, ldy);
}

/* int8 activations, int32 accumulation, no scales: the unique exact result. */
int msgemm_oracle_gemm_i32(int64_t m, int64_t k, int64_t b,
                           const uint8_t* codes,
                           const int8_t* X, int64_t ldx,
                           int32_t* Y, int64_t ldy)
{
    if (check_shape(m, k, b, 0) || !codes || !X || !Y) return -1;
    if (ldx < k || ldy < m) return -1;
#pragma omp parallel
    {
        int32_t* w = (int32_t*)malloc((size_t)k * sizeof(int32_t));
#pragma omp for schedule(static)
        for (int64_t i = 0; i < m; ++i) {
            for (int64_t j = 0; j < k; ++j)
                w[j] = msgemm_oracle_decode(code_at(codes, k, i, j));
            for (int64_t c = 0; c < b; ++c) {
                const int8_t* x = X + c * ldx;
                int32_t y = 0;
                for (int64_t j = 0; j < k; ++j) y += w[j] * (int32_t)x[j];
                Y[c * ldy + i] = y;
            }
        }
        free(w);
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Literal two-phase evaluation (Sections 3.1 and 3.2).                      */

static int64_t groups_per_block(int64_t block, int d) { return (block + d - 1) / d; }

/* Number of LUT groups (last dimension of L) for this k, d and scale block. */
int64_t msgemm_oracle_lut_groups(int64_t k, int d, int64_t scale_group)
{
    if (k <= 0 || d < 1 || d > 4 || scale_group < 0) return -1;
    const int64_t block = scale_group > 0 ? scale_group : k;
    if (k % block) return -1;
    return (k / block) * groups_per_block(block, d);
}

/* First column covered by group jg and the number of real columns in it. */
static void group_span(int64_t jg, int64_t k, int d, int64_t scale_group,
                       int64_t* first, int* len)
{
    const int64_t block = scale_group > 0 ? scale_group : k;
    const int64_t gpb = groups_per_block(block, d);
    const int64_t blk = jg / gpb, t = jg % gpb;
    int64_t lo = blk * block + t * d;
    int64_t hi = lo + d;
    if (hi > (blk + 1) * block) hi = (blk + 1) * block;
    *first = lo;
    *len = (int)(hi - lo);
}

/* Phase 1: L(i_0..i_{d-1}, j, c) = sum_r b(i_r) * X(j*d + r, c). */
int msgemm_oracle_lut_build_f64_values(int64_t k, int64_t b, int d, int64_t scale_group,
                                       const double* values16,
                                       const double* X, int64_t ldx, double* L)
{
    const int64_t G = msgemm_oracle_lut_groups(k, d, scale_group);
    if (G < 0 || b <= 0 || !X || !L || ldx < k) return -1;
    const int64_t E = (int64_t)1 << (4 * d);
    for (int64_t jg = 0; jg < G; ++jg) {
        int64_t first; int len;
        group_span(jg, k, d, scale_group, &first, &len);
        for (int64_t idx = 0; idx < E; ++idx)
            for (int64_t c = 0; c < b; ++c) {
                double s = 0.0;
                for (int r = 0; r < len; ++r) {
                    unsigned ir = (unsigned)(idx >> (4 * r)) & 15u;
                    const double w = values16 ? values16[ir] : (double)msgemm_oracle_decode(ir);
                    s += w * X[c * ldx + first + r];
                }
                L[(jg * E + idx) * b + c] = s;
            }
    }
    return 0;
}

int msgemm_oracle_lut_build_f64(int64_t k, int64_t b, int d, int64_t scale_group,
                                const double* X, int64_t ldx, double* L)
{
    return msgemm_oracle_lut_build_f64_values(k, b, d, scale_group, NULL, X, ldx, L);
}

int msgemm_oracle_lut_build_i32(int64_t k, int64_t b, int d,
                                const int8_t* X, int64_t ldx, int32_t* L)
{
    const int64_t G = msgemm_oracle_lut_groups(k, d, 0);
    if (G < 0 || b <= 0 || !X || !L || ldx < k) return -1;
    const int64_t E = (int64_t)1 << (4 * d);
    for (int64_t jg = 0; jg < G; ++jg) {
        int64_t first; int len;
        group_span(jg, k, d, 0, &first, &len);
        for (int64_t idx = 0; idx < E; ++idx)
            for (int64_t c = 0; c < b; ++c) {
                int32_t s = 0;
                for (int r = 0; r < len; ++r) {
                    unsigned ir = (unsigned)(idx >> (4 * r)) & 15u;
                    s += msgemm_oracle_decode(ir) * (int32_t)X[c * ldx + first + r];
                }
                L[(jg * E + idx) * b + c] = s;
            }
    }
    return 0;
}

/* The "int4d" index of row i at group jg: the d adjacent codes concatenated
 * (Section 4, indexing remark); short groups take digit 0 for missing places. */
static int64_t group_index(const uint8_t* codes, int64_t k, int64_t i,
                           int64_t first, int len)
{
    int64_t idx = 0;
    for (int r = 0; r < len; ++r)
        idx |= (int64_t)code_at(codes, k, i, first + r) << (4 * r);
    return idx;
}

/* Phase 2: y(i,c) = sum_j L(code digits of row i at group j, j, c), with the
 * block scale applied after the block's groups are consumed (Section 3.3). */
int msgemm_oracle_lut_consume_f64(int64_t m, int64_t k, int64_t b, int d,
                                  const uint8_t* codes,
                                  const double* scales, int64_t scale_group,
                                  const double* L, double* Y, int64_t ldy)
{
    const int64_t G = msgemm_oracle_lut_groups(k, d, scale_group);
    if (G < 0 || check_shape(m, k, b, scale_group) || !codes || !L || !Y || ldy < m)
        return -1;
    if (scale_group > 0 && !scales) return -1;
    const int64_t E = (int64_t)1 << (4 * d);
    const int64_t block = scale_group > 0 ? scale_group : k;
    const int64_t nblocks = k / block;
    const int64_t gpb = groups_per_block(block, d);
    for (int64_t i = 0; i < m; ++i)
        for (int64_t c = 0; c < b; ++c) {
            double y = 0.0;
            for (int64_t blk = 0; blk < nblocks; ++blk) {
                double s = 0.0;
                for (int64_t t = 0; t < gpb; ++t) {
                    int64_t jg = blk * gpb + t, first; int len;
                    group_span(jg, k, d, scale_group, &first, &len);
                    int64_t idx = group_index(codes, k, i, first, len);
                    s += L[(jg * E + idx) * b + c];
                }
                double q = scale_group > 0 ? scales[i * nblocks + blk] : 1.0;
                y += q * s;
            }
            Y[c * ldy + i] = y;
        }
    return 0;
}

int msgemm_oracle_lut_consume_i32(int64_t m, int64_t k, int64_t b, int d,
                                  const uint8_t* codes,
                                  const int32_t* L, int32_t* Y, int64_t ldy)
{
    const int64_t G = msgemm_oracle_lut_groups(k, d, 0);
    if (G < 0 || check_shape(m, k, b, 0) || !codes || !L || !Y || ldy < m) return -1;
    const int64_t E = (int64_t)1 << (4 * d);
    for (int64_t i = 0; i < m; ++i)
        for (int64_t c = 0; c < b; ++c) {
            int32_t y = 0;
            for (int64_t jg = 0; jg < G; ++jg) {
                int64_t first; int len;
                group_span(jg, k, d, 0, &first, &len);
                y += L[(jg * E + group_index(codes, k, i, first, len)) * b + c];
            }
            Y[c * ldy + i] = y;
        }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Final rounding of an fp64 result to the output type, round-to-nearest-even
 * straight from the double (no intermediate float, so no double rounding).  */

/* p = significand bits incl. the hidden one, emin/emax = exponent range of
 * normal numbers, ebits/mbits = field widths. */
static uint16_t round_to_small_float(double x, int p, int emin, int emax, int mbits)
{
    const int bias = emax;
    uint16_t sign = signbit(x) ? (uint16_t)0x8000u : 0;
    const uint16_t exp_all_ones = (uint16_t)(((1u << (15 - mbits)) - 1u) << mbits);
    if (isnan(x)) return (uint16_t)(sign | exp_all_ones | (1u << (mbits - 1)));
    double a = fabs(x);
    if (isinf(a)) return (uint16_t)(sign | exp_all_ones);
    if (a == 0.0) return sign;
    int ex;
    (void)frexp(a, &ex);          /* a = f * 2^ex, f in [0.5,1) */
    int e = ex - 1;               /* floor(log2(a)) */
    if (e < emin) e = emin;       /* subnormal range: fixed quantum */
    double quantum = ldexp(1.0, e - (p - 1));
    double q = nearbyint(a / quantum); /* exact scaling; default mode = RNE */
    double v = q * quantum;
    if (v >= ldexp(1.0, emax + 1)) return (uint16_t)(sign | exp_all_ones);
    if (v == 0.0) return sign;
    (void)frexp(v, &ex);
    e = ex - 1;
    if (e < emin) {               /* subnormal: field = v / 2^(emin-(p-1)) */
        uint16_t mant = (uint16_t)(v / ldexp(1.0, emin - (p - 1)));
        return (uint16_t)(sign | mant);
    }
    uint16_t mant = (uint16_t)(v / ldexp(1.0, e - (p - 1)) - ldexp(1.0, p - 1));
    return (uint16_t)(sign | ((uint16_t)(e + bias) << mbits) | mant);
}

uint16_t msgemm_oracle_f64_to_f16_bits(double x)
{
    return round_to_small_float(x, 11, -14, 15, 10);
}

uint16_t msgemm_oracle_f64_to_bf16_bits(double x)
{
    return round_to_small_float(x, 8, -126, 127, 7);
}

void msgemm_oracle_round_f16(const double* src, uint16_t* dst, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) dst[i] = msgemm_oracle_f64_to_f16_bits(src[i]);
}

void msgemm_oracle_round_bf16(const double* src, uint16_t* dst, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) dst[i] = msgemm_oracle_f64_to_bf16_bits(src[i]);
}

void msgemm_oracle_round_f32(const double* src, float* dst, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) dst[i] = (float)src[i]; /* C cast = RNE */
}
