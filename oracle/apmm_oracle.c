/*
 * CPU oracle for arbitrary-precision bipolar-INT matrix multiplication.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path, and nothing in the product path may call it.
 *
 * What is defined here (paper sections in brackets):
 *   - oracle_bipolar_value      : value of an n-bit bipolar-INT code   [Sec. 3.1, Eq. 1]
 *   - oracle_gemm_i64           : C = A * W^T on the decoded values,
 *                                 int64 triple loop                    [Sec. 3.2, Y = WX]
 *   - oracle_gemm_planes_i64    : the method's own three steps:
 *                                 decomposition into 1-bit planes,
 *                                 pairwise 1-bit products, shift-and-add
 *                                 recovery                             [Sec. 3.2, steps 1-3]
 *   - oracle_scale_f64          : per-token x per-channel scaling of
 *                                 the integer result in double
 *                                 (epilogue; not in the paper, defined
 *                                 by the build's problem statement)
 *
 * Orientation: activations A are M x K codes of p bits, weights W are N x K
 * codes of q bits, both K-contiguous; C is M x N row-major.  The paper writes
 * the same contraction as Y = W X with the weights on the left.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py
 * (closed forms, brute force over all codes, library matmul, invariants).
 * The paper's worked 2-bit example (Fig. 2) did not survive as numbers, so no
 * paper-printed value is used: "worked-example parity unpinned"; the n=2 value
 * table (-3,-1,+1,+3) that Eq. 1 fixes is stored in tests/golden/.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Eq. 1: (x)_D = sum_{i=0}^{n-1} (2 x^(i) - 1) * 2^i, x^(i) the i-th bit of the code. */
int64_t oracle_bipolar_value(uint32_t code, int nbits)
{
    int64_t v = 0;
    for (int i = 0; i < nbits; ++i) {
        int64_t bit = (code >> i) & 1u;
        v += (2 * bit - 1) * ((int64_t)1 << i);
    }
    return v;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Decode a rows x K matrix of codes (one uint8 per element, low nbits bits used)
 * into int64 values with Eq. 1, element by element. */
static int64_t *decode_matrix(const uint8_t *codes, int64_t rows, int64_t K, int nbits)
{
    int64_t *v = (int64_t *)malloc((size_t)rows * (size_t)K * sizeof(int64_t));
    if (!v) return NULL;
    uint32_t mask = (nbits >= 32) ? 0xffffffffu : ((1u << nbits) - 1u);
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t k = 0; k < K; ++k)
            v[r * K + k] = oracle_bipolar_value(codes[r * K + k] & mask, nbits);
    return v;
}

/* Sec. 3.2: Y = W X on decoded values.  Here C[m][n] = sum_k a[m][k] * w[n][k],
 * accumulated in int64.  Returns 0, or -1 on allocation failure. */
int oracle_gemm_i64(int64_t M, int64_t N, int64_t K, int p, int q,
                    const uint8_t *a_codes, const uint8_t *w_codes, int64_t *c)
{
    int64_t *a = decode_matrix(a_codes, M, K, p);
    int64_t *w = decode_matrix(w_codes, N, K, q);
    if (!a || !w) { free(a); free(w); return -1; }
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            int64_t acc = 0;
            for (int64_t k = 0; k < K; ++k)
                acc += a[m * K + k] * w[n * K + k];
            c[m * N + n] = acc;
        }
    }
    free(a);
    free(w);
    return 0;
}

/* Sec. 3.2, the method itself, in the paper's order:
 *   step 1 (decomposition): A^(j)[m][k] = bit j of the activation code,
 *                           W^(i)[n][k] = bit i of the weight code;
 *   step 2 (1-bit MatMul) : Y^(i,j)[m][n] = sum_k s(A^(j)[m][k]) * s(W^(i)[n][k]),
 *                           s(b) = 2b - 1, i.e. a product of +-1 entries; with the
 *                           XOR form of the 1-bit product this is
 *                           K - 2 * (number of k where the two bits differ);
 *   step 3 (recovery)     : Y = sum_i sum_j 2^(i+j) * Y^(i,j).
 * The differing-bit count is taken bit by bit (no packed words) so that this
 * routine stays a readable statement of the identity. */
int oracle_gemm_planes_i64(int64_t M, int64_t N, int64_t K, int p, int q,
                           const uint8_t *a_codes, const uint8_t *w_codes, int64_t *c)
{
    /* step 1: explicit plane matrices, one byte per bit */
    uint8_t *ap = (uint8_t *)malloc((size_t)p * (size_t)M * (size_t)K);
    uint8_t *wp = (uint8_t *)malloc((size_t)q * (size_t)N * (size_t)K);
    if (!ap || !wp) { free(ap); free(wp); return -1; }
    for (int j = 0; j < p; ++j)
        for (int64_t m = 0; m < M; ++m)
            for (int64_t k = 0; k < K; ++k)
                ap[((size_t)j * M + m) * K + k] = (a_codes[m * K + k] >> j) & 1u;
    for (int i = 0; i < q; ++i)
        for (int64_t n = 0; n < N; ++n)
            for (int64_t k = 0; k < K; ++k)
                wp[((size_t)i * N + n) * K + k] = (w_codes[n * K + k] >> i) & 1u;

#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            int64_t y = 0;
            for (int i = 0; i < q; ++i) {
                for (int j = 0; j < p; ++j) {
                    /* step 2: one plane pair */
                    const uint8_t *arow = ap + ((size_t)j * M + m) * K;
                    const uint8_t *wrow = wp + ((size_t)i * N + n) * K;
                    int64_t differ = 0;
                    for (int64_t k = 0; k < K; ++k)
                        differ += (arow[k] ^ wrow[k]);
                    int64_t y_ij = K - 2 * differ;
                    /* step 3: shift by the two bit positions and sum */
                    y += y_ij * ((int64_t)1 << (i + j));
                }
            }
            c[m * N + n] = y;
        }
    }
    free(ap);
    free(wp);
    return 0;
}

/* IEEE-754 binary16 bit pattern -> double, exact. */
double oracle_half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int exp = (h >> 10) & 0x1f;
    int man = h & 0x3ff;
    double v;
    if (exp == 0) {
        v = (double)man * (1.0 / 16777216.0);            /* man * 2^-24 (subnormal) */
    } else if (exp == 31) {
        v = man ? (0.0 / 0.0) : (1.0 / 0.0);
    } else {
        double scale = 1.0;
        int e = exp - 15;
        while (e > 0) { scale *= 2.0; --e; }
        while (e < 0) { scale *= 0.5; ++e; }
        v = (1.0 + (double)man / 1024.0) * scale;
    }
    return sign ? -v : v;
}

/* Epilogue reference: F[m][n] = C[m][n] * a_scale[m] * w_scale[n] in double.
 * Scales are given as binary16 bit patterns; a NULL scale vector means 1.
 * The result is NOT rounded to half: the GPU's half output is compared to it
 * with a relative tolerance. */
void oracle_scale_f64(int64_t M, int64_t N, const int64_t *c,
                      const uint16_t *a_scale, const uint16_t *w_scale, double *f)
{
    for (int64_t m = 0; m < M; ++m) {
        double sa = a_scale ? oracle_half_bits_to_double(a_scale[m]) : 1.0;
        for (int64_t n = 0; n < N; ++n) {
            double sw = w_scale ? oracle_half_bits_to_double(w_scale[n]) : 1.0;
            f[m * N + n] = (double)c[m * N + n] * sa * sw;
        }
    }
}

/* double -> IEEE-754 binary16 bit pattern, one rounding to nearest, ties to even (finite inputs;
 * values beyond the half range become infinity).  Every step is exact in double: the division is by a
 * power of two, so the rounding decision is taken on the exact value. */
uint16_t oracle_double_to_half_bits(double f)
{
    double a = f < 0 ? -f : f;
    uint16_t sign = (f < 0 || (f == 0 && 1.0 / f < 0)) ? 0x8000u : 0u;
    if (a != a) return (uint16_t)(sign | 0x7e00u);
    if (a == 0.0) return sign;
    /* spacing of half values around a: 2^-24 below 2^-14, else 2^(e-10) with 2^e <= a < 2^(e+1) */
    int e = -14;
    double pw = 1.0 / 16384.0;                          /* 2^-14 */
    while (a >= 2.0 * pw && e < 16) { pw *= 2.0; ++e; }
    double ulp = pw / 1024.0;
    double q = a / ulp;                                 /* exact: division by a power of two */
    if (q >= 4096.0) return (uint16_t)(sign | 0x7c00u); /* beyond twice the largest half: infinity */
    double fl = (double)(int64_t)q;                     /* q >= 0 */
    double frac = q - fl;
    int64_t n = (int64_t)fl;
    if (frac > 0.5 || (frac == 0.5 && (n & 1))) ++n;
    /* n counts ulps: below 2^-14 it is the subnormal mantissa; else 1024 <= n <= 2048 */
    if (a < 1.0 / 16384.0) return (uint16_t)(sign | (uint16_t)n);   /* n == 1024 rolls into the first normal */
    if (n == 2048) { n = 1024; ++e; }
    if (e > 15) return (uint16_t)(sign | 0x7c00u);
    return (uint16_t)(sign | (uint16_t)((e + 15) << 10) | (uint16_t)(n - 1024));
}

/* float -> binary16: a float is a double, so this is the same single rounding. */
uint16_t oracle_float_to_half_bits(float f) { return oracle_double_to_half_bits((double)f); }

/* Paper Sec. 3.1: the bipolar-INT grid is symmetric (the odd integers from -(2^p - 1) to 2^p - 1),
 * which suits symmetric quantisation of the feature matrix.  The paper gives no formula; the reading
 * taken is the plain symmetric per-token quantiser onto that grid:
 *   scale  s = max_k |x[k]| / (2^p - 1), rounded once to binary16 (it is stored as binary16);
 *   value    = the odd integer v of the grid nearest to x / s, ties to the upper one;
 *   code   u = (v + 2^p - 1) / 2.
 * Written out without any rounding in the decision: the grid point of code c is 2c - (2^p - 1), the
 * border between the cells of codes c - 1 and c is the even integer 2c - 2^p, and x / s >= border is the
 * same as x >= border * s because s > 0.  x and s are binary16 numbers and the border is a small integer,
 * so border * s and the comparison are exact in double: u is the number of borders at or below x.
 * (The division for the scale: the quotient of a binary16 number by an odd integer up to 255 is never
 * closer than 2^-19 relative to a binary16 rounding tie, so rounding the double quotient once gives the
 * correctly rounded binary16 scale.)
 * A row whose scale rounds to zero gets the code of +1 everywhere.
 * x: M x K binary16 bit patterns (finite); codes: M x K; scale_half: M binary16 bit patterns. */
void oracle_quantize_rows(int64_t M, int64_t K, int p, const uint16_t *x_half,
                          uint8_t *codes, uint16_t *scale_half)
{
    const int top = (1 << p) - 1;
    for (int64_t m = 0; m < M; ++m) {
        const uint16_t *x = x_half + m * K;
        double amax = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double v = oracle_half_bits_to_double(x[k]);
            if (v < 0) v = -v;
            if (v > amax) amax = v;
        }
        const uint16_t sh = oracle_double_to_half_bits(amax / (double)top);
        const double s = oracle_half_bits_to_double(sh);
        scale_half[m] = sh;
        for (int64_t k = 0; k < K; ++k) {
            int u = 1 << (p - 1);
            if (s > 0.0) {
                const double xv = oracle_half_bits_to_double(x[k]);
                u = 0;
                for (int c = 1; c <= top; ++c) {
                    const double border = (double)(2 * c - (1 << p)) * s;   /* exact */
                    if (xv >= border) u = c;
                }
            }
            codes[m * K + k] = (uint8_t)u;
        }
    }
}
