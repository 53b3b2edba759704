/*
 * CPU oracle for the tile-centric mixed-precision GEMM  C = alpha*A*B + beta*C
 * (paper Section 4, Algorithm 1).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It defines what the method computes, in
 * plain, slow, scalar C, so that the GPU library can be checked against it.
 * It shares no code, header, table or constant with the GPU library and is
 * never called by it; only the tests, the smoke check and the benchmark's
 * "cpu_baseline" leg load it.
 *
 * What the paper fixes (Section 4, Algorithm 1; Section 5.2):
 *   - A (MxK), B (KxN), C (MxN) are cut into square tiles of one size nb;
 *   - every tile has a storage precision taken from a per-matrix precision
 *     map (a 2-D integer array, 0 = FP64, 1 = FP32);
 *   - task (i,j,l) updates C(i,j) with A(i,l)*B(l,j); a tile travels in its
 *     stored precision and the receiving task converts it to the precision
 *     it computes in ("receiver-side conversion");
 *   - the result has the precision of the C tile.
 * Everything else (FP16 / FP8 tiles, how they are scaled, the product
 * precision once more than two formats exist, the accumulation order, the
 * norm-based precision rule) is this build's reading; each function below
 * states the reading it implements.
 *
 * Pins (tests/test_oracle_*.py): software rounding against numpy.float16 /
 * brute-force e4m3 search, all-FP64 and all-FP32 maps against an exact
 * rational-arithmetic fused-multiply-add triple loop, integer-valued inputs
 * against exact integer products for every map, the standard gamma_k error
 * bound, tile visit-order invariance, closed forms of the precision rule and
 * of the product-precision counts; the receiver-side FP64 -> FP32 down-cast on
 * FP32 midpoints against numpy's cast and an exact fmaf chain, the FP32 side
 * accumulator and its fold into an FP64 tile re-enacted with exact fused
 * multiply-adds, alpha and beta that FP32 cannot hold, BF16's rank and unit
 * roundoff in the rule against the formula written out in the test.  No
 * function here is "parity unpinned".
 *
 * Arithmetic rules used throughout: every fused multiply-add is an explicit
 * fma()/fmaf() call; the file must be compiled with -ffp-contract=off so that
 * nothing else is fused.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Precision codes: 0/1 as in the paper's description of the precision map
 * in Section 5.2; 2 and 3 extend it to FP16 and FP8 (OCP e4m3, "fn" variant:
 * no infinities, one NaN code per sign, max finite 448), 4 to BF16 (8 exponent
 * bits as FP32, 7 fraction bits).  The code is a name, not a rank: by unit
 * roundoff the formats order FP64 < FP32 < FP16 < BF16 < FP8.  5 is MXFP8: e4m3
 * elements with one power-of-two scale per block of 32 consecutive reduction
 * indices (the block-scaled format of the OCP microscaling specification)
 * instead of one per tile; 6 is MXFP4, the same with e2m1 elements (magnitudes
 * 0, 0.5, 1, 1.5, 2, 3, 4, 6); 7 is MXFP6, the same with e2m3 elements (two
 * exponent and three fraction bits: multiples of 1/8 below 2, of 1/4 below 4,
 * of 1/2 up to 7.5). */
enum { P_FP64 = 0, P_FP32 = 1, P_FP16 = 2, P_FP8 = 3, P_BF16 = 4, P_MXFP8 = 5, P_MXFP4 = 6, P_MXFP6 = 7 };

/* Which product-precision reading is applied (see orc_product_precision). */
enum { POLICY_OPERAND = 0, POLICY_C_TILE = 1 };

/* ------------------------------------------------------------------------ */
/* Software rounding to a small binary format, one rounding, from FP64.      */
/* mant_bits: stored fraction bits; emin: exponent of the smallest normal;   */
/* value returned is the rounded number itself (exactly representable in     */
/* FP64), before any overflow treatment.                                     */
static double round_to_format(double x, int mant_bits, int emin)
{
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    double a = fabs(x);
    int ex = ilogb(a);                 /* floor(log2 a), also for FP64 subnormals */
    if (ex < emin) ex = emin;          /* subnormals share the quantum of emin   */
    int qexp = ex - mant_bits;         /* spacing of the target grid near a      */
    double n = ldexp(a, -qexp);        /* exact: a power-of-two scaling          */
    double f = floor(n);
    double d = n - f;                  /* exact: n < 2^(mant_bits+1)             */
    if (d > 0.5 || (d == 0.5 && fmod(f, 2.0) == 1.0)) f += 1.0;   /* nearest, ties to even */
    double r = ldexp(f, qexp);
    return copysign(r, x);
}

/* FP16 (IEEE binary16): 10 fraction bits, emin -14, max finite 65504;
 * overflow goes to infinity, underflow is gradual. */
double orc_round_fp16(double x)
{
    if (isnan(x) || isinf(x)) return x;
    double r = round_to_format(x, 10, -14);
    if (fabs(r) > 65504.0) r = copysign(INFINITY, x);
    return r;
}

/* FP8 e4m3fn: 3 fraction bits, bias 7, emin -6, max finite 448 (the all-ones
 * pattern is NaN, there is no infinity).  Overflow, including an infinite
 * input, saturates to +-448; NaN stays NaN. */
double orc_round_fp8(double x)
{
    if (isnan(x)) return x;
    if (isinf(x)) return copysign(448.0, x);
    double r = round_to_format(x, 3, -6);
    if (fabs(r) > 448.0) r = copysign(448.0, x);
    return r;
}

/* BF16: 7 fraction bits, FP32's exponent range (emin -126), max finite
 * (2 - 2^-7) * 2^127; overflow goes to infinity, underflow is gradual. */
double orc_round_bf16(double x)
{
    if (isnan(x) || isinf(x)) return x;
    double r = round_to_format(x, 7, -126);
    if (fabs(r) > ldexp(2.0 - ldexp(1.0, -7), 127)) r = copysign(INFINITY, x);
    return r;
}

/* Bit patterns of values that are already exactly representable. */
uint16_t orc_bf16_bits(double y)
{
    uint16_t s = signbit(y) ? 0x8000u : 0u;
    if (isnan(y)) return (uint16_t)(s | 0x7fc0u);
    if (isinf(y)) return (uint16_t)(s | 0x7f80u);
    double a = fabs(y);
    if (a == 0.0) return s;
    int e = ilogb(a);
    if (e < -126) return (uint16_t)(s | (uint16_t)ldexp(a, 133));        /* subnormal: a / 2^-133 */
    double frac = ldexp(a, -e) - 1.0;
    return (uint16_t)(s | ((uint16_t)(e + 127) << 7) | (uint16_t)ldexp(frac, 7));
}

double orc_bf16_value(uint16_t h)
{
    int s = h >> 15, e = (h >> 7) & 255, m = h & 127;
    double v;
    if (e == 255) v = m ? NAN : INFINITY;
    else if (e == 0) v = ldexp((double)m, -133);
    else v = ldexp(1.0 + (double)m / 128.0, e - 127);
    return s ? -v : v;
}

uint16_t orc_fp16_bits(double y)
{
    uint16_t s = signbit(y) ? 0x8000u : 0u;
    if (isnan(y)) return (uint16_t)(s | 0x7e00u);
    if (isinf(y)) return (uint16_t)(s | 0x7c00u);
    double a = fabs(y);
    if (a == 0.0) return s;
    int e = ilogb(a);
    if (e < -14) return (uint16_t)(s | (uint16_t)ldexp(a, 24));          /* subnormal: a / 2^-24 */
    double frac = ldexp(a, -e) - 1.0;                                     /* in [0,1) */
    return (uint16_t)(s | ((uint16_t)(e + 15) << 10) | (uint16_t)ldexp(frac, 10));
}

double orc_fp16_value(uint16_t h)
{
    int s = h >> 15, e = (h >> 10) & 31, m = h & 1023;
    double v;
    if (e == 31) v = m ? NAN : INFINITY;
    else if (e == 0) v = ldexp((double)m, -24);
    else v = ldexp(1.0 + (double)m / 1024.0, e - 15);
    return s ? -v : v;
}

uint8_t orc_fp8_bits(double y)
{
    uint8_t s = signbit(y) ? 0x80u : 0u;
    if (isnan(y)) return (uint8_t)(s | 0x7fu);
    double a = fabs(y);
    if (a == 0.0) return s;
    int e = ilogb(a);
    if (e < -6) return (uint8_t)(s | (uint8_t)ldexp(a, 9));               /* subnormal: a / 2^-9 */
    double frac = ldexp(a, -e) - 1.0;
    return (uint8_t)(s | ((uint8_t)(e + 7) << 3) | (uint8_t)ldexp(frac, 3));
}

double orc_fp8_value(uint8_t b)
{
    int s = b >> 7, e = (b >> 3) & 15, m = b & 7;
    double v;
    if (e == 15 && m == 7) v = NAN;
    else if (e == 0) v = ldexp((double)m, -9);
    else v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return s ? -v : v;
}

/* MXFP8: one block of 32 numbers.  Reading (the paper names further formats
 * only as future work, Section 6; the format is the OCP microscaling one):
 * shared scale 2^s with s = floor(log2 max|x|) - 8 (8 = exponent of the
 * largest e4m3 binade), kept within the E8M0 range [-127, 127]; s = 0 for an
 * all-zero block or a non-finite maximum; elements = x * 2^-s rounded once to
 * e4m3, saturating.  y receives the element numbers, the return value is s. */
int32_t orc_mx_block(const double *x, int64_t stride, double *y, int64_t ystride)
{
    double mx = 0.0;
    for (int k = 0; k < 32; ++k) { double a = fabs(x[k * stride]); if (a > mx) mx = a; }   /* NaN never enters */
    int s = 0;
    if (mx != 0.0 && !isinf(mx)) {
        s = ilogb(mx) - 8;
        if (s < -127) s = -127;
        if (s > 127) s = 127;
    }
    for (int k = 0; k < 32; ++k) y[k * ystride] = orc_round_fp8(ldexp(x[k * stride], -s));
    return s;
}

/* FP4 e2m1: 1 fraction bit, emin 0, max finite 6, no infinity or NaN codes:
 * overflow and infinities saturate to +-6; a NaN has no code and is stored as 0. */
double orc_round_fp4(double x)
{
    if (isnan(x)) return 0.0;
    if (isinf(x)) return copysign(6.0, x);
    double r = round_to_format(x, 1, 0);
    if (fabs(r) > 6.0) r = copysign(6.0, x);
    return r;
}
uint8_t orc_fp4_bits(double y)
{
    uint8_t s = signbit(y) ? 8u : 0u;
    double a = fabs(y);
    if (a == 0.0) return s;
    if (a == 0.5) return (uint8_t)(s | 1u);
    int e = ilogb(a);
    return (uint8_t)(s | ((uint8_t)(e + 1) << 1) | (ldexp(a, -e) > 1.0 ? 1u : 0u));
}
/* MXFP4: as orc_mx_block with e2m1 elements; 2 = exponent of the largest e2m1 binade. */
int32_t orc_mx4_block(const double *x, int64_t stride, double *y, int64_t ystride)
{
    double mx = 0.0;
    for (int k = 0; k < 32; ++k) { double a = fabs(x[k * stride]); if (a > mx) mx = a; }
    int s = 0;
    if (mx != 0.0 && !isinf(mx)) {
        s = ilogb(mx) - 2;
        if (s < -127) s = -127;
        if (s > 127) s = 127;
    }
    for (int k = 0; k < 32; ++k) y[k * ystride] = orc_round_fp4(ldexp(x[k * stride], -s));
    return s;
}

/* FP6 e2m3: 3 fraction bits, emin 0 (bias 1: the smallest normal is 1, the subnormals are the
 * multiples of 1/8 below it), max finite 7.5, no infinity or NaN codes: overflow and infinities
 * saturate to +-7.5; a NaN has no code and is stored as 0. */
double orc_round_fp6(double x)
{
    if (isnan(x)) return 0.0;
    if (isinf(x)) return copysign(7.5, x);
    double r = round_to_format(x, 3, 0);
    if (fabs(r) > 7.5) r = copysign(7.5, x);
    return r;
}
/* sign, two exponent bits, three fraction bits */
uint8_t orc_fp6_bits(double y)
{
    uint8_t s = signbit(y) ? 32u : 0u;
    double a = fabs(y);
    if (a < 1.0) return (uint8_t)(s | (uint8_t)(a * 8.0));          /* subnormals and zero: a = m / 8 */
    int e = ilogb(a);
    return (uint8_t)(s | ((uint8_t)(e + 1) << 3) | (uint8_t)((ldexp(a, -e) - 1.0) * 8.0));
}
/* MXFP6: as orc_mx_block with e2m3 elements; 2 = exponent of the largest e2m3 binade. */
int32_t orc_mx6_block(const double *x, int64_t stride, double *y, int64_t ystride)
{
    double mx = 0.0;
    for (int k = 0; k < 32; ++k) { double a = fabs(x[k * stride]); if (a > mx) mx = a; }
    int s = 0;
    if (mx != 0.0 && !isinf(mx)) {
        s = ilogb(mx) - 2;
        if (s < -127) s = -127;
        if (s > 127) s = 127;
    }
    for (int k = 0; k < 32; ++k) y[k * ystride] = orc_round_fp6(ldexp(x[k * stride], -s));
    return s;
}

/* Vector forms for the tests. */
void orc_mx6_blocks_array(const double *x, int64_t nblocks, double *y, uint8_t *codes, uint8_t *scale_codes)
{
    for (int64_t b = 0; b < nblocks; ++b) {
        int32_t s = orc_mx6_block(x + 32 * b, 1, y + 32 * b, 1);
        scale_codes[b] = (uint8_t)(s + 127);
        for (int k = 0; k < 32; ++k) codes[32 * b + k] = orc_fp6_bits(y[32 * b + k]);
    }
}
void orc_mx4_blocks_array(const double *x, int64_t nblocks, double *y, uint8_t *codes, uint8_t *scale_codes)
{
    for (int64_t b = 0; b < nblocks; ++b) {
        int32_t s = orc_mx4_block(x + 32 * b, 1, y + 32 * b, 1);
        scale_codes[b] = (uint8_t)(s + 127);
        for (int k = 0; k < 32; ++k) codes[32 * b + k] = orc_fp4_bits(y[32 * b + k]);
    }
}
void orc_mx_blocks_array(const double *x, int64_t nblocks, double *y, uint8_t *codes, uint8_t *scale_codes)
{
    for (int64_t b = 0; b < nblocks; ++b) {
        int32_t s = orc_mx_block(x + 32 * b, 1, y + 32 * b, 1);
        scale_codes[b] = (uint8_t)(s + 127);
        for (int k = 0; k < 32; ++k) codes[32 * b + k] = orc_fp8_bits(y[32 * b + k]);
    }
}
void orc_round_fp16_array(const double *x, int64_t n, double *y, uint16_t *bits)
{
    for (int64_t i = 0; i < n; ++i) {
        y[i] = orc_round_fp16(x[i]);
        if (bits) bits[i] = orc_fp16_bits(y[i]);
    }
}
void orc_round_bf16_array(const double *x, int64_t n, double *y, uint16_t *bits)
{
    for (int64_t i = 0; i < n; ++i) {
        y[i] = orc_round_bf16(x[i]);
        if (bits) bits[i] = orc_bf16_bits(y[i]);
    }
}
void orc_round_fp8_array(const double *x, int64_t n, double *y, uint8_t *bits)
{
    for (int64_t i = 0; i < n; ++i) {
        y[i] = orc_round_fp8(x[i]);
        if (bits) bits[i] = orc_fp8_bits(y[i]);
    }
}

/* ------------------------------------------------------------------------ */
/* Tile scan: sum of squares and largest magnitude of every nb x nb tile of a */
/* dense row-major FP64 matrix (rows x cols, leading dimension ld).           */
/* Reading (the paper has no norm rule; it draws maps at random, Section 5.2, */
/* and leaves selection strategies to future work, Section 6): the sum of     */
/* squares of a tile is defined in one fixed order so that it is a single     */
/* number, not an interval:  per tile column, a running fma over the rows top */
/* to bottom; then the nb column sums are added pairwise, neighbours first    */
/* (level by level, an odd element is carried up unchanged).                  */
static double pairwise_neighbours(double *v, int64_t n)
{
    while (n > 1) {
        int64_t h = n / 2;
        for (int64_t i = 0; i < h; ++i) v[i] = v[2 * i] + v[2 * i + 1];
        if (n & 1) { v[h] = v[n - 1]; n = h + 1; } else n = h;
    }
    return v[0];
}

void orc_tile_scan(const double *X, int64_t ld, int64_t rows, int64_t cols, int32_t nb,
                   double *sumsq, double *maxabs)
{
    int64_t RT = rows / nb, CT = cols / nb;
#pragma omp parallel
    {
        double *col = (double *)malloc(sizeof(double) * (size_t)nb);
#pragma omp for collapse(2) schedule(dynamic)
        for (int64_t I = 0; I < RT; ++I)
            for (int64_t J = 0; J < CT; ++J) {
                double mx = 0.0;
                for (int32_t c = 0; c < nb; ++c) {
                    double s = 0.0;
                    for (int32_t r = 0; r < nb; ++r) {
                        double x = X[(I * nb + r) * ld + J * nb + c];
                        s = fma(x, x, s);
                        double ax = fabs(x);
                        if (ax > mx) mx = ax;        /* NaN never enters mx */
                    }
                    col[c] = s;
                }
                sumsq[I * CT + J] = pairwise_neighbours(col, nb);
                maxabs[I * CT + J] = mx;
            }
        free(col);
    }
}

/* Unit roundoff of each storage format. */
static double unit_roundoff(int p)
{
    switch (p) {
    case P_FP64: return ldexp(1.0, -53);
    case P_FP32: return ldexp(1.0, -24);
    case P_FP16: return ldexp(1.0, -11);
    case P_BF16: return ldexp(1.0, -8);
    case P_MXFP8: return ldexp(1.0, -4);
    case P_MXFP4: return ldexp(1.0, -2);
    case P_MXFP6: return ldexp(1.0, -4);
    default:     return ldexp(1.0, -4);      /* e4m3: 3 fraction bits */
    }
}

/* Norm-based tile precision rule.  Reading: the Frobenius-norm criterion of
 * the authors' earlier tile-adaptive work that the paper cites in Sections 1
 * and 2: a tile T of X may be stored at precision p when
 *     ||T||_F * sqrt(#tiles) / ||X||_F  <=  eps / u_p ,
 * which keeps  sum_T u_p(T)^2 ||T||_F^2 <= eps^2 ||X||_F^2.  The lowest
 * allowed precision that passes is taken, otherwise the highest allowed one.
 * The test is evaluated on squares, in FP64, in exactly this order:
 *     lhs = (S_T * ntiles) * (u_p * u_p);   rhs = (eps * eps) * S;
 * with S the sum of the S_T in row-major tile order.
 * allowed_mask: bit p set = precision code p may be used.  "Lowest" and
 * "highest" go by unit roundoff: FP8, BF16, FP16, FP32, FP64 from the lowest. */
void orc_precision_rule(const double *sumsq, int64_t ntiles, double eps, uint32_t allowed_mask,
                        uint16_t *map)
{
    static const int from_lowest[5] = {P_FP8, P_BF16, P_FP16, P_FP32, P_FP64};
    double S = 0.0;
    for (int64_t t = 0; t < ntiles; ++t) S = S + sumsq[t];
    int highest = P_FP64;
    for (int k = 0; k < 5; ++k)
        if (allowed_mask & (1u << from_lowest[k])) highest = from_lowest[k];
    double rhs = (eps * eps) * S;
    for (int64_t t = 0; t < ntiles; ++t) {
        int chosen = highest;
        for (int k = 0; k < 5; ++k) {
            int p = from_lowest[k];
            if (!(allowed_mask & (1u << p))) continue;
            double u = unit_roundoff(p);
            double lhs = (sumsq[t] * (double)ntiles) * (u * u);
            if (lhs <= rhs) { chosen = p; break; }
        }
        map[t] = (uint16_t)chosen;
    }
}

/* Per-tile power-of-two scale of FP16 / FP8 tiles.  Reading (the paper does
 * not treat these formats): the tile is stored as x * 2^-e with
 * e = floor(log2 max|x|) - E_p, E_FP16 = 14, E_FP8 = 7, so the largest scaled
 * magnitude lies in [2^14,2^15) resp. [2^7,2^8); e = 0 for an all-zero tile
 * or a non-finite maximum, and for FP64 / FP32 / BF16 tiles (BF16 has FP32's
 * range and needs no scale). */
int32_t orc_scale_exponent(double maxabs, int32_t p)
{
    if (p != P_FP16 && p != P_FP8) return 0;
    if (maxabs == 0.0 || isnan(maxabs) || isinf(maxabs)) return 0;
    return ilogb(maxabs) - (p == P_FP16 ? 14 : 7);
}

/* Storage rounding of a whole matrix, tile by tile (paper Section 5.2: matrix
 * values are initialised in the precision their map gives).  Y receives the
 * stored numbers y themselves as FP64 (each exactly representable in its tile's
 * format); the number a stored element stands for is y * 2^e with e = exps[tile].
 * FP64: copy.  FP32: C cast (round to nearest even, IEEE overflow / gradual
 * underflow).  FP16 / FP8: one direct rounding of x * 2^-e from FP64.
 * X and Y may be the same array. */
/* mx_axis: the blocks of block-scaled tiles run along a row (0: A, and C, which has no reduction
 * index: reading, Section 6 leaves such formats open) or down a column (1: B). */
void orc_store_tiles_axis(const double *X, int64_t ld, int64_t rows, int64_t cols, int32_t nb,
                          const uint16_t *map, const double *maxabs, double *Y, int64_t ldy,
                          int32_t *exps, int32_t mx_axis)
{
    int64_t RT = rows / nb, CT = cols / nb;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int64_t I = 0; I < RT; ++I)
        for (int64_t J = 0; J < CT; ++J) {
            int p = map[I * CT + J];
            int32_t e = orc_scale_exponent(maxabs[I * CT + J], p);
            exps[I * CT + J] = e;
            if (p == P_MXFP8 || p == P_MXFP4 || p == P_MXFP6) {
                /* the blocks run along the reduction index; Y receives the values the stored
                 * elements stand for, element * 2^s, which are exact in FP64 (and in FP32) */
                double yb[32];
                for (int32_t u = 0; u < nb; ++u)
                    for (int32_t k0 = 0; k0 < nb; k0 += 32) {
                        const double *x0 = mx_axis ? X + (I * nb + k0) * ld + J * nb + u : X + (I * nb + u) * ld + J * nb + k0;
                        int32_t s = p == P_MXFP8 ? orc_mx_block(x0, mx_axis ? ld : 1, yb, 1)
                                  : p == P_MXFP4 ? orc_mx4_block(x0, mx_axis ? ld : 1, yb, 1)
                                                 : orc_mx6_block(x0, mx_axis ? ld : 1, yb, 1);
                        for (int k = 0; k < 32; ++k) {
                            double *y0 = mx_axis ? Y + (I * nb + k0 + k) * ldy + J * nb + u : Y + (I * nb + u) * ldy + J * nb + k0 + k;
                            *y0 = ldexp(yb[k], s);
                        }
                    }
                continue;
            }
            for (int32_t r = 0; r < nb; ++r)
                for (int32_t c = 0; c < nb; ++c) {
                    double x = X[(I * nb + r) * ld + J * nb + c];
                    double y;
                    if (p == P_FP64) y = x;
                    else if (p == P_FP32) y = (double)(float)x;
                    else if (p == P_FP16) y = orc_round_fp16(ldexp(x, -e));
                    else if (p == P_BF16) y = orc_round_bf16(x);
                    else y = orc_round_fp8(ldexp(x, -e));
                    Y[(I * nb + r) * ldy + J * nb + c] = y;
                }
        }
}

void orc_store_tiles(const double *X, int64_t ld, int64_t rows, int64_t cols, int32_t nb,
                     const uint16_t *map, const double *maxabs, double *Y, int64_t ldy,
                     int32_t *exps)
{
    orc_store_tiles_axis(X, ld, rows, cols, nb, map, maxabs, Y, ldy, exps, 0);
}

/* Precision of the product A(I,L)*B(L,J) that updates C(I,J).
 * POLICY_C_TILE is the paper's literal statement (Section 5.2: the result
 * precision follows the C tile, operands are converted when their maps
 * differ): q = pC.
 * POLICY_OPERAND (default) is this build's reading once FP16 / FP8 exist:
 * compute at the precision of the better-stored operand, but never above
 * what the C tile keeps:  q = min(cap(pC), max(pA, pB)) in precision rank,
 * cap(FP64) = FP64 and FP32 otherwise.  With BF16 the formats no longer form a
 * chain (FP16 has more fraction bits, BF16 more range; neither holds the
 * other's numbers), so "the better of the two" becomes the smallest format
 * that holds both operands' numbers exactly: FP64 > FP32 > {FP16, BF16} > FP8,
 * and FP32 for the pair FP16, BF16. */
static int holds_both(int pA, int pB)
{
    if (pA == P_MXFP8 && pB == P_MXFP8) return P_MXFP8;
    if (pA == P_MXFP4 && pB == P_MXFP4) return P_MXFP4;
    if (pA == P_MXFP6 && pB == P_MXFP6) return P_MXFP6;
    if (pA >= P_MXFP8) pA = P_FP32;                      /* block-scaled numbers are FP32 numbers, and of */
    if (pB >= P_MXFP8) pB = P_FP32;                      /* no smaller format here                        */
    if (pA == P_FP64 || pB == P_FP64) return P_FP64;
    if (pA == P_FP32 || pB == P_FP32) return P_FP32;
    int h = (pA == P_FP16) || (pB == P_FP16), b = (pA == P_BF16) || (pB == P_BF16);
    if (h && b) return P_FP32;
    if (h) return P_FP16;
    if (b) return P_BF16;
    return P_FP8;
}
int32_t orc_product_precision(int32_t pA, int32_t pB, int32_t pC, int32_t policy)
{
    int cap = (pC == P_FP64) ? P_FP64 : P_FP32;
    if (policy == POLICY_C_TILE) return cap;
    int q = holds_both(pA, pB);
    return (q == P_FP64 && cap == P_FP32) ? P_FP32 : q;
}

/* ------------------------------------------------------------------------ */
/* The GEMM itself, for a list of jobs.  Job t computes the sub-rectangle     */
/* rows [r0,r1) x cols [c0,c1) (tile-local) of C tile (I,J) and writes it into */
/* Cout (dense, row-major, leading dimension ldc, global coordinates).        */
/*                                                                           */
/* Ay, By, Cy hold stored numbers as produced by orc_store_tiles; eA, eB the  */
/* tile scale exponents; mapA [MT][KT], mapB [KT][NT], mapC [MT][NT].         */
/*                                                                           */
/* Steps for one element (r,c) of C(I,J), following Algorithm 1 with the tile */
/* index L of the reduction dimension ascending and beta applied once (the    */
/* listing writes beta inside the loop; the definition C <- alpha*A*B+beta*C  */
/* in Section 4 applies it once):                                             */
/*   T = FP64 if pC = FP64 else FP32;  s = 0 in T                             */
/*   for L ascending:  q = product precision                                  */
/*     receiver-side conversion of both operand tiles to q:                   */
/*       q in {FP64,FP32}: value y*2^e formed in q (an up-cast is exact; the  */
/*                         only down-cast, FP64 -> FP32, rounds to nearest)   */
/*       q in {FP16,BF16,FP8}: operands stay in scaled form y; 2^(eA+eB) is   */
/*                         applied to the finished tile product (an FP8 tile  */
/*                         under a BF16 product keeps its scale, a BF16 tile  */
/*                         has none)                                          */
/*     q == T : s = fma_T(a, b, s) for k ascending (the running sum goes on)  */
/*     else   : t = 0 in FP32; t = fmaf(a, b, t) for k ascending;             */
/*              s = s +_T ldexp_T((T)t, eA+eB)   (the exponent sum is 0 when  */
/*              q = FP32)                                                     */
/*   v = alpha x_T s  (+_T  beta x_T c0  when beta != 0; c0 is never read     */
/*   when beta == 0);  alpha, beta are rounded to T;  C = v rounded to pC.    */
/* alpha == 0 skips the products (s = 0).                                     */
/* pC in {FP16, FP8, BF16} (a reading: the paper has FP64 / FP32 tiles only and     */
/* leaves further formats to Section 6): the tile is accumulated as an FP32   */
/* tile (T = FP32, product precisions as for pC = FP32), Cy holds the values   */
/* the old tile stands for (stored number * 2^e, see orc_stored_values), and  */
/* what a job returns is v in FP32; the rounding to pC needs the finished     */
/* tile's largest magnitude, so the caller applies orc_store_tiles to whole   */
/* tiles of v afterwards.  Returns 0, or -1 on a bad argument.                */
/*                                                                           */
/* So that a caller can also walk the loop nest exactly as Algorithm 1 prints */
/* it (reduction tile index outermost), a call may cover only the tile range  */
/* [L0,L1) of the reduction: with `resume` the running sums s start from      */
/* `state` instead of zero, and without `finish` they are written back to     */
/* `state` and the epilogue is left out.  `state` holds the sums of job after */
/* job, each nr*nc numbers row-major, as FP64 (exact for FP32 sums too).      */
int32_t orc_gemm_jobs(int64_t M, int64_t N, int64_t K, int32_t nb,
                      const double *Ay, int64_t lda, const uint16_t *mapA, const int32_t *eA,
                      const double *By, int64_t ldb, const uint16_t *mapB, const int32_t *eB,
                      const double *Cy, int64_t ldc0, const uint16_t *mapC,
                      double alpha, double beta, int32_t policy,
                      int64_t njobs, const int32_t *jobs /* [njobs][6]: I,J,r0,r1,c0,c1 */,
                      double *Cout, int64_t ldc,
                      int64_t L0, int64_t L1, double *state, int32_t resume, int32_t finish)
{
    int64_t MT = M / nb, NT = N / nb, KT = K / nb;
    if (MT * nb != M || NT * nb != N || KT * nb != K) return -1;
    if (L0 < 0 || L1 > KT || L0 > L1) return -1;
    if ((resume || !finish) && !state) return -1;
    int64_t state_pos = 0;
    for (int64_t t = 0; t < njobs; ++t) {
        const int32_t *jb = jobs + 6 * t;
        int64_t I = jb[0], J = jb[1];
        int32_t r0 = jb[2], r1 = jb[3], c0 = jb[4], c1 = jb[5];
        if (I < 0 || I >= MT || J < 0 || J >= NT || r0 < 0 || r1 > nb || r0 > r1 || c0 < 0 ||
            c1 > nb || c0 > c1)
            return -1;
        int pC = mapC[I * NT + J];
        if (pC < P_FP64 || pC > P_MXFP6) return -1;
        int T = pC == P_FP64 ? P_FP64 : P_FP32;       /* accumulate type: FP64 or FP32 */
        int64_t nr = r1 - r0, nc = c1 - c0;
        if (nr == 0 || nc == 0) continue;

        double *sD = NULL; float *sF = NULL;
        if (T == P_FP64) sD = (double *)calloc((size_t)(nr * nc), sizeof(double));
        else             sF = (float  *)calloc((size_t)(nr * nc), sizeof(float));
        double *bD = (double *)malloc(sizeof(double) * (size_t)nb * (size_t)nc);
        float  *bF = (float  *)malloc(sizeof(float)  * (size_t)nb * (size_t)nc);
        double *st = state ? state + state_pos : NULL;
        state_pos += nr * nc;
        if (resume)
            for (int64_t i = 0; i < nr * nc; ++i) {
                if (T == P_FP64) sD[i] = st[i]; else sF[i] = (float)st[i];
            }

        for (int64_t L = L0; alpha != 0.0 && L < L1; ++L) {
            int pA = mapA[I * KT + L], pB = mapB[L * NT + J];
            int q = orc_product_precision(pA, pB, pC, policy);
            int ea = eA[I * KT + L], eb = eB[L * NT + J];
            /* an MXFP8 product multiplies the values its operands stand for (Ay, By hold them,
             * exponents 0) exactly and accumulates in FP32, like the other low products */
            int esum = (q == P_FP16 || q == P_FP8 || q == P_BF16 || q == P_MXFP8 || q == P_MXFP4 || q == P_MXFP6) ? ea + eb : 0;

            /* receiver-side conversion of the B tile columns this job needs */
#pragma omp parallel for schedule(static)
            for (int32_t k = 0; k < nb; ++k)
                for (int64_t c = 0; c < nc; ++c) {
                    double y = By[(L * nb + k) * ldb + J * nb + c0 + c];
                    if (q == P_FP64) bD[k * nc + c] = ldexp(y, eb);
                    else if (q == P_FP32) bF[k * nc + c] = ldexpf((float)y, eb);
                    else bF[k * nc + c] = (float)y;          /* scaled form, exact */
                }

#pragma omp parallel
            {
                double *aD = (double *)malloc(sizeof(double) * (size_t)nb);
                float  *aF = (float  *)malloc(sizeof(float)  * (size_t)nb);
                float  *tF = (float  *)malloc(sizeof(float)  * (size_t)nc);
#pragma omp for schedule(dynamic, 4)
                for (int64_t r = 0; r < nr; ++r) {
                    /* receiver-side conversion of this row of the A tile */
                    for (int32_t k = 0; k < nb; ++k) {
                        double y = Ay[(I * nb + r0 + r) * lda + L * nb + k];
                        if (q == P_FP64) aD[k] = ldexp(y, ea);
                        else if (q == P_FP32) aF[k] = ldexpf((float)y, ea);
                        else aF[k] = (float)y;
                    }
                    if (q == P_FP64) {                         /* then T == FP64 */
                        double *s = sD + r * nc;
                        for (int32_t k = 0; k < nb; ++k) {
                            double a = aD[k];
                            const double *b = bD + (int64_t)k * nc;
                            for (int64_t c = 0; c < nc; ++c) s[c] = fma(a, b[c], s[c]);
                        }
                    } else if (q == P_FP32 && T == P_FP32) {
                        float *s = sF + r * nc;
                        for (int32_t k = 0; k < nb; ++k) {
                            float a = aF[k];
                            const float *b = bF + (int64_t)k * nc;
                            for (int64_t c = 0; c < nc; ++c) s[c] = fmaf(a, b[c], s[c]);
                        }
                    } else {
                        for (int64_t c = 0; c < nc; ++c) tF[c] = 0.0f;
                        for (int32_t k = 0; k < nb; ++k) {
                            float a = aF[k];
                            const float *b = bF + (int64_t)k * nc;
                            for (int64_t c = 0; c < nc; ++c) tF[c] = fmaf(a, b[c], tF[c]);
                        }
                        if (T == P_FP64) {
                            double *s = sD + r * nc;
                            for (int64_t c = 0; c < nc; ++c) s[c] = s[c] + ldexp((double)tF[c], esum);
                        } else {
                            float *s = sF + r * nc;
                            for (int64_t c = 0; c < nc; ++c) s[c] = s[c] + ldexpf(tF[c], esum);
                        }
                    }
                }
                free(aD); free(aF); free(tF);
            }
        }

        if (!finish) {
            for (int64_t i = 0; i < nr * nc; ++i) st[i] = (T == P_FP64) ? sD[i] : (double)sF[i];
            free(sD); free(sF); free(bD); free(bF);
            continue;
        }
        /* epilogue: two rounded products and one rounded sum in T, no fusion */
        for (int64_t r = 0; r < nr; ++r)
            for (int64_t c = 0; c < nc; ++c) {
                int64_t gi = I * nb + r0 + r, gj = J * nb + c0 + c;
                double v;
                if (T == P_FP64) {
                    double as = alpha * sD[r * nc + c];
                    if (beta != 0.0) { double bc = beta * Cy[gi * ldc0 + gj]; v = as + bc; }
                    else v = as;
                } else {
                    float af = (float)alpha, bf = (float)beta;
                    float as = af * sF[r * nc + c];
                    if (beta != 0.0) { float bc = bf * (float)Cy[gi * ldc0 + gj]; v = (double)(as + bc); }
                    else v = (double)as;
                }
                Cout[gi * ldc + gj] = v;     /* representable in T; FP16 / FP8 tiles: see above */
            }
        free(sD); free(sF); free(bD); free(bF);
    }
    return 0;
}

/* The values a stored matrix stands for: stored number times 2^e of its tile */
/* (exact in FP64; e = 0 for FP64 / FP32 tiles).                              */
void orc_stored_values(const double *Y, int64_t ldy, int64_t rows, int64_t cols, int32_t nb,
                       const int32_t *exps, double *X, int64_t ldx)
{
    int64_t CT = cols / nb;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c)
            X[r * ldx + c] = ldexp(Y[r * ldy + c], exps[(r / nb) * CT + c / nb]);
}

int32_t orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
