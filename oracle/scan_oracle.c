/*
 * CPU oracle for prefix sums.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the yardstick the GPU library is measured against.  It is a
 * plain sequential scan: one loop, one accumulator, no blocking, no SIMD
 * tricks, and it shares no code with the HIP kernels.  Only tests, the smoke
 * check and the benchmark's cpu-baseline leg may call it; the product path
 * never does.
 *
 * What it computes (paper, Section 1, notation paragraph: "prefix sum" means
 * the inclusive one, y[i] = x[0] + ... + x[i]; Section 2: L_s * w is the
 * prefix sum of w, and MatMulScan returns x overwritten by its prefix sums,
 * same length as the input):
 *
 *   inclusive : y[0] = x[0],  y[i] = y[i-1] + x[i]
 *   exclusive : y[0] = 0,     y[i] = y[i-1] + x[i-1]      (inclusive shifted by one)
 *   batched   : the above on each row of `cols` elements, accumulator reset
 *               at every row start (Section 2.2, step 1: independent segments)
 *
 * The paper's algorithm reaches exactly this result (it is a schedule, not an
 * approximation), so the oracle is the definition written out.
 *
 * Accumulators
 *   integers : 64-bit, output = low 32 bits (two's complement, i.e. the true
 *              sum modulo 2^32).
 *   floats   : fp64 over the exact values of the stored f16 / bf16 / f32
 *              inputs, with Neumaier compensation so the oracle's own error
 *              is O(2^-53 * sum|x|) whatever n is.
 *
 * Every function below is pinned by tests/test_oracle_pins.py against closed
 * forms, exact rational arithmetic, brute force and the worked example of the
 * paper's Figure 1(a); none is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

/* ---------------------------------------------------------------- formats */

/* IEEE binary16 bit pattern -> double, exact (every half is a double). */
static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);               /* subnormal: frac * 2^-24 */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(frac | 0x400), expo - 25); /* (1024+frac) * 2^(e-15-10) */
    }
    return sign ? -v : v;
}

/* bfloat16 bit pattern -> double, exact: bf16 is the top half of a binary32. */
static double bf16_bits_to_double(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

double oracle_half_to_double(uint16_t h) { return half_bits_to_double(h); }
double oracle_bf16_to_double(uint16_t b) { return bf16_bits_to_double(b); }

/* Input element kinds.  The numbering is the oracle's own. */
enum { K_I32 = 0, K_F16 = 1, K_I8 = 2, K_F32 = 3, K_BF16 = 4 };

static double load_float(const void *x, size_t i, int kind)
{
    switch (kind) {
    case K_F16:  return half_bits_to_double(((const uint16_t *)x)[i]);
    case K_BF16: return bf16_bits_to_double(((const uint16_t *)x)[i]);
    case K_F32:  return (double)((const float *)x)[i];
    default:     return NAN;
    }
}

static int64_t load_int(const void *x, size_t i, int kind)
{
    return kind == K_I8 ? (int64_t)((const int8_t *)x)[i]
                        : (int64_t)((const int32_t *)x)[i];
}

/* ------------------------------------------------ compensated accumulator */

typedef struct { double s, c; } nacc;   /* running sum and its correction */

static void nacc_add(nacc *a, double v)
{
    double t = a->s + v;
    if (fabs(a->s) >= fabs(v)) a->c += (a->s - t) + v;
    else                       a->c += (v - t) + a->s;
    a->s = t;
}
static double nacc_value(const nacc *a) { return a->s + a->c; }

/* ------------------------------------------------------------ integer scan */

/* y (int32) <- scan of x (int32 or int8), rows x cols, row-major dense. */
int oracle_scan_int(const void *x, int kind, int32_t *y,
                    size_t rows, size_t cols, int exclusive)
{
    if (kind != K_I32 && kind != K_I8) return 1;
    for (size_t r = 0; r < rows; ++r) {
        int64_t acc = 0;
        for (size_t j = 0; j < cols; ++j) {
            size_t i = r * cols + j;
            int64_t v = load_int(x, i, kind);
            if (exclusive) { y[i] = (int32_t)(uint32_t)(uint64_t)acc; acc += v; }
            else           { acc += v; y[i] = (int32_t)(uint32_t)(uint64_t)acc; }
        }
    }
    return 0;
}

/* Same, but the full 64-bit sums (to show that a configuration never wraps). */
int oracle_scan_int64(const void *x, int kind, int64_t *y,
                      size_t rows, size_t cols, int exclusive)
{
    if (kind != K_I32 && kind != K_I8) return 1;
    for (size_t r = 0; r < rows; ++r) {
        int64_t acc = 0;
        for (size_t j = 0; j < cols; ++j) {
            size_t i = r * cols + j;
            int64_t v = load_int(x, i, kind);
            if (exclusive) { y[i] = acc; acc += v; }
            else           { acc += v; y[i] = acc; }
        }
    }
    return 0;
}

/* -------------------------------------------------------------- float scan */

/* y (double) <- scan of x (f16 / bf16 / f32 bit patterns).  If l1 is not
 * NULL it receives the running L1 norm belonging to the same output index:
 * inclusive: sum_{j<=i}|x_j|, exclusive: sum_{j<i}|x_j|. */
int oracle_scan_float(const void *x, int kind, double *y, double *l1,
                      size_t rows, size_t cols, int exclusive)
{
    if (kind != K_F16 && kind != K_BF16 && kind != K_F32) return 1;
    for (size_t r = 0; r < rows; ++r) {
        nacc acc = {0.0, 0.0}, nrm = {0.0, 0.0};
        for (size_t j = 0; j < cols; ++j) {
            size_t i = r * cols + j;
            double v = load_float(x, i, kind);
            if (exclusive) {
                y[i] = nacc_value(&acc);
                if (l1) l1[i] = nacc_value(&nrm);
                nacc_add(&acc, v); nacc_add(&nrm, fabs(v));
            } else {
                nacc_add(&acc, v); nacc_add(&nrm, fabs(v));
                y[i] = nacc_value(&acc);
                if (l1) l1[i] = nacc_value(&nrm);
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------- comparators */
/*
 * Streaming comparison of a candidate output against the oracle, so that a
 * 2^28-element case needs no fp64 reference array.
 *
 * Floats.  The gate metric is
 *     E1 = max_i |got_i - ref_i| / S_i ,   S_i = running L1 norm at i,
 * which equals the element-wise relative error for non-negative data.  Where
 * S_i = 0 the exact result is 0 and the candidate must be exactly 0
 * (counted in zero_norm_bad otherwise).  Also reported: the largest absolute
 * error, the largest |ref|, and the index where E1 peaked.
 */
typedef struct {
    double e1;            /* max |got-ref| / S_i over S_i > 0        */
    double max_abs_err;   /* max |got-ref|                            */
    double max_abs_ref;   /* max |ref|                                */
    uint64_t worst_index; /* flat index of the E1 maximum             */
    uint64_t zero_norm_bad; /* outputs with S_i == 0 but got != 0     */
    uint64_t nonfinite;   /* candidate values that are NaN / Inf      */
} oracle_fcmp;

int oracle_compare_float(const void *x, int kind, const float *got,
                         size_t rows, size_t cols, int exclusive,
                         oracle_fcmp *out)
{
    if (kind != K_F16 && kind != K_BF16 && kind != K_F32) return 1;
    oracle_fcmp r = {0.0, 0.0, 0.0, 0, 0, 0};
    for (size_t row = 0; row < rows; ++row) {
        nacc acc = {0.0, 0.0}, nrm = {0.0, 0.0};
        for (size_t j = 0; j < cols; ++j) {
            size_t i = row * cols + j;
            double v = load_float(x, i, kind);
            if (!exclusive) { nacc_add(&acc, v); nacc_add(&nrm, fabs(v)); }
            double ref = nacc_value(&acc), s = nacc_value(&nrm);
            double g = (double)got[i];
            if (!isfinite(g)) { r.nonfinite++; }
            else {
                double d = fabs(g - ref);
                if (d > r.max_abs_err) r.max_abs_err = d;
                if (fabs(ref) > r.max_abs_ref) r.max_abs_ref = fabs(ref);
                if (s > 0.0) {
                    double e = d / s;
                    if (e > r.e1) { r.e1 = e; r.worst_index = i; }
                } else if (g != 0.0) {
                    r.zero_norm_bad++;
                }
            }
            if (exclusive) { nacc_add(&acc, v); nacc_add(&nrm, fabs(v)); }
        }
    }
    *out = r;
    return 0;
}

/* Integers: number of mismatching outputs and the first mismatching index
 * (or -1).  Bit-exact comparison of the low 32 bits. */
int oracle_compare_int(const void *x, int kind, const int32_t *got,
                       size_t rows, size_t cols, int exclusive,
                       uint64_t *n_bad, int64_t *first_bad)
{
    if (kind != K_I32 && kind != K_I8) return 1;
    uint64_t bad = 0; int64_t first = -1;
    for (size_t r = 0; r < rows; ++r) {
        int64_t acc = 0;
        for (size_t j = 0; j < cols; ++j) {
            size_t i = r * cols + j;
            int64_t v = load_int(x, i, kind);
            if (!exclusive) acc += v;
            int32_t ref = (int32_t)(uint32_t)(uint64_t)acc;
            if (got[i] != ref) { if (!bad) first = (int64_t)i; bad++; }
            if (exclusive) acc += v;
        }
    }
    *n_bad = bad; *first_bad = first;
    return 0;
}

/* Float candidate that must equal the oracle bit for bit (integer-valued
 * float inputs whose every partial sum is exactly representable in fp32). */
int oracle_compare_float_exact(const void *x, int kind, const float *got,
                               size_t rows, size_t cols, int exclusive,
                               uint64_t *n_bad, int64_t *first_bad)
{
    if (kind != K_F16 && kind != K_BF16 && kind != K_F32) return 1;
    uint64_t bad = 0; int64_t first = -1;
    for (size_t r = 0; r < rows; ++r) {
        nacc acc = {0.0, 0.0};
        for (size_t j = 0; j < cols; ++j) {
            size_t i = r * cols + j;
            double v = load_float(x, i, kind);
            if (!exclusive) nacc_add(&acc, v);
            float ref = (float)nacc_value(&acc);
            if (!(got[i] == ref)) { if (!bad) first = (int64_t)i; bad++; }
            if (exclusive) nacc_add(&acc, v);
        }
    }
    *n_bad = bad; *first_bad = first;
    return 0;
}

/* ------------------------------------------------- timed baseline entry */
/* The oracle exactly as above, writing the output type the GPU path writes
 * (int32 or fp32), for the benchmark's host-baseline leg. */
int oracle_scan_to_f32(const void *x, int kind, float *y,
                       size_t rows, size_t cols, int exclusive)
{
    if (kind != K_F16 && kind != K_BF16 && kind != K_F32) return 1;
    for (size_t r = 0; r < rows; ++r) {
        nacc acc = {0.0, 0.0};
        for (size_t j = 0; j < cols; ++j) {
            size_t i = r * cols + j;
            double v = load_float(x, i, kind);
            if (exclusive) { y[i] = (float)nacc_value(&acc); nacc_add(&acc, v); }
            else           { nacc_add(&acc, v); y[i] = (float)nacc_value(&acc); }
        }
    }
    return 0;
}
