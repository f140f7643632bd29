/*
 * CPU oracle for the LLM.int8() mixed-precision decomposition matmul
 * (arXiv 2208.07339, Section 3: vector-wise quantization, Eq. 7, and
 * mixed-precision decomposition, Eq. 8; absmax quantization, Section 2.1).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a slow, plain restatement of the method
 * used only to check the GPU library and to be timed as a CPU baseline.  It
 * shares no code with the GPU path and the GPU path never calls it.
 *
 * Conventions
 *   - fp16 values travel as their IEEE binary16 bit patterns (uint16_t) and
 *     are decoded/encoded by the two helpers below, written from the format
 *     definition (1 sign, 5 exponent, 10 fraction bits, bias 15).
 *   - X is [s x h] row-major, W is [h x o] row-major, as in the problem
 *     statement above Eq. 6 (s tokens, h features, o outputs).
 *   - A "constant" c_x / c_w is stored as the absolute maximum itself (an
 *     exact fp16 value); the paper's multiplier is 127 / absmax, so the
 *     denormalisation term S of Eq. 7 is c_x * c_w / 127^2 elementwise.
 *   - All floating point arithmetic is double precision with one rounding to
 *     fp16 at the very end.
 *
 * Pins (tests/test_oracle_*.py): fp16 helpers against every bit pattern,
 * Q() against pure-integer rational arithmetic, the integer GEMM against a
 * triple loop and closed forms, alpha = 0 against a float64 library matmul,
 * alpha = inf against Eq. 7 alone, the half-step error bound of rounding to
 * nearest; the int8-rows variant against exact rational arithmetic, its own
 * half-step bound and a float64 library matmul of the dequantized weights;
 * the row-wise and tensor-wise baselines against exact rational arithmetic,
 * closed forms on integer-valued inputs and the vector-wise functions on inputs
 * whose rows / columns share one maximum; the zeropoint variant against exact
 * rational arithmetic, the identity of Eq. 4 and Eq. 5, integer-grid inputs and
 * the absmax functions on ranges symmetric about zero.  Numbers printed by the paper: none exist for this path, so
 * end-to-end agreement with the authors' own runs is unpinned.
 */
#include <fenv.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- IEEE binary16 <-> double ------------------------------------------ */

/* value = (-1)^sign * 2^(e-15) * (1 + f/1024) for 0 < e < 31,
 *         (-1)^sign * 2^-14 * (f/1024)         for e == 0,
 *         inf / nan                             for e == 31.              */
double oracle_f16_to_double(uint16_t bits)
{
    int sign = (bits >> 15) & 1;
    int e = (bits >> 10) & 0x1f;
    int f = bits & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(1024 + f), e - 25);
    return sign ? -v : v;
}

/* round-to-nearest, ties-to-even; magnitudes that round past 65504 become
 * infinity, as IEEE 754 prescribes.                                          */
uint16_t oracle_double_to_f16(double v)
{
    uint16_t sign = signbit(v) ? 0x8000u : 0u;
    double a = fabs(v);
    if (isnan(v))
        return (uint16_t)(sign | 0x7e00u);
    if (isinf(v))
        return (uint16_t)(sign | 0x7c00u);
    if (a == 0.0)
        return sign;
    int ex;
    (void)frexp(a, &ex); /* a = m * 2^ex, 0.5 <= m < 1  =>  2^(ex-1) <= a   */
    int e = ex - 1;       /* unbiased exponent of a                          */
    if (e < -14)
        e = -14;          /* subnormal range: fixed quantum 2^-24            */
    /* quantum (spacing of fp16 values at this exponent) is 2^(e-10)         */
    double scaled = ldexp(a, 10 - e); /* exact: power-of-two scaling         */
    double r = nearbyint(scaled);     /* current mode is round-to-nearest-even */
    /* r is in [0, 2048]; r == 2048 means the mantissa carried               */
    long n = (long)r;
    if (n == 2048) {
        n = 1024;
        e += 1;
    }
    if (n >= 1024) { /* normal */
        if (e > 15)
            return (uint16_t)(sign | 0x7c00u);
        return (uint16_t)(sign | ((uint16_t)(e + 15) << 10) | (uint16_t)(n - 1024));
    }
    /* subnormal (e == -14, n < 1024)                                         */
    return (uint16_t)(sign | (uint16_t)n);
}

/* ---- absmax quantizer, Section 2.1 ------------------------------------- */

/* Q(x, c) = nearest integer to 127 * x / c, ties to even; 0 when c == 0.
 * 127 * x is exact in double (x has 11 significant bits); the division is
 * correctly rounded, a half-integer quotient is representable and therefore
 * produced exactly, and nearbyint() then applies ties-to-even.               */
int oracle_q(double x, double c)
{
    if (c == 0.0)
        return 0;
    return (int)nearbyint(127.0 * x / c);
}

/* ---- step 1: outlier feature dimensions, Section 3.2 -------------------- */

/* O = ascending list of feature columns j with |X[i][j]| >= alpha for at
 * least one row i.  Returns |O|; writes at most cap indices.                 */
int oracle_find_outliers(const uint16_t *X, int s, int h, double alpha, int32_t *idx, int cap)
{
    int count = 0;
    for (int j = 0; j < h; j++) {
        int hit = 0;
        for (int i = 0; i < s && !hit; i++)
            if (fabs(oracle_f16_to_double(X[(size_t)i * h + j])) >= alpha)
                hit = 1;
        if (hit) {
            if (count < cap)
                idx[count] = j;
            count++;
        }
    }
    return count;
}

/* ---- step 2: weights, one constant per output column (Section 3.1) ------ */

void oracle_quantize_weight(const uint16_t *W, int h, int o, int8_t *Wq, uint16_t *cw)
{
#pragma omp parallel for schedule(static)
    for (int j = 0; j < o; j++) {
        double m = 0.0;
        uint16_t mb = 0;
        for (int k = 0; k < h; k++) {
            double a = fabs(oracle_f16_to_double(W[(size_t)k * o + j]));
            if (a > m) {
                m = a;
                mb = (uint16_t)(W[(size_t)k * o + j] & 0x7fffu);
            }
        }
        cw[j] = mb;
        for (int k = 0; k < h; k++)
            Wq[(size_t)k * o + j] = (int8_t)oracle_q(oracle_f16_to_double(W[(size_t)k * o + j]), m);
    }
}

/* ---- step 3: hidden states, one constant per row over non-outlier columns */

void oracle_quantize_rows(const uint16_t *X, int s, int h, const int32_t *idx, int count,
                          int8_t *Xq, uint16_t *cx)
{
    uint8_t *is_out = (uint8_t *)calloc((size_t)h, 1);
    for (int t = 0; t < count; t++)
        is_out[idx[t]] = 1;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < s; i++) {
        double m = 0.0;
        uint16_t mb = 0;
        for (int j = 0; j < h; j++) {
            if (is_out[j])
                continue;
            double a = fabs(oracle_f16_to_double(X[(size_t)i * h + j]));
            if (a > m) {
                m = a;
                mb = (uint16_t)(X[(size_t)i * h + j] & 0x7fffu);
            }
        }
        cx[i] = mb;
        for (int j = 0; j < h; j++)
            Xq[(size_t)i * h + j] =
                is_out[j] ? (int8_t)0 : (int8_t)oracle_q(oracle_f16_to_double(X[(size_t)i * h + j]), m);
    }
    free(is_out);
}

/* ---- step 4: integer product with 32-bit accumulation (Eq. 7) ----------- */

/* C[i][j] = sum_k Xq[i][k] * Wq[k][j].  The k loop sits outside the j loop so
 * that memory is walked along rows; integer addition is exact in any order.
 * Accumulates in 64 bits and reports whether every sum fits in int32.
 * Returns 0 on success, 1 if some accumulator left the int32 range.          */
int oracle_igemm(const int8_t *Xq, const int8_t *Wq, int s, int h, int o, int32_t *C)
{
    int overflow = 0;
#pragma omp parallel for schedule(static) reduction(| : overflow)
    for (int i = 0; i < s; i++) {
        int64_t *acc = (int64_t *)calloc((size_t)o, sizeof(int64_t));
        for (int k = 0; k < h; k++) {
            int64_t a = Xq[(size_t)i * h + k];
            for (int j = 0; j < o; j++)
                acc[j] += a * (int64_t)Wq[(size_t)k * o + j];
        }
        for (int j = 0; j < o; j++) {
            if (acc[j] > INT32_MAX || acc[j] < INT32_MIN)
                overflow = 1;
            C[(size_t)i * o + j] = (int32_t)acc[j];
        }
        free(acc);
    }
    return overflow;
}

/* ---- steps 5 + 6: dequantize and add the 16-bit outlier product (Eq. 8) - */

void oracle_output(const int32_t *C, const uint16_t *cx, const uint16_t *cw, const uint16_t *X,
                   const uint16_t *W, const int32_t *idx, int count, int s, int h, int o,
                   uint16_t *Out)
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < s; i++) {
        double *acc = (double *)calloc((size_t)o, sizeof(double));
        for (int t = 0; t < count; t++) {
            int k = idx[t];
            double x = oracle_f16_to_double(X[(size_t)i * h + k]);
            for (int j = 0; j < o; j++)
                acc[j] += x * oracle_f16_to_double(W[(size_t)k * o + j]);
        }
        double ci = oracle_f16_to_double(cx[i]);
        for (int j = 0; j < o; j++) {
            double d = (double)C[(size_t)i * o + j] * ci * oracle_f16_to_double(cw[j]) / 16129.0;
            Out[(size_t)i * o + j] = oracle_double_to_f16(d + acc[j]);
        }
        free(acc);
    }
}

/* ---- variant: outlier rows of W rebuilt from the int8 codes ---------------- */

/* Section 3.2 puts the extra memory of the decomposition at roughly a tenth of a percent,
 * which keeping all of W in 16 bits would not give.  This variant stores no
 * 16-bit weights: the rows O of W are rebuilt from the codes by inverting the
 * absmax quantization of Section 2.1, W^[k][j] = fp16( W_i8[k][j] * c_w[j] / 127 )
 * (one rounding, to nearest even), and take the place of W_f16 in Eq. 8.      */
uint16_t oracle_dequant_weight(int8_t q, uint16_t cw_bits)
{
    return oracle_double_to_f16((double)q * oracle_f16_to_double(cw_bits) / 127.0);
}

/* rows[t][j] = W^[idx[t]][j] for t < count                                    */
void oracle_dequant_rows(const int8_t *Wq, const uint16_t *cw, int h, int o, const int32_t *idx, int count,
                         uint16_t *rows)
{
    (void)h;
    for (int t = 0; t < count; t++)
        for (int j = 0; j < o; j++)
            rows[(size_t)t * o + j] = oracle_dequant_weight(Wq[(size_t)idx[t] * o + j], cw[j]);
}

/* Eq. 8 with W^ in the 16-bit term                                            */
void oracle_output_dq(const int32_t *C, const uint16_t *cx, const uint16_t *cw, const uint16_t *X,
                      const int8_t *Wq, const int32_t *idx, int count, int s, int h, int o, uint16_t *Out)
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < s; i++) {
        double *acc = (double *)calloc((size_t)o, sizeof(double));
        for (int t = 0; t < count; t++) {
            int k = idx[t];
            double x = oracle_f16_to_double(X[(size_t)i * h + k]);
            for (int j = 0; j < o; j++)
                acc[j] += x * oracle_f16_to_double(oracle_dequant_weight(Wq[(size_t)k * o + j], cw[j]));
        }
        double ci = oracle_f16_to_double(cx[i]);
        for (int j = 0; j < o; j++) {
            double d = (double)C[(size_t)i * o + j] * ci * oracle_f16_to_double(cw[j]) / 16129.0;
            Out[(size_t)i * o + j] = oracle_double_to_f16(d + acc[j]);
        }
        free(acc);
    }
}

/* ---- the whole forward call ---------------------------------------------- */

/* Runs steps 1-6 on rows [0, s) of X.  Every output buffer is caller-owned.
 * idx must hold h entries (|O| can be as large as h).  Returns |O|, or -1 if
 * an int32 accumulator overflowed, or -2 if an input is not finite.          */
int oracle_linear(const uint16_t *X, const uint16_t *W, int s, int h, int o, double alpha,
                  int32_t *idx, int8_t *Xq, uint16_t *cx, int8_t *Wq, uint16_t *cw, int32_t *C,
                  uint16_t *Out)
{
    for (size_t n = 0; n < (size_t)s * h; n++)
        if ((X[n] & 0x7c00u) == 0x7c00u)
            return -2;
    for (size_t n = 0; n < (size_t)h * o; n++)
        if ((W[n] & 0x7c00u) == 0x7c00u)
            return -2;
    int count = oracle_find_outliers(X, s, h, alpha, idx, h);
    oracle_quantize_weight(W, h, o, Wq, cw);
    oracle_quantize_rows(X, s, h, idx, count, Xq, cx);
    if (oracle_igemm(Xq, Wq, s, h, o, C))
        return -1;
    oracle_output(C, cx, cw, X, W, idx, count, s, h, o, Out);
    return count;
}

/* ---- baselines of Table 1: coarser scaling constants ---------------------- */

/* Section 2.1 defines absmax quantization with ONE constant for a whole tensor
 * (127 over the largest magnitude of all its entries); Section 3 calls the
 * common refinement with one constant per row "row-wise" and its own, with a
 * constant per row of X and per column of W, "vector-wise".  Table 1 lists
 * all three, each with and without the decomposition of Section 3.2.  Here:
 *   granularity 0 (vector-wise): c_x per row of X, c_w per column of W
 *   granularity 1 (row-wise):    c_x per row of X, one c_w for all of W
 *   granularity 2 (tensor-wise): one c_x for all of X, one c_w for all of W
 * A shared constant is stored in every entry of the c_x / c_w vector, so Eq. 7
 * and Eq. 8 read the same way in all three.  With the decomposition the
 * constants of X are taken over the non-outlier columns only, as before.      */

/* one constant for the whole matrix */
void oracle_quantize_weight_tensor(const uint16_t *W, int h, int o, int8_t *Wq, uint16_t *cw)
{
    double m = 0.0;
    uint16_t mb = 0;
    for (size_t n = 0; n < (size_t)h * o; n++) {
        double a = fabs(oracle_f16_to_double(W[n]));
        if (a > m) {
            m = a;
            mb = (uint16_t)(W[n] & 0x7fffu);
        }
    }
    for (int j = 0; j < o; j++)
        cw[j] = mb;
#pragma omp parallel for schedule(static)
    for (int k = 0; k < h; k++)
        for (int j = 0; j < o; j++)
            Wq[(size_t)k * o + j] = (int8_t)oracle_q(oracle_f16_to_double(W[(size_t)k * o + j]), m);
}

/* one constant for all non-outlier entries of X; zeros in the outlier columns */
void oracle_quantize_rows_tensor(const uint16_t *X, int s, int h, const int32_t *idx, int count,
                                 int8_t *Xq, uint16_t *cx)
{
    uint8_t *is_out = (uint8_t *)calloc((size_t)h, 1);
    for (int t = 0; t < count; t++)
        is_out[idx[t]] = 1;
    double m = 0.0;
    uint16_t mb = 0;
    for (int i = 0; i < s; i++)
        for (int j = 0; j < h; j++) {
            if (is_out[j])
                continue;
            double a = fabs(oracle_f16_to_double(X[(size_t)i * h + j]));
            if (a > m) {
                m = a;
                mb = (uint16_t)(X[(size_t)i * h + j] & 0x7fffu);
            }
        }
    for (int i = 0; i < s; i++)
        cx[i] = mb;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < s; i++)
        for (int j = 0; j < h; j++)
            Xq[(size_t)i * h + j] =
                is_out[j] ? (int8_t)0 : (int8_t)oracle_q(oracle_f16_to_double(X[(size_t)i * h + j]), m);
    free(is_out);
}

/* oracle_linear with the constants at the given granularity (0, 1 or 2 as above);
 * same buffers and return values, -3 for an unknown granularity.              */
int oracle_linear_granular(const uint16_t *X, const uint16_t *W, int s, int h, int o, double alpha,
                           int granularity, int32_t *idx, int8_t *Xq, uint16_t *cx, int8_t *Wq,
                           uint16_t *cw, int32_t *C, uint16_t *Out)
{
    if (granularity < 0 || granularity > 2)
        return -3;
    for (size_t n = 0; n < (size_t)s * h; n++)
        if ((X[n] & 0x7c00u) == 0x7c00u)
            return -2;
    for (size_t n = 0; n < (size_t)h * o; n++)
        if ((W[n] & 0x7c00u) == 0x7c00u)
            return -2;
    int count = oracle_find_outliers(X, s, h, alpha, idx, h);
    if (granularity == 0)
        oracle_quantize_weight(W, h, o, Wq, cw);
    else
        oracle_quantize_weight_tensor(W, h, o, Wq, cw);
    if (granularity == 2)
        oracle_quantize_rows_tensor(X, s, h, idx, count, Xq, cx);
    else
        oracle_quantize_rows(X, s, h, idx, count, Xq, cx);
    if (oracle_igemm(Xq, Wq, s, h, o, C))
        return -1;
    oracle_output(C, cx, cw, X, W, idx, count, s, h, o, Out);
    return count;
}

/* ---- single outputs of a large problem ------------------------------------ */

/* Computes Out[i][j] and C[i][j] for n listed (i, j) pairs from the definition,
 * given the outlier set of the full X.  Each pair costs O(h): the row constant
 * of row i, the column constant of column j, then the two sums of Eq. 8.      */
void oracle_sampled(const uint16_t *X, const uint16_t *W, int s, int h, int o, const int32_t *idx,
                    int count, const int32_t *rows, const int32_t *cols, int n, int32_t *C_out,
                    uint16_t *Out_out)
{
    (void)s;
    uint8_t *is_out = (uint8_t *)calloc((size_t)h, 1);
    for (int t = 0; t < count; t++)
        is_out[idx[t]] = 1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int p = 0; p < n; p++) {
        int i = rows[p], j = cols[p];
        double mx = 0.0, mw = 0.0;
        for (int k = 0; k < h; k++) {
            double w = fabs(oracle_f16_to_double(W[(size_t)k * o + j]));
            if (w > mw)
                mw = w;
            if (is_out[k])
                continue;
            double x = fabs(oracle_f16_to_double(X[(size_t)i * h + k]));
            if (x > mx)
                mx = x;
        }
        int64_t acc = 0;
        double hi = 0.0;
        for (int k = 0; k < h; k++) {
            double x = oracle_f16_to_double(X[(size_t)i * h + k]);
            double w = oracle_f16_to_double(W[(size_t)k * o + j]);
            if (is_out[k])
                hi += x * w;
            else
                acc += (int64_t)oracle_q(x, mx) * (int64_t)oracle_q(w, mw);
        }
        C_out[p] = (int32_t)acc;
        Out_out[p] = oracle_double_to_f16((double)acc * mx * mw / 16129.0 + hi);
    }
    free(is_out);
}

/* oracle_sampled at a coarser granularity (1 or 2; 0 is oracle_sampled itself):
 * the shared constants are found once over the whole tensors, then every pair
 * is computed from the definition as above.                                   */
void oracle_sampled_granular(const uint16_t *X, const uint16_t *W, int s, int h, int o, const int32_t *idx,
                             int count, int granularity, const int32_t *rows, const int32_t *cols, int n,
                             int32_t *C_out, uint16_t *Out_out)
{
    uint8_t *is_out = (uint8_t *)calloc((size_t)h, 1);
    for (int t = 0; t < count; t++)
        is_out[idx[t]] = 1;
    double gw = 0.0, gx = 0.0;
    for (size_t q = 0; q < (size_t)h * o; q++) {
        double a = fabs(oracle_f16_to_double(W[q]));
        if (a > gw)
            gw = a;
    }
    for (int i = 0; i < s; i++)
        for (int k = 0; k < h; k++) {
            if (is_out[k])
                continue;
            double a = fabs(oracle_f16_to_double(X[(size_t)i * h + k]));
            if (a > gx)
                gx = a;
        }
#pragma omp parallel for schedule(dynamic, 1)
    for (int p = 0; p < n; p++) {
        int i = rows[p], j = cols[p];
        double mx = gx, mw = gw;
        if (granularity == 1) { /* row-wise: the row of X keeps its own constant */
            mx = 0.0;
            for (int k = 0; k < h; k++) {
                if (is_out[k])
                    continue;
                double x = fabs(oracle_f16_to_double(X[(size_t)i * h + k]));
                if (x > mx)
                    mx = x;
            }
        }
        int64_t acc = 0;
        double hi = 0.0;
        for (int k = 0; k < h; k++) {
            double x = oracle_f16_to_double(X[(size_t)i * h + k]);
            double w = oracle_f16_to_double(W[(size_t)k * o + j]);
            if (is_out[k])
                hi += x * w;
            else
                acc += (int64_t)oracle_q(x, mx) * (int64_t)oracle_q(w, mw);
        }
        C_out[p] = (int32_t)acc;
        Out_out[p] = oracle_double_to_f16((double)acc * mx * mw / 16129.0 + hi);
    }
    free(is_out);
}

/* ---- zeropoint quantization (Section 2.1, Eq. 1-5), vector-wise ------------ */

/* Asymmetric quantization of one vector v (a row of X without its outlier
 * columns, or a column of W) with lo = min v, hi = max v, D = hi - lo:
 *   Eq. 1  nd = 2 * 127 / D             (kept exact: the quotient is never rounded on its own)
 *   Eq. 3  u(x) = nearest integer to nd * x, ties to even
 *   Eq. 2  zp = u(lo) + 127             (the paper prints "X * min" where nd * min is meant; the
 *                                        127 recentres the stored byte into [-127, 127], the range
 *                                        the text names, instead of [0, 254])
 *   stored code = u(x) - zp in [-127, 127]; Eq. 4 adds zp back: code + zp = u(x).
 * D == 0 (a constant vector): codes 0, zp 0, and the vector counts as all zero.
 * lo and hi are exact fp16 values and travel as bit patterns (a zero as +0).
 *
 * 254 * x is exact in double, D = hi - lo is exact in double (at most 41
 * significant bits), the division is correctly rounded, and a quotient that is
 * not a tie lies at least 2^-50 (relative) from the nearest half-integer, so
 * nearbyint() of the double quotient is the exact answer.                     */
long long oracle_zp_u(double x, double D)
{
    if (D == 0.0)
        return 0;
    return llrint(254.0 * x / D);
}

static void zp_range(const uint16_t *v, size_t stride, int n, const uint8_t *skip, uint16_t *lo, uint16_t *hi)
{
    double mn = 0.0, mx = 0.0;
    uint16_t mnb = 0, mxb = 0;
    int first = 1;
    for (int q = 0; q < n; q++) {
        if (skip && skip[q])
            continue;
        uint16_t b = v[(size_t)q * stride];
        double x = oracle_f16_to_double(b);
        if (x == 0.0)
            b = 0;
        if (first || x < mn) {
            mn = x;
            mnb = b;
        }
        if (first || x > mx) {
            mx = x;
            mxb = b;
        }
        first = 0;
    }
    *lo = mnb;
    *hi = mxb;
}

/* columns of W: codes, range, zeropoint and the column sums of the codes over all h rows */
void oracle_zp_quantize_weight(const uint16_t *W, int h, int o, int8_t *Wq, uint16_t *lo, uint16_t *hi,
                               int32_t *zp, int32_t *colsum)
{
#pragma omp parallel for schedule(static)
    for (int j = 0; j < o; j++) {
        zp_range(W + j, (size_t)o, h, NULL, &lo[j], &hi[j]);
        double l = oracle_f16_to_double(lo[j]), D = oracle_f16_to_double(hi[j]) - l;
        long long z = D == 0.0 ? 0 : oracle_zp_u(l, D) + 127;
        long long sum = 0;
        for (int k = 0; k < h; k++) {
            long long c = D == 0.0 ? 0 : oracle_zp_u(oracle_f16_to_double(W[(size_t)k * o + j]), D) - z;
            Wq[(size_t)k * o + j] = (int8_t)c;
            sum += c;
        }
        zp[j] = (int32_t)z;
        colsum[j] = (int32_t)sum;
    }
}

/* rows of X over the non-outlier columns; code 0 in the outlier columns; row sums of the codes */
void oracle_zp_quantize_rows(const uint16_t *X, int s, int h, const int32_t *idx, int count, int8_t *Xq,
                             uint16_t *lo, uint16_t *hi, int32_t *zp, int32_t *rowsum)
{
    uint8_t *is_out = (uint8_t *)calloc((size_t)h, 1);
    for (int t = 0; t < count; t++)
        is_out[idx[t]] = 1;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < s; i++) {
        zp_range(X + (size_t)i * h, 1, h, is_out, &lo[i], &hi[i]);
        double l = oracle_f16_to_double(lo[i]), D = oracle_f16_to_double(hi[i]) - l;
        long long z = D == 0.0 ? 0 : oracle_zp_u(l, D) + 127;
        long long sum = 0;
        for (int j = 0; j < h; j++) {
            long long c = 0;
            if (!is_out[j] && D != 0.0)
                c = oracle_zp_u(oracle_f16_to_double(X[(size_t)i * h + j]), D) - z;
            Xq[(size_t)i * h + j] = (int8_t)c;
            sum += c;
        }
        zp[i] = (int32_t)z;
        rowsum[i] = (int32_t)sum;
    }
    free(is_out);
}

/* Eq. 4 over the non-outlier features: T[i][j] = sum_{k not in O} (A[i][k] + za[i]) (B[k][j] + zb[j]).
 * 64-bit sums: with zeropoints far from 0 the terms do not fit 32 bits.       */
void oracle_zp_gemm(const int8_t *Xq, const int32_t *za, const int8_t *Wq, const int32_t *zb, const int32_t *idx,
                    int count, int s, int h, int o, int64_t *T)
{
    uint8_t *is_out = (uint8_t *)calloc((size_t)h, 1);
    for (int t = 0; t < count; t++)
        is_out[idx[t]] = 1;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < s; i++) {
        int64_t *acc = (int64_t *)calloc((size_t)o, sizeof(int64_t));
        for (int k = 0; k < h; k++) {
            if (is_out[k])
                continue;
            int64_t a = (int64_t)Xq[(size_t)i * h + k] + za[i];
            for (int j = 0; j < o; j++)
                acc[j] += a * ((int64_t)Wq[(size_t)k * o + j] + zb[j]);
        }
        memcpy(T + (size_t)i * o, acc, (size_t)o * sizeof(int64_t));
        free(acc);
    }
    free(is_out);
}

/* Dequantization (division by nd_a nd_b, i.e. multiplication by D_a D_b / 254^2) plus the 16-bit
 * outlier product of Eq. 8                                                    */
void oracle_zp_output(const int64_t *T, const uint16_t *loa, const uint16_t *hia, const uint16_t *lob,
                      const uint16_t *hib, const uint16_t *X, const uint16_t *W, const int32_t *idx, int count,
                      int s, int h, int o, uint16_t *Out)
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < s; i++) {
        double *acc = (double *)calloc((size_t)o, sizeof(double));
        for (int t = 0; t < count; t++) {
            int k = idx[t];
            double x = oracle_f16_to_double(X[(size_t)i * h + k]);
            for (int j = 0; j < o; j++)
                acc[j] += x * oracle_f16_to_double(W[(size_t)k * o + j]);
        }
        double Da = oracle_f16_to_double(hia[i]) - oracle_f16_to_double(loa[i]);
        for (int j = 0; j < o; j++) {
            double Db = oracle_f16_to_double(hib[j]) - oracle_f16_to_double(lob[j]);
            double d = (double)T[(size_t)i * o + j] * Da * Db / 64516.0;
            Out[(size_t)i * o + j] = oracle_double_to_f16(d + acc[j]);
        }
        free(acc);
    }
}

/* The whole call with zeropoint quantization in place of absmax.  C receives the plain int8
 * product sum_k A B of Eq. 5 (what the matrix unit computes), T the full sum of Eq. 4.
 * Returns |O|, -1 if C leaves int32, -2 for non-finite input.                 */
int oracle_zp_linear(const uint16_t *X, const uint16_t *W, int s, int h, int o, double alpha, int32_t *idx,
                     int8_t *Xq, uint16_t *loa, uint16_t *hia, int32_t *za, int32_t *rowsum, int8_t *Wq,
                     uint16_t *lob, uint16_t *hib, int32_t *zb, int32_t *colsum, int32_t *C, int64_t *T,
                     uint16_t *Out)
{
    for (size_t n = 0; n < (size_t)s * h; n++)
        if ((X[n] & 0x7c00u) == 0x7c00u)
            return -2;
    for (size_t n = 0; n < (size_t)h * o; n++)
        if ((W[n] & 0x7c00u) == 0x7c00u)
            return -2;
    int count = oracle_find_outliers(X, s, h, alpha, idx, h);
    oracle_zp_quantize_weight(W, h, o, Wq, lob, hib, zb, colsum);
    oracle_zp_quantize_rows(X, s, h, idx, count, Xq, loa, hia, za, rowsum);
    if (oracle_igemm(Xq, Wq, s, h, o, C))
        return -1;
    oracle_zp_gemm(Xq, za, Wq, zb, idx, count, s, h, o, T);
    oracle_zp_output(T, loa, hia, lob, hib, X, W, idx, count, s, h, o, Out);
    return count;
}

/* single outputs of a large problem, each from the definition (as oracle_sampled) */
void oracle_zp_sampled(const uint16_t *X, const uint16_t *W, int s, int h, int o, const int32_t *idx, int count,
                       const int32_t *rows, const int32_t *cols, int n, int32_t *C_out, uint16_t *Out_out)
{
    (void)s;
    uint8_t *is_out = (uint8_t *)calloc((size_t)h, 1);
    for (int t = 0; t < count; t++)
        is_out[idx[t]] = 1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int p = 0; p < n; p++) {
        int i = rows[p], j = cols[p];
        uint16_t la, ha, lb, hb;
        zp_range(X + (size_t)i * h, 1, h, is_out, &la, &ha);
        zp_range(W + j, (size_t)o, h, NULL, &lb, &hb);
        double l_a = oracle_f16_to_double(la), Da = oracle_f16_to_double(ha) - l_a;
        double l_b = oracle_f16_to_double(lb), Db = oracle_f16_to_double(hb) - l_b;
        long long za = Da == 0.0 ? 0 : oracle_zp_u(l_a, Da) + 127;
        long long zb = Db == 0.0 ? 0 : oracle_zp_u(l_b, Db) + 127;
        int64_t acc = 0, T = 0;
        double hi = 0.0;
        for (int k = 0; k < h; k++) {
            double x = oracle_f16_to_double(X[(size_t)i * h + k]);
            double w = oracle_f16_to_double(W[(size_t)k * o + j]);
            if (is_out[k]) {
                hi += x * w;
                continue;
            }
            long long a = Da == 0.0 ? 0 : oracle_zp_u(x, Da) - za;
            long long b = Db == 0.0 ? 0 : oracle_zp_u(w, Db) - zb;
            acc += a * b;
            T += (a + za) * (b + zb);
        }
        C_out[p] = (int32_t)acc;
        Out_out[p] = oracle_double_to_f16((double)T * Da * Db / 64516.0 + hi);
    }
    free(is_out);
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    omp_set_num_threads(n);
#else
    (void)n;
#endif
}
