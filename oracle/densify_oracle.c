/*
 * CPU checker for "densify an assumed-sparse gradient and sum it with the dense one".
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition that the GPU
 * library is compared against.  Nothing in the product path may call it; it shares
 * no code, header, table or helper with the GPU sources.
 *
 * What it computes (the paper, Section 4, Listing 1: an IndexedSlices gradient is
 * converted to a dense tensor; Section 6, Algorithm 2, the added branch: every
 * gradient is converted to a dense tensor and the dense tensors are summed):
 *
 *   acc[V][d] = 0
 *   for each (id, row) pair, in input order:   acc[id][:] += row[:]
 *   out = acc + dense_in                        (dense_in absent: out = acc)
 *
 * Repeated ids add up: the gradient of a gather has one slice per looked-up
 * token (Section 3), and turning it into a dense tensor is a scatter-add.
 *
 * Precision: the paper fixes none.  Sums are kept in float64 and rounded to fp32
 * once, so this result is (to ~1e-16 relative) the exact one, and a tolerance on
 * the GPU's fp32 result is measured against the truth rather than against another
 * fp32 summation order.  abs[v][c] collects the sum of |terms| of each element,
 * the scale of the stated tolerance.
 *
 * Readings where the paper is silent:
 *   - ids outside [0, V) are skipped and counted (n_bad), never dereferenced;
 *   - rows that receive no pair are copied from dense_in bit for bit (so -0.0 and
 *     NaN payloads survive), or are +0.0 when dense_in is absent;
 *   - bf16 value rows are widened exactly (16-bit shift) before they are added.
 *
 * Pins (tests/test_oracle_pins.py): hand-worked cases under tests/golden/,
 * brute-force triple loop on tiny inputs, numpy.add.at and torch.index_add_ in
 * float64, column-sum / untouched-row / permutation invariants, exact results for
 * all-distinct ids and for small-integer data, exact power-of-two scaling,
 * decomposition into two calls, and the paper's 11.4 GB / 139 MB / 82x figures
 * for the byte-count formulas.  The scaled / bf16 finish: torch's CPU float32 ->
 * bfloat16 conversion, hand-worked ties and a double-rounding case, exact scaling by
 * powers of two, the average of k equal contributions, small-integer data.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_ROW_FP32 = 0, ORACLE_ROW_BF16 = 1 };

static double widen(const void* rows, int row_dtype, int64_t index)
{
    if (row_dtype == ORACLE_ROW_BF16) {
        uint32_t bits = (uint32_t)((const uint16_t*)rows)[index] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    return (double)((const float*)rows)[index];
}

/*
 * Adds one contribution (n pairs) into acc / abs_sum / count, in input order.
 * Calling it once per shard, shard after shard, is the definition of the
 * multi-shard result: the concatenation of the shards in shard order.
 * abs_sum may be NULL (then it is not maintained).
 */
void oracle_accumulate(const int32_t* ids, const void* rows, int64_t n, int32_t d, int32_t V,
                       int32_t row_dtype, double* acc, double* abs_sum, int32_t* count,
                       int64_t* n_bad)
{
    for (int64_t t = 0; t < n; ++t) {
        int32_t v = ids[t];
        if (v < 0 || v >= V) {
            *n_bad += 1;
            continue;
        }
        count[v] += 1;
        double* a = acc + (int64_t)v * d;
        double* s = abs_sum ? abs_sum + (int64_t)v * d : NULL;
        for (int32_t c = 0; c < d; ++c) {
            double x = widen(rows, row_dtype, t * (int64_t)d + c);
            a[c] += x;
            if (s) s[c] += fabs(x);
        }
    }
}

/*
 * out = acc + dense_in, rounded once to fp32 (round to nearest even, the C
 * double -> float conversion).  Rows with count 0 are bit copies of dense_in.
 * exact (may be NULL) receives the unrounded float64 value; abs_sum (may be
 * NULL) additionally receives |dense_in| for rows that were summed.
 */
void oracle_finish(const double* acc, double* abs_sum, const int32_t* count, const float* dense_in,
                   int32_t d, int32_t V, float* out, double* exact)
{
    for (int32_t v = 0; v < V; ++v) {
        for (int32_t c = 0; c < d; ++c) {
            int64_t i = (int64_t)v * d + c;
            if (count[v] == 0) {
                if (dense_in)
                    memcpy(&out[i], &dense_in[i], sizeof(float));
                else
                    out[i] = 0.0f;
                if (exact) exact[i] = (double)out[i];
                if (abs_sum) abs_sum[i] = dense_in ? fabs((double)dense_in[i]) : 0.0;
            } else {
                double e = acc[i] + (dense_in ? (double)dense_in[i] : 0.0);
                out[i] = (float)e;
                if (exact) exact[i] = e;
                if (abs_sum && dense_in) abs_sum[i] += fabs((double)dense_in[i]);
            }
        }
    }
}

/*
 * Rounds a real number to bf16 (1 sign, 8 exponent, 7 fraction bits: the upper half of
 * an fp32), nearest with ties to even, in ONE step from the float64 value: the multiple
 * of the format's spacing at that magnitude that lies nearest.  Below 2^-126 the spacing
 * stays 2^-133 (subnormals); 2^128 and beyond is infinity.
 */
uint16_t oracle_bf16_from_double(double e)
{
    if (isnan(e)) return 0x7FC0;
    uint16_t sign = signbit(e) ? 0x8000 : 0;
    double a = fabs(e);
    if (a == 0.0) return sign;
    if (isinf(a)) return (uint16_t)(sign | 0x7F80);
    int ex;
    (void)frexp(a, &ex);                    /* a = m * 2^ex with 0.5 <= m < 1 */
    int eq = ex - 8;                        /* spacing 2^eq leaves 8 significant bits */
    if (eq < -133) eq = -133;
    double q = nearbyint(ldexp(a, -eq));    /* default rounding mode: ties to even; 0 <= q <= 256 */
    if (q == 256.0) {
        q = 128.0;
        eq += 1;
    }
    if (q < 128.0) return (uint16_t)(sign | (uint16_t)q);     /* subnormal or zero (only when eq == -133) */
    int field = eq + 7 + 127;               /* value = (q / 128) * 2^(eq + 7) */
    if (field >= 255) return (uint16_t)(sign | 0x7F80);
    return (uint16_t)(sign | (field << 7) | ((int)q - 128));
}

void oracle_bf16_from_double_array(const double* x, int64_t n, uint16_t* out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = oracle_bf16_from_double(x[i]);
}

enum { ORACLE_OUT_FP32 = 0, ORACLE_OUT_BF16 = 1 };

/*
 * The finish step with a write-back epilogue (a reduction buffer that wants the average
 * instead of the sum, or a 16-bit copy of it: Section 4 hands the converted gradient to a
 * dense reduction; Section 1 mentions reduced precision):
 *
 *   rows that received pairs:  e = (acc + dense_in) * scale in float64, rounded ONCE to
 *                              the output type (fp32: C conversion; bf16: the function
 *                              above);
 *   other rows:                y = scale * dense_in as an fp32 product (the float64
 *                              product of two fp32 numbers is exact, so converting it to
 *                              float is the correctly rounded product); fp32 output is y
 *                              (a bit copy of dense_in when scale == 1), bf16 output is
 *                              y rounded to bf16.
 * exact receives the unrounded value, abs_sum the sum of |terms| times |scale|.
 * Exactly one of out_f32 / out_bf16 is used, according to out_dtype.
 */
void oracle_finish_scaled(const double* acc, double* abs_sum, const int32_t* count, const float* dense_in,
                          int32_t d, int32_t V, float scale, int32_t out_dtype, float* out_f32,
                          uint16_t* out_bf16, double* exact)
{
    const double sc = (double)scale;
    for (int32_t v = 0; v < V; ++v) {
        for (int32_t c = 0; c < d; ++c) {
            int64_t i = (int64_t)v * d + c;
            double x = dense_in ? (double)dense_in[i] : 0.0;
            if (count[v] == 0) {
                float y = (float)(sc * x);
                if (out_dtype == ORACLE_OUT_BF16) {
                    out_bf16[i] = oracle_bf16_from_double((double)y);
                } else if (scale == 1.0f && dense_in) {
                    memcpy(&out_f32[i], &dense_in[i], sizeof(float));
                } else {
                    out_f32[i] = y;
                }
                if (exact) exact[i] = sc * x;
                if (abs_sum) abs_sum[i] = fabs(sc * x);
            } else {
                double e = (acc[i] + x) * sc;
                if (out_dtype == ORACLE_OUT_BF16)
                    out_bf16[i] = oracle_bf16_from_double(e);
                else
                    out_f32[i] = (float)e;
                if (exact) exact[i] = e;
                if (abs_sum) abs_sum[i] = (abs_sum[i] + fabs(x)) * fabs(sc);
            }
        }
    }
}

/*
 * The whole definition in one call, with its own zeroed float64 array: this is
 * the form that is timed as the CPU baseline.  Returns 0, or -1 when the
 * accumulator cannot be allocated.  count must hold V zeros on entry.
 */
int oracle_densify(const int32_t* ids, const void* rows, int64_t n, int32_t d, int32_t V,
                   int32_t row_dtype, const float* dense_in, float* out, int32_t* count,
                   int64_t* n_bad)
{
    double* acc = (double*)calloc((size_t)V * (size_t)d, sizeof(double));
    if (!acc) return -1;
    oracle_accumulate(ids, rows, n, d, V, row_dtype, acc, NULL, count, n_bad);
    oracle_finish(acc, NULL, count, dense_in, d, V, out, NULL);
    free(acc);
    return 0;
}

/* Ascending list of the ids that received at least one pair; returns how many. */
int32_t oracle_unique_ids(const int32_t* count, int32_t V, int32_t* unique_out)
{
    int32_t m = 0;
    for (int32_t v = 0; v < V; ++v)
        if (count[v] > 0) unique_out[m++] = v;
    return m;
}

/*
 * Bytes of the two accumulate buffers the paper compares (Section 4, Fig. 5a):
 * a gather concatenates every one of k workers' N (id, row) pairs, an int32 id
 * plus d values each; a reduce moves one dense [V, d] fp32 tensor whatever k is.
 */
void oracle_buffer_bytes(int64_t k, int64_t N, int32_t d, int32_t V, int32_t row_dtype,
                         int64_t* gathered, int64_t* dense)
{
    int64_t elem = (row_dtype == ORACLE_ROW_BF16) ? 2 : 4;
    *gathered = k * N * (4 + elem * (int64_t)d);
    *dense = 4 * (int64_t)V * (int64_t)d;
}
