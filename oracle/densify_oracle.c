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
 * for the byte-count formulas.
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
