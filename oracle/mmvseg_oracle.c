/*
 * CPU oracle for segmented inclusive scan, segmented sum and COO SpMV.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, sequential, obviously
 * correct statement of what the GPU library must compute.  It shares no code,
 * header, table or helper with the HIP path and is never linked into it.
 * Only the test-suite, the smoke check and the benchmark's cpu_baseline leg
 * may call it.
 *
 * What it follows:
 *  - segmented inclusive scan: the recurrence of Problem 2.1 (Sec. 2,
 *    "Segmented Scan"): z(i) = x(i) if i == 0 or f(i) == 1, else
 *    z(i-1) + x(i).
 *  - segmented sum: Sec. 2, the last element of every segment of the segmented
 *    scan, in segment order (worked example: x=(2,2,3,3,1,3,1,2),
 *    f=(1,0,1,0,0,1,0,0) -> scan (2,4,3,6,7,3,4,6), sum (4,7,6)).
 *  - SpMV: y = A x (Theorem "SpMV", Sec. 4.3), written as the plain
 *    accumulation over the coordinate triples; rows without entries stay 0
 *    (appendix "SpMV implementation").
 *
 * Readings taken where the paper is silent:
 *  - position 0 always opens a segment, whatever f(0) holds;
 *  - int8 inputs accumulate in 32-bit two's complement with wrap-around
 *    (Z/2^32 is a group, as Sec. 2 requires); the add is done on uint32_t so
 *    that the C arithmetic has no undefined behaviour;
 *  - floating-point inputs are widened exactly to double and accumulated in
 *    double; results are returned as double (never rounded to fp32).
 *
 * No blocking, no reordering, one thread.
 */
#include <stddef.h>
#include <stdint.h>

/* ---- int8 -> int32 ------------------------------------------------------ */

/* z[i] for all i; flags: one byte per element, non-zero = segment start. */
void oracle_segscan_i8(const int8_t *x, const uint8_t *f, uint64_t n, int32_t *z)
{
    uint32_t acc = 0;
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t xi = (uint32_t)(int32_t)x[i];
        if (i == 0 || f[i])
            acc = xi;
        else
            acc = acc + xi;
        z[i] = (int32_t)acc;
    }
}

/* out[k] = sum of segment k; returns the number of segments. */
uint64_t oracle_segsum_i8(const int8_t *x, const uint8_t *f, uint64_t n, int32_t *out)
{
    uint32_t acc = 0;
    uint64_t k = 0;
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t xi = (uint32_t)(int32_t)x[i];
        if (i == 0 || f[i])
            acc = xi;
        else
            acc = acc + xi;
        if (i == n - 1 || f[i + 1])
            out[k++] = (int32_t)acc;
    }
    return k;
}

/* ---- floating point (values already widened exactly to double) ---------- */

void oracle_segscan_f64(const double *x, const uint8_t *f, uint64_t n, double *z)
{
    double acc = 0.0;
    for (uint64_t i = 0; i < n; ++i) {
        if (i == 0 || f[i])
            acc = x[i];
        else
            acc = acc + x[i];
        z[i] = acc;
    }
}

uint64_t oracle_segsum_f64(const double *x, const uint8_t *f, uint64_t n, double *out)
{
    double acc = 0.0;
    uint64_t k = 0;
    for (uint64_t i = 0; i < n; ++i) {
        if (i == 0 || f[i])
            acc = x[i];
        else
            acc = acc + x[i];
        if (i == n - 1 || f[i + 1])
            out[k++] = acc;
    }
    return k;
}

/* Same recurrence reading fp32 input directly (widening float->double is
 * exact), so that very long inputs need no fp64 copy of x. */
void oracle_segscan_f32in(const float *x, const uint8_t *f, uint64_t n, double *z)
{
    double acc = 0.0;
    for (uint64_t i = 0; i < n; ++i) {
        double xi = (double)x[i];
        if (i == 0 || f[i])
            acc = xi;
        else
            acc = acc + xi;
        z[i] = acc;
    }
}

/* ---- COO SpMV ------------------------------------------------------------ */

/* y[0..n_rows) = A x with A given as nnz (row, col, val) triples in any order.
 * The product of two fp32 numbers is exact in double.  Returns 0, or 1 if an
 * index is out of range (nothing is written for that triple). */
int oracle_spmv_coo(uint64_t n_rows, uint64_t n_cols, uint64_t nnz,
                    const int32_t *row, const int32_t *col, const float *val,
                    const float *x, double *y)
{
    int bad = 0;
    for (uint64_t r = 0; r < n_rows; ++r)
        y[r] = 0.0;
    for (uint64_t k = 0; k < nnz; ++k) {
        int64_t r = row[k], c = col[k];
        if (r < 0 || (uint64_t)r >= n_rows || c < 0 || (uint64_t)c >= n_cols) {
            bad = 1;
            continue;
        }
        y[r] += (double)val[k] * (double)x[c];
    }
    return bad;
}
