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
 *    accumulation over the coordinate triples (COO) or over the entries of
 *    each row (CSR, Algorithm "MMV-RAM CSR SpMV"); rows without entries stay 0
 *    (appendix "SpMV implementation").
 *  - the parallel primitives that Algorithms SCD and SSCR (Sec. 4.1) are
 *    composed of, each as its plain definition: SCAN z(i) = sum of x(j), j <= i
 *    (Sec. 1.1, Notation); COMPRESS = the entries of x whose mask entry is 1,
 *    in order (Sec. 2; example COMPRESS((2,2,3,3,1,3,1,2), (1,0,1,0,0,1,0,0))
 *    = (2,3,3)); DIFF z(i) = x(i) - x(i-1) with x(-1) = 0 (Sec. 4.1); REVERT
 *    (Sec. 4.1) subtracts from every element the speculative scan value at the
 *    last position of the previous segment.
 *
 *  - the same segmented scan / sum over another group, bytes under bit-wise
 *    exclusive or (Sec. 2 states the problem for any group).
 *
 * Readings taken where the paper is silent:
 *  - position 0 always opens a segment, whatever f(0) holds;
 *  - int8 inputs accumulate in 32-bit two's complement with wrap-around
 *    (Z/2^32 is a group, as Sec. 2 requires); the add is done on uint32_t so
 *    that the C arithmetic has no undefined behaviour;
 *  - floating-point inputs are widened exactly to double and accumulated in
 *    double; results are returned as double (never rounded to fp32);
 *  - REVERT as printed compares the inclusive flag count with idx + 1 for idx
 *    from 0, which would subtract w(0) from the first segment of the paper's
 *    own worked example; here an element whose inclusive flag count (with
 *    position 0 counted as a segment start) is k >= 2 gets w(k - 2) subtracted
 *    and k == 1 is left alone.
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

/* ---- another group: bytes under bit-wise exclusive or ---------------------- */

/* Problem 2.1 asks only for a group (Sec. 2): here ((Z_2)^8, xor).  The same
 * recurrence with xor for +; the result byte in the low bits of a 32-bit word. */
void oracle_segscan_xor_u8(const uint8_t *x, const uint8_t *f, uint64_t n, uint32_t *z)
{
    uint32_t acc = 0;
    for (uint64_t i = 0; i < n; ++i) {
        if (i == 0 || f[i])
            acc = x[i];
        else
            acc = acc ^ x[i];
        z[i] = acc;
    }
}

uint64_t oracle_segsum_xor_u8(const uint8_t *x, const uint8_t *f, uint64_t n, uint32_t *out)
{
    uint32_t acc = 0;
    uint64_t k = 0;
    for (uint64_t i = 0; i < n; ++i) {
        if (i == 0 || f[i])
            acc = x[i];
        else
            acc = acc ^ x[i];
        if (i == n - 1 || f[i + 1])
            out[k++] = acc;
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

/* ---- parallel primitives of Algorithms SCD and SSCR (Sec. 4.1) ------------- */

/* SCAN: z(i) = x(0) + ... + x(i), int8 in, int32 out with wrap-around. */
void oracle_scan_i8(const int8_t *x, uint64_t n, int32_t *z)
{
    uint32_t acc = 0;
    for (uint64_t i = 0; i < n; ++i) {
        acc = acc + (uint32_t)(int32_t)x[i];
        z[i] = (int32_t)acc;
    }
}

/* SCAN of fp32 input accumulated in double. */
void oracle_scan_f32in(const float *x, uint64_t n, double *z)
{
    double acc = 0.0;
    for (uint64_t i = 0; i < n; ++i) {
        acc = acc + (double)x[i];
        z[i] = acc;
    }
}

void oracle_scan_f64(const double *x, uint64_t n, double *z)
{
    double acc = 0.0;
    for (uint64_t i = 0; i < n; ++i) {
        acc = acc + x[i];
        z[i] = acc;
    }
}

/* COMPRESS: the 32-bit entries of x whose mask byte is non-zero, in order.
 * Returns how many there are. */
uint64_t oracle_compress_u32(const uint32_t *x, const uint8_t *m, uint64_t n, uint32_t *out)
{
    uint64_t k = 0;
    for (uint64_t i = 0; i < n; ++i)
        if (m[i])
            out[k++] = x[i];
    return k;
}

/* DIFF on int32 with wrap-around: z(i) = x(i) - x(i-1), x(-1) = 0. */
void oracle_diff_i32(const int32_t *x, uint64_t n, int32_t *z)
{
    uint32_t prev = 0;
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t cur = (uint32_t)x[i];
        z[i] = (int32_t)(cur - prev);
        prev = cur;
    }
}

/* DIFF on fp32 input, exact in double (the difference of two floats is
 * representable in double unless their exponents differ by more than 29;
 * it is rounded once in that case). */
void oracle_diff_f32in(const float *x, uint64_t n, double *z)
{
    double prev = 0.0;
    for (uint64_t i = 0; i < n; ++i) {
        double cur = (double)x[i];
        z[i] = cur - prev;
        prev = cur;
    }
}

/* REVERT on int32 with wrap-around.  xhat = SCAN(x), fhat = inclusive count of
 * segment starts up to and including i (position 0 counted), w = the values of
 * xhat at the segment ends, one per segment.  Returns 1 if a count points
 * outside w (nothing subtracted there), else 0. */
int oracle_revert_i32(const int32_t *xhat, const int32_t *fhat, const int32_t *w, uint64_t n,
                      uint64_t nw, int32_t *z)
{
    int bad = 0;
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t v = (uint32_t)xhat[i];
        int64_t k = fhat[i];
        if (k >= 2) {
            if ((uint64_t)(k - 2) < nw)
                v = v - (uint32_t)w[k - 2];
            else
                bad = 1;
        }
        z[i] = (int32_t)v;
    }
    return bad;
}

/* REVERT on fp32 inputs, subtraction in double. */
int oracle_revert_f32in(const float *xhat, const int32_t *fhat, const float *w, uint64_t n,
                        uint64_t nw, double *z)
{
    int bad = 0;
    for (uint64_t i = 0; i < n; ++i) {
        double v = (double)xhat[i];
        int64_t k = fhat[i];
        if (k >= 2) {
            if ((uint64_t)(k - 2) < nw)
                v = v - (double)w[k - 2];
            else
                bad = 1;
        }
        z[i] = v;
    }
    return bad;
}

/* ---- CSR SpMV --------------------------------------------------------------- */

/* y(r) = sum over k in [rowptr(r), rowptr(r+1)) of val(k) * x(col(k)); rowptr has
 * n_rows + 1 non-decreasing entries, rowptr(0) = 0.  Returns 0, or 1 if the
 * row pointers are not monotone or an index is out of range (that entry is
 * skipped). */
int oracle_spmv_csr(uint64_t n_rows, uint64_t n_cols, const int32_t *rowptr, const int32_t *col,
                    const float *val, const float *x, double *y)
{
    int bad = 0;
    for (uint64_t r = 0; r < n_rows; ++r) {
        double acc = 0.0;
        if (rowptr[r + 1] < rowptr[r] || rowptr[r] < 0)
            bad = 1;
        for (int64_t k = rowptr[r]; k < rowptr[r + 1]; ++k) {
            int64_t c = col[k];
            if (c < 0 || (uint64_t)c >= n_cols) {
                bad = 1;
                continue;
            }
            acc += (double)val[k] * (double)x[c];
        }
        y[r] = acc;
    }
    return bad;
}
