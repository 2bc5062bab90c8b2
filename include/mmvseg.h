/*
 * libmmvseg - segmented inclusive scan, segmented sum and COO SpMV on AMD
 * MI355X (gfx950), computed as small matrix products (tile times triangular
 * all-ones matrix) on the matrix cores plus vector masking and carry steps,
 * after "Segmented Operations using Matrix Multiplications" (MMV-RAM).
 *
 * Conventions shared by every call
 * --------------------------------
 *  - Every pointer whose name starts with d_ is DEVICE memory owned by the
 *    caller.  The library allocates nothing, on the device or on the host, and
 *    what it keeps between calls is fixed in size and holds no result: per kernel
 *    one word per device (how many of its workgroups the device holds at once,
 *    asked from the runtime on first use), the device address of the array behind
 *    mmv_segscan_static, and the per-thread timing events of mmv_set_kernel_events.
 *  - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL =
 *    the default stream).  Calls return as soon as the kernels are enqueued;
 *    results are valid once the caller has synchronised that stream.
 *  - `d_ws` is scratch of at least mmv_workspace_bytes(...) bytes, 256-byte
 *    aligned.  The library resets what it needs on every call (inside the
 *    stream, by a small fill kernel); contents are undefined afterwards, except
 *    for the status word read by mmv_workspace_status() and for the plan that
 *    mmv_spmv_coo_prepare / mmv_spmv_csr_prepare leave for their _run calls.
 *    Two calls that share a workspace must not overlap in time.
 *  - Value, flag, index and output pointers must be 16-byte aligned.  Inputs are read
 *    in aligned 16-byte blocks: the block that holds the last element is read whole
 *    (up to 15 bytes beyond the last element, never beyond that block) and the
 *    surplus is ignored.
 *  - Errors are returned as mmv_status; nothing aborts or throws.  Argument
 *    errors are detected on the host before anything is launched.
 *  - Position 0 always opens a segment, whatever its flag says (Problem 2.1 of
 *    Sec. 2 lets a segment begin at the first position or at a set flag).
 *  - n == 0 (nnz == 0) is valid: nothing is read, *d_nseg = 0, y is zero filled.
 */
#ifndef MMVSEG_H
#define MMVSEG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Enum arguments: every enum below ends in an enumerator of value 0x7fffffff that no call accepts.  It gives the
 * type the full non-negative range of an int, so that a caller who passes a number that is not one of the listed
 * values gets MMV_ERR_INVALID_ARG (or 0 from the sizing functions) instead of undefined behaviour inside the library. */
typedef enum {
    MMV_OK = 0,
    MMV_ERR_INVALID_ARG = 1, /* bad enum value, misaligned pointer, size out of range */
    MMV_ERR_NULL = 2,        /* a required pointer is NULL */
    MMV_ERR_UNSUPPORTED = 3, /* valid but not implemented combination */
    MMV_ERR_WORKSPACE = 4,   /* workspace too small or misaligned */
    MMV_ERR_HIP = 5,         /* a HIP launch failed */
    MMV_ERR_TOO_LARGE = 6,   /* mmv_segscan_static: the input needs more scratch than the built-in array holds */
    MMV_STATUS_INT_MAX = 0x7fffffff /* (not a status; see "enum arguments" below) */
} mmv_status;

/* Input element type / accumulator-and-output type (appendix "Implementation of
 * operators": fp16 in, fp32 out; int8 in, int32 out; fp32 added for SpMV). */
typedef enum {
    MMV_F32_F32 = 0,
    MMV_F16_F32 = 1,
    MMV_BF16_F32 = 2,
    MMV_I8_I32 = 3, /* 32-bit two's complement, wraps (Z/2^32 is a group, Sec. 2) */
    MMV_U8_XOR = 4  /* another group (Sec. 2 asks only for a group): bytes under bit-wise exclusive or; the
                       result byte comes in the low bits of a 32-bit word.  mmv_segscan, mmv_segsum and
                       mmv_scan only; the un-fused compositions and SpMV answer MMV_ERR_UNSUPPORTED.
                       The matrix cores only add, so MMV_VARIANT_MFMA takes the running exclusive or as the
                       parity of bit-plane sums (four products per 32x32 tile and the vector work of making
                       the planes and gathering the parities): correct, but on this chip slower than
                       MMV_VARIANT_SHUFFLE (62 % against 73 % of the HBM peak at 2^28 elements); callers that
                       only want the result should pass MMV_VARIANT_SHUFFLE for this type. */
    ,
    MMV_DTYPE_INT_MAX = 0x7fffffff
} mmv_dtype;

/* Segment-start flags f of Problem 2.1. */
typedef enum {
    MMV_FLAGS_U8 = 0,      /* one byte per element, non-zero = segment start */
    MMV_FLAGS_PACKED32 = 1 /* bit (i mod 32) of 32-bit word floor(i/32), LSB first;
                              ceil(n/32) words, bits beyond n ignored */
    ,
    MMV_FLAGS_INT_MAX = 0x7fffffff
} mmv_flag_fmt;

/* How the speculative s-block scans x-bar = MATMUL(x, U_s) (Sec. 1.1, first line
 * of BlockSegScan in the block-recursive algorithm) are computed. */
typedef enum {
    MMV_VARIANT_MFMA = 0,   /* matrix cores: tile times triangular ones matrix, s = 32 */
    MMV_VARIANT_SHUFFLE = 1, /* ablation: same rows scanned with vector adds and lane shuffles */
    MMV_VARIANT_INT_MAX = 0x7fffffff
} mmv_variant;

typedef enum {
    MMV_OP_SEGSCAN = 0,
    MMV_OP_SEGSUM = 1,
    MMV_OP_SPMV_COO = 2,
    MMV_OP_SCAN = 3,         /* mmv_scan */
    MMV_OP_COMPRESS = 4,     /* mmv_compress (dt ignored) */
    MMV_OP_SEGSUM_SCD = 5,   /* mmv_segsum_scd, sized for out_capacity = n */
    MMV_OP_SEGSCAN_SSCR = 6, /* mmv_segscan_sscr */
    MMV_OP_SPMV_CSR = 7,     /* sized by mmv_spmv_csr_workspace_bytes */
    MMV_OP_INT_MAX = 0x7fffffff
} mmv_op;

/* Element type of the 32-bit vectors that DIFF and REVERT work on. */
typedef enum { MMV_ELEM_I32 = 0 /* wraps */, MMV_ELEM_F32 = 1, MMV_ELEM_INT_MAX = 0x7fffffff } mmv_elem;

/* Bytes of scratch needed for one call.  `n` is the vector length (nnz for
 * SpMV).  Pure host function; returns 0 for invalid arguments and for
 * MMV_OP_SPMV_CSR, whose size depends on two lengths. */
size_t mmv_workspace_bytes(mmv_op op, mmv_dtype dt, mmv_flag_fmt ff, uint64_t n);
size_t mmv_spmv_csr_workspace_bytes(uint64_t n_rows, uint64_t nnz);

/* Segmented inclusive scan (Problem 2.1, Sec. 2):
 *   z(i) = x(i) if i == 0 or f(i) == 1, else z(i-1) + x(i).
 * Computed by the block-recursive scheme of Sec. 4.2 (steps 1-6): speculative
 * scans of rows of s = 32 elements as a matrix product with U_s, REVSPEC to undo
 * the mis-speculation inside a row, a segmented scan of the row aggregates
 * (registers, LDS, then decoupled look-back between workgroups instead of the
 * paper's recursion passes) and the first-segment carry update.
 *   d_x      n input values of the type `dt` names
 *   d_flags  n flags in format `ff`
 *   d_z      n outputs (fp32 or int32); may alias d_x only for MMV_F32_F32
 * Integers (and bytes under exclusive or) are exact: they form a group, as Sec. 2 requires.  Floats do not, and
 * the method subtracts two speculative prefixes of a row of 32 elements: a result is off by the rounding of that
 * row's prefix (about 32 * 2^-24 of the row's sum of |x|; the carries add one rounding per level), not by the
 * rounding of its own segment alone, so a segment of small values behind large ones in the same row of 32
 * loses relative accuracy.  With fp32 inputs a position that starts a segment receives its input bit for bit.
 * An infinity or NaN makes the rest of its own segment non-finite, as the definition does, and can in addition turn
 * later positions of the same row of 32 into NaN (Inf - Inf); positions outside that row are not affected unless
 * its own segment reaches them.  A block of 2048 positions that all start segments is copied exactly. */
mmv_status mmv_segscan(const void *d_x, const void *d_flags, uint64_t n, void *d_z,
                       mmv_dtype dt, mmv_flag_fmt ff, mmv_variant v,
                       void *d_ws, size_t ws_bytes, void *hip_stream);

/* mmv_segscan for callers that cannot allocate device memory and have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and error
 * behaviour as mmv_segscan, without d_ws / ws_bytes: the tile descriptors (and, for MMV_FLAGS_U8, the packed
 * copy of the flags) live in an array of MMV_STATIC_SCRATCH_BYTES bytes that is part of the library's device
 * code, so every GPU the library runs on holds that much memory from the first call on it until the process
 * ends.  The call allocates and frees nothing, on the device or through any library.
 *   limit   mmv_workspace_bytes(MMV_OP_SEGSCAN, dt, ff, n) <= MMV_STATIC_SCRATCH_BYTES, else
 *           MMV_ERR_TOO_LARGE is returned and nothing is launched.  With packed flags that is about 2^31
 *           fp32, 2^32 16-bit or 2^33 int8 elements; with one flag byte per element about 8 million.
 *   sharing every call on one GPU uses that GPU's one array, which keeps the last call's contents: each
 *           call clears what it needs inside its stream, and two calls that overlap in time on one GPU
 *           (two streams, two host threads) race and give undefined results.  Calls on different GPUs
 *           are independent.  A time-out of the look-back cannot be read back (there is no workspace to
 *           hand to mmv_workspace_status). */
#define MMV_STATIC_SCRATCH_BYTES (1u << 20)
mmv_status mmv_segscan_static(const void *d_x, const void *d_flags, uint64_t n, void *d_z,
                              mmv_dtype dt, mmv_flag_fmt ff, mmv_variant v, void *hip_stream);

/* Segmented sum (Sec. 2): the last element of every segment of the segmented
 * scan, in segment order; equals Algorithm SCD (Sec. 4.1) with the compress
 * step fused (output index = number of segment ends before the element).
 *   d_out         room for `out_capacity` sums (fp32 or int32)
 *   d_nseg        device uint64: receives the true number of segments,
 *                 1 + #{i >= 1 : f(i) = 1} for n >= 1
 * Floating point: as for mmv_segscan (a sum is off by the rounding of the prefixes of the rows of 32 it starts
 * and ends in; a non-finite value can reach the sums of the segments that share its row of 32).  16-bit inputs
 * on vectors longer than one round of workgroups (either variant) speculate over chunks of 2048 elements
 * (2048-aligned): there a sum is the difference of two prefixes of its chunk and is off by their rounding
 * (2^-24 of the chunk's running sum each), and a non-finite value reaches the other sums of its chunk.
 * Sums with index >= out_capacity are not written (d_nseg still holds the true
 * count); pass out_capacity = n to be safe.  The number of segments must be
 * below 2^32 (counts are carried in 32 bits).
 * Speed on long vectors (n = 2^28, 0.1 % of the flags set, % of the HBM peak): 8- and 16-bit inputs are fastest
 * with MMV_VARIANT_MFMA (bytes 59 % against 52 %, fp16 69 % against 60 %: the same kernel, its 32x32 tiles scanned
 * by the matrix cores or by vector instructions), fp32 inputs with MMV_VARIANT_SHUFFLE (74 % against 51 %: its
 * tiles are twice as long, which the registers of the matrix-core variant do not allow). */
mmv_status mmv_segsum(const void *d_x, const void *d_flags, uint64_t n,
                      void *d_out, uint64_t out_capacity, uint64_t *d_nseg,
                      mmv_dtype dt, mmv_flag_fmt ff, mmv_variant v,
                      void *d_ws, size_t ws_bytes, void *hip_stream);

/* y = A x for a row-sorted COO matrix through the segmented sum (Algorithm
 * "MMV-RAM CSR SpMV", Sec. 4.3: gather x by column, multiply by the values,
 * segmented sum over rows; the row indices play the part of the flags:
 * f(i) = [i == 0 or row(i) != row(i-1)]).
 *   d_row, d_col  nnz int32 indices, rows non-decreasing (otherwise the result
 *                 is undefined), 0 <= row < n_rows, 0 <= col < n_cols (not checked)
 *   d_val, d_x    fp32; d_y  n_rows fp32, fully written: rows without entries
 *                 are exactly 0 (appendix "SpMV implementation"); duplicate
 *                 (row, col) pairs add up.
 * n_rows, n_cols < 2^31. */
mmv_status mmv_spmv_coo(uint64_t n_rows, uint64_t n_cols, uint64_t nnz,
                        const int32_t *d_row, const int32_t *d_col, const float *d_val,
                        const float *d_x, float *d_y, mmv_variant v,
                        void *d_ws, size_t ws_bytes, void *hip_stream);

/* y = A x for a CSR matrix (Algorithm "MMV-RAM CSR SpMV", Sec. 4.3: the row
 * vector holds the segment start indices instead of flags), rows without
 * entries allowed (appendix "SpMV implementation").  The row pointers are turned
 * into segment-start flags over the non-zeros and into the list of rows that have
 * entries (a COMPRESS of the row indices); the sum of the k-th segment goes to
 * the k-th such row.
 *   d_rowptr  n_rows + 1 int32, non-decreasing, d_rowptr[0] = 0,
 *             d_rowptr[n_rows] = nnz (not checked; otherwise undefined)
 *   d_col, d_val, d_x, d_y  as for mmv_spmv_coo; d_y is fully written.
 * n_rows, n_cols, nnz < 2^31. */
mmv_status mmv_spmv_csr(uint64_t n_rows, uint64_t n_cols, uint64_t nnz,
                        const int32_t *d_rowptr, const int32_t *d_col, const float *d_val,
                        const float *d_x, float *d_y, mmv_variant v,
                        void *d_ws, size_t ws_bytes, void *hip_stream);

/* SpMV in two steps, for a matrix that is multiplied more than once (an iterative solver, an attention mask): what
 * depends on the matrix alone (Sec. 4.3: the segment-start flags from the row indices or row pointers; for CSR also the
 * number of segment starts per tile and the list of rows that have entries) is made once by the `_prepare` call and
 * stays in the workspace; every `_run` call then resets the tile descriptors, zeroes y and runs the product kernel
 * alone.  Arguments as for mmv_spmv_coo / mmv_spmv_csr; the results are theirs (the same kernel on the same flags;
 * as with every floating-point result of this library, the carries of rows that cross tile borders may be added in
 * another order from one run to the next, so the last bits can differ between any two calls).
 *   workspace  the same size as for the one-step call; it belongs to this matrix from `_prepare` on: any other call
 *              that uses it as its workspace destroys the plan.  `_run` calls on one workspace must not overlap in time.
 *   errors     `_run` with a workspace that `_prepare` has not prepared for a matrix of this n_rows and nnz (the
 *              library keeps a mark of both in the workspace; it cannot tell two matrices of the same shape apart)
 *              writes zeros to y and sets the status word to 2 (mmv_workspace_status); nothing is read out of bounds.
 *              The index arrays passed to `_run` must be the ones that were prepared (not checked). */
mmv_status mmv_spmv_coo_prepare(uint64_t n_rows, uint64_t n_cols, uint64_t nnz,
                                const int32_t *d_row, const int32_t *d_col,
                                void *d_ws, size_t ws_bytes, void *hip_stream);
mmv_status mmv_spmv_coo_run(uint64_t n_rows, uint64_t n_cols, uint64_t nnz,
                            const int32_t *d_row, const int32_t *d_col, const float *d_val,
                            const float *d_x, float *d_y, mmv_variant v,
                            void *d_ws, size_t ws_bytes, void *hip_stream);
mmv_status mmv_spmv_csr_prepare(uint64_t n_rows, uint64_t n_cols, uint64_t nnz,
                                const int32_t *d_rowptr, const int32_t *d_col,
                                void *d_ws, size_t ws_bytes, void *hip_stream);
mmv_status mmv_spmv_csr_run(uint64_t n_rows, uint64_t n_cols, uint64_t nnz,
                            const int32_t *d_rowptr, const int32_t *d_col, const float *d_val,
                            const float *d_x, float *d_y, mmv_variant v,
                            void *d_ws, size_t ws_bytes, void *hip_stream);

/* ---- The parallel primitives of Sec. 4.1, one call each, and the paper's
 * ---- un-fused compositions of them (for comparison with the fused calls above).

 * SCAN: unsegmented inclusive scan z(i) = x(0) + ... + x(i) (Sec. 1.1;
 * Algorithm "Scan in MMV-RAM", Sec. 4): the same single-pass kernel as
 * mmv_segscan without a flag vector.  Types and aliasing as for mmv_segscan. */
mmv_status mmv_scan(const void *d_x, uint64_t n, void *d_z, mmv_dtype dt, mmv_variant v,
                    void *d_ws, size_t ws_bytes, void *hip_stream);

/* COMPRESS (Sec. 2: keeps the entries of x at which the mask is set, in order; the worked example there:
 * COMPRESS((2,2,3,3,1,3,1,2), (1,0,1,0,0,1,0,0)) = (2,3,3)); the output position
 * of an entry is the number of selected entries before it (the scan of the mask
 * in the proof of the SCD / SSCR theorem).
 *   d_x      n 32-bit entries of any type, copied bit for bit; NULL = compress
 *            the positions 0 .. n-1 themselves (uint32)
 *   d_mask   n mask entries in format `ff` (position 0 has no special role here)
 *   d_out    room for `out_capacity` entries; entries with index >= out_capacity
 *            are not written
 *   d_count  device uint64: receives the number of selected entries, which
 *            must be below 2^32 */
mmv_status mmv_compress(const void *d_x, const void *d_mask, uint64_t n,
                        void *d_out, uint64_t out_capacity, uint64_t *d_count,
                        mmv_flag_fmt ff, void *d_ws, size_t ws_bytes, void *hip_stream);

/* DIFF (Sec. 4.1, the differentiation of a vector): z(i) = x(i) - x(i-1), x(-1) = 0.
 * d_z must not alias d_x.  No workspace. */
mmv_status mmv_diff(const void *d_x, uint64_t n, void *d_z, mmv_elem et, void *hip_stream);

/* REVERT (Sec. 4.1): undoes the speculation of an unsegmented scan,
 *   z(i) = xhat(i) - w(fhat(i) - 2)  if fhat(i) >= 2,   z(i) = xhat(i) otherwise,
 * where fhat(i) is the number of segment starts at positions 0 .. i (position 0
 * counted) and w(k) is xhat at the last position of segment k.  (The printed
 * procedure compares fhat with idx + 1; that would also subtract from the first
 * segment, so the index is read shifted by one.)  A count that points beyond
 * w(nw - 1) subtracts nothing.  d_z may alias d_xhat.  No workspace. */
mmv_status mmv_revert(const void *d_xhat, const int32_t *d_fhat, const void *d_w,
                      uint64_t n, uint64_t nw, void *d_z, mmv_elem et, void *hip_stream);

/* Algorithm SCD (Sec. 4.1) as printed: segmented sum = DIFF(COMPRESS(SCAN(x),
 * f^-)), four kernels and three passes over HBM.  Same arguments and results as
 * mmv_segsum (entries of d_out beyond the segment count are left untouched).  The
 * speculative scan runs over the whole vector, so floating-point sums carry the
 * rounding error of the global prefix (up to ulp(|xhat|) per sum); integers are
 * exact. */
mmv_status mmv_segsum_scd(const void *d_x, const void *d_flags, uint64_t n,
                          void *d_out, uint64_t out_capacity, uint64_t *d_nseg,
                          mmv_dtype dt, mmv_flag_fmt ff, mmv_variant v,
                          void *d_ws, size_t ws_bytes, void *hip_stream);

/* Algorithm SSCR (Sec. 4.1) as printed: segmented scan = REVERT(SCAN(x), SCAN(f),
 * COMPRESS(SCAN(x), f^-)).  Same arguments and results as mmv_segscan, same
 * remark on floating point as mmv_segsum_scd (and a non-finite value reaches every later position). */
mmv_status mmv_segscan_sscr(const void *d_x, const void *d_flags, uint64_t n, void *d_z,
                            mmv_dtype dt, mmv_flag_fmt ff, mmv_variant v,
                            void *d_ws, size_t ws_bytes, void *hip_stream);

/* Reads the status word the last call on this workspace left behind: 0 = fine,
 * 1 = a workgroup gave up waiting for a predecessor tile's carry (should
 * never happen; the result of that call is then invalid), 2 = mmv_spmv_*_run on a
 * workspace that was not prepared for this matrix (y holds zeros).  Synchronises
 * `hip_stream`.  *h_status is HOST memory. */
mmv_status mmv_workspace_status(const void *d_ws, void *hip_stream, uint32_t *h_status);

/* Streaming reference for the roofline (the paper compares every primitive with
 * a memcopy operator, Sec. 5.2.2): reads `in_bytes` from d_src and writes
 * `out_bytes` to d_dst with 128-bit accesses, each output chunk derived from the
 * input chunk at the same relative position.  Both sizes must be multiples of
 * 16; either may be 0. */
mmv_status mmv_stream_copy(const void *d_src, size_t in_bytes, void *d_dst, size_t out_bytes,
                           void *hip_stream);

/* Random-access reference for SpMV (the product vector val(i) * x(col(i)) of Sec. 4.3
 * without the segmented sum that follows it): streams the first nnz - nnz % 4 entries
 * of d_val and d_col (16-byte aligned), gathers x[col] from the n_cols entries of d_x
 * and leaves one partial sum per thread in d_partial, which must hold
 * MMV_GATHER_REFERENCE_PARTIALS floats.  Its time is what the random accesses to x
 * cost on their own; mmv_spmv_coo / mmv_spmv_csr cannot be faster.  A column index
 * outside [0, n_cols) reads x[0]. */
#define MMV_GATHER_REFERENCE_PARTIALS (8192 * 256)
mmv_status mmv_gather_reference(uint64_t nnz, const float *d_val, const int32_t *d_col, uint64_t n_cols,
                                const float *d_x, float *d_partial, void *hip_stream);

/* Instrumentation for benchmarks: from now on, every mmv_segscan / mmv_segsum /
 * mmv_spmv_coo call made by the calling host thread records `ev_start` (a
 * hipEvent_t passed as void*) on the call's stream immediately before its main
 * kernel and `ev_stop` immediately after it, so that the kernel can be timed
 * apart from the workspace reset.  The events stay owned by the caller.  Pass
 * NULL, NULL to switch it off (the default).  Per-thread setting. */
mmv_status mmv_set_kernel_events(void *ev_start, void *ev_stop);

const char *mmv_status_string(mmv_status s);

/* Elements per workgroup tile for an operation, input type and length (tiles are
 * smaller for short inputs so that every compute unit gets one).  For tests that want
 * to straddle tile borders and for sizing: the workspace holds one 8-byte descriptor
 * per tile (the segmented sum 40 more bytes of counts per tile).  The value is that
 * of the matrix-core variant (the other one differs for fp32 sums and for bytes under exclusive or).
 * The segmented sum of 8- and 16-bit inputs has longer tiles than the scan; mmv_scan of 16- and
 * 32-bit inputs has longer tiles than mmv_segscan.
 * 0 for invalid arguments. */
uint32_t mmv_tile_elems(mmv_op op, mmv_dtype dt, uint64_t n);

#ifdef __cplusplus
}
#endif
#endif /* MMVSEG_H */
