// libmmvseg: segmented inclusive scan, segmented sum and SpMV (row-sorted COO, CSR) for
// gfx950 (MI355X), after the block-recursive segmented scan of "Segmented
// Operations using Matrix Multiplications" (Sec. 4.2 and the appendix algorithm
// "Block-recursive segmented scan"); plus the paper's stand-alone primitives
// (SCAN, COMPRESS, DIFF, REVERT, Sec. 4.1) and its un-fused compositions SCD and SSCR.
//
// One kernel launch (seg_kernel) does a whole segmented operation in a single pass over HBM:
//
//   step 1  speculative row scans  x-bar = MATMUL(x, U_s), s = 32          MFMA
//           (computed transposed: Z^T = U_s^T X^T, so that every lane ends up
//           with four consecutive positions of one row per 128-bit LDS write)
//   step 2  REVSPEC: subtract x-bar(start-1) inside the row                 VALU + LDS gather
//   step 3  row aggregates (last element of each reverted row)              one lane per row
//   step 4  OR of the row's flags                                           one lane per row
//   step 5  segmented scan of the aggregates: lanes -> waves -> workgroup,
//           then decoupled look-back over tile descriptors in HBM
//           (replaces the paper's recursion passes over global memory)
//   step 6  UpdateFirstSegment: add the carry to the elements before the
//           row's first flag (folded into step 2 through a per-row slot that
//           holds the negated carry)
//
// Layout of a workgroup tile: 8 waves x (1 to 4) chunks x 64 rows x 32 elements.
// Lane r of a wave owns row r of the wave's current 2048-element chunk for steps 3-5;
// one packed flag word is exactly one row.
//
// Small kernels around it: workspace reset, flag packing (bytes, COO row indices, CSR row
// pointers), per-tile counts of segment starts (the output positions of the segmented sum),
// COMPRESS, DIFF, REVERT, and two reference kernels for the benchmark: a streaming copy
// (bandwidth) and a gather of x[col] (what the random accesses of SpMV cost on their own).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <mutex>
#include <type_traits>

#include "mmvseg.h"

#include "tunables.h"
#include "lanes.h"
#include "tile_math.h"
#include "seg_kernel.h"
#include "sum_kernel.h"
#include "seg_entry.h"
#include "aux_kernels.h"
#include "primitives.h"
#include "host.h"


// ---- scratch for callers that cannot allocate (mmv_segscan_static) -------------------------------------------
//
// Device memory that exists from the moment the library is loaded: every GPU that runs this code object
// holds its own copy of the array at its own address until the process ends.  In host code the array's
// name is only a handle for hipGetSymbolAddress, never an address: the device address is asked once per
// device, with that device current, and kept.
static __device__ __align__(256) unsigned char scratch[MMV_STATIC_SCRATCH_BYTES];

namespace {

std::atomic<void *> g_scratch_ptr[kMaxDevices];   // device address of `scratch`, per device; null = not asked yet

// Address of the current device's copy of `scratch` (nullptr on failure).
void *static_scratch() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    void *q = nullptr;
    if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) return nullptr;
    g_scratch_ptr[dev].store(q, std::memory_order_release);   // (two threads asking at once store the same address)
    return q;
}

mmv_status segscan_call(const void *d_x, const void *d_flags, uint64_t n, void *d_z, mmv_dtype dt, mmv_flag_fmt ff,
                        mmv_variant v, void *d_ws, size_t ws_bytes, hipStream_t s) {
    Params P = {};
    const mmv_status st = prepare(MMV_OP_SEGSCAN, d_x, d_flags, n, dt, ff, v, d_ws, ws_bytes, s, P);
    if (st != MMV_OK) return st;
    P.z = d_z;
    return launch_dt<kScan>(P, dt, v, s) == hipSuccess ? MMV_OK : MMV_ERR_HIP;
}

}  // namespace

// ---- C ABI ------------------------------------------------------------------------------------------------------

extern "C" {

size_t mmv_workspace_bytes(mmv_op op, mmv_dtype dt, mmv_flag_fmt ff, uint64_t n) {
    if (!valid_dtype(dt) || !valid_ff(ff) || n > kMaxN) return 0;
    switch (op) {
        case MMV_OP_SEGSCAN:
        case MMV_OP_SEGSUM:
        case MMV_OP_SCAN: return ws_layout(op, dt, ff, n).total;
        case MMV_OP_SPMV_COO: return ws_layout(op, MMV_F32_F32, ff, n).total;
        case MMV_OP_COMPRESS: return compress_layout(ff, n).total;
        case MMV_OP_SEGSUM_SCD: return scd_layout(dt, ff, n, n).total;
        case MMV_OP_SEGSCAN_SSCR: return sscr_layout(dt, ff, n).total;
        case MMV_OP_SPMV_CSR: return 0;  // two sizes: see mmv_spmv_csr_workspace_bytes
        default: break;
    }
    return 0;
}

size_t mmv_spmv_csr_workspace_bytes(uint64_t n_rows, uint64_t nnz) {
    if (n_rows >= (1ull << 31) || nnz >= (1ull << 31)) return 0;
    return csr_layout(n_rows, nnz).total;
}

mmv_status mmv_segscan(const void *d_x, const void *d_flags, uint64_t n, void *d_z, mmv_dtype dt, mmv_flag_fmt ff,
                       mmv_variant v, void *d_ws, size_t ws_bytes, void *hip_stream) {
    if (n == 0) return (valid_dtype(dt) && valid_ff(ff) && valid_variant(v)) ? MMV_OK : MMV_ERR_INVALID_ARG;
    if (!d_z) return MMV_ERR_NULL;
    if (!aligned16(d_z)) return MMV_ERR_INVALID_ARG;
    if (d_z == d_x && valid_dtype(dt) && dt != MMV_F32_F32) return MMV_ERR_INVALID_ARG;
    return segscan_call(d_x, d_flags, n, d_z, dt, ff, v, d_ws, ws_bytes, (hipStream_t)hip_stream);
}

mmv_status mmv_segscan_static(const void *d_x, const void *d_flags, uint64_t n, void *d_z, mmv_dtype dt,
                              mmv_flag_fmt ff, mmv_variant v, void *hip_stream) {
    if (!valid_dtype(dt) || !valid_ff(ff) || !valid_variant(v) || n > kMaxN) return MMV_ERR_INVALID_ARG;
    if (n == 0) return MMV_OK;
    if (!d_z) return MMV_ERR_NULL;
    if (!aligned16(d_z)) return MMV_ERR_INVALID_ARG;
    if (d_z == d_x && dt != MMV_F32_F32) return MMV_ERR_INVALID_ARG;
    // the tile descriptors (and the packed copy of one-byte flags) must fit the built-in array
    if (ws_layout(MMV_OP_SEGSCAN, dt, ff, n).total > (size_t)MMV_STATIC_SCRATCH_BYTES) return MMV_ERR_TOO_LARGE;
    void *ws = static_scratch();
    if (!ws) return MMV_ERR_HIP;
    return segscan_call(d_x, d_flags, n, d_z, dt, ff, v, ws, (size_t)MMV_STATIC_SCRATCH_BYTES, (hipStream_t)hip_stream);
}

mmv_status mmv_segsum(const void *d_x, const void *d_flags, uint64_t n, void *d_out, uint64_t out_capacity,
                      uint64_t *d_nseg, mmv_dtype dt, mmv_flag_fmt ff, mmv_variant v, void *d_ws, size_t ws_bytes,
                      void *hip_stream) {
    if (!valid_dtype(dt) || !valid_ff(ff) || !valid_variant(v) || n > kMaxN) return MMV_ERR_INVALID_ARG;
    if (!d_nseg) return MMV_ERR_NULL;
    hipStream_t s = (hipStream_t)hip_stream;
    if (n == 0) {
        fill_zero_kernel<<<1, 256, 0, s>>>((uint32_t *)d_nseg, 2, nullptr, 0);
        return hipGetLastError() == hipSuccess ? MMV_OK : MMV_ERR_HIP;
    }
    if (!d_out && out_capacity > 0) return MMV_ERR_NULL;
    if (!aligned16(d_out) || ((uintptr_t)d_nseg & 7u)) return MMV_ERR_INVALID_ARG;
    Params P = {};
    const mmv_status st = prepare(MMV_OP_SEGSUM, d_x, d_flags, n, dt, ff, v, d_ws, ws_bytes, s, P);
    if (st != MMV_OK) return st;
    P.out = d_out;
    P.out_cap = out_capacity;
    P.nseg = d_nseg;
    // number of segment starts before every tile: per-tile counts, then their exclusive scan
    const TilePlan plan = tile_plan(MMV_OP_SEGSUM, dt, n, v == MMV_VARIANT_MFMA);
    const WsLayout L = ws_layout(MMV_OP_SEGSUM, dt, ff, n);
    uint32_t *tile_count = (uint32_t *)((char *)d_ws + L.desc_c);
    if (plan.tiles > 0x7fffffffull) return MMV_ERR_INVALID_ARG;
    uint32_t *span_count = (uint32_t *)((char *)d_ws + L.span_c);
    count_tiles_kernel<<<(unsigned)plan.tiles, 256, 0, s>>>((uint32_t *)d_ws, L.desc_c / 4, P.fw, n, plan.reg,
                                                             plan.unit, tile_count, span_count);
    if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    // few tiles: every tile of the main kernel adds up the counts before it; many: one more small kernel
    // turns the counts into prefix sums first
    P.count_is_prefix = plan.tiles > kCountSumTiles ? 1u : 0u;
    if (P.count_is_prefix) {
        scan_counts_kernel<<<1, 1024, 0, s>>>(tile_count, (uint32_t)plan.tiles, d_nseg);
        if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    }
    P.tile_count = tile_count;
    P.span_count = span_count;
    return launch_dt<kSum>(P, dt, v, s) == hipSuccess ? MMV_OK : MMV_ERR_HIP;
}

mmv_status mmv_spmv_coo(uint64_t n_rows, uint64_t n_cols, uint64_t nnz, const int32_t *d_row, const int32_t *d_col,
                        const float *d_val, const float *d_x, float *d_y, mmv_variant v, void *d_ws, size_t ws_bytes,
                        void *hip_stream) {
    if (!valid_variant(v) || n_rows >= (1ull << 31) || n_cols >= (1ull << 31) || nnz > kMaxN) return MMV_ERR_INVALID_ARG;
    if (n_rows == 0) return MMV_OK;
    if (!d_y) return MMV_ERR_NULL;
    if (!aligned16(d_y)) return MMV_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    if (nnz == 0) {
        fill_zero_kernel<<<grid_for(n_rows), 256, 0, s>>>((uint32_t *)d_y, n_rows, nullptr, 0);
        return hipGetLastError() == hipSuccess ? MMV_OK : MMV_ERR_HIP;
    }
    if (!d_row || !d_col || !d_val || !d_x || !d_ws) return MMV_ERR_NULL;
    if (!aligned16(d_row) || !aligned16(d_col) || !aligned16(d_val) || !aligned16(d_x)) return MMV_ERR_INVALID_ARG;
    const WsLayout L = ws_layout(MMV_OP_SPMV_COO, MMV_F32_F32, MMV_FLAGS_PACKED32, nnz);
    if (((uintptr_t)d_ws & 255u) != 0 || ws_bytes < L.total) return MMV_ERR_WORKSPACE;
    char *ws = (char *)d_ws;
    Params P = {};
    P.x = d_val;
    P.n = nnz;
    P.row = d_row;
    P.col = d_col;
    P.xv = d_x;
    P.y = d_y;
    P.hdr = (uint32_t *)ws;
    P.desc_v = (uint64_t *)(ws + L.desc_v);
    P.num_tiles = (uint32_t)tiles_for(nnz, MMV_OP_SPMV_COO, MMV_F32_F32);
    P.fw = (const uint32_t *)(ws + L.packed);
    // one launch ahead of the main kernel: header and descriptors and y zeroed, the flag words made from the row indices
    const uint64_t zero_words = L.packed / 4;
    uint64_t flag_blocks = (nnz + 8191) / 8192;
    if (flag_blocks > 0x7fffffffull) return MMV_ERR_INVALID_ARG;
    const uint64_t fill_blocks = (uint64_t)grid_for(zero_words > n_rows ? zero_words : n_rows);   // (few entries, many rows)
    if (flag_blocks < fill_blocks) flag_blocks = fill_blocks;
    row_flags_kernel<<<(unsigned)flag_blocks, 256, 0, s>>>(d_row, nnz, (uint32_t *)(ws + L.packed), d_col, (uint32_t *)ws,
                                                           zero_words, (uint32_t *)d_y, n_rows);
    if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    return launch_seg<TSpmv, kSpmv>(P, v, s) == hipSuccess ? MMV_OK : MMV_ERR_HIP;
}

// SpMV in two steps: the mark that the first step leaves in the header for this matrix shape (never 0).
static uint32_t prepared_mark(mmv_op op, uint64_t n_rows, uint64_t nnz) {
    uint64_t h = (nnz + 0x9E3779B97F4A7C15ull) * 0xD6E8FEB86659FD93ull + n_rows * 0xCA5A826395121157ull + (uint64_t)op;
    h ^= h >> 32;
    return (uint32_t)h | 1u;
}

mmv_status mmv_spmv_coo_prepare(uint64_t n_rows, uint64_t n_cols, uint64_t nnz, const int32_t *d_row,
                                const int32_t *d_col, void *d_ws, size_t ws_bytes, void *hip_stream) {
    if (n_rows >= (1ull << 31) || n_cols >= (1ull << 31) || nnz > kMaxN) return MMV_ERR_INVALID_ARG;
    if (n_rows == 0 || nnz == 0) return MMV_OK;
    if (!d_row || !d_col || !d_ws) return MMV_ERR_NULL;
    if (!aligned16(d_row) || !aligned16(d_col)) return MMV_ERR_INVALID_ARG;
    const WsLayout L = ws_layout(MMV_OP_SPMV_COO, MMV_F32_F32, MMV_FLAGS_PACKED32, nnz);
    if (((uintptr_t)d_ws & 255u) != 0 || ws_bytes < L.total) return MMV_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    char *ws = (char *)d_ws;
    const uint64_t zero_words = L.packed / 4;
    uint64_t flag_blocks = (nnz + 8191) / 8192;
    if (flag_blocks > 0x7fffffffull) return MMV_ERR_INVALID_ARG;
    const uint64_t fill_blocks = (uint64_t)grid_for(zero_words);
    if (flag_blocks < fill_blocks) flag_blocks = fill_blocks;
    row_flags_kernel<<<(unsigned)flag_blocks, 256, 0, s>>>(d_row, nnz, (uint32_t *)(ws + L.packed), d_col, (uint32_t *)ws,
                                                           zero_words, nullptr, 0);
    if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    mark_prepared_kernel<<<1, 64, 0, s>>>((uint32_t *)ws, prepared_mark(MMV_OP_SPMV_COO, n_rows, nnz));
    return hipGetLastError() == hipSuccess ? MMV_OK : MMV_ERR_HIP;
}

mmv_status mmv_spmv_coo_run(uint64_t n_rows, uint64_t n_cols, uint64_t nnz, const int32_t *d_row, const int32_t *d_col,
                            const float *d_val, const float *d_x, float *d_y, mmv_variant v, void *d_ws, size_t ws_bytes,
                            void *hip_stream) {
    if (!valid_variant(v) || n_rows >= (1ull << 31) || n_cols >= (1ull << 31) || nnz > kMaxN) return MMV_ERR_INVALID_ARG;
    if (n_rows == 0) return MMV_OK;
    if (!d_y) return MMV_ERR_NULL;
    if (!aligned16(d_y)) return MMV_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    if (nnz == 0) {
        fill_zero_kernel<<<grid_for(n_rows), 256, 0, s>>>((uint32_t *)d_y, n_rows, nullptr, 0);
        return hipGetLastError() == hipSuccess ? MMV_OK : MMV_ERR_HIP;
    }
    if (!d_row || !d_col || !d_val || !d_x || !d_ws) return MMV_ERR_NULL;
    if (!aligned16(d_row) || !aligned16(d_col) || !aligned16(d_val) || !aligned16(d_x)) return MMV_ERR_INVALID_ARG;
    const WsLayout L = ws_layout(MMV_OP_SPMV_COO, MMV_F32_F32, MMV_FLAGS_PACKED32, nnz);
    if (((uintptr_t)d_ws & 255u) != 0 || ws_bytes < L.total) return MMV_ERR_WORKSPACE;
    char *ws = (char *)d_ws;
    Params P = {};
    P.x = d_val;
    P.n = nnz;
    P.row = d_row;
    P.col = d_col;
    P.xv = d_x;
    P.y = d_y;
    P.hdr = (uint32_t *)ws;
    P.desc_v = (uint64_t *)(ws + L.desc_v);
    P.num_tiles = (uint32_t)tiles_for(nnz, MMV_OP_SPMV_COO, MMV_F32_F32);
    P.fw = (const uint32_t *)(ws + L.packed);
    P.prepared = prepared_mark(MMV_OP_SPMV_COO, n_rows, nnz);
    const uint64_t zero_words = L.packed / 4;   // header and descriptors; the flag words behind them stay
    reset_prepared_kernel<<<grid_for(zero_words > n_rows ? zero_words : n_rows), 256, 0, s>>>(
        (uint32_t *)ws, zero_words, (uint32_t *)d_y, n_rows, P.prepared);
    if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    return launch_seg<TSpmv, kSpmv>(P, v, s) == hipSuccess ? MMV_OK : MMV_ERR_HIP;
}

mmv_status mmv_scan(const void *d_x, uint64_t n, void *d_z, mmv_dtype dt, mmv_variant v, void *d_ws, size_t ws_bytes,
                    void *hip_stream) {
    if (!valid_dtype(dt) || !valid_variant(v) || n > kMaxN) return MMV_ERR_INVALID_ARG;
    if (n == 0) return MMV_OK;
    if (!d_x || !d_z || !d_ws) return MMV_ERR_NULL;
    if (!aligned16(d_x) || !aligned16(d_z)) return MMV_ERR_INVALID_ARG;
    if (d_z == d_x && dt != MMV_F32_F32) return MMV_ERR_INVALID_ARG;
    return scan_impl(d_x, n, d_z, dt, v, d_ws, ws_bytes, (hipStream_t)hip_stream, false);
}

mmv_status mmv_compress(const void *d_x, const void *d_mask, uint64_t n, void *d_out, uint64_t out_capacity,
                        uint64_t *d_count, mmv_flag_fmt ff, void *d_ws, size_t ws_bytes, void *hip_stream) {
    if (!valid_ff(ff) || n > kMaxN) return MMV_ERR_INVALID_ARG;
    if (!d_count) return MMV_ERR_NULL;
    if ((uintptr_t)d_count & 7u) return MMV_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    if (n == 0) {
        fill_zero_kernel<<<1, 256, 0, s>>>((uint32_t *)d_count, 2, nullptr, 0);
        return hipGetLastError() == hipSuccess ? MMV_OK : MMV_ERR_HIP;
    }
    if (!d_mask || !d_ws || (!d_out && out_capacity > 0)) return MMV_ERR_NULL;
    if (!aligned16(d_x) || !aligned16(d_mask) || !aligned16(d_out)) return MMV_ERR_INVALID_ARG;
    return compress_impl(d_x, d_mask, n, d_out, out_capacity, d_count, ff, d_ws, ws_bytes, s);
}

mmv_status mmv_diff(const void *d_x, uint64_t n, void *d_z, mmv_elem et, void *hip_stream) {
    if (!valid_elem(et) || n > kMaxN) return MMV_ERR_INVALID_ARG;
    if (n == 0) return MMV_OK;
    if (!d_x || !d_z) return MMV_ERR_NULL;
    if (!aligned16(d_x) || !aligned16(d_z) || d_x == d_z) return MMV_ERR_INVALID_ARG;
    return diff_impl(d_x, n, d_z, et, (hipStream_t)hip_stream);
}

mmv_status mmv_revert(const void *d_xhat, const int32_t *d_fhat, const void *d_w, uint64_t n, uint64_t nw,
                      void *d_z, mmv_elem et, void *hip_stream) {
    if (!valid_elem(et) || n > kMaxN) return MMV_ERR_INVALID_ARG;
    if (n == 0) return MMV_OK;
    if (!d_xhat || !d_fhat || !d_z || (!d_w && nw > 0)) return MMV_ERR_NULL;
    if (!aligned16(d_xhat) || !aligned16(d_fhat) || !aligned16(d_z) || ((uintptr_t)d_w & 3u)) return MMV_ERR_INVALID_ARG;
    return revert_impl(d_xhat, d_fhat, d_w, n, nw, d_z, et, (hipStream_t)hip_stream);
}

mmv_status mmv_segsum_scd(const void *d_x, const void *d_flags, uint64_t n, void *d_out, uint64_t out_capacity,
                          uint64_t *d_nseg, mmv_dtype dt, mmv_flag_fmt ff, mmv_variant v, void *d_ws, size_t ws_bytes,
                          void *hip_stream) {
    if (!valid_dtype(dt) || !valid_ff(ff) || !valid_variant(v) || n > kMaxN) return MMV_ERR_INVALID_ARG;
    if (dt == MMV_U8_XOR) return MMV_ERR_UNSUPPORTED;   // DIFF subtracts
    if (!d_nseg) return MMV_ERR_NULL;
    hipStream_t s = (hipStream_t)hip_stream;
    if (n == 0) {
        fill_zero_kernel<<<1, 256, 0, s>>>((uint32_t *)d_nseg, 2, nullptr, 0);
        return hipGetLastError() == hipSuccess ? MMV_OK : MMV_ERR_HIP;
    }
    if (!d_x || !d_flags || !d_ws || (!d_out && out_capacity > 0)) return MMV_ERR_NULL;
    if (!aligned16(d_x) || !aligned16(d_flags) || !aligned16(d_out) || ((uintptr_t)d_nseg & 7u)) return MMV_ERR_INVALID_ARG;
    const ScdLayout L = scd_layout(dt, ff, n, out_capacity);
    if (((uintptr_t)d_ws & 255u) != 0 || ws_bytes < L.total) return MMV_ERR_WORKSPACE;
    char *ws = (char *)d_ws;
    EventsOff quiet;
    const uint64_t nwords = (n + 31) / 32;
    const uint64_t cap = out_capacity < n ? out_capacity : n;
    // 1. speculative scan of the whole vector
    mmv_status st = scan_impl(d_x, n, ws + L.xhat, dt, v, ws + L.scan_ws, L.xhat - L.scan_ws, s, false);
    if (st != MMV_OK) return st;
    // 2. end markers f^- (from packed flags)
    const uint32_t *fw = (const uint32_t *)d_flags;
    if (ff == MMV_FLAGS_U8) {
        uint32_t *packed = (uint32_t *)(ws + L.packed);
        pack_flags_kernel<<<grid_for(nwords), 256, 0, s>>>((const uint8_t *)d_flags, n, packed, nwords);
        if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
        fw = packed;
    }
    end_markers_kernel<<<grid_for(nwords), 256, 0, s>>>(fw, n, (uint32_t *)(ws + L.fminus), nwords);
    if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    // 3. scanned values at the segment ends
    st = compress_impl(ws + L.xhat, ws + L.fminus, n, ws + L.w, cap, d_nseg, MMV_FLAGS_PACKED32, ws + L.compress_ws,
                       L.w - L.compress_ws, s);
    if (st != MMV_OK) return st;
    // 4. adjacent differences of the first min(nseg, capacity) of them
    if (cap == 0) return MMV_OK;
    return diff_impl(ws + L.w, cap, d_out, dt == MMV_I8_I32 ? MMV_ELEM_I32 : MMV_ELEM_F32, s, d_nseg);
}

mmv_status mmv_segscan_sscr(const void *d_x, const void *d_flags, uint64_t n, void *d_z, mmv_dtype dt, mmv_flag_fmt ff,
                            mmv_variant v, void *d_ws, size_t ws_bytes, void *hip_stream) {
    if (!valid_dtype(dt) || !valid_ff(ff) || !valid_variant(v) || n > kMaxN) return MMV_ERR_INVALID_ARG;
    if (dt == MMV_U8_XOR) return MMV_ERR_UNSUPPORTED;   // REVERT subtracts
    if (n == 0) return MMV_OK;
    if (!d_x || !d_flags || !d_z || !d_ws) return MMV_ERR_NULL;
    if (!aligned16(d_x) || !aligned16(d_flags) || !aligned16(d_z)) return MMV_ERR_INVALID_ARG;
    if (d_z == d_x && dt != MMV_F32_F32) return MMV_ERR_INVALID_ARG;
    const SscrLayout L = sscr_layout(dt, ff, n);
    if (((uintptr_t)d_ws & 255u) != 0 || ws_bytes < L.total) return MMV_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    char *ws = (char *)d_ws;
    EventsOff quiet;
    const uint64_t nwords = (n + 31) / 32;
    // flags in both encodings: bits for the end markers, 0 / 1 bytes for SCAN(f) (the caller's
    // bytes may hold any non-zero value for "set", so they are not summed as they are)
    const uint32_t *fw = (const uint32_t *)d_flags;
    if (ff == MMV_FLAGS_U8) {
        uint32_t *packed = (uint32_t *)(ws + L.packed);
        pack_flags_kernel<<<grid_for(nwords), 256, 0, s>>>((const uint8_t *)d_flags, n, packed, nwords);
        if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
        fw = packed;
    }
    unpack_flags_kernel<<<grid_for((n + 3) / 4), 256, 0, s>>>(fw, n, (int8_t *)(ws + L.f8));
    if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    const void *f8 = ws + L.f8;
    // 1. (SCAN(x), SCAN(f)); the speculative scan goes straight to z and is reverted in place
    mmv_status st = scan_impl(d_x, n, d_z, dt, v, ws + L.scan_ws_x, L.scan_ws_f - L.scan_ws_x, s, false);
    if (st != MMV_OK) return st;
    st = scan_impl(f8, n, ws + L.fhat, MMV_I8_I32, v, ws + L.scan_ws_f, L.fhat - L.scan_ws_f, s, true);
    if (st != MMV_OK) return st;
    // 2. end markers, 3. w = scanned values at the segment ends
    end_markers_kernel<<<grid_for(nwords), 256, 0, s>>>(fw, n, (uint32_t *)(ws + L.fminus), nwords);
    if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    uint64_t *d_nw = (uint64_t *)(ws + L.w);          // the count sits in front of w
    st = compress_impl(d_z, ws + L.fminus, n, ws + L.w + 16, n, d_nw, MMV_FLAGS_PACKED32, ws + L.compress_ws,
                       L.w - L.compress_ws, s);
    if (st != MMV_OK) return st;
    // 4. REVERT; every count is at most the number of segments, so nw = n is a safe bound
    return revert_impl(d_z, (const int32_t *)(ws + L.fhat), ws + L.w + 16, n, n, d_z,
                       dt == MMV_I8_I32 ? MMV_ELEM_I32 : MMV_ELEM_F32, s);
}

mmv_status mmv_spmv_csr(uint64_t n_rows, uint64_t n_cols, uint64_t nnz, const int32_t *d_rowptr, const int32_t *d_col,
                        const float *d_val, const float *d_x, float *d_y, mmv_variant v, void *d_ws, size_t ws_bytes,
                        void *hip_stream) {
    if (!valid_variant(v) || n_rows >= (1ull << 31) || n_cols >= (1ull << 31) || nnz >= (1ull << 31))
        return MMV_ERR_INVALID_ARG;
    if (n_rows == 0) return MMV_OK;
    if (!d_y) return MMV_ERR_NULL;
    if (!aligned16(d_y)) return MMV_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    if (nnz == 0) {
        fill_zero_kernel<<<grid_for(n_rows), 256, 0, s>>>((uint32_t *)d_y, n_rows, nullptr, 0);
        return hipGetLastError() == hipSuccess ? MMV_OK : MMV_ERR_HIP;
    }
    if (!d_rowptr || !d_col || !d_val || !d_x || !d_ws) return MMV_ERR_NULL;
    if (!aligned16(d_rowptr) || !aligned16(d_col) || !aligned16(d_val) || !aligned16(d_x)) return MMV_ERR_INVALID_ARG;
    const CsrLayout C = csr_layout(n_rows, nnz);
    if (((uintptr_t)d_ws & 255u) != 0 || ws_bytes < C.total) return MMV_ERR_WORKSPACE;
    char *ws = (char *)d_ws;
    const WsLayout L = ws_layout(MMV_OP_SPMV_CSR, MMV_F32_F32, MMV_FLAGS_PACKED32, nnz);
    // zero: the main kernel's header, descriptors and flag words, the header and descriptors of COMPRESS; y
    const uint64_t zero_words = (C.compress_ws + compress_layout(MMV_FLAGS_PACKED32, n_rows).packed) / 4;
    fill_zero_kernel<<<grid_for(zero_words > n_rows ? zero_words : n_rows), 256, 0, s>>>((uint32_t *)ws, zero_words,
                                                                                      (uint32_t *)d_y, n_rows);
    if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    // segment-start flags over the non-zeros, their number per tile of the main kernel, and the mask of
    // rows that have entries
    const TilePlan plan = tile_plan(MMV_OP_SPMV_CSR, MMV_F32_F32, nnz);
    uint32_t *fw = (uint32_t *)(ws + C.main_ws + L.packed);
    uint32_t *tile_count = (uint32_t *)(ws + C.main_ws + L.desc_c);
    const uint64_t row_blocks = (n_rows + 255) / 256;
    csr_flags_kernel<<<(unsigned)row_blocks, 256, 0, s>>>(d_rowptr, n_rows, fw, (uint32_t *)(ws + C.rowmask),
                                                          (uint32_t *)(ws + C.main_ws), plan.reg, plan.unit,
                                                          tile_count, d_col, nnz);
    if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    // rowmap = COMPRESS(0 .. n_rows - 1, rowmask): the k-th segment belongs to row rowmap[k]
    {
        EventsOff quiet;
        const mmv_status st = compress_impl(nullptr, ws + C.rowmask, n_rows, ws + C.rowmap, n_rows,
                                            (uint64_t *)(ws + C.rowcount), MMV_FLAGS_PACKED32, ws + C.compress_ws,
                                            C.rowmask - C.compress_ws, s, true,
                                            (const uint32_t *)(ws + C.main_ws) + kHdrEmptyRows);
        if (st != MMV_OK) return st;
    }
    Params P = {};
    P.x = d_val;
    P.n = nnz;
    P.col = d_col;
    P.xv = d_x;
    P.y = d_y;
    P.rowmap = (const uint32_t *)(ws + C.rowmap);
    P.out_cap = n_rows;
    P.hdr = (uint32_t *)(ws + C.main_ws);
    P.desc_v = (uint64_t *)(ws + C.main_ws + L.desc_v);
    P.fw = fw;
    P.count_is_prefix = plan.tiles > kCountSumTilesCsr ? 1u : 0u;
    if (P.count_is_prefix) {
        scan_counts_kernel<<<1, 1024, 0, s>>>(tile_count, (uint32_t)plan.tiles, (uint64_t *)(ws + C.rowcount));
        if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    }
    P.tile_count = tile_count;
    return launch_seg<TSpmv, kSpmvCsr>(P, v, s) == hipSuccess ? MMV_OK : MMV_ERR_HIP;
}

mmv_status mmv_spmv_csr_prepare(uint64_t n_rows, uint64_t n_cols, uint64_t nnz, const int32_t *d_rowptr,
                                const int32_t *d_col, void *d_ws, size_t ws_bytes, void *hip_stream) {
    if (n_rows >= (1ull << 31) || n_cols >= (1ull << 31) || nnz >= (1ull << 31)) return MMV_ERR_INVALID_ARG;
    if (n_rows == 0 || nnz == 0) return MMV_OK;
    if (!d_rowptr || !d_col || !d_ws) return MMV_ERR_NULL;
    if (!aligned16(d_rowptr) || !aligned16(d_col)) return MMV_ERR_INVALID_ARG;
    const CsrLayout C = csr_layout(n_rows, nnz);
    if (((uintptr_t)d_ws & 255u) != 0 || ws_bytes < C.total) return MMV_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    char *ws = (char *)d_ws;
    const WsLayout L = ws_layout(MMV_OP_SPMV_CSR, MMV_F32_F32, MMV_FLAGS_PACKED32, nnz);
    const uint64_t zero_words = (C.compress_ws + compress_layout(MMV_FLAGS_PACKED32, n_rows).packed) / 4;
    fill_zero_kernel<<<grid_for(zero_words), 256, 0, s>>>((uint32_t *)ws, zero_words, nullptr, 0);
    if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    const TilePlan plan = tile_plan(MMV_OP_SPMV_CSR, MMV_F32_F32, nnz);
    uint32_t *fw = (uint32_t *)(ws + C.main_ws + L.packed);
    uint32_t *tile_count = (uint32_t *)(ws + C.main_ws + L.desc_c);
    const uint64_t row_blocks = (n_rows + 255) / 256;
    csr_flags_kernel<<<(unsigned)row_blocks, 256, 0, s>>>(d_rowptr, n_rows, fw, (uint32_t *)(ws + C.rowmask),
                                                          (uint32_t *)(ws + C.main_ws), plan.reg, plan.unit,
                                                          tile_count, d_col, nnz);
    if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    {
        EventsOff quiet;
        const mmv_status st = compress_impl(nullptr, ws + C.rowmask, n_rows, ws + C.rowmap, n_rows,
                                            (uint64_t *)(ws + C.rowcount), MMV_FLAGS_PACKED32, ws + C.compress_ws,
                                            C.rowmask - C.compress_ws, s, true,
                                            (const uint32_t *)(ws + C.main_ws) + kHdrEmptyRows);
        if (st != MMV_OK) return st;
    }
    if (plan.tiles > kCountSumTilesCsr) {
        scan_counts_kernel<<<1, 1024, 0, s>>>(tile_count, (uint32_t)plan.tiles, (uint64_t *)(ws + C.rowcount));
        if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    }
    mark_prepared_kernel<<<1, 64, 0, s>>>((uint32_t *)(ws + C.main_ws), prepared_mark(MMV_OP_SPMV_CSR, n_rows, nnz));
    return hipGetLastError() == hipSuccess ? MMV_OK : MMV_ERR_HIP;
}

mmv_status mmv_spmv_csr_run(uint64_t n_rows, uint64_t n_cols, uint64_t nnz, const int32_t *d_rowptr, const int32_t *d_col,
                            const float *d_val, const float *d_x, float *d_y, mmv_variant v, void *d_ws, size_t ws_bytes,
                            void *hip_stream) {
    if (!valid_variant(v) || n_rows >= (1ull << 31) || n_cols >= (1ull << 31) || nnz >= (1ull << 31))
        return MMV_ERR_INVALID_ARG;
    if (n_rows == 0) return MMV_OK;
    if (!d_y) return MMV_ERR_NULL;
    if (!aligned16(d_y)) return MMV_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    if (nnz == 0) {
        fill_zero_kernel<<<grid_for(n_rows), 256, 0, s>>>((uint32_t *)d_y, n_rows, nullptr, 0);
        return hipGetLastError() == hipSuccess ? MMV_OK : MMV_ERR_HIP;
    }
    if (!d_rowptr || !d_col || !d_val || !d_x || !d_ws) return MMV_ERR_NULL;
    if (!aligned16(d_rowptr) || !aligned16(d_col) || !aligned16(d_val) || !aligned16(d_x)) return MMV_ERR_INVALID_ARG;
    const CsrLayout C = csr_layout(n_rows, nnz);
    if (((uintptr_t)d_ws & 255u) != 0 || ws_bytes < C.total) return MMV_ERR_WORKSPACE;
    char *ws = (char *)d_ws;
    const WsLayout L = ws_layout(MMV_OP_SPMV_CSR, MMV_F32_F32, MMV_FLAGS_PACKED32, nnz);
    const TilePlan plan = tile_plan(MMV_OP_SPMV_CSR, MMV_F32_F32, nnz);
    Params P = {};
    P.x = d_val;
    P.n = nnz;
    P.col = d_col;
    P.xv = d_x;
    P.y = d_y;
    P.rowmap = (const uint32_t *)(ws + C.rowmap);
    P.out_cap = n_rows;
    P.hdr = (uint32_t *)(ws + C.main_ws);
    P.desc_v = (uint64_t *)(ws + C.main_ws + L.desc_v);
    P.fw = (const uint32_t *)(ws + C.main_ws + L.packed);
    P.count_is_prefix = plan.tiles > kCountSumTilesCsr ? 1u : 0u;
    P.tile_count = (const uint32_t *)(ws + C.main_ws + L.desc_c);
    P.prepared = prepared_mark(MMV_OP_SPMV_CSR, n_rows, nnz);
    // header and value descriptors of the main kernel; the counts, flag words, row mask and row map behind them stay
    const uint64_t zero_words = L.desc_c / 4;
    reset_prepared_kernel<<<grid_for(zero_words > n_rows ? zero_words : n_rows), 256, 0, s>>>(
        (uint32_t *)(ws + C.main_ws), zero_words, (uint32_t *)d_y, n_rows, P.prepared);
    if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    return launch_seg<TSpmv, kSpmvCsr>(P, v, s) == hipSuccess ? MMV_OK : MMV_ERR_HIP;
}

mmv_status mmv_workspace_status(const void *d_ws, void *hip_stream, uint32_t *h_status) {
    if (!d_ws || !h_status) return MMV_ERR_NULL;
    hipStream_t s = (hipStream_t)hip_stream;
    uint32_t hdr[2] = {0, 0};
    if (hipMemcpyAsync(hdr, d_ws, sizeof(hdr), hipMemcpyDeviceToHost, s) != hipSuccess) return MMV_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return MMV_ERR_HIP;
    *h_status = hdr[kHdrError];
    return MMV_OK;
}

mmv_status mmv_stream_copy(const void *d_src, size_t in_bytes, void *d_dst, size_t out_bytes, void *hip_stream) {
    if ((in_bytes & 15u) || (out_bytes & 15u)) return MMV_ERR_INVALID_ARG;
    if (in_bytes == 0 && out_bytes == 0) return MMV_OK;
    if ((in_bytes && !d_src) || !d_dst) return MMV_ERR_NULL;
    if (!aligned16(d_src) || !aligned16(d_dst)) return MMV_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    const uint64_t ni = in_bytes / 16, no = out_bytes / 16;
    const v4u *src = (const v4u *)d_src;
    v4u *dst = (v4u *)d_dst;
#define MMV_COPY(KI, KO, UNITS)                                                                          \
    do {                                                                                                 \
        const uint64_t units_ = (UNITS);                                                                 \
        const uint64_t blocks_ = (units_ + 255) / 256;                                                   \
        if (blocks_ > 0x7fffffffull) return MMV_ERR_INVALID_ARG;                                         \
        stream_copy_kernel<KI, KO><<<(unsigned)blocks_, 256, 0, s>>>(src, dst, units_);                  \
    } while (0)
    if (no == 0) MMV_COPY(1, 0, ni);
    else if (ni == 0) MMV_COPY(0, 1, no);
    else if (ni == no) MMV_COPY(1, 1, ni);
    else if (no == 4 * ni) MMV_COPY(1, 4, ni);
    else if (no == 2 * ni) MMV_COPY(1, 2, ni);
    else if (ni == 2 * no) MMV_COPY(2, 1, no);
    else if (ni == 4 * no) MMV_COPY(4, 1, no);
    else return MMV_ERR_UNSUPPORTED;
#undef MMV_COPY
    return hipGetLastError() == hipSuccess ? MMV_OK : MMV_ERR_HIP;
}

mmv_status mmv_gather_reference(uint64_t nnz, const float *d_val, const int32_t *d_col, uint64_t n_cols,
                                const float *d_x, float *d_partial, void *hip_stream) {
    if (nnz == 0) return MMV_OK;
    if (!d_val || !d_col || !d_x || !d_partial) return MMV_ERR_NULL;
    if (!aligned16(d_val) || !aligned16(d_col) || !aligned4(d_x) || !aligned4(d_partial)) return MMV_ERR_INVALID_ARG;
    if (n_cols == 0 || n_cols > 0x7fffffffull) return MMV_ERR_INVALID_ARG;
    gather_reference_kernel<<<kGatherRefBlocks, 256, 0, (hipStream_t)hip_stream>>>(
        (const v4u *)d_val, (const v4u *)d_col, nnz / 4, (uint32_t)n_cols, d_x, d_partial);
    return hipGetLastError() == hipSuccess ? MMV_OK : MMV_ERR_HIP;
}

mmv_status mmv_set_kernel_events(void *ev_start, void *ev_stop) {
    tl_ev_start = (hipEvent_t)ev_start;
    tl_ev_stop = (hipEvent_t)ev_stop;
    return MMV_OK;
}

const char *mmv_status_string(mmv_status s) {
    switch (s) {
        case MMV_OK: return "ok";
        case MMV_ERR_INVALID_ARG: return "invalid argument";
        case MMV_ERR_NULL: return "null pointer";
        case MMV_ERR_UNSUPPORTED: return "unsupported";
        case MMV_ERR_WORKSPACE: return "workspace too small or misaligned";
        case MMV_ERR_HIP: return "HIP error";
        case MMV_ERR_TOO_LARGE: return "input too large for the built-in scratch of mmv_segscan_static";
        default: break;
    }
    return "unknown status";
}

uint32_t mmv_tile_elems(mmv_op op, mmv_dtype dt, uint64_t n) {
    if (!valid_dtype(dt)) return 0;
    if (op == MMV_OP_COMPRESS) return (uint32_t)compress_tile(n);
    if (op != MMV_OP_SEGSCAN && op != MMV_OP_SEGSUM && op != MMV_OP_SCAN && !is_spmv(op)) return 0;
    return tile_plan(op, is_spmv(op) ? MMV_F32_F32 : dt, n).body_elems;
}

}  // extern "C"
