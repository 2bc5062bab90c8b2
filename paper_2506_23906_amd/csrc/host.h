// libmmvseg, part of the one translation unit mmvseg.hip (included there, in order).
// Host side: argument checks, workspace layouts, tile plans and the launch sequences behind the C ABI.
#pragma once

namespace {

// ---- host side -------------------------------------------------------------------------------------------------

inline size_t round256(size_t b) { return (b + 255) & ~(size_t)255; }
// Tile plan.  A tile costs one ticket (about 11 ns, serialised), so tiles are as large as the registers
// allow: kMaxCpw chunks of 2048 elements per wave.  Inputs that fit into one round of resident workgroups
// get equal tiles of just the size that gives every workgroup one.  A longer vector starts with groups of
// tiles of 1, 2, ... chunks per wave and ends with groups of ..., 2, 1: started together on full tiles, the
// workgroups of the first round all load, then all compute, then all store (nothing overlaps for a whole
// tile time), and those of the last round would leave most of the chip idle while the last ones finish.
// (Measured on the int8 scan: the time of a launch is a fixed 22 us plus 0.216 ms per 2^28 elements with
// full tiles throughout and one group of short tiles at the end.)
constexpr uint64_t kResident = MMV_MIN_TILES;   // workgroups resident at once (2 per compute unit)
#ifndef MMV_HEAD_GROUP
#define MMV_HEAD_GROUP 128   // tiles per length at the start of a long vector (0: full tiles from the start)
#endif
#ifndef MMV_TAIL_GROUP
#define MMV_TAIL_GROUP 64    // tiles per length (2 chunks per wave and more) at the end of a long vector
#endif
#ifndef MMV_TAIL_TILES
#define MMV_TAIL_TILES 128   // tiles of one chunk per wave at the very end (the last of them is ragged)
#endif
// Up to this many tiles the segmented sum needs no prefix kernel: every wave of the main kernel adds up the counts of
// the tiles before its own.  That loop costs in proportion to the number of tiles (1224 tiles: 5.6 us of a 42 us
// kernel; 2448: 15 us), the prefix kernel 3 us of the call.
constexpr uint64_t kCountSumTiles = 768;
// CSR SpMV: one wave per tile adds up (959 tiles: the loop 1.4 us of the kernel, the prefix kernel 3 us of the call)
constexpr uint64_t kCountSumTilesCsr = 2048;
inline bool is_spmv(mmv_op op) { return op == MMV_OP_SPMV_COO || op == MMV_OP_SPMV_CSR; }
// Most chunks per wave of the tile body that carries its pair from row to row (seg_tile): what the kernel
// instantiation for this operation, type and variant is built with.
template <typename TT> inline int row_form_cpw_of(mmv_op op, bool mfma) {
    switch (op) {
        case MMV_OP_SCAN: return mfma ? chunks_per_wave<TT, kPlainScan, true>() : chunks_per_wave<TT, kPlainScan, false>();
        case MMV_OP_SEGSUM: return mfma ? chunks_per_wave<TT, kSum, true>() : chunks_per_wave<TT, kSum, false>();
        default: return mfma ? chunks_per_wave<TT, kScan, true>() : chunks_per_wave<TT, kScan, false>();
    }
}
inline int row_form_cpw(mmv_op op, mmv_dtype dt, bool mfma) {
    if (is_spmv(op)) return TSpmv::kMaxCpw;
    switch (dt) {
        case MMV_F32_F32: return row_form_cpw_of<TF32>(op, mfma);
        case MMV_F16_F32: return row_form_cpw_of<TF16>(op, mfma);
        case MMV_BF16_F32: return row_form_cpw_of<TBF16>(op, mfma);
        case MMV_I8_I32: return row_form_cpw_of<TI8>(op, mfma);
        case MMV_U8_XOR: return row_form_cpw_of<TX8>(op, mfma);
        default: break;
    }
    return 1;
}
// Most chunks per wave of the segmented sum that speculates over whole chunks and streams through its spans
// (sum_tile; 0: this operation, type or variant has no such form).
inline int chunk_form_cpw(mmv_op op, mmv_dtype dt, bool mfma) {
    (void)mfma;   // both variants have it
    if (op != MMV_OP_SEGSUM) return 0;
    if (dt == MMV_I8_I32 && chunk_sum_kernel<TI8, kSum, true>()) return sum_cpw<TI8>();
    if (dt == MMV_U8_XOR && chunk_sum_kernel<TX8, kSum, true>()) return sum_cpw<TX8>();
    if (dt == MMV_F16_F32 && chunk_sum_kernel<TF16, kSum, true>()) return sum_cpw<TF16>();
    if (dt == MMV_BF16_F32 && chunk_sum_kernel<TBF16, kSum, true>()) return sum_cpw<TBF16>();
    return 0;
}
inline int waves_of(mmv_op op, mmv_dtype dt) {
    if (is_spmv(op)) return TSpmv::kWaves;
    switch (dt) {
        case MMV_F32_F32: return TF32::kWaves;
        case MMV_F16_F32: return TF16::kWaves;
        case MMV_BF16_F32: return TBF16::kWaves;
        case MMV_I8_I32: return TI8::kWaves;
        case MMV_U8_XOR: return TX8::kWaves;
        default: break;
    }
    return 1;
}
struct TilePlan {
    TileRegions reg;
    uint64_t tiles;        // all tiles (reg.num_tiles holds it when it fits 31 bits)
    uint32_t unit;         // elements of one chunk per wave
    uint32_t body_elems;   // elements of a tile in the middle of the vector
    bool chunk_form;       // segmented sum: the kernel that streams through long spans (sum_kernel) takes it
};
inline TilePlan tile_plan(mmv_op op, mmv_dtype dt, uint64_t n, bool mfma = true) {
    TilePlan p = {};
    const uint64_t unit = (uint64_t)waves_of(op, dt) * kChunkElems;  // one chunk per wave
    // A sum that fits one round of workgroups is bound by the life of one tile, and the tile that holds all its
    // values, publishes its aggregate and then walks its ends has the shorter life (workload 2, fp16 2^24: 12.4
    // against 15.5 us); longer vectors go to the kernel that streams.
    int cpw = row_form_cpw(op, dt, mfma);
    const int chunk_cpw = chunk_form_cpw(op, dt, mfma);
    p.chunk_form = chunk_cpw > 0 && (MMV_SHORT_SUMS_ROW_FORM == 0 || n > MMV_SHORT_SUMS_ROW_FORM * kResident * unit * (uint64_t)cpw);
    if (p.chunk_form) cpw = chunk_cpw;
    p.unit = (uint32_t)unit;
    TileRegions &R = p.reg;
    uint64_t tiles = 0, at = 0;
    auto add = [&](uint32_t c, uint64_t count) {   // `count` tiles of c chunks per wave from element `at` on
        if (count == 0) return;
        R.base[R.count] = at;
        R.first[R.count] = (uint32_t)tiles;
        R.cpw[R.count] = c;
        ++R.count;
        tiles += count;
        at += count * c * unit;
    };
    // The sum kernel of 8-bit inputs has four workgroups per compute unit, not two: a vector that is too long for
    // one round of 512 workgroups still gets one round, of up to 1024 (n = 2^27: 0.0485 -> 0.0445 ms whole call);
    // shorter ones keep the 512 longer tiles (as fast, and below the number of tiles that needs the prefix kernel).
    const uint64_t resident = p.chunk_form && dt == MMV_I8_I32 && n > kResident * unit * cpw ? 2 * kResident : kResident;
    if (n <= resident * unit * cpw) {
        // one round: equal tiles, as small as gives every resident workgroup at most one
        uint64_t c = (n + resident * unit - 1) / (resident * unit);
        if (c < 1) c = 1;
        if (c > (uint64_t)cpw) c = cpw;
        p.body_elems = (uint32_t)(unit * c);
        add((uint32_t)c, (n + unit * c - 1) / (unit * c));
    } else {
        p.body_elems = (uint32_t)(unit * cpw);
        // lengths of the short tiles: a quarter, a half and three quarters of the full length
        int steps[3], nsteps = 0;
        for (int q = 1; q <= 3; ++q) {
            const int c = cpw * q / 4;
            if (c >= 1 && c < cpw && (nsteps == 0 || steps[nsteps - 1] != c)) steps[nsteps++] = c;
        }
        uint64_t head = 0, tail = (uint64_t)MMV_TAIL_TILES * unit;   // elements in the short tiles of both ends
        for (int i = 0; i < nsteps; ++i) {
            head += (uint64_t)MMV_HEAD_GROUP * steps[i] * unit;
            if (steps[i] >= 2) tail += (uint64_t)MMV_TAIL_GROUP * steps[i] * unit;
        }
        const bool graded = nsteps > 0 && head + tail <= n;
        if (!graded) head = 0, tail = (uint64_t)MMV_TAIL_TILES * unit < n ? (uint64_t)MMV_TAIL_TILES * unit : n;
        if (graded)
            for (int i = 0; i < nsteps; ++i) add((uint32_t)steps[i], MMV_HEAD_GROUP);
        add((uint32_t)cpw, (n - head - tail) / (unit * cpw));
        if (graded)
            for (int i = nsteps - 1; i >= 0; --i)
                if (steps[i] >= 2) add((uint32_t)steps[i], MMV_TAIL_GROUP);
        if (cpw > 1 || R.count == 0) {
            add(1u, (n - at + unit - 1) / unit);          // what is left, the last tile ragged
        } else {
            tiles += (n - at + unit - 1) / unit;          // (tiles of one chunk per wave throughout: one region)
        }
    }
    p.tiles = tiles;
    R.num_tiles = (uint32_t)(tiles < 0x7fffffffull ? tiles : 0x7fffffffull);
    return p;
}
// (for sizing: the variant with the shorter tiles needs more descriptors)
inline uint64_t tiles_for(uint64_t n, mmv_op op, mmv_dtype dt) {
    const uint64_t a = tile_plan(op, dt, n, true).tiles, b = tile_plan(op, dt, n, false).tiles;
    return a > b ? a : b;
}
inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }
inline bool aligned4(const void *p) { return ((uintptr_t)p & 3u) == 0; }

struct WsLayout {
    size_t desc_v, desc_c, span_c, packed, total;
};

WsLayout ws_layout(mmv_op op, mmv_dtype dt, mmv_flag_fmt ff, uint64_t n) {
    WsLayout L;
    const uint64_t t = tiles_for(n, op, dt);
    size_t off = kHdrBytes;
    L.desc_v = off;
    off += round256(t * 8);
    L.desc_c = off;   // counts of segment starts: per tile, and (segmented sum) per wave span
    if (op == MMV_OP_SEGSUM || op == MMV_OP_SPMV_CSR) off += round256(t * 8);
    L.span_c = off;
    if (op == MMV_OP_SEGSUM) off += round256(t * 4 * (uint64_t)waves_of(op, dt));
    L.packed = off;
    if (is_spmv(op) || (ff == MMV_FLAGS_U8 && op != MMV_OP_SCAN)) off += round256(((n + 63) / 64) * 8);
    L.total = off;
    return L;
}

// Workspace of COMPRESS: header, one count descriptor per tile, packed mask if the caller gave bytes.
struct CompressLayout {
    size_t desc, packed, total;
    uint64_t tiles;
};
CompressLayout compress_layout(mmv_flag_fmt ff, uint64_t n) {
    CompressLayout L;
    L.tiles = (n + compress_tile(n) - 1) / compress_tile(n);
    size_t off = kHdrBytes;
    L.desc = off;
    off += round256(L.tiles * 8);
    L.packed = off;
    if (ff == MMV_FLAGS_U8) off += round256(((n + 63) / 64) * 8);
    L.total = off;
    return L;
}

// Workspaces of the un-fused compositions: the sub-workspaces of the primitives they call and
// their intermediate vectors, one after the other (every offset a multiple of 256).
struct ScdLayout {
    size_t scan_ws, xhat, packed, fminus, compress_ws, w, total;
};
ScdLayout scd_layout(mmv_dtype dt, mmv_flag_fmt ff, uint64_t n, uint64_t cap) {
    ScdLayout L;
    size_t off = 0;
    L.scan_ws = off;
    off += round256(ws_layout(MMV_OP_SCAN, dt, MMV_FLAGS_PACKED32, n).total);
    L.xhat = off;
    off += round256(n * 4);
    L.packed = off;
    if (ff == MMV_FLAGS_U8) off += round256(((n + 63) / 64) * 8);
    L.fminus = off;
    off += round256(((n + 63) / 64) * 8);
    L.compress_ws = off;
    off += round256(compress_layout(MMV_FLAGS_PACKED32, n).total);
    L.w = off;
    off += round256((cap < n ? cap : n) * 4 + 16);
    L.total = off;
    return L;
}
struct SscrLayout {
    size_t scan_ws_x, scan_ws_f, fhat, f8, packed, fminus, compress_ws, w, total;
};
SscrLayout sscr_layout(mmv_dtype dt, mmv_flag_fmt ff, uint64_t n) {
    SscrLayout L;
    size_t off = 0;
    L.scan_ws_x = off;
    off += round256(ws_layout(MMV_OP_SCAN, dt, MMV_FLAGS_PACKED32, n).total);
    L.scan_ws_f = off;
    off += round256(ws_layout(MMV_OP_SCAN, MMV_I8_I32, MMV_FLAGS_PACKED32, n).total);
    L.fhat = off;
    off += round256(n * 4);
    L.f8 = off;
    off += round256(n + 16);   // flags as one 0 / 1 byte per element for SCAN(f)
    L.packed = off;
    if (ff == MMV_FLAGS_U8) off += round256(((n + 63) / 64) * 8);
    L.fminus = off;
    off += round256(((n + 63) / 64) * 8);
    L.compress_ws = off;
    off += round256(compress_layout(MMV_FLAGS_PACKED32, n).total);
    L.w = off;
    off += round256(n * 4 + 16);   // one entry per segment, at most n
    L.total = off;
    return L;
}
// CSR SpMV: the main kernel's workspace (flags over the non-zeros included), the mask of rows
// with entries, their indices (rowmap) and the workspace of the COMPRESS that makes them.
struct CsrLayout {
    size_t main_ws, rowmask, rowmap, rowcount, compress_ws, total;
};
CsrLayout csr_layout(uint64_t n_rows, uint64_t nnz) {
    CsrLayout L;
    size_t off = 0;
    L.main_ws = off;   // the two workspaces that hold tickets and descriptors lie next to each other:
    off += round256(ws_layout(MMV_OP_SPMV_CSR, MMV_F32_F32, MMV_FLAGS_PACKED32, nnz).total);
    L.compress_ws = off;   // one fill clears both (and the flag words between them)
    off += round256(compress_layout(MMV_FLAGS_PACKED32, n_rows).total);
    L.rowmask = off;
    off += round256(((n_rows + 63) / 64) * 8);
    L.rowmap = off;
    off += round256(n_rows * 4 + 16);
    L.rowcount = off;
    off += 256;
    L.total = off;
    return L;
}

// Optional instrumentation (mmv_set_kernel_events): events recorded right before and
// right after the main kernel of a call made by this host thread.
thread_local hipEvent_t tl_ev_start = nullptr, tl_ev_stop = nullptr;

// Workgroups of `kernel` that the current device holds at once (0 when a query fails).  `cache` is the
// caller's table for this kernel, one word per device (0 = not asked yet, else the value + 1): a fixed
// array per kernel instantiation, so nothing grows and nothing is allocated after the library is loaded.
constexpr int kMaxDevices = 64;
uint32_t resident_workgroups(const void *kernel, int threads, std::atomic<uint32_t> (&cache)[kMaxDevices]) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
    const uint32_t known = cache[dev].load(std::memory_order_relaxed);
    if (known) return known - 1u;
    int per_cu = 0, cus = 0;
    uint32_t value = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && per_cu > 0 && cus > 0)
        value = (uint32_t)per_cu * (uint32_t)cus;
    cache[dev].store(value + 1u, std::memory_order_relaxed);   // (two threads asking at once store the same value)
    return value;
}

template <typename TT, int kOp, bool kMfma> hipError_t launch_variant(Params P, bool chunk_form, hipStream_t s) {
    static std::atomic<uint32_t> occupancy[2][kMaxDevices];
    void (*kernel)(Params, const uint32_t *) = seg_kernel<TT, kOp, kMfma>;
    if constexpr (chunk_sum_kernel<TT, kOp, kMfma>()) {
        if (chunk_form) kernel = sum_kernel<TT, kMfma>;
    }
    const uint32_t resident = resident_workgroups((const void *)kernel, TT::kWaves * 64, occupancy[chunk_form ? 1 : 0]);
    P.first_round = P.num_tiles < resident ? P.num_tiles : resident;
    // SpMV: the workgroups of the first round start spread over about one tile time.  Started together
    // they stay in step (load, gather, compute all at the same time) and the memory pipe idles half the
    // time; measured 4 to 7 % on the long SpMV kernels, nothing on the scans.
    P.stagger_wgs = resident;
    P.stagger_ticks = ((kOp == kSpmv || kOp == kSpmvCsr) && P.num_tiles > resident) ? MMV_SPMV_STAGGER_US * 100u : 0u;
    kernel<<<P.num_tiles, TT::kWaves * 64, 0, s>>>(P, P.hdr + kHdrHints);
    return hipGetLastError();
}

template <typename TT, int kOp>
hipError_t launch_seg(Params P, mmv_variant v, hipStream_t s) {
    const TilePlan plan = tile_plan((mmv_op)kOp, TT::kDtype, P.n, v == MMV_VARIANT_MFMA);
    if (plan.tiles > 0x7fffffffull) return hipErrorInvalidValue;
    P.num_tiles = (uint32_t)plan.tiles;
    P.reg = plan.reg;
    if (tl_ev_start && hipEventRecord(tl_ev_start, s) != hipSuccess) return hipErrorUnknown;
    if (v == MMV_VARIANT_MFMA) {
        if (launch_variant<TT, kOp, true>(P, plan.chunk_form, s) != hipSuccess) return hipErrorUnknown;
    } else {
        if (launch_variant<TT, kOp, false>(P, plan.chunk_form, s) != hipSuccess) return hipErrorUnknown;
    }
    const hipError_t e = hipGetLastError();
    if (tl_ev_stop && hipEventRecord(tl_ev_stop, s) != hipSuccess) return hipErrorUnknown;
    return e;
}

template <int kOp> hipError_t launch_dt(const Params &P, mmv_dtype dt, mmv_variant v, hipStream_t s) {
    switch (dt) {
        case MMV_F32_F32: return launch_seg<TF32, kOp>(P, v, s);
        case MMV_F16_F32: return launch_seg<TF16, kOp>(P, v, s);
        case MMV_BF16_F32: return launch_seg<TBF16, kOp>(P, v, s);
        case MMV_I8_I32: return launch_seg<TI8, kOp>(P, v, s);
        case MMV_U8_XOR: return launch_seg<TX8, kOp>(P, v, s);
        default: break;
    }
    return hipErrorInvalidValue;
}

int grid_for(uint64_t items_per_thread_total) {
    uint64_t blocks = (items_per_thread_total + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 2048) blocks = 2048;
    return (int)blocks;
}

bool valid_dtype(int dt) { return dt >= 0 && dt <= 4; }
bool valid_ff(int ff) { return ff == 0 || ff == 1; }
bool valid_variant(int v) { return v == 0 || v == 1; }
bool valid_elem(int et) { return et == 0 || et == 1; }
constexpr uint64_t kMaxN = 1ull << 40;

// Common part of scan and sum: checks, workspace reset, flag packing.
mmv_status prepare(mmv_op op, const void *d_x, const void *d_flags, uint64_t n, mmv_dtype dt, mmv_flag_fmt ff,
                   mmv_variant v, void *d_ws, size_t ws_bytes, hipStream_t s, Params &P) {
    if (!valid_dtype(dt) || !valid_ff(ff) || !valid_variant(v) || n > kMaxN) return MMV_ERR_INVALID_ARG;
    if (!d_x || !d_flags) return MMV_ERR_NULL;
    if (!aligned16(d_x) || !aligned16(d_flags)) return MMV_ERR_INVALID_ARG;
    if (!d_ws) return MMV_ERR_NULL;
    const WsLayout L = ws_layout(op, dt, ff, n);
    if (((uintptr_t)d_ws & 255u) != 0 || ws_bytes < L.total) return MMV_ERR_WORKSPACE;
    char *ws = (char *)d_ws;
    P.x = d_x;
    P.n = n;
    P.hdr = (uint32_t *)ws;
    P.desc_v = (uint64_t *)(ws + L.desc_v);
    P.num_tiles = (uint32_t)tiles_for(n, op, dt);
    if (op != MMV_OP_SEGSUM) {   // the segmented sum zeroes them in its tile-count kernel
        const uint64_t zero_words = L.packed / 4;  // header + descriptors
        fill_zero_kernel<<<grid_for(zero_words), 256, 0, s>>>((uint32_t *)ws, zero_words, nullptr, 0);
        if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    }
    if (ff == MMV_FLAGS_U8) {
        const uint64_t nwords = (n + 31) / 32;
        uint32_t *packed = (uint32_t *)(ws + L.packed);
        pack_flags_kernel<<<grid_for(nwords), 256, 0, s>>>((const uint8_t *)d_flags, n, packed, nwords);
        if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
        P.fw = packed;
    } else {
        P.fw = (const uint32_t *)d_flags;
    }
    return MMV_OK;
}

// Turns timing events off for the sub-calls of a composition (each would re-record them).
struct EventsOff {
    hipEvent_t a, b;
    EventsOff() : a(tl_ev_start), b(tl_ev_stop) { tl_ev_start = tl_ev_stop = nullptr; }
    ~EventsOff() {
        tl_ev_start = a;
        tl_ev_stop = b;
    }
};

// SCAN on an input that is already checked; first_one makes element 0 count as 1 (flag bytes).
mmv_status scan_impl(const void *d_x, uint64_t n, void *d_z, mmv_dtype dt, mmv_variant v, void *d_ws,
                     size_t ws_bytes, hipStream_t s, bool first_one) {
    const WsLayout L = ws_layout(MMV_OP_SCAN, dt, MMV_FLAGS_PACKED32, n);
    if (((uintptr_t)d_ws & 255u) != 0 || ws_bytes < L.total) return MMV_ERR_WORKSPACE;
    char *ws = (char *)d_ws;
    Params P = {};
    P.x = d_x;
    P.n = n;
    P.z = d_z;
    P.hdr = (uint32_t *)ws;
    P.desc_v = (uint64_t *)(ws + L.desc_v);
    P.first_one = first_one ? 1u : 0u;
    const uint64_t zero_words = L.total / 4;
    fill_zero_kernel<<<grid_for(zero_words), 256, 0, s>>>((uint32_t *)ws, zero_words, nullptr, 0);
    if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    return launch_dt<kPlainScan>(P, dt, v, s) == hipSuccess ? MMV_OK : MMV_ERR_HIP;
}

// COMPRESS on checked arguments; d_x == nullptr compresses the positions.
mmv_status compress_impl(const void *d_x, const void *d_mask, uint64_t n, void *d_out, uint64_t out_capacity,
                         uint64_t *d_count, mmv_flag_fmt ff, void *d_ws, size_t ws_bytes, hipStream_t s,
                         bool ws_is_reset = false, const uint32_t *d_needed = nullptr) {
    const CompressLayout L = compress_layout(ff, n);
    if (((uintptr_t)d_ws & 255u) != 0 || ws_bytes < L.total) return MMV_ERR_WORKSPACE;
    if (L.tiles > 0x7fffffffull) return MMV_ERR_INVALID_ARG;
    char *ws = (char *)d_ws;
    if (!ws_is_reset) {
        const uint64_t zero_words = L.packed / 4;
        fill_zero_kernel<<<grid_for(zero_words), 256, 0, s>>>((uint32_t *)ws, zero_words, nullptr, 0);
        if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    }
    const uint32_t *mw = (const uint32_t *)d_mask;
    if (ff == MMV_FLAGS_U8) {
        const uint64_t nwords = (n + 31) / 32;
        uint32_t *packed = (uint32_t *)(ws + L.packed);
        pack_flags_kernel<<<grid_for(nwords), 256, 0, s>>>((const uint8_t *)d_mask, n, packed, nwords);
        if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
        mw = packed;
    }
    if (tl_ev_start && hipEventRecord(tl_ev_start, s) != hipSuccess) return MMV_ERR_HIP;
    // the workgroups that are resident from the start take the tile of their own index, the others a ticket
    static std::atomic<uint32_t> occupancy[4][kMaxDevices];
    void (*kernel)(const uint32_t *, const uint32_t *, uint64_t, uint32_t *, uint64_t, uint64_t *, uint32_t *, uint64_t *,
                   uint32_t, const uint32_t *, uint32_t) = compress_kernel<64, 1>;
    int which = 1;
    if (compress_words(n) == 16) kernel = compress_kernel<16, 1>, which = 0;
    else if (compress_groups(n) == 2) kernel = compress_kernel<64, 2>, which = 2;
    else if (compress_groups(n) == 4) kernel = compress_kernel<64, 4>, which = 3;
    const uint32_t resident = resident_workgroups((const void *)kernel, kCompressWaves * 64, occupancy[which]);
    const uint32_t first_round = (uint32_t)L.tiles < resident ? (uint32_t)L.tiles : resident;
    kernel<<<(unsigned)L.tiles, kCompressWaves * 64, 0, s>>>((const uint32_t *)d_x, mw, n, (uint32_t *)d_out, out_capacity,
                                                             d_count, (uint32_t *)ws, (uint64_t *)(ws + L.desc),
                                                             (uint32_t)L.tiles, d_needed, first_round);
    const hipError_t e = hipGetLastError();
    if (tl_ev_stop && hipEventRecord(tl_ev_stop, s) != hipSuccess) return MMV_ERR_HIP;
    return e == hipSuccess ? MMV_OK : MMV_ERR_HIP;
}

mmv_status diff_impl(const void *d_x, uint64_t n, void *d_z, mmv_elem et, hipStream_t s,
                     const uint64_t *d_limit = nullptr) {
    const uint64_t blocks = (n + 1023) / 1024;
    if (blocks > 0x7fffffffull) return MMV_ERR_INVALID_ARG;
    if (tl_ev_start && hipEventRecord(tl_ev_start, s) != hipSuccess) return MMV_ERR_HIP;
    if (et == MMV_ELEM_I32)
        diff_kernel<uint32_t><<<(unsigned)blocks, 256, 0, s>>>((const uint32_t *)d_x, n, (uint32_t *)d_z, d_limit);
    else
        diff_kernel<float><<<(unsigned)blocks, 256, 0, s>>>((const uint32_t *)d_x, n, (uint32_t *)d_z, d_limit);
    const hipError_t e = hipGetLastError();
    if (tl_ev_stop && hipEventRecord(tl_ev_stop, s) != hipSuccess) return MMV_ERR_HIP;
    return e == hipSuccess ? MMV_OK : MMV_ERR_HIP;
}

mmv_status revert_impl(const void *d_xhat, const int32_t *d_fhat, const void *d_w, uint64_t n, uint64_t nw,
                       void *d_z, mmv_elem et, hipStream_t s) {
    const uint64_t blocks = (n + 1023) / 1024;
    if (blocks > 0x7fffffffull) return MMV_ERR_INVALID_ARG;
    if (tl_ev_start && hipEventRecord(tl_ev_start, s) != hipSuccess) return MMV_ERR_HIP;
    if (et == MMV_ELEM_I32)
        revert_kernel<uint32_t><<<(unsigned)blocks, 256, 0, s>>>((const uint32_t *)d_xhat, d_fhat, (const uint32_t *)d_w,
                                                                  n, nw, (uint32_t *)d_z);
    else
        revert_kernel<float><<<(unsigned)blocks, 256, 0, s>>>((const uint32_t *)d_xhat, d_fhat, (const uint32_t *)d_w, n,
                                                               nw, (uint32_t *)d_z);
    const hipError_t e = hipGetLastError();
    if (tl_ev_stop && hipEventRecord(tl_ev_stop, s) != hipSuccess) return MMV_ERR_HIP;
    return e == hipSuccess ? MMV_OK : MMV_ERR_HIP;
}

}  // namespace
