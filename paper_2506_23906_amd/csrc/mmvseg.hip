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

#include <mutex>
#include <vector>

#include "mmvseg.h"

namespace {

// Tunables (the defaults are the measured best on MI355X; -D overrides are for experiments).
#ifndef MMV_WAVES
#define MMV_WAVES 8      // waves per workgroup (int8)
#endif
#ifndef MMV_WAVES_F16
#define MMV_WAVES_F16 8
#endif
#ifndef MMV_WAVES_F32
#define MMV_WAVES_F32 8
#endif
#ifndef MMV_WAVES_SPMV
#define MMV_WAVES_SPMV 8
#endif
#ifndef MMV_CPW_I8
#define MMV_CPW_I8 4     // most chunks per wave, int8 inputs (6 spills registers)
#endif
#ifndef MMV_CPW_F16
#define MMV_CPW_F16 2    // most chunks per wave, 16-bit inputs (4 spills registers)
#endif
#ifndef MMV_CPW_F32
#define MMV_CPW_F32 1    // most chunks per wave, fp32 inputs (2 spills registers)
#endif
#ifndef MMV_CPW_SPMV
#define MMV_CPW_SPMV 1
#endif
#ifndef MMV_UNROLL_CHUNKS
#define MMV_UNROLL_CHUNKS 1   // 1: the chunk loops of the sum / SpMV kernels are unrolled (see kUnrollChunks)
#endif
#ifndef MMV_MIN_WAVES_PER_SIMD
#define MMV_MIN_WAVES_PER_SIMD 4   // register budget: 512 / 4 = 128 VGPRs per lane
#endif
#ifndef MMV_SPMV_STAGGER_US
#define MMV_SPMV_STAGGER_US 15   // SpMV: start times of the first round spread over this many microseconds
#endif
#ifndef MMV_KEEP_ROWS
#define MMV_KEEP_ROWS 1   // 1: single-chunk waves of the matrix-core variant keep their row scans in LDS (see kKeepRows)
#endif
#ifndef MMV_DPP_SCAN
#define MMV_DPP_SCAN 1   // 1: the sum-type kernels exchange lanes with DPP moves and v_permlane32_swap, 0: with lane shuffles through the LDS hardware
#endif
#ifndef MMV_ROLL_STEP
#define MMV_ROLL_STEP 2
#endif
#ifndef MMV_LOAD_PRIO
#define MMV_LOAD_PRIO 1   // wave priority while a workgroup takes its ticket and issues its loads (0: off)
#endif
#ifndef MMV_MIN_TILES
#define MMV_MIN_TILES 512   // workgroups resident at once: 2 per compute unit (LDS)
#endif

constexpr int kS = 32;                          // row length = MFMA tile edge
constexpr int kRowsPerChunk = 64;               // a chunk = 64 rows, one per lane = two 32x32 tiles
constexpr int kChunkElems = kS * kRowsPerChunk; // 2048
constexpr int kRowStride = 36;                  // dwords per LDS row: 4 meta + 32 values
constexpr int kSlotF = 0;                       // flag word of the row
constexpr int kSlotNegCarry = 2;                // minus the carry into the row
constexpr int kSlotZero = 3;                    // x-bar(-1) = 0
constexpr int kRowData = 4;

constexpr uint32_t kHdrTicket = 0;              // workspace header words
constexpr uint32_t kHdrError = 1;
constexpr uint32_t kHdrHints = 32;              // first of the words the SpMV kernels read as hints (a cache line of
                                                // their own: the line of the ticket is busy with atomics):
constexpr uint32_t kHdrEmptyRows = 32;          // CSR SpMV: set when some row of the matrix has no entries
constexpr uint32_t kHdrColumnRuns = 33;         // SpMV: set when neighbouring entries mostly have consecutive columns
constexpr size_t kHdrBytes = 256;

constexpr uint64_t kStatusInvalid = 0;          // descriptor not written yet
constexpr uint64_t kStatusAggregate = 1;        // payload = aggregate of a tile without any flag
constexpr uint64_t kStatusPrefix = 2;           // payload = carry out of the tile, look-back stops here
constexpr uint32_t kMaxSpins = 1u << 20;        // bounded wait, then the status word is set

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef short v8s __attribute__((ext_vector_type(8)));

// What a kernel instantiation computes (values match mmv_op where there is one):
//   kScan       segmented inclusive scan
//   kSum        segmented sum (one output per segment, index = number of segment ends before it)
//   kSpmv       row-sorted COO SpMV: products val * x[col], sums scattered to y[row]
//   kPlainScan  unsegmented inclusive scan (no flag vector: every row aggregate is carried on)
//   kSpmvCsr    CSR SpMV: as kSpmv, but the sum of the k-th segment goes to y[rowmap[k]]
enum Op { kScan = 0, kSum = 1, kSpmv = 2, kPlainScan = 3, kSpmvCsr = 7 };

struct Params {
    const void *x;          // values (scan, sum) / val (spmv)
    const uint32_t *fw;     // packed flag words (scan, sum)
    uint64_t n;             // elements / nnz
    void *z;                // scan output
    void *out;              // sum output
    uint64_t out_cap;
    uint64_t *nseg;
    const int32_t *row;     // spmv (coo)
    const uint32_t *rowmap; // spmv (csr): row index of the k-th non-empty row
    uint32_t first_one;     // plain scan of a flag vector: element 0 counts as 1 whatever it holds
    const int32_t *col;
    const float *xv;
    float *y;
    uint32_t *hdr;          // workspace header
    uint64_t *desc_v;       // value descriptors, one per tile
    const uint32_t *tile_count;  // sum: segment starts per tile (position 0 not counted), or ...
    uint32_t count_is_prefix;    // ... their exclusive prefix sums already (long vectors)
    uint32_t num_tiles;
    uint32_t big_tiles;     // tiles [0, big_tiles) have the full number of chunks per wave ...
    uint32_t tail_cpw;      // ... the rest have this many (shorter tiles at the end shorten the tail)
    uint32_t ordered;       // the whole grid is resident at once: workgroup b takes tile b, no ticket
    uint32_t stagger_wgs;   // workgroups [0, stagger_wgs) start after a delay of up to ...
    uint32_t stagger_ticks; // ... this many ticks of the 100 MHz clock, spread evenly over them
#ifdef MMV_TRACE
    uint64_t *trace;        // 8 timestamps per tile (development builds only)
#endif
};

#ifdef MMV_TRACE
#define MMV_STAMP(k)                                                                     \
    do {                                                                                 \
        if (tid == 0 && P.trace) P.trace[(uint64_t)tile * 8 + (k)] = wall_clock64();     \
    } while (0)
#else
#define MMV_STAMP(k) do { } while (0)
#endif

// ---- small helpers -----------------------------------------------------------------------

template <typename T> __device__ __forceinline__ T from_bits(uint32_t b) { return __builtin_bit_cast(T, b); }
template <typename T> __device__ __forceinline__ uint32_t to_bits(T v) { return __builtin_bit_cast(uint32_t, v); }

// Orders LDS traffic between the lanes of one wave (no s_barrier needed: a wave's
// LDS instructions execute in order).
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ uint64_t desc_load(const uint64_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void desc_store(uint64_t *p, uint64_t status, uint32_t payload) {
    __hip_atomic_store(p, (status << 62) | payload, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Data-parallel-primitive move: every lane reads the lane the control word names (row_shr n = 0x110 + n
// inside rows of 16 lanes, row_bcast 15 / 31 = 0x142 / 0x143, wave_shr 1 = 0x138); a lane that has
// no source, or whose row of lanes is not in kRowMask, reads 0.
template <int kCtrl, int kRowMask> __device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, kCtrl, kRowMask, 0xF, false);
}

// Both halves of the wave, each broadcast to all 64 lanes: lo[l] = v[l mod 32], hi[l] = v[32 + l mod 32]
// (one v_permlane32_swap, no LDS hardware).
// Lane exchanges come in two forms: through the vector ALU (DPP moves, v_permlane32_swap) or through
// the LDS hardware (ds_bpermute: what __shfl compiles to).  The ALU form has a tenth of the latency and
// made the segmented sum 10 % faster; the scan kernels, which wait for memory anyway, ran 0.9 % slower
// with it (the extra ALU instructions compete with the address arithmetic of the stores) and keep the
// LDS form.  kAlu selects.
struct Halves {
    uint32_t lo, hi;
};
template <bool kAlu> __device__ __forceinline__ Halves wave_halves(uint32_t v, int lane) {
    if constexpr (kAlu) {
        const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
        return {(uint32_t)r[0], (uint32_t)r[1]};
    } else {
        const uint32_t o = __shfl_xor(v, 32);
        return {lane < 32 ? v : o, lane < 32 ? o : v};
    }
}

// Sum over the 64 lanes, the same value in every lane: DPP adds inside the rows of 16 lanes, row totals
// passed on with row_bcast 15 / 31, the total read from lane 63.
template <typename T, bool kAlu = true> __device__ __forceinline__ T wave_sum(T v) {
    if constexpr (!kAlu) {
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) v += from_bits<T>(__shfl_xor(to_bits(v), d));
        return v;
    }
    v += from_bits<T>(dpp_or_zero<0x111, 0xF>(to_bits(v)));
    v += from_bits<T>(dpp_or_zero<0x112, 0xF>(to_bits(v)));
    v += from_bits<T>(dpp_or_zero<0x114, 0xF>(to_bits(v)));
    v += from_bits<T>(dpp_or_zero<0x118, 0xF>(to_bits(v)));
    v += from_bits<T>(dpp_or_zero<0x142, 0xA>(to_bits(v)));
    v += from_bits<T>(dpp_or_zero<0x143, 0xC>(to_bits(v)));
    return from_bits<T>((uint32_t)__builtin_amdgcn_readlane((int)to_bits(v), 63));
}

// Sum of the payloads of the predecessor tiles back to (and including) the first
// one whose descriptor says "prefix".  The whole wave polls 64 descriptors at a
// time.  Tile -1 counts as prefix 0, so the loop always ends there at the latest.
// (Polling 128 or 256 descriptors per round trip was measured 3-9 % slower on long
// chains: the polls are served by the memory side and compete with the streams,
// and in steady state the nearest "prefix" is within 64 tiles anyway.)
template <typename T, bool kAlu = true>
__device__ T lookback(const uint64_t *desc, int tile, int lane, uint32_t *hdr) {
    T carry = T(0);
    int pos = tile - 1;
    uint32_t spins = 0;
    while (true) {
        const int idx = pos - lane;
        const uint64_t d = idx >= 0 ? desc_load(desc + idx) : (kStatusPrefix << 62);
        const uint32_t st = (uint32_t)(d >> 62);
        const uint64_t invalid = __ballot(st == kStatusInvalid);
        const uint64_t stop = __ballot(st == kStatusPrefix);
        const int first_stop = stop ? (__ffsll((unsigned long long)stop) - 1) : 64;
        const uint64_t need = first_stop >= 63 ? ~0ull : ((2ull << first_stop) - 1ull);
        if (invalid & need) {
            if (++spins > kMaxSpins) {
                if (lane == 0) __hip_atomic_store(hdr + kHdrError, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(2);
            continue;
        }
        const T v = lane <= first_stop ? from_bits<T>((uint32_t)d) : T(0);
        carry += wave_sum<T, kAlu>(v);
        if (stop) break;
        pos -= 64;
    }
    return carry;
}

// ---- element types ------------------------------------------------------------------------------

struct TI8 {
    typedef int8_t in_t;
    typedef uint32_t acc_t;  // int32 with wrap-around
    static constexpr int kEpl = 16;  // elements per 128-bit load
    static constexpr int kMaxCpw = MMV_CPW_I8;  // most chunks of 2048 elements a wave takes (raw inputs sit in registers)
    static constexpr int kWaves = MMV_WAVES;
    static constexpr mmv_dtype kDtype = MMV_I8_I32;
    static __device__ __forceinline__ acc_t widen(in_t v) { return (acc_t)(int32_t)v; }
};
struct TF16 {
    typedef _Float16 in_t;
    typedef float acc_t;
    static constexpr int kEpl = 8;
    static constexpr int kMaxCpw = MMV_CPW_F16;
    static constexpr int kWaves = MMV_WAVES_F16;
    static constexpr mmv_dtype kDtype = MMV_F16_F32;
    static __device__ __forceinline__ acc_t widen(in_t v) { return (float)v; }
};
struct TBF16 {
    typedef __bf16 in_t;
    typedef float acc_t;
    static constexpr int kEpl = 8;
    static constexpr int kMaxCpw = MMV_CPW_F16;
    static constexpr int kWaves = MMV_WAVES_F16;
    static constexpr mmv_dtype kDtype = MMV_BF16_F32;
    static __device__ __forceinline__ acc_t widen(in_t v) { return (float)v; }
};
struct TF32 {
    typedef float in_t;
    typedef float acc_t;
    static constexpr int kEpl = 4;
    static constexpr int kMaxCpw = MMV_CPW_F32;
    static constexpr int kWaves = MMV_WAVES_F32;
    static constexpr mmv_dtype kDtype = MMV_F32_F32;
    static __device__ __forceinline__ acc_t widen(in_t v) { return v; }
};
struct TSpmv : TF32 {  // COO SpMV: values and column indices both sit in registers, so fewer chunks
    static constexpr int kMaxCpw = MMV_CPW_SPMV;
    static constexpr int kWaves = MMV_WAVES_SPMV;
};
struct TInt {  // column indices of the COO matrix, loaded in the same layout as its values
    typedef int32_t in_t;
    static constexpr int kEpl = 4;
};

// ---- raw inputs of one wave chunk (2048 elements), kept in registers ---------------------------------
//
// A lane holds 2 * K 128-bit words, K = 1 (int8), 2 (fp16, bf16), 4 (fp32) per
// 32x32 tile.  They are loaded one tile ahead of their use (software pipeline of
// the persistent workgroup loop), so that HBM latency overlaps the previous
// tile's look-back and stores.
//
// Matrix-core layout: one 32x32 tile = 32 rows ("runs") of 32 consecutive
// elements.  D = A B with A = U_s^T (lower-triangular ones, M x K) and B = X^T
// (K x N, column n = run n): D(m, n) = sum_{k <= m} X(n, k) = x-bar at position m
// of run n.  Lane (c = lane % 32, h = lane / 32) holds row c of A and column c of
// B for the K indices half h owns; A and B use the same (half, register, byte) ->
// K map, so only "which positions does half h hold" has to agree between them.
// Result: acc[v] of lane (n, h) = D(8 (v / 4) + 4 h + v % 4, n).
//
// Shuffle layout (ablation): lane l holds kEpl consecutive elements, striped.

// 16- and 32-bit values are loaded striped in both variants (rows of 64 or 128 bytes would
// otherwise make every load instruction touch 32 cache lines for 1 KiB) and the matrix-core
// variant moves them into the operand layout through LDS (to_operand_layout).
template <typename TT, bool kMfma> __device__ __forceinline__ int raw_offset(int i, int lane) {
    constexpr int K = 16 / TT::kEpl;
    if (kMfma && K == 1) return 32 * (lane & 31) + 16 * (lane >> 5);  // int8: 32-byte rows, already contiguous
    return (1024 / K) * i + TT::kEpl * lane;
}

// One chunk from the striped layout (word w of lane l = elements (2048 / W) w + kEpl l ..,
// W = 2 K words per lane) to the operand layout, through the wave's LDS rows.
//   fp32 (K = 4): word 4t+q of lane (c, h) = positions 16h + 4q .. +3 of row 32t + c
//   16-bit (K = 2): word 2t+ks of lane (c, h) = positions 16ks + 8h .. +7 of row 32t + c
// The padded row strides keep the 128-bit accesses (almost) free of bank conflicts.
template <int K> __device__ __forceinline__ void to_operand_layout(v4u (&raw)[2 * K], uint32_t *rows, int lane);

template <> __device__ __forceinline__ void to_operand_layout<4>(v4u (&raw)[8], uint32_t *rows, int lane) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
        *reinterpret_cast<v4u *>(rows + (8 * i + (lane >> 3)) * kRowStride + kRowData + 4 * (lane & 7)) = raw[i];
    wave_lds_sync();
    const int c = lane & 31, h = lane >> 5;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int q = 0; q < 4; ++q)
            raw[4 * t + q] = *reinterpret_cast<const v4u *>(rows + (32 * t + c) * kRowStride + kRowData + 16 * h + 4 * q);
    wave_lds_sync();
}

template <> __device__ __forceinline__ void to_operand_layout<2>(v4u (&raw)[4], uint32_t *rows, int lane) {
    constexpr int kStride = 20;  // dwords per row of 32 halves (16) + padding
#pragma unroll
    for (int i = 0; i < 4; ++i)
        *reinterpret_cast<v4u *>(rows + (16 * i + (lane >> 2)) * kStride + 4 * (lane & 3)) = raw[i];
    wave_lds_sync();
    const int c = lane & 31, h = lane >> 5;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
            raw[2 * t + ks] = *reinterpret_cast<const v4u *>(rows + (32 * t + c) * kStride + 8 * ks + 4 * h);
    wave_lds_sync();
}

// 128 bits = 16 / sizeof(T) consecutive elements starting at element e0 (a multiple
// of 16 bytes); elements at or beyond n read as zero.  The aligned 16-byte block that
// holds the last element is read whole (it cannot straddle a page) and masked.
template <typename T> __device__ __forceinline__ v4u load128(const T *x, uint64_t e0, uint64_t n, bool full) {
    // streamed once: non-temporal, so that the inputs do not push the gather vector (spmv)
    // and the descriptors out of L2
    if (full) return __builtin_nontemporal_load(reinterpret_cast<const v4u *>(x + e0));
    v4u w = {0, 0, 0, 0};
    if (e0 < n) {
        w = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(x + e0));
        const uint64_t valid_bytes = (n - e0) * sizeof(T);
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int vb = valid_bytes >= 4u * d + 4u ? 4 : (valid_bytes > 4u * d ? (int)(valid_bytes - 4u * d) : 0);
            w[d] &= vb == 4 ? ~0u : ((1u << (8 * vb)) - 1u);
        }
    }
    return w;
}

// The 2 * K words of one chunk (two 32x32 tiles) starting at element chunk_base.
template <typename TT, bool kMfma>
__device__ __forceinline__ void load_raw(const typename TT::in_t *x, uint64_t chunk_base, uint64_t n, int lane,
                                         v4u (&raw)[2 * (16 / TT::kEpl)]) {
    constexpr int K = 16 / TT::kEpl;
    const bool full = chunk_base + kChunkElems <= n;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < K; ++i)
            raw[t * K + i] = load128(x, chunk_base + 1024u * t + raw_offset<TT, kMfma>(i, lane), n, full);
}

// ---- step 1, matrix-core form: x-bar of 32x32 tile t from the raw registers ------------------------------

template <typename TT> struct SpecMfma;

template <> struct SpecMfma<TI8> {
    static __device__ __forceinline__ void run(const v4u *raw, int lane, uint32_t (&acc)[16]) {
        const int c = lane & 31, h = lane >> 5;
        v4i a;  // bytes 4d..4d+3 = positions 16h+4d+j: one where position <= c
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            int cnt = c - (16 * h + 4 * d) + 1;
            cnt = cnt < 0 ? 0 : (cnt > 4 ? 4 : cnt);
            a[d] = cnt == 4 ? 0x01010101 : (int)(0x01010101u & ((1u << (8 * cnt)) - 1u));
        }
        v16i r = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        r = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, __builtin_bit_cast(v4i, raw[0]), r, 0, 0, 0);
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = (uint32_t)r[v];
    }
};

template <> struct SpecMfma<TF16> {
    // two K-steps of 16: in step ks half h supplies positions 16 ks + 8 h .. + 7
    static __device__ __forceinline__ void run(const v4u *raw, int lane, float (&acc)[16]) {
        const int c = lane & 31, h = lane >> 5;
        v16f r = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v8h a;
#pragma unroll
            for (int j = 0; j < 8; ++j) a[j] = (16 * ks + 8 * h + j <= c) ? (_Float16)1.0f : (_Float16)0.0f;
            r = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, __builtin_bit_cast(v8h, raw[ks]), r, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = r[v];
    }
};

template <> struct SpecMfma<TBF16> {
    static __device__ __forceinline__ void run(const v4u *raw, int lane, float (&acc)[16]) {
        const int c = lane & 31, h = lane >> 5;
        v16f r = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v8s a;
#pragma unroll
            for (int j = 0; j < 8; ++j) a[j] = (16 * ks + 8 * h + j <= c) ? (short)0x3F80 : (short)0;  // bf16 1.0
            r = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a),
                                                        __builtin_bit_cast(v8bf, raw[ks]), r, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = r[v];
    }
};

template <> struct SpecMfma<TF32> {
    // fp32 through the bf16 matrix pipe, exactly: every value is split into three bf16 pieces
    // (8 + 8 + 8 significand bits, x = hi + mid + lo with no rounding), the pieces are
    // multiplied by the 0/1 matrix (exact products) and accumulated in fp32.  Six
    // 32x32x16 instructions of 8 passes instead of sixteen 32x32x2 fp32 ones of 16 passes.
    // In K-step ks half h supplies positions 16 h + 8 ks .. + 7 (the lane's own words 2 ks, 2 ks + 1).
    static __device__ __forceinline__ void run(const v4u *raw, int lane, float (&acc)[16]) {
        const int c = lane & 31, h = lane >> 5;
        v16f r = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            // the eight values of this K-step (words 2 ks and 2 ks + 1), split and packed in pairs
            uint32_t hi[4], mid[4], lo[4];
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int pr = 0; pr < 2; ++pr) {
                    uint32_t ph[2], pm[2], pl[2];
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const uint32_t xb = raw[2 * ks + q][2 * pr + e];
                        ph[e] = xb & 0xFFFF0000u;
                        const float r1 = from_bits<float>(xb) - from_bits<float>(ph[e]);
                        pm[e] = to_bits(r1) & 0xFFFF0000u;
                        pl[e] = to_bits(r1 - from_bits<float>(pm[e]));  // at most 8 significant bits left
                    }
                    hi[2 * q + pr] = __builtin_amdgcn_perm(ph[1], ph[0], 0x07060302u);
                    mid[2 * q + pr] = __builtin_amdgcn_perm(pm[1], pm[0], 0x07060302u);
                    lo[2 * q + pr] = __builtin_amdgcn_perm(pl[1], pl[0], 0x07060302u);
                }
            v8s a;
#pragma unroll
            for (int j = 0; j < 8; ++j) a[j] = (16 * h + 8 * ks + j <= c) ? (short)0x3F80 : (short)0;  // bf16 1.0
            const v8bf ab = __builtin_bit_cast(v8bf, a);
            const v4u wl = {lo[0], lo[1], lo[2], lo[3]};
            const v4u wm = {mid[0], mid[1], mid[2], mid[3]};
            const v4u wh = {hi[0], hi[1], hi[2], hi[3]};
            r = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ab, __builtin_bit_cast(v8bf, wl), r, 0, 0, 0);
            r = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ab, __builtin_bit_cast(v8bf, wm), r, 0, 0, 0);
            r = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ab, __builtin_bit_cast(v8bf, wh), r, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = r[v];
    }
};

template <> struct SpecMfma<TSpmv> : SpecMfma<TF32> {};

// ---- steps 2-4 without the detour through LDS: row aggregates from the raw registers -----------------
//
// The aggregate of a row after the revert is x-bar(31) - x-bar(start - 1) = the sum of
// the elements from the row's last flag on.  In the matrix-core layout a lane holds 16
// consecutive positions of one row per 32x32 tile, so this is a masked dot product of
// its own elements plus one exchange with the lane that holds the other half.  Returns
// the aggregate of the row this lane owns (row r of the chunk for lane r).
template <typename TT> struct RowAgg;

__device__ __forceinline__ int last_flag_pos(uint32_t f) { return f ? 31 - __clz(f) : 0; }

template <> struct RowAgg<TI8> {
    template <bool kAlu> static __device__ __forceinline__ uint32_t run(const v4u *raw, uint32_t F, int lane) {
        const int h = lane >> 5;
        const Halves Fh = wave_halves<kAlu>(F, lane);   // flag words of rows c and 32 + c
        uint32_t tot[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int st = last_flag_pos(t ? Fh.hi : Fh.lo);
            // my 16 bytes are positions 16h .. 16h+15; the first k of them lie before the start and
            // get weight 0, the others weight 1: two 64-bit shifts of a word of ones
            int k = st - 16 * h;
            k = k < 0 ? 0 : (k > 16 ? 16 : k);
            const uint64_t ones = 0x0101010101010101ull;
            const uint64_t m_lo = k >= 8 ? 0ull : ones << (8 * k);
            const uint64_t m_hi = k >= 16 ? 0ull : ones << (8 * (k > 8 ? k - 8 : 0));
            int part = 0;
            part = __builtin_amdgcn_sdot4((int)raw[t][0], (int)(uint32_t)m_lo, part, false);
            part = __builtin_amdgcn_sdot4((int)raw[t][1], (int)(uint32_t)(m_lo >> 32), part, false);
            part = __builtin_amdgcn_sdot4((int)raw[t][2], (int)(uint32_t)m_hi, part, false);
            part = __builtin_amdgcn_sdot4((int)raw[t][3], (int)(uint32_t)(m_hi >> 32), part, false);
            const Halves ph = wave_halves<kAlu>((uint32_t)part, lane);
            tot[t] = ph.lo + ph.hi;
        }
        return lane < 32 ? tot[0] : tot[1];
    }
};

template <bool kBf16> struct RowAggHalf {
    template <bool kAlu> static __device__ __forceinline__ float run(const v4u *raw, uint32_t F, int lane) {
        typedef _Float16 v2h __attribute__((ext_vector_type(2)));
        typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
        constexpr uint32_t kOne = kBf16 ? 0x3F80u : 0x3C00u;
        const int h = lane >> 5;
        const Halves Fh = wave_halves<kAlu>(F, lane);   // flag words of rows c and 32 + c
        float tot[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int st = last_flag_pos(t ? Fh.hi : Fh.lo);
            float part = 0.0f;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int d = 0; d < 4; ++d) {  // positions 16ks+8h+2d and +1
                    const int p = 16 * ks + 8 * h + 2 * d;
                    const uint32_t mask = (p >= st ? kOne : 0u) | (p + 1 >= st ? kOne << 16 : 0u);
                    const uint32_t pair = raw[2 * t + ks][d];  // by value: bit_cast of a vector element miscompiles
                    if (kBf16)
                        part = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(v2bf, pair),
                                                               __builtin_bit_cast(v2bf, mask), part, false);
                    else
                        part = __builtin_amdgcn_fdot2(__builtin_bit_cast(v2h, pair), __builtin_bit_cast(v2h, mask),
                                                      part, false);
                }
            const Halves ph = wave_halves<kAlu>(to_bits(part), lane);
            tot[t] = from_bits<float>(ph.lo) + from_bits<float>(ph.hi);
        }
        return lane < 32 ? tot[0] : tot[1];
    }
};
template <> struct RowAgg<TF16> : RowAggHalf<false> {};
template <> struct RowAgg<TBF16> : RowAggHalf<true> {};

template <> struct RowAgg<TF32> {
    template <bool kAlu> static __device__ __forceinline__ float run(const v4u *raw, uint32_t F, int lane) {
        const int h = lane >> 5;
        const Halves Fh = wave_halves<kAlu>(F, lane);   // flag words of rows c and 32 + c
        float tot[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int st = last_flag_pos(t ? Fh.hi : Fh.lo);
            float part = 0.0f;
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int i = 0; i < 4; ++i)  // position 16h+4q+i
                    part += (16 * h + 4 * q + i >= st) ? from_bits<float>(raw[4 * t + q][i]) : 0.0f;
            const Halves ph = wave_halves<kAlu>(to_bits(part), lane);
            tot[t] = from_bits<float>(ph.lo) + from_bits<float>(ph.hi);
        }
        return lane < 32 ? tot[0] : tot[1];
    }
};
template <> struct RowAgg<TSpmv> : RowAgg<TF32> {};


// Writes the 16 results of a lane into the LDS rows of 32x32 tile t of this wave.
template <typename A>
__device__ __forceinline__ void store_spec_rows(uint32_t *rows, int t, int lane, const A (&acc)[16]) {
    const int c = lane & 31, h = lane >> 5;
    uint32_t *rp = rows + (32 * t + c) * kRowStride + kRowData + 4 * h;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        v4u w = {to_bits(acc[4 * q]), to_bits(acc[4 * q + 1]), to_bits(acc[4 * q + 2]), to_bits(acc[4 * q + 3])};
        *reinterpret_cast<v4u *>(rp + 8 * q) = w;
    }
}

// ---- step 1, vector-only form (ablation) --------------------------------------------------------------------
//
// Every lane prefix-sums its kEpl consecutive elements in registers and the
// 32 / kEpl lanes that share a row combine with lane shuffles.
template <typename TT> __device__ __forceinline__ typename TT::acc_t raw_elem(const v4u &w, int i);
template <> __device__ __forceinline__ uint32_t raw_elem<TI8>(const v4u &w, int i) {
    return (uint32_t)(int32_t)(int8_t)(w[i >> 2] >> (8 * (i & 3)));
}
template <> __device__ __forceinline__ float raw_elem<TF16>(const v4u &w, int i) {
    return (float)__builtin_bit_cast(_Float16, (unsigned short)(w[i >> 1] >> (16 * (i & 1))));
}
template <> __device__ __forceinline__ float raw_elem<TBF16>(const v4u &w, int i) {
    return from_bits<float>((w[i >> 1] >> (16 * (i & 1))) << 16);
}
template <> __device__ __forceinline__ float raw_elem<TF32>(const v4u &w, int i) { return from_bits<float>(w[i]); }
template <> __device__ __forceinline__ float raw_elem<TSpmv>(const v4u &w, int i) { return from_bits<float>(w[i]); }

template <typename TT, bool kAlu>
__device__ __forceinline__ void spec_shuffle_tile(const v4u *raw, int lane, uint32_t *rows, int t) {
    typedef typename TT::acc_t A;
    constexpr int kEpl = TT::kEpl;
    constexpr int K = 16 / kEpl;
    constexpr int kLpr = 32 / kEpl;  // lanes per row
    constexpr int kRowsPerLoad = 64 / kLpr;
#pragma unroll
    for (int ld = 0; ld < K; ++ld) {
        A p[kEpl];
        p[0] = raw_elem<TT>(raw[ld], 0);
#pragma unroll
        for (int i = 1; i < kEpl; ++i) p[i] = p[i - 1] + raw_elem<TT>(raw[ld], i);
        A inc = p[kEpl - 1];
        // prefix over the kLpr lanes of a row (a lane whose source lies in another row does not add)
        if constexpr (!kAlu) {
#pragma unroll
            for (int d = 1; d < kLpr; d <<= 1) {
                const A o = from_bits<A>(__shfl_up(to_bits(inc), d));
                if ((lane & (kLpr - 1)) >= d) inc += o;
            }
        } else {
        if constexpr (kLpr > 1) {
            const A o = from_bits<A>(dpp_or_zero<0x111, 0xF>(to_bits(inc)));
            if ((lane & (kLpr - 1)) >= 1) inc += o;
        }
        if constexpr (kLpr > 2) {
            const A o = from_bits<A>(dpp_or_zero<0x112, 0xF>(to_bits(inc)));
            if ((lane & (kLpr - 1)) >= 2) inc += o;
        }
        if constexpr (kLpr > 4) {
            const A o = from_bits<A>(dpp_or_zero<0x114, 0xF>(to_bits(inc)));
            if ((lane & (kLpr - 1)) >= 4) inc += o;
        }
        }
        const A ex = inc - p[kEpl - 1];
        uint32_t *rp = rows + (32 * t + kRowsPerLoad * ld + lane / kLpr) * kRowStride + kRowData + kEpl * (lane % kLpr);
#pragma unroll
        for (int q = 0; q < kEpl / 4; ++q) {
            v4u w = {to_bits(p[4 * q] + ex), to_bits(p[4 * q + 1] + ex), to_bits(p[4 * q + 2] + ex),
                     to_bits(p[4 * q + 3] + ex)};
            *reinterpret_cast<v4u *>(rp + 4 * q) = w;
        }
    }
}

// ---- the kernel ---------------------------------------------------------------------------------------
//
// One workgroup = one tile = kWaves waves x kCpw chunks x 2048 elements, taken from
// an atomic ticket counter (a tile only ever waits for tiles held by workgroups that
// are already running).  A same-address device-scope atomic costs about 11 ns on
// this chip and they serialise, which is why a ticket covers tens of thousands of
// elements.  Every wave owns a contiguous span of the tile and
//   A. loads all its inputs at once, then for each chunk computes the speculative
//      row scans (matrix cores), the row aggregates and their segmented scan; only
//      a few registers per chunk are kept, the row scans themselves are dropped;
//   -  the wave aggregates are combined and the tile's descriptor is published;
//   B. recomputes the row scans of each chunk from the raw registers (cheaper than
//      holding them: LDS is the scarce resource), reverts the mis-speculation, adds
//      the carries and stores.  Chunks that start after a flag of the tile go first;
//      chunks that continue a segment of an earlier tile go last, after wave 0 has
//      looked back for the carry of the predecessor tiles.
// The chunk loops of the scan kernels are rolled: the per-chunk registers are rotated so that
// the loop body always works on the first slots (unrolled, these kernels spill).

template <typename T, int N> __device__ __forceinline__ void rotate(T (&a)[N]) {
    const T first = a[0];
#pragma unroll
    for (int i = 0; i + 1 < N; ++i) a[i] = a[i + 1];
    a[N - 1] = first;
}
template <int N, int M> __device__ __forceinline__ void rotate_rows(v4u (&a)[N][M]) {
#pragma unroll
    for (int m = 0; m < M; ++m) {
        const v4u first = a[0][m];
#pragma unroll
        for (int i = 0; i + 1 < N; ++i) a[i][m] = a[i + 1][m];
        a[N - 1][m] = first;
    }
}

// LDS of one workgroup: the row buffers of the waves and the words the waves exchange.
template <int kWaves> struct SegShared {
    __attribute__((aligned(16))) uint32_t rows[kWaves][kRowsPerChunk * kRowStride];
    uint32_t wave_v[kWaves], wave_f[kWaves], wave_c[kWaves];
    uint32_t tile, carry_v, carry_c, ready;
};

// One tile, from the loads on.  kLateVal (SpMV only): the values are loaded behind the gathers of
// x[col] instead of beside the columns.
template <typename TT, int kOp, bool kMfma, bool kLateVal>
__device__ __forceinline__ void seg_tile(const Params &P, const uint32_t *__restrict__ hints, SegShared<TT::kWaves> &sm,
                                         const uint32_t tile) {
    typedef typename TT::acc_t A;
    typedef typename TT::in_t In;
    constexpr int kWaves = TT::kWaves;
    constexpr int kCpw = TT::kMaxCpw;            // most chunks a wave takes (register arrays)
    constexpr int K = 16 / TT::kEpl;             // 128-bit words per lane and 32x32 tile
    constexpr bool kScanLike = kOp == kScan || kOp == kPlainScan;   // every element is an output
    // The chunk loops are either rolled, with the per-chunk registers rotated so that the body always
    // works on the first slot(s) (about 45 moves per rotation and phase, small code), or unrolled.  Unrolled, the
    // scan kernels spill registers (measured: 100 to 700 bytes per lane) and so does the shuffle-only
    // int8 sum kernel with its four chunks; the other sum / SpMV kernels do not.
    constexpr bool kUnrollChunks = MMV_UNROLL_CHUNKS != 0 && !kScanLike && (kMfma || kCpw <= 2);
    // chunks per iteration of the chunk loops: all (unrolled), or MMV_ROLL_STEP with the registers
    // rotated by as many slots afterwards (the moves of a rotation do not depend on the distance)
    constexpr int kStep = kUnrollChunks ? kCpw : (kCpw >= 2 * MMV_ROLL_STEP && kCpw % MMV_ROLL_STEP == 0 ? MMV_ROLL_STEP : 1);
    // A wave with a single chunk (fp32, SpMV) keeps the row scans of phase A in its LDS rows for
    // phase B instead of making them a second time; with more chunks LDS holds only the last one made.
    // Matrix-core variant only: there it saves the second 3-way split and 50 registers (fp32 scan
    // 4-5 % faster); in the shuffle variant the same change was measured 3 % slower.
    constexpr bool kKeepRows = MMV_KEEP_ROWS != 0 && kCpw == 1 && kMfma;
    // lane exchanges through the vector ALU for the sum-type kernels and the 16-bit scans (measured 2 %
    // faster), through the LDS hardware for the int8 and fp32 scans (0.9 % faster / no difference)
    constexpr bool kAluLanes = MMV_DPP_SCAN != 0 && (!kScanLike || TT::kEpl == 8);
    constexpr bool kCounts = kOp == kSum || kOp == kSpmvCsr;        // output index = segment ordinal
    // the count of the segments before the tile comes from a table of per-tile counts made by a
    // small kernel before this one, so that no chunk has to wait for it
    constexpr bool kProduct = kOp == kSpmv || kOp == kSpmvCsr;      // values are val * x[col]

    // the wave index as a scalar: everything derived from it (the wave's span, chunk bases, the
    // "whole chunk inside the vector" tests, base addresses of loads and stores) then lives in scalar
    // registers and costs no vector instructions
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint64_t n = P.n;
    uint32_t *rows = sm.rows[wave];
    MMV_STAMP(1);
    // tiles at the end of the vector are shorter (fewer chunks per wave)
    const bool big_tile = tile < P.big_tiles;
    const int cpw_t = big_tile ? kCpw : (int)P.tail_cpw;
    const uint64_t tile_base =
        big_tile ? (uint64_t)tile * (kWaves * kCpw * kChunkElems)
                 : (uint64_t)P.big_tiles * (kWaves * kCpw * kChunkElems) +
                       (uint64_t)(tile - P.big_tiles) * ((uint64_t)kWaves * P.tail_cpw * kChunkElems);
    const uint64_t wave_base = tile_base + (uint64_t)wave * cpw_t * kChunkElems;

    // ---- all inputs of my span: flag word of my row and raw values (and columns) per chunk ----
    uint32_t F[kCpw];
    v4u raw[kCpw][2 * K];
    v4u rawc[kProduct ? kCpw : 1][2 * K];  // column indices (spmv)
#pragma unroll
    for (int c = 0; c < kCpw; ++c) {
        const uint64_t cb = wave_base + (uint64_t)c * kChunkElems;
        F[c] = 0;
        if (c < cpw_t) {
            const uint64_t rs = cb + 32u * lane;
            if constexpr (kOp != kPlainScan) {
                if (rs < n) F[c] = __builtin_nontemporal_load(P.fw + (rs >> 5));
            }
            if constexpr (kProduct) load_raw<TInt, kMfma>(P.col, cb, n, lane, rawc[c]);
            if constexpr (!kProduct || !kLateVal) load_raw<TT, kMfma>((const In *)P.x, cb, n, lane, raw[c]);
        }
    }

#if MMV_LOAD_PRIO
    __builtin_amdgcn_s_setprio(0);
#endif
    if constexpr (kOp == kPlainScan && sizeof(In) == 1) {
        // counting segment starts: position 0 always opens a segment (byte 0 of the first word, both layouts)
        if (P.first_one && tile == 0 && tid == 0) raw[0][0][0] = (raw[0][0][0] & ~0xFFu) | 1u;
    }

    // CSR SpMV: without empty rows the k-th segment is row k and the row map was not made
    bool rows_dense = false;
    if constexpr (kOp == kSpmvCsr) rows_dense = hints[kHdrEmptyRows - kHdrHints] == 0;
    if constexpr (kCounts) {
        // number of segment starts before my tile, while the loads are in flight: either the table
        // holds the prefix sums already, or (few tiles) wave 1 adds up the counts of the tiles before
        if (wave == 1) {
            uint32_t c = 0;
            if (P.count_is_prefix) {
                c = P.tile_count[tile];
            } else {
                for (uint32_t i = lane; i < tile; i += 64) c += P.tile_count[i];
                c = wave_sum<uint32_t, kAluLanes>(c);
            }
            if (lane == 0) sm.carry_c = c;
        }
    }

    // per chunk: exclusive segmented prefix of my row inside the chunk, and of the chunk inside
    // my span; run_* = running aggregate of the span
    A ex_v[kCpw], pre_v[kCpw];
    uint32_t ex_f[kCpw], pre_f[kCpw], ex_c[kCpw];
#pragma unroll
    for (int c = 0; c < kCpw; ++c) {
        ex_v[c] = pre_v[c] = A(0);
        ex_f[c] = pre_f[c] = ex_c[c] = 0;
    }
    A run_v = A(0);
    uint32_t run_f = 0, run_c = 0;

    // ================= phase A: aggregates =================
#pragma unroll 1
    for (int c0 = 0; c0 < kCpw; c0 += kStep) {
#pragma unroll
     for (int u = 0; u < kStep; ++u) {
      const int c = c0 + u;
      const int S = kUnrollChunks ? c : u;   // register slot of this chunk
      if (c < cpw_t) {
        const uint64_t cb = wave_base + (uint64_t)c * kChunkElems;
        const uint64_t row_start = cb + 32u * lane;  // first element of the row this lane owns
        // ---- flags of my row (one 32-bit word = one row); bits beyond n do not count ----
        if (row_start + 32 > n) F[S] = row_start < n ? (F[S] & ((1u << (uint32_t)(n - row_start)) - 1u)) : 0u;
        if constexpr (kProduct && kLateVal) {
            // product vector p(i) = val(i) * x(col(i)), in the layout the columns were loaded in: the
            // gathers go out as soon as the columns are there, the loads of the values right behind them
            float xg[2 * K][4];
            if (cb + kChunkElems <= n) {   // all of the chunk lies inside the matrix: no checks
#pragma unroll
                for (int i = 0; i < 2 * K; ++i)
#pragma unroll
                    for (int k = 0; k < 4; ++k) xg[i][k] = P.xv[rawc[S][i][k]];
            } else {
#pragma unroll
                for (int i = 0; i < 2 * K; ++i)
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const uint64_t e = cb + 1024u * (i / K) + raw_offset<TT, kMfma>(i % K, lane) + k;
                        xg[i][k] = e < n ? P.xv[rawc[S][i][k]] : 0.0f;
                    }
            }
            __builtin_amdgcn_sched_barrier(0);
            load_raw<TT, kMfma>((const In *)P.x, cb, n, lane, raw[S]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 2 * K; ++i)
#pragma unroll
                for (int k = 0; k < 4; ++k) raw[S][i][k] = to_bits(from_bits<float>(raw[S][i][k]) * xg[i][k]);
        } else if constexpr (kProduct) {
            // product vector p(i) = val(i) * x(col(i)), in the layout the values were loaded in (the
            // checks stay even in full chunks: without them the compiler issues all gathers of the chunk
            // at once, which was measured 4 % slower with scattered columns)
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int i = 0; i < K; ++i) {
                    const uint64_t e0 = cb + 1024u * t + raw_offset<TT, kMfma>(i, lane);
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const float p =
                            (e0 + k < n) ? from_bits<float>(raw[S][t * K + i][k]) * P.xv[rawc[S][t * K + i][k]] : 0.0f;
                        raw[S][t * K + i][k] = to_bits(p);
                    }
                }
        }

        // ---- steps 1-4 for the aggregate of my row: last element after the revert, any flag ----
        const uint32_t has_flag = F[S] != 0;
        A agg_v;
        if constexpr (kMfma && kKeepRows) {
            // one chunk per wave: the row scans made here stay in the wave's LDS rows until phase B
            if constexpr (K > 1) to_operand_layout<K>(raw[S], rows, lane);
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                A acc[16];
                SpecMfma<TT>::run(raw[S] + t * K, lane, acc);
                store_spec_rows(rows, t, lane, acc);
            }
            rows[lane * kRowStride + kSlotZero] = 0;
            wave_lds_sync();
            const A last = from_bits<A>(rows[lane * kRowStride + kRowData + 31]);
            const int slot = kSlotZero + last_flag_pos(F[S]);  // x-bar(start - 1)
            agg_v = last - from_bits<A>(rows[lane * kRowStride + slot]);
        } else if constexpr (kMfma) {
            if constexpr (K > 1) to_operand_layout<K>(raw[S], rows, lane);
            agg_v = RowAgg<TT>::template run<kAluLanes>(raw[S], F[S], lane);
        } else {
#pragma unroll
            for (int t = 0; t < 2; ++t) spec_shuffle_tile<TT, kAluLanes>(raw[S] + t * K, lane, rows, t);
            rows[lane * kRowStride + kSlotZero] = 0;
            wave_lds_sync();
            const A last = from_bits<A>(rows[lane * kRowStride + kRowData + 31]);
            const int slot = kSlotZero + last_flag_pos(F[S]);  // x-bar(start - 1)
            agg_v = last - from_bits<A>(rows[lane * kRowStride + slot]);
            if constexpr (!kKeepRows) wave_lds_sync();  // the rows are read before the next chunk overwrites them
        }
        // segment starts in my row, position 0 of the whole vector not counted (sum only)
        const uint32_t cnt = __popc(row_start == 0 ? (F[S] & ~1u) : F[S]);

        // ---- step 5a: segmented inclusive scan of (value, flag) over the 64 rows of the chunk ----
        A inc_v = agg_v;
        uint32_t inc_f = has_flag;
        uint32_t inc_c = cnt;
      if constexpr (kAluLanes) {
        // Kogge-Stone inside the rows of 16 lanes (row_shr 1, 2, 4, 8), then the total of a row of lanes
        // to the next one (row_bcast 15 into lane rows 1 and 3) and of the first 32 lanes to the last 32
        // (row_bcast 31 into lane rows 2 and 3).  A lane without a source gets (0, no flag, 0).
#define MMV_SCAN_STEP(CTRL, ROWS)                                                                  \
        {                                                                                          \
            const A ov = from_bits<A>(dpp_or_zero<CTRL, ROWS>(to_bits(inc_v)));                    \
            const uint32_t of = dpp_or_zero<CTRL, ROWS>(inc_f);                                    \
            if (kCounts) inc_c += dpp_or_zero<CTRL, ROWS>(inc_c);                                  \
            if (!inc_f) inc_v = ov + inc_v;                                                        \
            inc_f |= of;                                                                           \
        }
        MMV_SCAN_STEP(0x111, 0xF)
        MMV_SCAN_STEP(0x112, 0xF)
        MMV_SCAN_STEP(0x114, 0xF)
        MMV_SCAN_STEP(0x118, 0xF)
        MMV_SCAN_STEP(0x142, 0xA)
        MMV_SCAN_STEP(0x143, 0xC)
#undef MMV_SCAN_STEP
        ex_v[S] = from_bits<A>(dpp_or_zero<0x138, 0xF>(to_bits(inc_v)));   // wave_shr 1: lane 0 gets 0
        ex_f[S] = dpp_or_zero<0x138, 0xF>(inc_f);
        ex_c[S] = run_c + inc_c - cnt;
        pre_v[S] = run_v;
        pre_f[S] = run_f;
        // chunk aggregate = inclusive value of the last row; fold it into the span's running aggregate
        const A ca_v = from_bits<A>((uint32_t)__builtin_amdgcn_readlane((int)to_bits(inc_v), 63));
        const uint32_t ca_f = (uint32_t)__builtin_amdgcn_readlane((int)inc_f, 63);
        run_v = ca_f ? ca_v : run_v + ca_v;
        run_f |= ca_f;
        if (kCounts) run_c += (uint32_t)__builtin_amdgcn_readlane((int)inc_c, 63);
      } else {
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const A ov = from_bits<A>(__shfl_up(to_bits(inc_v), d));
            const uint32_t of = __shfl_up(inc_f, d);
            if (lane >= d) {
                if (!inc_f) inc_v = ov + inc_v;
                inc_f |= of;
            }
            if (kCounts) {
                const uint32_t oc = __shfl_up(inc_c, d);
                if (lane >= d) inc_c += oc;
            }
        }
        ex_v[S] = from_bits<A>(__shfl_up(to_bits(inc_v), 1));
        ex_f[S] = __shfl_up(inc_f, 1);
        if (lane == 0) {
            ex_v[S] = A(0);
            ex_f[S] = 0;
        }
        ex_c[S] = run_c + inc_c - cnt;
        pre_v[S] = run_v;
        pre_f[S] = run_f;
        // chunk aggregate = inclusive value of the last row; fold it into the span's running aggregate
        const A ca_v = from_bits<A>(__shfl(to_bits(inc_v), 63));
        const uint32_t ca_f = __shfl(inc_f, 63);
        run_v = ca_f ? ca_v : run_v + ca_v;
        run_f |= ca_f;
        if (kCounts) run_c += __shfl(inc_c, 63);
      }
      }
     }
        if constexpr (!kUnrollChunks) {
#pragma unroll
            for (int r = 0; r < kStep; ++r) {
                rotate(F);
                rotate_rows(raw);
                if constexpr (kProduct) rotate_rows(rawc);
                rotate(ex_v);
                rotate(ex_f);
                rotate(pre_v);
                rotate(pre_f);
                if (kCounts) rotate(ex_c);
            }
        }
    }
    MMV_STAMP(2);
    if (lane == 0) {
        sm.wave_v[wave] = to_bits(run_v);
        sm.wave_f[wave] = run_f;
        sm.wave_c[wave] = run_c;
    }
    __syncthreads();
    MMV_STAMP(3);

    // ---- step 5b: waves of the tile ----
    A wex_v = A(0);
    uint32_t wex_f = 0, wex_c = 0;
    A tagg_v = A(0);
    uint32_t tagg_f = 0, tagg_c = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        if (w == wave) {
            wex_v = tagg_v;
            wex_f = tagg_f;
            wex_c = tagg_c;
        }
        const A wv = from_bits<A>(sm.wave_v[w]);
        const uint32_t wf = sm.wave_f[w];
        tagg_v = wf ? wv : tagg_v + wv;
        tagg_f |= wf;
        tagg_c += sm.wave_c[w];
    }
    wex_f = __builtin_amdgcn_readfirstlane(wex_f);

    if constexpr (kCounts) {
        if (kOp == kSum && !P.count_is_prefix && tile == P.num_tiles - 1 && tid == 0) *P.nseg = (uint64_t)sm.carry_c + tagg_c + 1u;
    }

    // ---- step 5c, first half: publish this tile ----
    const bool final_now = tile == 0 || tagg_f;  // carry out does not depend on predecessors
    if (tid == 0) desc_store(P.desc_v + tile, final_now ? kStatusPrefix : kStatusAggregate, to_bits(tagg_v));

    // carry into my span (used only by rows with no flag before them in the tile); the carry of
    // the predecessor tiles is added once it is known
    A span_carry = wex_v;
    uint32_t count_carry = 0;
    if constexpr (kCounts) count_carry = sm.carry_c;

    // ================= phase B: recompute, revert, add carries, store =================
#pragma unroll 1
    for (int pass = 0; pass < 2; ++pass) {
        if (pass == 1) {
            // ---- step 5c, second half: carry of the predecessor tiles by decoupled look-back ----
            A tile_carry = A(0);
            if (wave == 0) {
                if (tile > 0) tile_carry = lookback<A, kAluLanes>(P.desc_v, (int)tile, lane, P.hdr);
                MMV_STAMP(4);
                if (lane == 0) {
                    if (!final_now) desc_store(P.desc_v + tile, kStatusPrefix, to_bits(tile_carry + tagg_v));
                    sm.carry_v = to_bits(tile_carry);
                    __hip_atomic_store(&sm.ready, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
            }
            if (wave != 0 && !wex_f) {
                // my span starts inside a segment that began in an earlier tile: wait for wave 0
                while (__hip_atomic_load(&sm.ready, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) == 0)
                    __builtin_amdgcn_s_sleep(1);
                tile_carry = from_bits<A>(sm.carry_v);
            }
            if (!wex_f) span_carry = tile_carry + wex_v;
            MMV_STAMP(5);
        }
#pragma unroll 1
        for (int c0 = 0; c0 < kCpw; c0 += kStep) {
#pragma unroll
          for (int u = 0; u < kStep; ++u) {
            const int c = c0 + u;
            const int S = kUnrollChunks ? c : u;
            // a chunk is "open" when no flag of the tile precedes it
            const bool chunk_open = !(wex_f || __builtin_amdgcn_readfirstlane(pre_f[S]));
            if (c < cpw_t && chunk_open == (pass == 1)) {
                const uint64_t cb = wave_base + (uint64_t)c * kChunkElems;
                const bool chunk_full = cb + kChunkElems <= n;
                const uint64_t row_start = cb + 32u * lane;
                // sum, spmv: end mask of my row, bit p set iff position p + 1 starts a segment or p is
                // the last element; a 32x32 tile none of whose rows holds a segment end needs no x-bar
                uint32_t E = 0;
                uint64_t rows_with_ends = ~0ull;
                if constexpr (!kScanLike) {
                    uint32_t next0 = dpp_or_zero<0x130, 0xF>(F[S]) & 1u;   // wave_shl 1: the word of the next row
                    if (lane == 63) {
                        const uint64_t en = cb + kChunkElems;
                        next0 = 0;
                        if (en < n) next0 = P.fw[en >> 5] & 1u;
                    }
                    E = (F[S] >> 1) | (next0 << 31);
                    if (row_start < n) {
                        if (row_start + 32 >= n) {
                            const uint32_t last = (uint32_t)(n - 1 - row_start);
                            E = (E & ((1u << last) - 1u)) | (1u << last);
                        }
                    } else {
                        E = 0;
                    }
                    rows_with_ends = __ballot(E != 0);
                }
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    if (kKeepRows) continue;   // still there from phase A
                    if (((rows_with_ends >> (32 * t)) & 0xFFFFFFFFull) == 0) continue;
                    if (kMfma) {
                        A acc[16];
                        SpecMfma<TT>::run(raw[S] + t * K, lane, acc);
                        store_spec_rows(rows, t, lane, acc);
                    } else {
                        spec_shuffle_tile<TT, kAluLanes>(raw[S] + t * K, lane, rows, t);
                    }
                }
                // ---- step 6: carry into my row ----
                const A carry = ex_f[S] ? ex_v[S] : (pre_f[S] ? pre_v[S] + ex_v[S] : (span_carry + pre_v[S]) + ex_v[S]);
                if constexpr (kScanLike) {
                    // stored negated in the slot before x-bar(-1), so that the revert subtracts it
                    rows[lane * kRowStride + kSlotZero] = 0;
                    rows[lane * kRowStride + kSlotF] = F[S];
                    rows[lane * kRowStride + kSlotNegCarry] = to_bits(A(0) - carry);
                    const uint64_t row_any = __ballot(F[S] != 0);
                    wave_lds_sync();

                    // ---- steps 2 + 6 on every element, then store; a lane owns 4 consecutive positions ----
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const int R = 8 * j + (lane >> 3), p0 = 4 * (lane & 7);
                        const uint32_t *rp = rows + R * kRowStride;
                        const v4u xb = *reinterpret_cast<const v4u *>(rp + kRowData + p0);
                        A o[4];
                        if (((row_any >> (8 * j)) & 0xFFull) == 0) {
                            // none of these eight rows has a flag: the speculation stands, only the carry is added
                            const A nc = from_bits<A>(rp[kSlotNegCarry]);
#pragma unroll
                            for (int i = 0; i < 4; ++i) o[i] = from_bits<A>(xb[i]) - nc;
                        } else {
                            const uint32_t Fr = rp[kSlotF];
                            const uint32_t m = Fr & ((2u << p0) - 1u);  // flags at or before my first position
                            const int slot = m ? kSlotZero + (31 - __clz(m)) : kSlotNegCarry;
                            A b = from_bits<A>(rp[slot]);
                            o[0] = from_bits<A>(xb[0]) - b;
#pragma unroll
                            for (int i = 1; i < 4; ++i) {
                                if ((Fr >> (p0 + i)) & 1u) b = from_bits<A>(xb[i - 1]);
                                o[i] = from_bits<A>(xb[i]) - b;
                            }
                        }
                        const uint64_t e0 = cb + 256u * j + 4u * lane;
                        A *z = (A *)P.z;
                        if (chunk_full) {
                            v4u w = {to_bits(o[0]), to_bits(o[1]), to_bits(o[2]), to_bits(o[3])};
                            __builtin_nontemporal_store(w, reinterpret_cast<v4u *>(z + e0));
                        } else {
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                if (e0 + i < n) z[e0 + i] = o[i];
                        }
                    }
                } else {
                    // ---- sum, spmv: only the segment ends produce output; the lane that owns a row
                    // walks the ends of its row (steps 2 + 6 for those positions only) ----
                    wave_lds_sync();
                    const uint32_t *rp = rows + lane * kRowStride + kRowData;
                    const uint32_t Fc = row_start == 0 ? (F[S] & ~1u) : F[S];  // position 0 is not counted
                    const uint64_t count_base = (uint64_t)count_carry + wex_c + ex_c[S];
                    while (E) {
                        const int e = __builtin_ctz(E);
                        E &= E - 1u;
                        const uint32_t m = F[S] & ((2u << e) - 1u);  // flags at or before the end
                        A v = from_bits<A>(rp[e]);
                        if (m) {
                            const int st = 31 - __clz(m);
                            if (st > 0) v -= from_bits<A>(rp[st - 1]);   // REVSPEC: x-bar(e) - x-bar(start - 1)
                        } else {
                            v += carry;                                  // the segment began before this row
                        }
                        if (kOp == kSum) {
                            const uint64_t k = count_base + __popc(Fc & ((2u << e) - 1u));
                            if (k < P.out_cap) ((A *)P.out)[k] = v;
                        } else if (kOp == kSpmvCsr) {
                            const uint64_t k = count_base + __popc(Fc & ((2u << e) - 1u));
                            if (k < P.out_cap) P.y[rows_dense ? (uint32_t)k : P.rowmap[k]] = from_bits<float>(to_bits(v));
                        } else {
                            P.y[P.row[row_start + e]] = from_bits<float>(to_bits(v));
                        }
                    }
                }
                wave_lds_sync();  // the rows are read before the next chunk overwrites them
            }
          }
            if constexpr (!kUnrollChunks) {
#pragma unroll
                for (int r = 0; r < kStep; ++r) {
                    rotate(F);
                    rotate_rows(raw);
                    rotate(ex_v);
                    rotate(ex_f);
                    rotate(pre_v);
                    rotate(pre_f);
                    if (kCounts) rotate(ex_c);
                }
            }
        }
    }
    MMV_STAMP(6);
#ifdef MMV_TRACE
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    MMV_STAMP(7);
#endif
}

template <typename TT, int kOp, bool kMfma>
__global__ __launch_bounds__(TT::kWaves * 64, MMV_MIN_WAVES_PER_SIMD) void seg_kernel(Params P, const uint32_t *__restrict__ hints) {
    __shared__ SegShared<TT::kWaves> sm;
    constexpr bool kProduct = kOp == kSpmv || kOp == kSpmvCsr;
    const int tid = threadIdx.x;
#ifdef MMV_TRACE
    const uint64_t t_begin = wall_clock64();
#endif
    // A workgroup that starts competes with the ones in the middle of their arithmetic: its ticket
    // and its loads go first (measured: 2 to 3 % on the long scans)
#if MMV_LOAD_PRIO
    __builtin_amdgcn_s_setprio(MMV_LOAD_PRIO);
#endif
    // SpMV, where neighbouring entries mostly sit in consecutive columns (blocked, banded matrices): the
    // gathers are cheap and the memory pipe is the limit, so the values are loaded behind the gathers
    // instead of beside the columns: half the burst at the start of the tile, the columns arrive
    // sooner (measured 11-15 % on the blocked sparse-attention matrices).  With scattered columns the
    // gathers are the limit and values loaded that late only add to their burst (4-8 % slower).
    // Uniform words, written by the kernel that makes the flags.
    bool late_val = false;
    if constexpr (kProduct) late_val = hints[kHdrColumnRuns - kHdrHints] != 0;

    // Tiles are handed out by an atomic ticket, so that a tile never waits for a predecessor that
    // has not started (workgroups need not start in index order).  The tickets of the workgroups
    // that start together are served one after the other (about 11 ns each): a grid that is resident
    // as a whole cannot block itself that way and skips them.
    if (tid == 0) {
        sm.ready = 0;
        if (!P.ordered) {
            if (blockIdx.x < P.stagger_wgs) {
                // low-discrepancy spread of the start times: fraction of blockIdx * golden ratio
                const uint32_t frac = blockIdx.x * 2654435769u;
                const uint64_t wait = ((uint64_t)frac * P.stagger_ticks) >> 32;
                const uint64_t t0 = wall_clock64();
                while (wall_clock64() - t0 < wait) __builtin_amdgcn_s_sleep(8);
            }
            sm.tile = __hip_atomic_fetch_add(P.hdr + kHdrTicket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (!P.ordered) __syncthreads();
    const uint32_t tile = __builtin_amdgcn_readfirstlane(P.ordered ? blockIdx.x : sm.tile);   // a scalar, like the wave index
#ifdef MMV_TRACE
    if (tid == 0 && P.trace) P.trace[(uint64_t)tile * 8] = t_begin;
#endif
    if (kProduct && late_val)
        seg_tile<TT, kOp, kMfma, kProduct>(P, hints, sm, tile);
    else
        seg_tile<TT, kOp, kMfma, false>(P, hints, sm, tile);
}

// ---- auxiliary kernels -------------------------------------------------------------------------------------

// Zero fills two ranges (workspace words and, for SpMV, y) with 32-bit stores.
__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t *a, uint64_t na, uint32_t *b, uint64_t nb) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < na; i += stride) a[i] = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nb; i += stride) b[i] = 0;
}

// Segmented sum, step "scan of the end markers" of COMPRESS (proof of the SCD / SSCR theorem)
// at tile granularity: workgroup b counts the segment starts inside tile b (position 0 is not
// counted: it opens segment 0 whatever its flag says; bits at or beyond n are not counted).  The
// same launch zeroes the header and the descriptors of the main kernel.
__global__ __launch_bounds__(256) void count_tiles_kernel(uint32_t *zero, uint64_t zero_words, const uint32_t *fw,
                                                          uint64_t n, uint32_t big_tiles, uint32_t big_elems,
                                                          uint32_t tail_elems, uint32_t *cnt) {
    __shared__ uint32_t s_part[4];
    const uint32_t b = blockIdx.x, tid = threadIdx.x;
    for (uint64_t i = (uint64_t)b * 256 + tid; i < zero_words; i += (uint64_t)gridDim.x * 256) zero[i] = 0;
    const uint64_t base = b < big_tiles ? (uint64_t)b * big_elems
                                        : (uint64_t)big_tiles * big_elems + (uint64_t)(b - big_tiles) * tail_elems;
    const uint64_t elems = b < big_tiles ? big_elems : tail_elems;
    const uint64_t end = base + elems < n ? base + elems : n;
    uint32_t sum = 0;
    for (uint64_t w = (base >> 5) + tid; w < ((end + 31) >> 5); w += 256) {   // tiles begin on word borders
        uint32_t v = fw[w];
        if (w == 0) v &= ~1u;
        if ((w + 1) * 32 > n) v &= (1u << (uint32_t)(n - w * 32)) - 1u;
        sum += __popc(v);
    }
    sum = wave_sum(sum);
    if ((tid & 63) == 0) s_part[tid >> 6] = sum;
    __syncthreads();
    if (tid == 0) cnt[b] = s_part[0] + s_part[1] + s_part[2] + s_part[3];
}

// Exclusive prefix sums of the per-tile counts, in place, by one workgroup; the total (+ 1 for
// segment 0) is the number of segments.
__global__ __launch_bounds__(1024) void scan_counts_kernel(uint32_t *cnt, uint32_t num_tiles, uint64_t *nseg) {
    __shared__ uint32_t s_wave[16];
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t running = 0;
    for (uint32_t base = 0; base < num_tiles; base += 1024) {
        const uint32_t i = base + tid;
        const uint32_t v = i < num_tiles ? cnt[i] : 0u;
        uint32_t inc = v;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t o = __shfl_up(inc, d);
            if (lane >= (uint32_t)d) inc += o;
        }
        if (lane == 63) s_wave[wave] = inc;
        __syncthreads();
        uint32_t before = 0, total = 0;
#pragma unroll
        for (uint32_t w = 0; w < 16; ++w) {
            if (w == wave) before = total;
            total += s_wave[w];
        }
        if (i < num_tiles) cnt[i] = running + before + inc - v;
        running += total;
        __syncthreads();
    }
    if (tid == 0) *nseg = (uint64_t)running + 1u;
}

// One byte per element -> one bit per element; a thread builds one 32-bit word.
__global__ __launch_bounds__(256) void pack_flags_kernel(const uint8_t *f, uint64_t n, uint32_t *words,
                                                         uint64_t nwords) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t w = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; w < nwords; w += stride) {
        uint32_t bits = 0;
        const uint64_t e0 = w * 32;
        if (e0 + 32 <= n) {
            const v4u a = *reinterpret_cast<const v4u *>(f + e0), b = *reinterpret_cast<const v4u *>(f + e0 + 16);
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    bits |= (((a[k] >> (8 * j)) & 0xFFu) ? 1u : 0u) << (4 * k + j);
                    bits |= (((b[k] >> (8 * j)) & 0xFFu) ? 1u : 0u) << (16 + 4 * k + j);
                }
        } else {
            for (int i = 0; i < 32 && e0 + i < n; ++i) bits |= (f[e0 + i] ? 1u : 0u) << i;
        }
        words[w] = bits;
    }
}

// One wave looks at 512 pairs of neighbouring column indices spread over the matrix and notes in the
// (zeroed) workspace header whether most of them are consecutive, as in blocked and banded matrices.
__device__ __forceinline__ void sample_column_runs(const int32_t *col, uint64_t nnz, uint32_t *hdr, int lane) {
    const uint64_t stride = nnz / 512 > 0 ? nnz / 512 : 1;
    uint32_t runs = 0, pairs = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint64_t p = (uint64_t)(lane * 8 + j) * stride;
        if (p + 1 < nnz) {
            ++pairs;
            runs += col[p + 1] == col[p] + 1 ? 1u : 0u;
        }
    }
    runs = wave_sum(runs);
    pairs = wave_sum(pairs);
    if (lane == 0 && 2 * runs > pairs) hdr[kHdrColumnRuns] = 1u;
}

// Segment-start flags of a row-sorted COO matrix, f(e) = [e == 0 or row(e) != row(e-1)],
// bit-packed.  A lane takes four consecutive entries (one 128-bit load) and the entry before
// them from the lane below; eight lanes OR their nibbles into one flag word.
__global__ __launch_bounds__(256) void row_flags_kernel(const int32_t *row, uint64_t nnz, uint32_t *words,
                                                        const int32_t *col, uint32_t *hdr) {
    const int lane = threadIdx.x & 63;
    if (blockIdx.x == 0 && threadIdx.x < 64) sample_column_runs(col, nnz, hdr, lane);
    const uint64_t wave0 = ((uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 1024;  // four rounds of 256 entries
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint64_t e0 = wave0 + 256u * j + 4u * lane;
        v4i r = {0, 0, 0, 0};
        if (e0 + 4 <= nnz) {
            r = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(row + e0));
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (e0 + i < nnz) r[i] = row[e0 + i];
        }
        int prev = __shfl_up(r[3], 1);
        if (lane == 0) prev = (e0 > 0 && e0 - 1 < nnz) ? row[e0 - 1] : r[0];
        uint32_t nib = (e0 == 0 || r[0] != prev) ? 1u : 0u;
#pragma unroll
        for (int i = 1; i < 4; ++i) nib |= (r[i] != r[i - 1] ? 1u : 0u) << i;
        const uint32_t valid = e0 >= nnz ? 0u : (nnz - e0 >= 4 ? 0xFu : (1u << (uint32_t)(nnz - e0)) - 1u);
        uint32_t v = (nib & valid) << (4 * (lane & 7));
        v |= __shfl_xor(v, 1);
        v |= __shfl_xor(v, 2);
        v |= __shfl_xor(v, 4);
        const uint64_t w = ((wave0 + 256u * j) >> 5) + (lane >> 3);
        if ((lane & 7) == 0 && w * 32 < nnz) words[w] = v;
    }
}

// ---- the stand-alone primitives of Algorithms SCD and SSCR (Sec. 4.1) ------------------------------------
//
// SCAN is the main kernel without a flag vector (kPlainScan).  COMPRESS, DIFF and REVERT follow.
// They exist so that the paper's un-fused compositions (SCD = DIFF o COMPRESS o SCAN, SSCR =
// REVERT o COMPRESS o (SCAN, SCAN)) can be run and timed next to the fused single-pass kernel.

// End markers f^- of Algorithm SCD: f shifted left by one position with a 1 appended, bit-packed.
__global__ __launch_bounds__(256) void end_markers_kernel(const uint32_t *fw, uint64_t n, uint32_t *out,
                                                          uint64_t nwords) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t w = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; w < nwords; w += stride) {
        const uint32_t next = w + 1 < nwords ? fw[w + 1] : 0u;
        uint32_t e = (fw[w] >> 1) | (next << 31);
        if (w == nwords - 1) {
            const uint32_t last = (uint32_t)((n - 1) & 31u);   // position of element n - 1 in this word
            e = (e & ((1u << last) - 1u)) | (1u << last);
        }
        out[w] = e;
    }
}

// Bit-packed flags -> one int8 (0 / 1) per element, for the count scan SCAN(f) of Algorithm SSCR.
__global__ __launch_bounds__(256) void unpack_flags_kernel(const uint32_t *fw, uint64_t n, int8_t *out) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    const uint64_t nquads = (n + 3) / 4;   // a thread writes four bytes; out has room for the padding
    for (uint64_t q = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; q < nquads; q += stride) {
        const uint32_t bits = (fw[q >> 3] >> (4 * (q & 7))) & 0xFu;
        reinterpret_cast<uint32_t *>(out)[q] = (bits & 1u) | ((bits & 2u) << 7) | ((bits & 4u) << 14) | ((bits & 8u) << 21);
    }
}

// COMPRESS (Sec. 2): out = the 32-bit entries of x whose mask bit is set, in order; with
// x == nullptr the positions themselves are compressed.  The mask is bit-packed; the output
// index of an entry is the number of set bits before it (the scan of the mask in the paper's
// COMPRESS), found per tile from popcounts and across tiles by decoupled look-back.
// A wave owns 64 * kWords consecutive positions (kWords = 64 or 16): lane j < kWords holds the
// 64-bit mask word j, and for every word the wave reads only the selected entries (one coalesced
// load, skipped when the word is empty) and writes them to consecutive output slots; a wave with
// few selected entries lets every lane walk its own word instead.  Short masks take the short
// spans: four times the waves, a quarter of the words each wave visits one after the other.
constexpr int kCompressWaves = 8;
constexpr int kCompressTile = kCompressWaves * 4096;
constexpr uint64_t kCompressShortN = 1ull << 22;   // masks up to this length take 16 words per wave
inline int compress_words(uint64_t n) { return n <= kCompressShortN ? 16 : 64; }
inline uint64_t compress_tile(uint64_t n) { return (uint64_t)kCompressWaves * 64u * compress_words(n); }

template <int kWords>
__global__ __launch_bounds__(kCompressWaves * 64) void compress_kernel(
    const uint32_t *__restrict__ x, const uint32_t *__restrict__ mw, uint64_t n, uint32_t *__restrict__ out,
    uint64_t out_cap, uint64_t *__restrict__ count, uint32_t *hdr, uint64_t *desc, uint32_t num_tiles,
    const uint32_t *needed) {
    __shared__ uint32_t s_tile, s_wave[kCompressWaves], s_carry;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (needed && *needed == 0) return;   // CSR SpMV without empty rows: nobody reads the row map
    if (tid == 0) s_tile = __hip_atomic_fetch_add(hdr + kHdrTicket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const uint32_t tile = s_tile;
    constexpr uint32_t kSpan = 64u * kWords;                                        // positions of a wave
    const uint64_t span = ((uint64_t)tile * kCompressWaves + wave) * kSpan;          // first position of my wave
    const uint64_t p0 = span + 64u * lane;                                          // first position of my word
    uint64_t m = 0;
    if (lane < kWords && p0 < n) {
        const uint64_t wi = p0 >> 5;
        m = mw[wi];
        if (p0 + 32 < n) m |= (uint64_t)mw[wi + 1] << 32;
        if (p0 + 64 > n) m &= (1ull << (n - p0)) - 1ull;
    }
    const uint32_t cnt = (uint32_t)__popcll((unsigned long long)m);
    uint32_t inc = cnt;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(inc, d);
        if (lane >= d) inc += o;
    }
    if (lane == 63) s_wave[wave] = inc;
    __syncthreads();
    uint32_t wave_ex = 0, tile_cnt = 0;
#pragma unroll
    for (int w = 0; w < kCompressWaves; ++w) {
        if (w == wave) wave_ex = tile_cnt;
        tile_cnt += s_wave[w];
    }
    if (tid == 0) desc_store(desc + tile, tile == 0 ? kStatusPrefix : kStatusAggregate, tile_cnt);
    if (wave == 0) {
        uint32_t carry = 0;
        if (tile > 0) carry = lookback<uint32_t>(desc, (int)tile, lane, hdr);
        if (lane == 0) {
            if (tile > 0) desc_store(desc + tile, kStatusPrefix, carry + tile_cnt);
            s_carry = carry;
            if (tile == num_tiles - 1) *count = (uint64_t)carry + tile_cnt;
        }
    }
    __syncthreads();
    // output index of the first selected entry of word j of my wave (lane j holds it)
    const uint64_t word_base = (uint64_t)s_carry + wave_ex + (inc - cnt);
    if (__builtin_amdgcn_readlane((int)inc, 63) <= 4 * kWords) {
        // few selected entries in my wave's positions: every lane walks the set bits of its own
        // word (a handful of independent loads per lane) instead of the wave visiting all 64 words
        uint64_t mm = m, k = word_base;
        while (mm) {
            const uint64_t p = p0 + (uint32_t)__builtin_ctzll((unsigned long long)mm);
            mm &= mm - 1;
            const uint32_t v = x ? __builtin_nontemporal_load(x + p) : (uint32_t)p;
            if (k < out_cap) out[k] = v;
            ++k;
        }
        return;
    }
    const uint32_t m_lo = (uint32_t)m, m_hi = (uint32_t)(m >> 32);
    const uint32_t base_lo = (uint32_t)word_base, base_hi = (uint32_t)(word_base >> 32);
    const uint64_t lane_below = (1ull << lane) - 1ull;
#pragma unroll 8
    for (int j = 0; j < kWords; ++j) {
        const uint64_t mj = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)m_hi, j) << 32) |
                            (uint32_t)__builtin_amdgcn_readlane((int)m_lo, j);
        const uint64_t bj = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)base_hi, j) << 32) |
                            (uint32_t)__builtin_amdgcn_readlane((int)base_lo, j);
        if ((mj >> lane) & 1ull) {
            const uint64_t p = span + 64u * j + lane;
            const uint32_t v = x ? __builtin_nontemporal_load(x + p) : (uint32_t)p;
            const uint64_t k = bj + (uint32_t)__popcll((unsigned long long)(mj & lane_below));
            if (k < out_cap) out[k] = v;
        }
    }
}

// DIFF (Sec. 4.1): z(i) = x(i) - x(i-1) with x(-1) = 0, on int32 (wrap-around) or fp32.  The
// paper writes it as the product with the bidiagonal matrix D_s plus a vector fix of the block
// borders; here a lane takes four consecutive elements and gets the element before them from
// its neighbour lane (one extra load at the wave border).
// With `limit` the vector ends at min(n, *limit) (a count that an earlier kernel left on the device).
template <typename A>
__global__ __launch_bounds__(256) void diff_kernel(const uint32_t *__restrict__ x, uint64_t n, uint32_t *__restrict__ z,
                                                   const uint64_t *__restrict__ limit) {
    const int lane = threadIdx.x & 63;
    if (limit) {
        const uint64_t m = *limit;
        n = m < n ? m : n;
    }
    const uint64_t e0 = ((uint64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    v4u w = {0, 0, 0, 0};
    if (e0 + 4 <= n) {
        w = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(x + e0));
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (e0 + i < n) w[i] = x[e0 + i];
    }
    uint32_t prev = __shfl_up(w[3], 1);
    if (lane == 0) prev = (e0 > 0 && e0 - 1 < n) ? x[e0 - 1] : 0u;
    v4u o;
    o[0] = to_bits(from_bits<A>(w[0]) - from_bits<A>(prev));
#pragma unroll
    for (int i = 1; i < 4; ++i) o[i] = to_bits(from_bits<A>(w[i]) - from_bits<A>(w[i - 1]));
    if (e0 + 4 <= n) {
        __builtin_nontemporal_store(o, reinterpret_cast<v4u *>(z + e0));
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (e0 + i < n) z[e0 + i] = o[i];
    }
}

// REVERT (Sec. 4.1): z(i) = xhat(i) - w(fhat(i) - 2) where the inclusive count of segment
// starts fhat(i) is at least 2 (the printed index is read shifted by one: the first segment is
// left alone).  A count that points outside w subtracts nothing and raises the error word.
template <typename A>
__global__ __launch_bounds__(256) void revert_kernel(const uint32_t *xhat, const int32_t *__restrict__ fhat,
                                                     const uint32_t *__restrict__ w, uint64_t n, uint64_t nw,
                                                     uint32_t *z, uint32_t *err) {
    const uint64_t e0 = ((uint64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (e0 >= n) return;
    v4u xv = {0, 0, 0, 0};
    v4i kv = {0, 0, 0, 0};
    const bool full = e0 + 4 <= n;
    if (full) {
        xv = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(xhat + e0));
        kv = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(fhat + e0));
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (e0 + i < n) {
                xv[i] = xhat[e0 + i];
                kv[i] = fhat[e0 + i];
            }
    }
    v4u o;
    bool bad = false;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        A v = from_bits<A>(xv[i]);
        const int64_t k = kv[i];
        if (k >= 2) {
            if ((uint64_t)(k - 2) < nw) v -= from_bits<A>(w[k - 2]);
            else if (e0 + i < n) bad = true;
        }
        o[i] = to_bits(v);
    }
    if (bad && err) __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (full) {
        __builtin_nontemporal_store(o, reinterpret_cast<v4u *>(z + e0));
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (e0 + i < n) z[e0 + i] = o[i];
    }
}

// Row pointers of a CSR matrix -> (a) bit-packed segment-start flags over the non-zeros (a row
// with entries sets the bit of its first entry; rows that share a word meet in an atomic OR on
// a zeroed word), (b) the bit-packed mask of rows that have entries (one ballot per 64 rows),
// (c) the number of segment starts inside every tile of the main kernel (position 0 not counted,
// as in count_tiles_kernel; the rows of a wave that start in the same tile share one atomic add
// on a zeroed table) and (d) the mark that some row is empty.
__global__ __launch_bounds__(256) void csr_flags_kernel(const int32_t *rowptr, uint64_t n_rows, uint32_t *fw,
                                                        uint32_t *rowmask, uint32_t *hdr, uint32_t big_tiles,
                                                        uint32_t big_elems, uint32_t tail_elems, uint32_t *tile_count,
                                                        const int32_t *col, uint64_t nnz) {
    const int lane = threadIdx.x & 63;
    if (blockIdx.x == 0 && threadIdx.x < 64) sample_column_runs(col, nnz, hdr, lane);
    const uint64_t r = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    bool nonempty = false;
    uint32_t tile = 0xFFFFFFFFu;   // tile of the first entry of a row that is counted
    if (r < n_rows) {
        const int32_t a = rowptr[r], b = rowptr[r + 1];
        nonempty = b > a;
        if (nonempty) {
            atomicOr(fw + ((uint32_t)a >> 5), 1u << ((uint32_t)a & 31u));
            const uint64_t big_total = (uint64_t)big_tiles * big_elems;
            if (a > 0) tile = (uint32_t)a < big_total ? (uint32_t)a / big_elems
                                                      : big_tiles + (uint32_t)(((uint32_t)a - big_total) / tail_elems);
        }
    }
    const uint64_t m = __ballot(nonempty);
    // a matrix none of whose rows is empty needs no row map: segment k is row k
    if (__ballot(r < n_rows && !nonempty) != 0 && lane == 0) hdr[kHdrEmptyRows] = 1u;
    uint64_t todo = __ballot(tile != 0xFFFFFFFFu);
    while (todo) {   // one round per distinct tile among the rows of the wave
        const int first = __ffsll((unsigned long long)todo) - 1;
        const uint32_t t = __shfl(tile, first);
        const uint64_t same = __ballot(tile == t);
        if (lane == first) atomicAdd(tile_count + t, (uint32_t)__popcll((unsigned long long)same));
        todo &= ~same;
    }
    const uint64_t r0 = r - lane;
    if (lane == 0 && r0 < n_rows) {
        rowmask[r0 >> 5] = (uint32_t)m;
        if (r0 + 32 < n_rows) rowmask[(r0 >> 5) + 1] = (uint32_t)(m >> 32);
    }
}

// Random-access reference for SpMV: streams val and col with 128-bit loads, gathers x[col] and
// keeps one partial sum per thread: everything the product vector of SpMV costs, and nothing of
// the segmented sum.  A column index at or beyond n_cols reads x[0] instead (no access out of bounds).
constexpr int kGatherRefBlocks = 8192;
__global__ __launch_bounds__(256) void gather_reference_kernel(const v4u *val, const v4u *col, uint64_t quads,
                                                               uint32_t n_cols, const float *x, float *partial) {
    float acc = 0.0f;
    const uint64_t stride = (uint64_t)gridDim.x * 256;
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < quads; i += stride) {
        const v4u v = __builtin_nontemporal_load(val + i);
        const v4u c = __builtin_nontemporal_load(col + i);
#pragma unroll
        for (int k = 0; k < 4; ++k) acc += from_bits<float>(v[k]) * x[c[k] < n_cols ? c[k] : 0u];
    }
    partial[(uint64_t)blockIdx.x * 256 + threadIdx.x] = acc;
}

// Streaming reference: 128-bit non-temporal reads and writes, kIn input chunks and kOut
// output chunks per thread, both striped across the workgroup; one workgroup per 256
// units (measured faster than a persistent grid-stride loop on this chip).
template <int kIn, int kOut>
__global__ __launch_bounds__(256) void stream_copy_kernel(const v4u *src, v4u *dst, uint64_t units) {
    const uint64_t u0 = (uint64_t)blockIdx.x * 256;
    v4u acc = {0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < kIn; ++i) {
        const uint64_t idx = u0 * kIn + (uint64_t)i * 256 + threadIdx.x;
        if (idx < units * kIn) acc ^= __builtin_nontemporal_load(src + idx);
    }
#pragma unroll
    for (int i = 0; i < kOut; ++i) {
        const uint64_t idx = u0 * kOut + (uint64_t)i * 256 + threadIdx.x;
        if (idx < units * kOut) __builtin_nontemporal_store(acc + (unsigned)i, dst + idx);
    }
    if (kOut == 0 && acc[0] == 0x9E3779B9u && acc[1] == 0x7F4A7C15u && acc[2] == 1u && acc[3] == 2u)
        dst[0] = acc;  // keeps the reads alive; practically never taken
}

// ---- host side -------------------------------------------------------------------------------------------------

inline size_t round256(size_t b) { return (b + 255) & ~(size_t)255; }
// Tile plan.  A tile costs one ticket (about 11 ns, serialised), so tiles are as large as the
// registers allow: kMaxCpw chunks of 2048 elements per wave.  The workgroups of the last round
// would leave most of the chip idle while they finish, so the end of the vector is cut into
// shorter tiles (one chunk per wave); inputs that fit into one round of resident workgroups
// get equal tiles of just the size that gives every workgroup one.
constexpr uint64_t kResident = MMV_MIN_TILES;   // workgroups resident at once (2 per compute unit)
#ifndef MMV_TAIL_ROUNDS
#define MMV_TAIL_ROUNDS 1
#endif
#ifndef MMV_TAIL_TILES
#define MMV_TAIL_TILES (MMV_TAIL_ROUNDS * kResident / 2)   // half a round measured best (256, 512, 768 within 1.5 %)
#endif
#ifndef MMV_TAIL_CPW
#define MMV_TAIL_CPW 1
#endif
constexpr uint64_t kTailTiles = MMV_TAIL_TILES;  // short tiles at the end of a long vector
constexpr uint64_t kCountSumTiles = 2048;        // up to this many tiles the segmented sum needs no prefix kernel
inline bool is_spmv(mmv_op op) { return op == MMV_OP_SPMV_COO || op == MMV_OP_SPMV_CSR; }
inline int max_cpw(mmv_op op, mmv_dtype dt) {
    if (is_spmv(op)) return TSpmv::kMaxCpw;
    switch (dt) {
        case MMV_F32_F32: return TF32::kMaxCpw;
        case MMV_F16_F32: return TF16::kMaxCpw;
        case MMV_BF16_F32: return TBF16::kMaxCpw;
        case MMV_I8_I32: return TI8::kMaxCpw;
    }
    return 1;
}
inline int waves_of(mmv_op op, mmv_dtype dt) {
    if (is_spmv(op)) return TSpmv::kWaves;
    switch (dt) {
        case MMV_F32_F32: return TF32::kWaves;
        case MMV_F16_F32: return TF16::kWaves;
        case MMV_BF16_F32: return TBF16::kWaves;
        case MMV_I8_I32: return TI8::kWaves;
    }
    return 1;
}
struct TilePlan {
    uint64_t big_tiles, tail_tiles;
    uint32_t big_elems, tail_cpw, tail_elems;
    uint64_t tiles() const { return big_tiles + tail_tiles; }
};
inline TilePlan tile_plan(mmv_op op, mmv_dtype dt, uint64_t n) {
    TilePlan p;
    const uint64_t unit = (uint64_t)waves_of(op, dt) * kChunkElems;  // one chunk per wave
    const int cpw = max_cpw(op, dt);
    p.big_elems = (uint32_t)(unit * cpw);
    if (n <= kResident * p.big_elems) {
        // one round: equal tiles, as small as gives every resident workgroup at most one
        uint64_t c = (n + kResident * unit - 1) / (kResident * unit);
        if (c < 1) c = 1;
        if (c > (uint64_t)cpw) c = cpw;
        p.tail_cpw = (uint32_t)c;
        p.big_tiles = 0;
    } else {
        p.tail_cpw = MMV_TAIL_CPW < cpw ? MMV_TAIL_CPW : cpw;
        const uint64_t tail = kTailTiles * unit * p.tail_cpw < n ? kTailTiles * unit * p.tail_cpw : n;
        p.big_tiles = (n - tail) / p.big_elems;
    }
    p.tail_elems = (uint32_t)(unit * p.tail_cpw);
    const uint64_t rest = n - p.big_tiles * p.big_elems;
    p.tail_tiles = (rest + p.tail_elems - 1) / p.tail_elems;
    return p;
}
inline uint64_t tiles_for(uint64_t n, mmv_op op, mmv_dtype dt) { return tile_plan(op, dt, n).tiles(); }
inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }
inline bool aligned4(const void *p) { return ((uintptr_t)p & 3u) == 0; }

struct WsLayout {
    size_t desc_v, desc_c, packed, total;
};

WsLayout ws_layout(mmv_op op, mmv_dtype dt, mmv_flag_fmt ff, uint64_t n) {
    WsLayout L;
    const uint64_t t = tiles_for(n, op, dt);
    size_t off = kHdrBytes;
    L.desc_v = off;
    off += round256(t * 8);
    L.desc_c = off;
    if (op == MMV_OP_SEGSUM || op == MMV_OP_SPMV_CSR) off += round256(t * 8);
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

#ifdef MMV_TRACE
uint64_t *g_trace = nullptr;
#endif

// Optional instrumentation (mmv_set_kernel_events): events recorded right before and
// right after the main kernel of a call made by this host thread.
thread_local hipEvent_t tl_ev_start = nullptr, tl_ev_stop = nullptr;

// Workgroups of `kernel` that the current device holds at once (0 when a query fails); asked once
// per kernel and device.
uint32_t resident_workgroups(const void *kernel, int threads) {
    struct Entry {
        const void *kernel;
        int device;
        uint32_t value;
    };
    static std::mutex mu;
    static std::vector<Entry> known;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    std::lock_guard<std::mutex> lock(mu);
    for (const Entry &e : known)
        if (e.kernel == kernel && e.device == dev) return e.value;
    int per_cu = 0, cus = 0;
    uint32_t value = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && per_cu > 0 && cus > 0)
        value = (uint32_t)per_cu * (uint32_t)cus;
    known.push_back({kernel, dev, value});
    return value;
}

template <typename TT, int kOp, bool kMfma> hipError_t launch_variant(Params P, hipStream_t s) {
#ifdef MMV_TRACE
    P.trace = g_trace;
#endif
    const uint32_t resident = resident_workgroups((const void *)seg_kernel<TT, kOp, kMfma>, TT::kWaves * 64);
    P.ordered = P.num_tiles <= resident ? 1u : 0u;
    // SpMV: the workgroups of the first round start spread over about one tile time.  Started together
    // they stay in step (load, gather, compute all at the same time) and the memory pipe idles half the
    // time; measured 4 to 7 % on the long SpMV kernels, nothing on the scans.
    P.stagger_wgs = resident;
    P.stagger_ticks = (kOp == kSpmv || kOp == kSpmvCsr) ? MMV_SPMV_STAGGER_US * 100u : 0u;
    seg_kernel<TT, kOp, kMfma><<<P.num_tiles, TT::kWaves * 64, 0, s>>>(P, P.hdr + kHdrHints);
    return hipGetLastError();
}

template <typename TT, int kOp>
hipError_t launch_seg(Params P, mmv_variant v, hipStream_t s) {
    const TilePlan plan = tile_plan((mmv_op)kOp, TT::kDtype, P.n);
    if (plan.tiles() > 0x7fffffffull) return hipErrorInvalidValue;
    P.num_tiles = (uint32_t)plan.tiles();
    P.big_tiles = (uint32_t)plan.big_tiles;
    P.tail_cpw = plan.tail_cpw;
    if (tl_ev_start && hipEventRecord(tl_ev_start, s) != hipSuccess) return hipErrorUnknown;
    if (v == MMV_VARIANT_MFMA) {
        if (launch_variant<TT, kOp, true>(P, s) != hipSuccess) return hipErrorUnknown;
    } else {
        if (launch_variant<TT, kOp, false>(P, s) != hipSuccess) return hipErrorUnknown;
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
    }
    return hipErrorInvalidValue;
}

int grid_for(uint64_t items_per_thread_total) {
    uint64_t blocks = (items_per_thread_total + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 2048) blocks = 2048;
    return (int)blocks;
}

bool valid_dtype(int dt) { return dt >= 0 && dt <= 3; }
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
    if (compress_words(n) == 16)
        compress_kernel<16><<<(unsigned)L.tiles, kCompressWaves * 64, 0, s>>>(
            (const uint32_t *)d_x, mw, n, (uint32_t *)d_out, out_capacity, d_count, (uint32_t *)ws,
            (uint64_t *)(ws + L.desc), (uint32_t)L.tiles, d_needed);
    else
        compress_kernel<64><<<(unsigned)L.tiles, kCompressWaves * 64, 0, s>>>(
            (const uint32_t *)d_x, mw, n, (uint32_t *)d_out, out_capacity, d_count, (uint32_t *)ws,
            (uint64_t *)(ws + L.desc), (uint32_t)L.tiles, d_needed);
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
                                                                  n, nw, (uint32_t *)d_z, nullptr);
    else
        revert_kernel<float><<<(unsigned)blocks, 256, 0, s>>>((const uint32_t *)d_xhat, d_fhat, (const uint32_t *)d_w, n,
                                                               nw, (uint32_t *)d_z, nullptr);
    const hipError_t e = hipGetLastError();
    if (tl_ev_stop && hipEventRecord(tl_ev_stop, s) != hipSuccess) return MMV_ERR_HIP;
    return e == hipSuccess ? MMV_OK : MMV_ERR_HIP;
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
    hipStream_t s = (hipStream_t)hip_stream;
    Params P = {};
    const mmv_status st = prepare(MMV_OP_SEGSCAN, d_x, d_flags, n, dt, ff, v, d_ws, ws_bytes, s, P);
    if (st != MMV_OK) return st;
    P.z = d_z;
    return launch_dt<kScan>(P, dt, v, s) == hipSuccess ? MMV_OK : MMV_ERR_HIP;
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
    const TilePlan plan = tile_plan(MMV_OP_SEGSUM, dt, n);
    const WsLayout L = ws_layout(MMV_OP_SEGSUM, dt, ff, n);
    uint32_t *tile_count = (uint32_t *)((char *)d_ws + L.desc_c);
    if (plan.tiles() > 0x7fffffffull) return MMV_ERR_INVALID_ARG;
    count_tiles_kernel<<<(unsigned)plan.tiles(), 256, 0, s>>>((uint32_t *)d_ws, L.desc_c / 4, P.fw, n,
                                                               (uint32_t)plan.big_tiles, plan.big_elems,
                                                               plan.tail_elems, tile_count);
    if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    // few tiles: every tile of the main kernel adds up the counts before it; many: one more small kernel
    // turns the counts into prefix sums first
    P.count_is_prefix = plan.tiles() > kCountSumTiles ? 1u : 0u;
    if (P.count_is_prefix) {
        scan_counts_kernel<<<1, 1024, 0, s>>>(tile_count, (uint32_t)plan.tiles(), d_nseg);
        if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    }
    P.tile_count = tile_count;
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
    const uint64_t zero_words = L.packed / 4;  // header + descriptors; the flag words are all written below
    fill_zero_kernel<<<grid_for(zero_words > n_rows ? zero_words : n_rows), 256, 0, s>>>((uint32_t *)ws, zero_words,
                                                                                      (uint32_t *)d_y, n_rows);
    if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    const uint64_t flag_blocks = (nnz + 4095) / 4096;
    if (flag_blocks > 0x7fffffffull) return MMV_ERR_INVALID_ARG;
    row_flags_kernel<<<(unsigned)flag_blocks, 256, 0, s>>>(d_row, nnz, (uint32_t *)(ws + L.packed), d_col, (uint32_t *)ws);
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
                                                          (uint32_t *)(ws + C.main_ws), (uint32_t)plan.big_tiles,
                                                          plan.big_elems, plan.tail_elems, tile_count, d_col, nnz);
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
    P.count_is_prefix = plan.tiles() > kCountSumTiles ? 1u : 0u;
    if (P.count_is_prefix) {
        scan_counts_kernel<<<1, 1024, 0, s>>>(tile_count, (uint32_t)plan.tiles(), (uint64_t *)(ws + C.rowcount));
        if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    }
    P.tile_count = tile_count;
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

#ifdef MMV_TRACE
// Development builds only: device buffer of 8 uint64 per tile that receives phase timestamps.
void mmv_trace_buffer(void *d_trace) { g_trace = (uint64_t *)d_trace; }
#endif

const char *mmv_status_string(mmv_status s) {
    switch (s) {
        case MMV_OK: return "ok";
        case MMV_ERR_INVALID_ARG: return "invalid argument";
        case MMV_ERR_NULL: return "null pointer";
        case MMV_ERR_UNSUPPORTED: return "unsupported";
        case MMV_ERR_WORKSPACE: return "workspace too small or misaligned";
        case MMV_ERR_HIP: return "HIP error";
    }
    return "unknown status";
}

uint32_t mmv_tile_elems(mmv_op op, mmv_dtype dt, uint64_t n) {
    if (!valid_dtype(dt)) return 0;
    if (op == MMV_OP_COMPRESS) return (uint32_t)compress_tile(n);
    if (op != MMV_OP_SEGSCAN && op != MMV_OP_SEGSUM && op != MMV_OP_SCAN && !is_spmv(op)) return 0;
    const TilePlan p = tile_plan(op, is_spmv(op) ? MMV_F32_F32 : dt, n);
    return p.big_tiles ? p.big_elems : p.tail_elems;
}

}  // extern "C"
