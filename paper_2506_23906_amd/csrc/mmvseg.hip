// libmmvseg: segmented inclusive scan, segmented sum and row-sorted COO SpMV for
// gfx950 (MI355X), after the block-recursive segmented scan of "Segmented
// Operations using Matrix Multiplications" (Sec. 4.2 and the appendix algorithm
// "Block-recursive segmented scan").
//
// One kernel launch does the whole operation (single pass over HBM):
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
// Layout of a workgroup tile: 4 waves x 64 rows x 32 elements = 8192 elements.
// Lane r of a wave owns row r of the wave's 2048-element chunk for steps 3-5;
// one packed flag word is exactly one row.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mmvseg.h"

namespace {

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kS = 32;                          // row length = MFMA tile edge
constexpr int kRowsPerWave = 64;                // one row per lane
constexpr int kWaveElems = kS * kRowsPerWave;   // 2048
constexpr int kTileElems = kWaves * kWaveElems; // 8192
constexpr int kRowStride = 36;                  // dwords per LDS row: 4 meta + 32 values
constexpr int kSlotF = 0;                       // flag word of the row
constexpr int kSlotE = 1;                       // segment-end mask of the row
constexpr int kSlotNegCarry = 2;                // minus the carry into the row
constexpr int kSlotZero = 3;                    // x-bar(-1) = 0
constexpr int kRowData = 4;

constexpr uint32_t kHdrTicket = 0;              // workspace header words
constexpr uint32_t kHdrError = 1;
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

enum Op { kScan = 0, kSum = 1, kSpmv = 2 };

struct Params {
    const void *x;          // values (scan, sum) / val (spmv)
    const uint32_t *fw;     // packed flag words (scan, sum)
    uint64_t n;             // elements / nnz
    void *z;                // scan output
    void *out;              // sum output
    uint64_t out_cap;
    uint64_t *nseg;
    const int32_t *row;     // spmv
    const int32_t *col;
    const float *xv;
    float *y;
    uint32_t *hdr;          // workspace header
    uint64_t *desc_v;       // value descriptors, one per tile
    uint64_t *desc_c;       // count descriptors (sum)
    uint32_t num_tiles;
};

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

template <typename T> __device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += from_bits<T>(__shfl_xor(to_bits(v), d));
    return v;
}

// Sum of the payloads of the predecessor tiles back to (and including) the first
// one whose descriptor says "prefix".  The whole wave polls 64 descriptors at a
// time.  Tile -1 counts as prefix 0, so the loop always ends there at the latest.
template <typename T>
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
        carry += wave_sum(v);
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
    static __device__ __forceinline__ acc_t widen(in_t v) { return (acc_t)(int32_t)v; }
};
struct TF16 {
    typedef _Float16 in_t;
    typedef float acc_t;
    static constexpr int kEpl = 8;
    static __device__ __forceinline__ acc_t widen(in_t v) { return (float)v; }
};
struct TBF16 {
    typedef __bf16 in_t;
    typedef float acc_t;
    static constexpr int kEpl = 8;
    static __device__ __forceinline__ acc_t widen(in_t v) { return (float)v; }
};
struct TF32 {
    typedef float in_t;
    typedef float acc_t;
    static constexpr int kEpl = 4;
    static __device__ __forceinline__ acc_t widen(in_t v) { return v; }
};

// Loads kCount consecutive elements starting at element index e0 (e0 * sizeof is a
// multiple of 16 when kCount * sizeof == 16); elements at or beyond n read as zero.
template <typename T, int kCount>
__device__ __forceinline__ void load_elems(const T *x, uint64_t e0, uint64_t n, bool full, T (&dst)[kCount]) {
    static_assert(kCount * sizeof(T) == 16, "one 128-bit load");
    if (full) {
        *reinterpret_cast<v4u *>(dst) = *reinterpret_cast<const v4u *>(x + e0);
    } else {
#pragma unroll
        for (int i = 0; i < kCount; ++i) dst[i] = (e0 + i < n) ? x[e0 + i] : T(0);
    }
}

// ---- step 1, matrix-core form ---------------------------------------------------------------------
//
// One 32x32 tile = 32 rows ("runs") of 32 consecutive elements.  D = A B with
// A = U_s^T (lower-triangular ones, M x K) and B = X^T (K x N, column n = run n):
// D(m, n) = sum_{k <= m} X(n, k) = x-bar at position m of run n.
// Operand registers: lane (c = lane % 32, h = lane / 32) holds, for A, row c and
// for B, column c, with the K indices that half h owns.  A and B use the same
// (half, register, byte) -> K map, so only "which positions does half h hold"
// has to agree between the two operands.
// Result registers: acc[v] of lane (n, h) = D(8 (v / 4) + 4 h + v % 4, n).

template <typename TT> struct Spec;

template <> struct Spec<TI8> {
    // lane (n, h) loads positions 16 h .. 16 h + 15 of run n: one 128-bit load
    static __device__ __forceinline__ void run(const int8_t *x, uint64_t tile0, uint64_t n, bool full, int lane,
                                               uint32_t (&acc)[16]) {
        const int c = lane & 31, h = lane >> 5;
        alignas(16) int8_t b[16];
        load_elems<int8_t, 16>(x, tile0 + 32 * c + 16 * h, n, full, b);
        v4i a;
#pragma unroll
        for (int d = 0; d < 4; ++d) {  // bytes 4d..4d+3 = positions 16h+4d+j: one where position <= c
            int cnt = c - (16 * h + 4 * d) + 1;
            cnt = cnt < 0 ? 0 : (cnt > 4 ? 4 : cnt);
            a[d] = cnt == 4 ? 0x01010101 : (int)(0x01010101u & ((1u << (8 * cnt)) - 1u));
        }
        v16i r = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        r = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, *reinterpret_cast<v4i *>(b), r, 0, 0, 0);
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = (uint32_t)r[v];
    }
};

template <> struct Spec<TF16> {
    // two K-steps of 16: lane (n, h) loads positions 16 ks + 8 h .. + 7 of run n
    static __device__ __forceinline__ void run(const _Float16 *x, uint64_t tile0, uint64_t n, bool full, int lane,
                                               float (&acc)[16]) {
        const int c = lane & 31, h = lane >> 5;
        v16f r = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            alignas(16) _Float16 b[8];
            load_elems<_Float16, 8>(x, tile0 + 32 * c + 16 * ks + 8 * h, n, full, b);
            v8h a;
#pragma unroll
            for (int j = 0; j < 8; ++j) a[j] = (16 * ks + 8 * h + j <= c) ? (_Float16)1.0f : (_Float16)0.0f;
            r = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, *reinterpret_cast<v8h *>(b), r, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = r[v];
    }
};

template <> struct Spec<TBF16> {
    static __device__ __forceinline__ void run(const __bf16 *x, uint64_t tile0, uint64_t n, bool full, int lane,
                                               float (&acc)[16]) {
        const int c = lane & 31, h = lane >> 5;
        v16f r = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            alignas(16) __bf16 b[8];
            load_elems<__bf16, 8>(x, tile0 + 32 * c + 16 * ks + 8 * h, n, full, b);
            v8s a;
#pragma unroll
            for (int j = 0; j < 8; ++j) a[j] = (16 * ks + 8 * h + j <= c) ? (short)0x3F80 : (short)0;  // bf16 1.0
            r = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), *reinterpret_cast<v8bf *>(b), r,
                                                        0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = r[v];
    }
};

// fp32: sixteen K-steps of 2; in step t half h supplies position 16 h + t.
__device__ __forceinline__ void spec_f32_from_regs(const float (&b)[16], int lane, float (&acc)[16]) {
    const int c = lane & 31, h = lane >> 5;
    v16f r = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        const float a = (16 * h + t <= c) ? 1.0f : 0.0f;
        r = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b[t], r, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = r[v];
}

template <> struct Spec<TF32> {
    static __device__ __forceinline__ void run(const float *x, uint64_t tile0, uint64_t n, bool full, int lane,
                                               float (&acc)[16]) {
        const int c = lane & 31, h = lane >> 5;
        float b[16];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            alignas(16) float t4[4];
            load_elems<float, 4>(x, tile0 + 32 * c + 16 * h + 4 * q, n, full, t4);
#pragma unroll
            for (int i = 0; i < 4; ++i) b[4 * q + i] = t4[i];
        }
        spec_f32_from_regs(b, lane, acc);
    }
};

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

// ---- step 1, vector-only form (ablation) ------------------------------------------------------------
//
// Every lane loads 128 bits = kEpl consecutive elements, prefix-sums them in
// registers, and the 32 / kEpl lanes that share a row combine with lane shuffles.
template <typename TT>
__device__ __forceinline__ void spec_shuffle_tile(const typename TT::in_t *x, uint64_t tile0, uint64_t n, bool full,
                                                  int lane, uint32_t *rows, int t) {
    typedef typename TT::acc_t A;
    constexpr int kEpl = TT::kEpl;
    constexpr int kLpr = 32 / kEpl;         // lanes per row
    constexpr int kRowsPerLoad = 64 / kLpr;
    constexpr int kLoads = 32 / kRowsPerLoad;
#pragma unroll
    for (int ld = 0; ld < kLoads; ++ld) {
        alignas(16) typename TT::in_t b[kEpl];
        load_elems<typename TT::in_t, kEpl>(x, tile0 + (uint64_t)(kRowsPerLoad * 32 * ld + kEpl * lane), n, full, b);
        A p[kEpl];
        p[0] = TT::widen(b[0]);
#pragma unroll
        for (int i = 1; i < kEpl; ++i) p[i] = p[i - 1] + TT::widen(b[i]);
        A inc = p[kEpl - 1];
#pragma unroll
        for (int d = 1; d < kLpr; d <<= 1) {
            const A o = from_bits<A>(__shfl_up(to_bits(inc), d));
            if ((lane & (kLpr - 1)) >= d) inc += o;
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

template <typename TT, int kOp, bool kMfma>
__global__ __launch_bounds__(kThreads) void seg_kernel(Params P) {
    typedef typename TT::acc_t A;
    typedef typename TT::in_t In;

    __shared__ __attribute__((aligned(16))) uint32_t s_rows[kWaves][kRowsPerWave * kRowStride];
    __shared__ uint32_t s_cnt[kWaves * kRowsPerWave];  // segment starts before each row (sum)
    __shared__ uint32_t s_wave_v[kWaves], s_wave_f[kWaves], s_wave_c[kWaves];
    __shared__ uint32_t s_tile, s_carry_v, s_carry_c;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) s_tile = __hip_atomic_fetch_add(P.hdr + kHdrTicket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const int tile = (int)s_tile;
    const uint64_t n = P.n;
    const uint64_t wave_base = (uint64_t)tile * kTileElems + (uint64_t)wave * kWaveElems;
    const bool wave_full = wave_base + kWaveElems <= n;
    uint32_t *rows = s_rows[wave];
    const uint64_t row_start = wave_base + 32u * lane;  // first element of the row this lane owns

    // ---- flags of my row (one 32-bit word = one row) ----
    uint32_t F = 0;
    if (kOp == kSpmv) {
        // f(e) = [e == 0 or row(e) != row(e-1)], 64 elements per ballot
        int prev_last = wave_base > 0 && wave_base - 1 < n ? P.row[wave_base - 1] : -1;
        for (int j = 0; j < 32; ++j) {
            const uint64_t e = wave_base + 64u * j + lane;
            const int r = e < n ? P.row[e] : 0;
            int rp = __shfl_up(r, 1);
            if (lane == 0) rp = prev_last;
            const uint64_t m = __ballot(e < n && (e == 0 || r != rp));
            if (lane == 2 * j) F = (uint32_t)m;
            if (lane == 2 * j + 1) F = (uint32_t)(m >> 32);
            prev_last = __shfl(r, 63);
        }
    } else {
        if (row_start < n) {
            F = P.fw[row_start >> 5];
            if (row_start + 32 > n) F &= (1u << (uint32_t)(n - row_start)) - 1u;
        }
    }

    // ---- step 1: speculative row scans into LDS ----
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const uint64_t tile0 = wave_base + 1024u * t;
        if (kOp == kSpmv) {
            // product vector p(i) = val(i) * x(col(i)), built in the layout step 1 needs
            if (kMfma) {
                const int c = lane & 31, h = lane >> 5;
                float b[16];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    alignas(16) float v4[4];
                    alignas(16) int c4[4];
                    const uint64_t e0 = tile0 + 32 * c + 16 * h + 4 * q;
                    load_elems<float, 4>((const float *)P.x, e0, n, wave_full, v4);
                    load_elems<int, 4>(P.col, e0, n, wave_full, c4);
#pragma unroll
                    for (int i = 0; i < 4; ++i) b[4 * q + i] = (e0 + i < n) ? v4[i] * P.xv[c4[i]] : 0.0f;
                }
                float acc[16];
                spec_f32_from_regs(b, lane, acc);
                store_spec_rows(rows, t, lane, acc);
            } else {
#pragma unroll
                for (int ld = 0; ld < 4; ++ld) {
                    alignas(16) float v4[4];
                    float p[4];
                    alignas(16) int c4[4];
                    const uint64_t e0 = tile0 + 256 * ld + 4 * lane;
                    load_elems<float, 4>((const float *)P.x, e0, n, wave_full, v4);
                    load_elems<int, 4>(P.col, e0, n, wave_full, c4);
#pragma unroll
                    for (int i = 0; i < 4; ++i) p[i] = (e0 + i < n) ? v4[i] * P.xv[c4[i]] : 0.0f;
                    p[1] += p[0];
                    p[2] += p[1];
                    p[3] += p[2];
                    float inc = p[3];
#pragma unroll
                    for (int d = 1; d < 8; d <<= 1) {
                        const float o = __shfl_up(inc, d);
                        if ((lane & 7) >= d) inc += o;
                    }
                    const float ex = inc - p[3];
                    v4u w = {to_bits(p[0] + ex), to_bits(p[1] + ex), to_bits(p[2] + ex), to_bits(p[3] + ex)};
                    *reinterpret_cast<v4u *>(rows + (32 * t + 8 * ld + lane / 8) * kRowStride + kRowData +
                                             4 * (lane & 7)) = w;
                }
            }
        } else if (kMfma) {
            A acc[16];
            Spec<TT>::run((const In *)P.x, tile0, n, wave_full, lane, acc);
            store_spec_rows(rows, t, lane, acc);
        } else {
            spec_shuffle_tile<TT>((const In *)P.x, tile0, n, wave_full, lane, rows, t);
        }
    }
    rows[lane * kRowStride + kSlotZero] = 0;
    rows[lane * kRowStride + kSlotF] = F;
    wave_lds_sync();

    // ---- steps 2-4 for the aggregate of my row: last element after the revert, any flag ----
    const bool has_flag = F != 0;
    A agg_v;
    {
        const A last = from_bits<A>(rows[lane * kRowStride + kRowData + 31]);
        const int slot = has_flag ? kSlotZero + (31 - __clz(F)) : kSlotZero;  // x-bar(start - 1)
        agg_v = last - from_bits<A>(rows[lane * kRowStride + slot]);
    }
    // segment starts in my row, position 0 of the whole vector not counted (sum only)
    const uint32_t Fc = row_start == 0 ? (F & ~1u) : F;
    uint32_t cnt = __popc(Fc);

    // ---- step 5a: segmented inclusive scan of (value, flag) over the 64 rows of the wave ----
    A inc_v = agg_v;
    uint32_t inc_f = has_flag;
    uint32_t inc_c = cnt;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const A ov = from_bits<A>(__shfl_up(to_bits(inc_v), d));
        const uint32_t of = __shfl_up(inc_f, d);
        if (lane >= d) {
            if (!inc_f) inc_v = ov + inc_v;
            inc_f |= of;
        }
        if (kOp == kSum) {
            const uint32_t oc = __shfl_up(inc_c, d);
            if (lane >= d) inc_c += oc;
        }
    }
    A ex_v = from_bits<A>(__shfl_up(to_bits(inc_v), 1));
    uint32_t ex_f = __shfl_up(inc_f, 1);
    if (lane == 0) {
        ex_v = A(0);
        ex_f = 0;
    }
    const uint32_t ex_c = inc_c - cnt;
    if (lane == 63) {
        s_wave_v[wave] = to_bits(inc_v);
        s_wave_f[wave] = inc_f;
        s_wave_c[wave] = inc_c;
    }

    // segment-end mask of my row (sum, spmv): bit p set iff position p + 1 starts a segment
    // or p is the last element of the vector
    if (kOp != kScan) {
        uint32_t next0 = __shfl_down(F, 1) & 1u;
        if (lane == 63) {
            const uint64_t en = wave_base + kWaveElems;
            next0 = 0;
            if (en < n) next0 = kOp == kSpmv ? (P.row[en] != P.row[en - 1]) : (P.fw[en >> 5] & 1u);
        }
        uint32_t E = (F >> 1) | (next0 << 31);
        if (row_start < n) {
            if (row_start + 32 >= n) E = (E & ((1u << (uint32_t)(n - 1 - row_start)) - 1u)) | (1u << (uint32_t)(n - 1 - row_start));
        } else {
            E = 0;
        }
        rows[lane * kRowStride + kSlotE] = E;
    }
    __syncthreads();

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
        const A wv = from_bits<A>(s_wave_v[w]);
        const uint32_t wf = s_wave_f[w];
        tagg_v = wf ? wv : tagg_v + wv;
        tagg_f |= wf;
        tagg_c += s_wave_c[w];
    }

    // ---- step 5c: tiles, by decoupled look-back ----
    if (wave == 0) {
        const bool final_now = tile == 0 || tagg_f;  // carry out does not depend on predecessors
        if (lane == 0) desc_store(P.desc_v + tile, final_now ? kStatusPrefix : kStatusAggregate, to_bits(tagg_v));
        A carry = A(0);
        if (tile > 0) carry = lookback<A>(P.desc_v, tile, lane, P.hdr);
        if (lane == 0) {
            if (!final_now) desc_store(P.desc_v + tile, kStatusPrefix, to_bits(carry + tagg_v));
            s_carry_v = to_bits(carry);
        }
    }
    if (kOp == kSum && wave == 1) {
        if (lane == 0) desc_store(P.desc_c + tile, tile == 0 ? kStatusPrefix : kStatusAggregate, tagg_c);
        uint32_t carry = 0;
        if (tile > 0) carry = lookback<uint32_t>(P.desc_c, tile, lane, P.hdr);
        if (lane == 0) {
            if (tile > 0) desc_store(P.desc_c + tile, kStatusPrefix, carry + tagg_c);
            s_carry_c = carry;
            if ((uint32_t)tile == P.num_tiles - 1) *P.nseg = (uint64_t)carry + tagg_c + 1u;
        }
    }
    __syncthreads();

    // ---- step 6: carry into my row; stored negated so that the revert subtracts it ----
    {
        const A tile_carry = from_bits<A>(s_carry_v);
        const A carry = ex_f ? ex_v : (wex_f ? wex_v + ex_v : tile_carry + wex_v + ex_v);
        rows[lane * kRowStride + kSlotNegCarry] = to_bits(A(0) - carry);
        if (kOp == kSum) s_cnt[wave * kRowsPerWave + lane] = s_carry_c + wex_c + ex_c;
    }
    const uint64_t row_any = __ballot(has_flag);
    wave_lds_sync();

    // ---- steps 2 + 6 on every element, then store; lane owns 4 consecutive positions ----
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int R = 8 * j + (lane >> 3), p0 = 4 * (lane & 7);
        const uint32_t *rp = rows + R * kRowStride;
        const v4u xb = *reinterpret_cast<const v4u *>(rp + kRowData + p0);
        A o[4];
        uint32_t Fr = 0;
        if (((row_any >> (8 * j)) & 0xFFull) == 0) {
            // none of these eight rows has a flag: the speculation stands, only the carry is added
            const A nc = from_bits<A>(rp[kSlotNegCarry]);
#pragma unroll
            for (int i = 0; i < 4; ++i) o[i] = from_bits<A>(xb[i]) - nc;
        } else {
            Fr = rp[kSlotF];
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
        const uint64_t e0 = wave_base + 256u * j + 4u * lane;
        if (kOp == kScan) {
            A *z = (A *)P.z;
            if (wave_full) {
                v4u w = {to_bits(o[0]), to_bits(o[1]), to_bits(o[2]), to_bits(o[3])};
                *reinterpret_cast<v4u *>(z + e0) = w;
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (e0 + i < n) z[e0 + i] = o[i];
            }
        } else {
            const uint32_t ends = (rp[kSlotE] >> p0) & 0xFu;
            if (ends) {
                if (kOp == kSum) {
                    if (!Fr) Fr = rp[kSlotF];
                    const uint32_t Frc = (wave_base == 0 && R == 0) ? (Fr & ~1u) : Fr;
                    const uint32_t base = s_cnt[wave * kRowsPerWave + R];
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if ((ends >> i) & 1u) {
                            const uint64_t k = (uint64_t)base + __popc(Frc & ((2u << (p0 + i)) - 1u));
                            if (k < P.out_cap) ((A *)P.out)[k] = o[i];
                        }
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if ((ends >> i) & 1u) P.y[P.row[e0 + i]] = from_bits<float>(to_bits(o[i]));
                }
            }
        }
    }
}

// ---- auxiliary kernels -------------------------------------------------------------------------------------

// Zero fills two ranges (workspace words and, for SpMV, y) with 32-bit stores.
__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t *a, uint64_t na, uint32_t *b, uint64_t nb) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < na; i += stride) a[i] = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nb; i += stride) b[i] = 0;
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

// Streaming reference: 128-bit reads and writes, kIn input chunks and kOut output
// chunks per thread and step, both striped across the workgroup.
template <int kIn, int kOut>
__global__ __launch_bounds__(256) void stream_copy_kernel(const v4u *src, v4u *dst, uint64_t units) {
    const uint64_t nblocks = (units + 255) / 256;
    for (uint64_t blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
        const uint64_t u0 = blk * 256;
        v4u acc = {0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < kIn; ++i) {
            const uint64_t idx = u0 * kIn + (uint64_t)i * 256 + threadIdx.x;
            if (idx < units * kIn) acc ^= src[idx];
        }
#pragma unroll
        for (int i = 0; i < kOut; ++i) {
            const uint64_t idx = u0 * kOut + (uint64_t)i * 256 + threadIdx.x;
            if (idx < units * kOut) dst[idx] = acc + (unsigned)i;
        }
        if (kOut == 0 && acc[0] == 0x9E3779B9u && acc[1] == 0x7F4A7C15u && acc[2] == 1u && acc[3] == 2u)
            dst[0] = acc;  // keeps the reads alive; practically never taken
    }
}

// ---- host side -------------------------------------------------------------------------------------------------

inline size_t round256(size_t b) { return (b + 255) & ~(size_t)255; }
inline uint64_t tiles_for(uint64_t n) { return (n + kTileElems - 1) / kTileElems; }
inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

struct WsLayout {
    size_t desc_v, desc_c, packed, total;
};

WsLayout ws_layout(mmv_op op, mmv_flag_fmt ff, uint64_t n) {
    WsLayout L;
    const uint64_t t = tiles_for(n);
    size_t off = kHdrBytes;
    L.desc_v = off;
    off += round256(t * 8);
    L.desc_c = off;
    if (op == MMV_OP_SEGSUM) off += round256(t * 8);
    L.packed = off;
    if (op != MMV_OP_SPMV_COO && ff == MMV_FLAGS_U8) off += round256(((n + 31) / 32) * 4);
    L.total = off;
    return L;
}

// Optional instrumentation (mmv_set_kernel_events): events recorded right before and
// right after the main kernel of a call made by this host thread.
thread_local hipEvent_t tl_ev_start = nullptr, tl_ev_stop = nullptr;

template <typename TT, int kOp>
hipError_t launch_seg(const Params &P, mmv_variant v, hipStream_t s) {
    if (tl_ev_start && hipEventRecord(tl_ev_start, s) != hipSuccess) return hipErrorUnknown;
    if (v == MMV_VARIANT_MFMA)
        seg_kernel<TT, kOp, true><<<P.num_tiles, kThreads, 0, s>>>(P);
    else
        seg_kernel<TT, kOp, false><<<P.num_tiles, kThreads, 0, s>>>(P);
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
constexpr uint64_t kMaxN = 1ull << 40;

// Common part of scan and sum: checks, workspace reset, flag packing.
mmv_status prepare(mmv_op op, const void *d_x, const void *d_flags, uint64_t n, mmv_dtype dt, mmv_flag_fmt ff,
                   mmv_variant v, void *d_ws, size_t ws_bytes, hipStream_t s, Params &P) {
    if (!valid_dtype(dt) || !valid_ff(ff) || !valid_variant(v) || n > kMaxN) return MMV_ERR_INVALID_ARG;
    if (!d_x || !d_flags) return MMV_ERR_NULL;
    if (!aligned16(d_x) || !aligned16(d_flags)) return MMV_ERR_INVALID_ARG;
    if (!d_ws) return MMV_ERR_NULL;
    const WsLayout L = ws_layout(op, ff, n);
    if (((uintptr_t)d_ws & 255u) != 0 || ws_bytes < L.total) return MMV_ERR_WORKSPACE;
    char *ws = (char *)d_ws;
    P.x = d_x;
    P.n = n;
    P.hdr = (uint32_t *)ws;
    P.desc_v = (uint64_t *)(ws + L.desc_v);
    P.desc_c = (uint64_t *)(ws + L.desc_c);
    P.num_tiles = (uint32_t)tiles_for(n);
    const uint64_t zero_words = L.packed / 4;  // header + descriptors
    fill_zero_kernel<<<grid_for(zero_words), 256, 0, s>>>((uint32_t *)ws, zero_words, nullptr, 0);
    if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
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

}  // namespace

// ---- C ABI ------------------------------------------------------------------------------------------------------

extern "C" {

size_t mmv_workspace_bytes(mmv_op op, mmv_dtype dt, mmv_flag_fmt ff, uint64_t n) {
    if ((int)op < 0 || (int)op > 2 || !valid_dtype(dt) || !valid_ff(ff) || n > kMaxN) return 0;
    return ws_layout(op, ff, n).total;
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
    if (!valid_dtype(dt) || !valid_ff(ff) || !valid_variant(v)) return MMV_ERR_INVALID_ARG;
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
    const WsLayout L = ws_layout(MMV_OP_SPMV_COO, MMV_FLAGS_PACKED32, nnz);
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
    P.desc_c = nullptr;
    P.num_tiles = (uint32_t)tiles_for(nnz);
    const uint64_t zero_words = L.total / 4;
    fill_zero_kernel<<<grid_for(zero_words > n_rows ? zero_words : n_rows), 256, 0, s>>>((uint32_t *)ws, zero_words,
                                                                                      (uint32_t *)d_y, n_rows);
    if (hipGetLastError() != hipSuccess) return MMV_ERR_HIP;
    return launch_seg<TF32, kSpmv>(P, v, s) == hipSuccess ? MMV_OK : MMV_ERR_HIP;
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
        uint64_t blocks_ = (units_ + 255) / 256;                                                         \
        if (blocks_ > 16384) blocks_ = 16384;                                                            \
        stream_copy_kernel<KI, KO><<<(int)blocks_, 256, 0, s>>>(src, dst, units_);                       \
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
    }
    return "unknown status";
}

uint32_t mmv_tile_elems(void) { return kTileElems; }

}  // extern "C"
