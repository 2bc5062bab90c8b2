// libmmvseg, part of the one translation unit mmvseg.hip (included there, in order).
// Element types, the raw registers of a wave chunk, step 1 on the matrix cores, row aggregates straight
// from the raw registers, and the vector-only form of step 1 (the ablation variant).
#pragma once

namespace {

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
// Another group on the same skeleton (Sec. 2 asks only for a group): bit-wise exclusive or on bytes,
// (Z_2)^8.  "Addition" and "subtraction" are both XOR, the neutral element is 0, so the revert
// z(j) = x-bar(j) - x-bar(start - 1) and the carries work unchanged through the operators below.
struct XorWord {
    uint32_t v;
    XorWord() = default;
    __device__ __host__ constexpr explicit XorWord(uint32_t x) : v(x) {}
    __device__ __host__ constexpr explicit XorWord(int x) : v((uint32_t)x) {}
    friend __device__ __forceinline__ XorWord operator+(XorWord a, XorWord b) { return XorWord(a.v ^ b.v); }
    friend __device__ __forceinline__ XorWord operator-(XorWord a, XorWord b) { return XorWord(a.v ^ b.v); }
    __device__ __forceinline__ XorWord &operator+=(XorWord b) { v ^= b.v; return *this; }
    __device__ __forceinline__ XorWord &operator-=(XorWord b) { v ^= b.v; return *this; }
};
struct TX8 {
    typedef uint8_t in_t;
    typedef XorWord acc_t;   // the result byte in the low bits of a 32-bit word
    static constexpr int kEpl = 16;
    static constexpr int kMaxCpw = MMV_CPW_I8;
    static constexpr int kWaves = MMV_WAVES;
    static constexpr mmv_dtype kDtype = MMV_U8_XOR;
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
// Most chunks a wave of seg_tile takes.  Bytes under exclusive or in the matrix-core variant hold four accumulators
// of bit-plane sums per tile next to the raw words: two chunks fit the registers, four spill.  The scan without a
// flag vector keeps no flag words and no carried flags, which leaves room for longer tiles of 16- and 32-bit inputs; so does
// the segmented sum of fp32 values in the variant without the matrix cores.
template <typename TT, int kOp, bool kMfma> constexpr int chunks_per_wave() {
    if (TT::kDtype == MMV_U8_XOR && kMfma) return MMV_CPW_X8_MFMA;
    if (kOp == kPlainScan && sizeof(typename TT::in_t) == 2) return MMV_CPW_F16_SCAN;
    if (kOp == kPlainScan && sizeof(typename TT::in_t) == 4) return MMV_CPW_F32_SCAN;
    if (kOp == kSum && TT::kDtype == MMV_F32_F32 && !kMfma) return MMV_CPW_F32_SUM_SHUFFLE;
    return TT::kMaxCpw;
}

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

// (the two halves of the fp32 form are also called one by one: between them the registers still hold the
// striped layout)
__device__ __forceinline__ void operand_layout_write4(const v4u (&raw)[8], uint32_t *rows, int lane) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
        *reinterpret_cast<v4u *>(rows + (8 * i + (lane >> 3)) * kRowStride + kRowData + 4 * (lane & 7)) = raw[i];
}
__device__ __forceinline__ void operand_layout_read4(v4u (&raw)[8], const uint32_t *rows, int lane) {
    wave_lds_sync();
    const int c = lane & 31, h = lane >> 5;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int q = 0; q < 4; ++q)
            raw[4 * t + q] = *reinterpret_cast<const v4u *>(rows + (32 * t + c) * kRowStride + kRowData + 16 * h + 4 * q);
    wave_lds_sync();
}
template <> __device__ __forceinline__ void to_operand_layout<4>(v4u (&raw)[8], uint32_t *rows, int lane) {
    operand_layout_write4(raw, rows, lane);
    operand_layout_read4(raw, rows, lane);
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

template <> struct SpecMfma<TX8> {
    // Exclusive or through integer sums: the running XOR of a bit is the parity of its running count.
    // Two bit planes share one product (bit b in bit 0 and bit b + 1 in bit 6 of the int8 operand: counts
    // of up to 32 need six bits each), so a byte takes four matrix instructions.  Two results are packed
    // into one word (fields at bits 0, 6, 12, 18), whose four parity bits a 24-bit multiplication moves
    // next to each other: bit 6 i times 2^(15 - 5 i) lands at bit 15 + i, and no two partial products meet.
    static __device__ __forceinline__ v16i planes(const v4u &w, v4i a, int p) {   // sums of planes p and p + 1
        v4i b;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t t = w[d] >> p;
            b[d] = (int)((t & 0x01010101u) | ((t << 5) & 0x40404040u));
        }
        v16i r = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, r, 0, 0, 0);
    }
    static __device__ __forceinline__ void run(const v4u *raw, int lane, XorWord (&acc)[16]) {
        const int c = lane & 31, h = lane >> 5;
        v4i a;  // as for int8 sums: one where position <= c
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            int cnt = c - (16 * h + 4 * d) + 1;
            cnt = cnt < 0 ? 0 : (cnt > 4 ? 4 : cnt);
            a[d] = cnt == 4 ? 0x01010101 : (int)(0x01010101u & ((1u << (8 * cnt)) - 1u));
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = XorWord(0u);
#pragma unroll 1
        for (int nib = 0; nib < 2; ++nib) {   // (rolled: one nibble at a time, or the registers do not suffice)
            const v16i r0 = planes(raw[0], a, 4 * nib);
            const v16i r1 = planes(raw[0], a, 4 * nib + 2);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const uint32_t packed = (((uint32_t)r1[v] << 12) + (uint32_t)r0[v]) & 0x041041u;
                acc[v].v |= (((packed * 0x8421u) >> 15) & 0xFu) << (4 * nib);
            }
        }
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
    // the 0 / 1 operand of the two K-steps (lower-triangular ones, as bf16); the same for every tile of a lane
    struct Operand {
        v4u a[2];
    };
    static __device__ __forceinline__ Operand operand(int lane) {
        const int c = lane & 31, h = lane >> 5;
        Operand op;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v8s a;
#pragma unroll
            for (int j = 0; j < 8; ++j) a[j] = (16 * h + 8 * ks + j <= c) ? (short)0x3F80 : (short)0;  // bf16 1.0
            op.a[ks] = __builtin_bit_cast(v4u, a);
        }
        return op;
    }
    // keeps the compiler from moving the making of the operand past this point
    static __device__ __forceinline__ void pin(Operand &op) { asm volatile("" : "+v"(op.a[0]), "+v"(op.a[1])); }
    static __device__ __forceinline__ void run(const v4u *raw, int lane, float (&acc)[16]) {
        run(raw, lane, acc, operand(lane));
    }
    static __device__ __forceinline__ void run(const v4u *raw, int lane, float (&acc)[16], const Operand &op) {
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
            const v8bf ab = __builtin_bit_cast(v8bf, op.a[ks]);
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

// ---- plain sum of the raw registers of one chunk (for the aggregate of a tile that holds no flag) ----------
//
// A lane's partial sum over its 2 * K words; the layout does not matter.  Elements beyond n were loaded as zeros.
template <typename TT> struct RawSum;
template <> struct RawSum<TI8> {
    static __device__ __forceinline__ uint32_t run(const v4u *raw) {
        int s = 0;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int d = 0; d < 4; ++d) s = __builtin_amdgcn_sdot4((int)raw[i][d], 0x01010101, s, false);
        return (uint32_t)s;
    }
};
template <> struct RawSum<TX8> {
    static __device__ __forceinline__ XorWord run(const v4u *raw) {
        uint32_t x = 0;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int d = 0; d < 4; ++d) x ^= raw[i][d];
        x ^= x >> 16;
        x ^= x >> 8;
        return XorWord(x & 0xFFu);
    }
};
template <bool kBf16> struct RawSumHalf {
    static __device__ __forceinline__ float run(const v4u *raw) {
        typedef _Float16 v2h __attribute__((ext_vector_type(2)));
        typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
        constexpr uint32_t kOnes = kBf16 ? 0x3F803F80u : 0x3C003C00u;
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const uint32_t pair = raw[i][d];
                if (kBf16)
                    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(v2bf, pair), __builtin_bit_cast(v2bf, kOnes), s, false);
                else
                    s = __builtin_amdgcn_fdot2(__builtin_bit_cast(v2h, pair), __builtin_bit_cast(v2h, kOnes), s, false);
            }
        return s;
    }
};
template <> struct RawSum<TF16> : RawSumHalf<false> {};
template <> struct RawSum<TBF16> : RawSumHalf<true> {};
template <> struct RawSum<TF32> {
    static __device__ __forceinline__ float run(const v4u *raw) {
        float s[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int d = 0; d < 4; ++d) s[d] += from_bits<float>(raw[i][d]);
        return (s[0] + s[1]) + (s[2] + s[3]);
    }
};
template <> struct RawSum<TSpmv> : RawSum<TF32> {};

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

template <> struct RowAgg<TX8> {
    // as RowAgg<TI8>, with the masked bytes folded by XOR instead of summed
    template <bool kAlu> static __device__ __forceinline__ XorWord run(const v4u *raw, uint32_t F, int lane) {
        const int h = lane >> 5;
        const Halves Fh = wave_halves<kAlu>(F, lane);
        uint32_t tot[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int st = last_flag_pos(t ? Fh.hi : Fh.lo);
            int k = st - 16 * h;
            k = k < 0 ? 0 : (k > 16 ? 16 : k);
            const uint64_t ones = ~0ull;
            const uint64_t m_lo = k >= 8 ? 0ull : ones << (8 * k);
            const uint64_t m_hi = k >= 16 ? 0ull : ones << (8 * (k > 8 ? k - 8 : 0));
            uint32_t x = (raw[t][0] & (uint32_t)m_lo) ^ (raw[t][1] & (uint32_t)(m_lo >> 32)) ^
                         (raw[t][2] & (uint32_t)m_hi) ^ (raw[t][3] & (uint32_t)(m_hi >> 32));
            x ^= x >> 16;
            x ^= x >> 8;
            const Halves ph = wave_halves<kAlu>(x & 0xFFu, lane);
            tot[t] = ph.lo ^ ph.hi;
        }
        return XorWord(lane < 32 ? tot[0] : tot[1]);
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
template <> __device__ __forceinline__ XorWord raw_elem<TX8>(const v4u &w, int i) {
    return XorWord((w[i >> 2] >> (8 * (i & 3))) & 0xFFu);
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

}  // namespace
