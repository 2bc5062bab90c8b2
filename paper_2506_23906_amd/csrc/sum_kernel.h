// libmmvseg, part of the one translation unit mmvseg.hip (included there, in order).
// The tile body of the segmented sum for 8- and 16-bit inputs on long vectors (both variants: the 32x32 tiles that
// hold segment ends are scanned by the matrix cores, SpecMfma, or by vector instructions, SpecVector).
#pragma once

namespace {

// ---- segmented sum: speculation over a whole chunk -------------------------------------------------------------
//
// A segmented sum only has an output where a segment ends, so what every row needs in phase A is little: its plain
// total (a dot product with ones) and the number of segment starts it holds, both scanned WITHOUT regard to the
// flags over the 64 rows of the chunk (the speculative scan of Sec. 4.2, one level up: over row totals).  The sum of
// a segment that ends at position p of row r and starts at position s of row r' is then
//     [T(r) + x-bar_r(p)] - [T(r') + x-bar_r'(s - 1)],        T = exclusive scan of the row totals,
// the difference of two speculative prefixes of the chunk, exactly as Algorithm SCD takes the difference of two
// prefixes of the whole vector; if no flag of the chunk precedes p, it is carry + T(r) + x-bar_r(p).  The row
// scans x-bar come from the matrix cores (vector instructions in the ablation variant) and are made only for
// 32x32 tiles that the ends of the chunk need.
// Between chunks, waves and tiles the segmented pair (value after the last flag, any flag) is carried as in the
// scan; the one row of a chunk whose last flag matters there is known to the whole wave, so its masked dot
// product uses masks made on the scalar unit.
// Integers and bytes under exclusive or are exact (groups); 16-bit floats see the rounding of a prefix of up to
// 2048 terms instead of 32, which for values that are exact in fp32 products stays far inside the tolerance.
// Compared with carrying the segmented pair from row to row (what the scan kernels and the 32-bit sums do):
// 60 instead of 160 vector instructions per chunk in phase A.

// Sum of the K words a lane holds of one 32x32 tile (operand layout; elements beyond n are zeros).
template <typename TT> struct TilePart;
template <> struct TilePart<TI8> {
    static __device__ __forceinline__ uint32_t run(const v4u *raw) {
        int s = 0;
#pragma unroll
        for (int d = 0; d < 4; ++d) s = __builtin_amdgcn_sdot4((int)raw[0][d], 0x01010101, s, false);
        return (uint32_t)s;
    }
};
template <> struct TilePart<TX8> {
    static __device__ __forceinline__ XorWord run(const v4u *raw) {
        uint32_t x = raw[0][0] ^ raw[0][1] ^ raw[0][2] ^ raw[0][3];
        x ^= x >> 16;
        x ^= x >> 8;
        return XorWord(x & 0xFFu);
    }
};
template <bool kBf16> struct TilePartHalf {
    static __device__ __forceinline__ float run(const v4u *raw) {
        typedef _Float16 v2h __attribute__((ext_vector_type(2)));
        typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
        constexpr uint32_t kOnes = kBf16 ? 0x3F803F80u : 0x3C003C00u;
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < 2; ++i)
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
template <> struct TilePart<TF16> : TilePartHalf<false> {};
template <> struct TilePart<TBF16> : TilePartHalf<true> {};

// The row scans of one 32x32 tile without the matrix cores, for the ablation variant of this kernel: same input
// (operand layout: lane (c, h) holds one half of row c) and same output layout as SpecMfma (lane (c, h) gets
// positions 8 q + 4 h .. + 3 of row c in acc[4 q .. 4 q + 3]).  One v_permlane32_swap per register gives both
// lanes of a row all of it; each then scans the row with vector instructions and keeps its sixteen positions.
template <typename TT> struct SpecVector;
// (a register of the half-wave that holds the lower half-rows / the upper half-rows, in every lane)
__device__ __forceinline__ void both_halves(uint32_t mine, uint32_t &lower, uint32_t &upper) {
    const auto sw = __builtin_amdgcn_permlane32_swap(mine, mine, false, false);
    lower = (uint32_t)sw[0];
    upper = (uint32_t)sw[1];
}
template <> struct SpecVector<TI8> {
    static __device__ __forceinline__ void run(const v4u *raw, int lane, uint32_t (&acc)[16]) {
        const bool h = lane >= 32;
        // words of the row in position order: w[2 q] = positions 8 q .. + 3, w[2 q + 1] = 8 q + 4 .. + 7
        uint32_t w[8];
#pragma unroll
        for (int d = 0; d < 4; ++d) both_halves(raw[0][d], w[d], w[4 + d]);
        int before = 0;   // sum of the words before the one at hand
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int s0 = __builtin_amdgcn_sdot4((int)w[2 * q], 0x01010101, before, false);   // ... up to and with word 2 q
            const uint32_t word = h ? w[2 * q + 1] : w[2 * q];
            const int base = h ? s0 : before;
            acc[4 * q + 0] = (uint32_t)__builtin_amdgcn_sdot4((int)word, 0x00000001, base, false);
            acc[4 * q + 1] = (uint32_t)__builtin_amdgcn_sdot4((int)word, 0x00000101, base, false);
            acc[4 * q + 2] = (uint32_t)__builtin_amdgcn_sdot4((int)word, 0x00010101, base, false);
            acc[4 * q + 3] = (uint32_t)__builtin_amdgcn_sdot4((int)word, 0x01010101, base, false);
            before = __builtin_amdgcn_sdot4((int)w[2 * q + 1], 0x01010101, s0, false);
        }
    }
};
template <> struct SpecVector<TX8> {
    static __device__ __forceinline__ uint32_t fold(uint32_t x) {   // xor of the four bytes, in the low byte
        x ^= x >> 16;
        x ^= x >> 8;
        return x & 0xFFu;
    }
    static __device__ __forceinline__ void run(const v4u *raw, int lane, XorWord (&acc)[16]) {
        const bool h = lane >= 32;
        uint32_t w[8];
#pragma unroll
        for (int d = 0; d < 4; ++d) both_halves(raw[0][d], w[d], w[4 + d]);
        uint32_t before = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t s0 = before ^ fold(w[2 * q]);
            const uint32_t word = h ? w[2 * q + 1] : w[2 * q];
            const uint32_t base = h ? s0 : before;
            // byte j of `run` = xor of bytes 0 .. j of the word
            uint32_t run = word ^ (word << 8);
            run ^= run << 16;
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[4 * q + j] = XorWord(((run >> (8 * j)) & 0xFFu) ^ base);
            before = s0 ^ fold(w[2 * q + 1]);
        }
    }
};
template <bool kBf16> struct SpecVectorHalf {
    static __device__ __forceinline__ float lo(uint32_t pair) {
        return kBf16 ? from_bits<float>(pair << 16) : (float)__builtin_bit_cast(_Float16, (uint16_t)(pair & 0xFFFFu));
    }
    static __device__ __forceinline__ float hi(uint32_t pair) {
        return kBf16 ? from_bits<float>(pair & 0xFFFF0000u) : (float)__builtin_bit_cast(_Float16, (uint16_t)(pair >> 16));
    }
    static __device__ __forceinline__ void run(const v4u *raw, int lane, float (&acc)[16]) {
        const bool h = lane >= 32;
        // run q of eight positions (8 q .. 8 q + 7) is word ks = q / 2 of the half-wave q % 2: four pairs each
        uint32_t r[4][4];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int d = 0; d < 4; ++d) both_halves(raw[ks][d], r[2 * ks][d], r[2 * ks + 1][d]);
        float before = 0.0f;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            // my four positions of this run: pairs 2 h and 2 h + 1; the pairs before them belong to the other lane
            const float first = (lo(r[q][0]) + hi(r[q][0])) + (lo(r[q][1]) + hi(r[q][1]));   // positions 8 q .. + 3
            const uint32_t p0 = h ? r[q][2] : r[q][0], p1 = h ? r[q][3] : r[q][1];
            float s = h ? before + first : before;
            s += lo(p0);
            acc[4 * q + 0] = s;
            s += hi(p0);
            acc[4 * q + 1] = s;
            s += lo(p1);
            acc[4 * q + 2] = s;
            s += hi(p1);
            acc[4 * q + 3] = s;
            before = (before + first) + ((lo(r[q][2]) + hi(r[q][2])) + (lo(r[q][3]) + hi(r[q][3])));
        }
    }
};
template <> struct SpecVector<TF16> : SpecVectorHalf<false> {};
template <> struct SpecVector<TBF16> : SpecVectorHalf<true> {};

// Sum of the elements a lane holds of one 32x32 tile that lie at positions below p of their row (p is the same
// for all lanes, so the masks of both half-waves are made on the scalar unit and a lane picks its own).
template <typename TT> struct HeadPart;
// (bytes: bit i of `below` says whether position i lies below p; the four bits of a word's positions are spread to
// the low bits of its four bytes by one multiplication -- the copies of the four bits, 7 places apart, do not overlap)
__device__ __forceinline__ uint32_t byte_mask_of_bits(uint32_t bits4) { return (bits4 * 0x00204081u) & 0x01010101u; }
template <> struct HeadPart<TI8> {
    static __device__ __forceinline__ uint32_t run(const v4u *raw, int p, int h) {
        const uint32_t mine = ((1u << p) - 1u) >> (16 * h);   // half h holds positions 16 h + 4 d .. + 3 in word d; p < 32
        int s = 0;
#pragma unroll
        for (int d = 0; d < 4; ++d)
            s = __builtin_amdgcn_sdot4((int)raw[0][d], (int)byte_mask_of_bits((mine >> (4 * d)) & 0xFu), s, false);
        return (uint32_t)s;
    }
};
template <> struct HeadPart<TX8> {
    static __device__ __forceinline__ XorWord run(const v4u *raw, int p, int h) {
        const uint32_t mine = ((1u << p) - 1u) >> (16 * h);
        uint32_t x = 0;
#pragma unroll
        for (int d = 0; d < 4; ++d) x ^= raw[0][d] & (byte_mask_of_bits((mine >> (4 * d)) & 0xFu) * 0xFFu);
        x ^= x >> 16;
        x ^= x >> 8;
        return XorWord(x & 0xFFu);
    }
};
template <bool kBf16> struct HeadPartHalf {
    static __device__ __forceinline__ float run(const v4u *raw, int p, int h) {
        typedef _Float16 v2h __attribute__((ext_vector_type(2)));
        typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
        constexpr uint32_t kOne = kBf16 ? 0x3F80u : 0x3C00u;
        // word ks of half h holds positions 16 ks + 8 h + 2 d and + 1 in dword d; the two bits that say whether they lie
        // below p become a 1.0 in the low and in the high half of the mask word
        const uint32_t mine = ((1u << p) - 1u) >> (8 * h);   // p < 32
        float s = 0.0f;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const uint32_t two = (mine >> (16 * ks + 2 * d)) & 3u;
                const uint32_t mask = ((two * 0x8001u) & 0x10001u) * kOne;
                const uint32_t pair = raw[ks][d];
                if (kBf16)
                    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(v2bf, pair), __builtin_bit_cast(v2bf, mask), s, false);
                else
                    s = __builtin_amdgcn_fdot2(__builtin_bit_cast(v2h, pair), __builtin_bit_cast(v2h, mask), s, false);
            }
        return s;
    }
};
template <> struct HeadPart<TF16> : HeadPartHalf<false> {};
template <> struct HeadPart<TBF16> : HeadPartHalf<true> {};

template <typename A> __device__ __forceinline__ A read_lane(A v, int l) {
    return from_bits<A>((uint32_t)__builtin_amdgcn_readlane((int)to_bits(v), l));
}

// Inclusive scan over the 64 lanes without regard to anything (DPP: inside the rows of 16 lanes, then row to row).
template <typename A> __device__ __forceinline__ A wave_inclusive_scan(A v) {
    v += from_bits<A>(dpp_or_zero<0x111, 0xF>(to_bits(v)));
    v += from_bits<A>(dpp_or_zero<0x112, 0xF>(to_bits(v)));
    v += from_bits<A>(dpp_or_zero<0x114, 0xF>(to_bits(v)));
    v += from_bits<A>(dpp_or_zero<0x118, 0xF>(to_bits(v)));
    v += from_bits<A>(dpp_or_zero<0x142, 0xA>(to_bits(v)));
    v += from_bits<A>(dpp_or_zero<0x143, 0xC>(to_bits(v)));
    return v;
}

// Inclusive scans over the 64 lanes of a row total and a count of at most 32 per lane, together.  Totals of rows of
// 32 bytes and their sums over a chunk fit 20 bits, the counts 12, so the 8-bit sums scan both in one word.
template <typename TT> struct ScanPair {
    typedef typename TT::acc_t A;
    static __device__ __forceinline__ void run(A tot, uint32_t cnt, A &inc_t, uint32_t &inc_c) {
        inc_t = wave_inclusive_scan(tot);
        inc_c = wave_inclusive_scan(cnt);
    }
};
template <> struct ScanPair<TI8> {
    static __device__ __forceinline__ void run(uint32_t tot, uint32_t cnt, uint32_t &inc_t, uint32_t &inc_c) {
        const uint32_t both = wave_inclusive_scan((tot << 12) + cnt);
        inc_c = both & 0xFFFu;
        inc_t = (uint32_t)((int32_t)both >> 12);
    }
};

// Most chunks per wave of this tile body: a wave holds only the chunks whose loads are in flight, whatever the
// length of its span, so the tiles can be longer than those of the scan (fewer tickets, and the fixed costs of a
// tile spread over more elements).
template <typename TT> constexpr int sum_cpw() { return sizeof(typename TT::in_t) == 1 ? MMV_SUM_CPW_I8 : MMV_SUM_CPW_F16; }
template <typename TT, int kOp, bool kMfma> constexpr bool chunk_sum_kernel() {
    return MMV_CHUNK_SUM != 0 && kOp == kSum && sizeof(typename TT::in_t) <= 2;
}

// The LDS rows of one wave: the row scans x-bar of the chunk at hand.  Row scans of 32 bytes fit 16 bits
// (|x-bar| <= 32 * 128), which halves the rows of the 8-bit inputs; 16-bit inputs keep 32-bit rows in the layout of
// the scan kernels (they also pass through them on their way into the operand layout).
template <typename TT, bool kNarrow = sizeof(typename TT::in_t) == 1> struct SumRows;
template <typename TT> struct SumRows<TT, false> {
    typedef typename TT::acc_t A;
    static constexpr int kWords = kRowsPerChunk * kRowStride;
    static __device__ __forceinline__ void store(uint32_t *rows, int t, int lane, const A (&acc)[16]) { store_spec_rows(rows, t, lane, acc); }
    static __device__ __forceinline__ A x_bar(const uint32_t *rows, int r, int p) { return from_bits<A>(rows[r * kRowStride + kRowData + p]); }
};
template <typename TT> struct SumRows<TT, true> {
    typedef typename TT::acc_t A;
    static constexpr int kStride = 18;   // words per row: 16 of values, 2 of padding (64-bit stores of a half-wave hit every bank once)
    static constexpr int kWords = kRowsPerChunk * kStride;
    // lane (c, h) holds positions 8 q + 4 h .. + 3 of row 32 t + c in acc[4 q .. 4 q + 3]
    static __device__ __forceinline__ void store(uint32_t *rows, int t, int lane, const A (&acc)[16]) {
        const int c = lane & 31, h = lane >> 5;
        uint32_t *rp = rows + (32 * t + c) * kStride + 2 * h;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            v2u w = {__builtin_amdgcn_perm(to_bits(acc[4 * q + 1]), to_bits(acc[4 * q]), 0x05040100u),
                     __builtin_amdgcn_perm(to_bits(acc[4 * q + 3]), to_bits(acc[4 * q + 2]), 0x05040100u)};
            *reinterpret_cast<v2u *>(rp + 4 * q) = w;
        }
    }
    static __device__ __forceinline__ A x_bar(const uint32_t *rows, int r, int p) {
        return from_bits<A>((uint32_t)(int32_t) reinterpret_cast<const int16_t *>(rows)[r * (2 * kStride) + p]);
    }
};

// LDS of one workgroup of the sum kernel.
template <typename TT> struct SumShared {
    __attribute__((aligned(16))) uint32_t rows[TT::kWaves][SumRows<TT>::kWords];
    uint32_t wave_v[TT::kWaves], wave_f[TT::kWaves];
    // per wave: the one output that needs the sum carried into the wave's span (its value so far, its index in the
    // output, whether there is one)
    uint32_t late_v[TT::kWaves], late_k[TT::kWaves], late_on[TT::kWaves];
    uint32_t tile, carry_v, ready, arrived;
};
// Waves per SIMD the compiler is to leave room for: four workgroups of eight waves per compute unit for 8-bit sums
// (narrow rows: 37 KB of LDS each; measured against three with one more chunk in flight: 4 to 6 % faster), two
// where the rows are wide (74 KB).
template <typename TT> constexpr int sum_waves_per_simd() { return MMV_MIN_WAVES_PER_SIMD; }
template <> constexpr int sum_waves_per_simd<TI8>() { return MMV_SUM_WAVES_PER_SIMD_I8; }
// Chunks of a wave whose loads are in flight at once (their values wait in registers).
template <typename TT> constexpr int sum_load_depth() { return sizeof(typename TT::in_t) == 1 ? MMV_SUM_LOAD_DEPTH_I8 : MMV_SUM_LOAD_DEPTH_F16; }
template <> constexpr int sum_load_depth<TX8>() { return 2; }

// What a wave holds of one chunk while its loads are in flight: the flag word of its row, the flag word of the row
// after it (whose lowest bit says whether the row's last position ends a segment), and the values.
template <typename TT> struct SumSlot {
    uint32_t F, Fnext;
    v4u raw[2 * (16 / TT::kEpl)];
};
template <typename TT>
__device__ __forceinline__ void sum_load_slot(const Params &P, uint64_t chunk_base, int lane, SumSlot<TT> &slot) {
    const uint64_t rs = chunk_base + 32u * lane;
    slot.F = slot.Fnext = 0;
    if (rs < P.n) slot.F = __builtin_nontemporal_load(P.fw + (rs >> 5));
    if (rs + 32 < P.n) slot.Fnext = __builtin_nontemporal_load(P.fw + (rs >> 5) + 1);
    load_raw<TT, true>((const typename TT::in_t *)P.x, chunk_base, P.n, lane, slot.raw);
}

// One tile.  A wave takes the chunks of its span one after the other, a few of them in flight ahead of the one at
// hand, and is done with a chunk's values when it moves on: everything a segment end needs lies inside its chunk,
// except for the first end of a chunk when the segment began before the chunk, and of those only the one with no
// flag of the wave's span before it needs anything from other waves or tiles (at most one per wave: after that
// end comes a flag; kept in LDS and written at the end, when the carry is known).  The index of an output is the
// number of segment starts before its segment; the starts before a wave's span come from the counting kernel.
// So a tile can be long (few tickets, barriers and look-backs per element) without holding more in registers.
template <typename TT, bool kMfma>
__device__ __forceinline__ void sum_tile(const Params &P, SumShared<TT> &sm, const uint32_t tile) {
    typedef SumRows<TT> Rows;
    typedef typename std::conditional<kMfma, SpecMfma<TT>, SpecVector<TT>>::type Spec;   // how a 32x32 tile is scanned
    typedef typename TT::acc_t A;
    constexpr int kWaves = TT::kWaves;
    constexpr int kDepth = sum_load_depth<TT>();
    constexpr int K = 16 / TT::kEpl;
    static_assert(K <= 2, "8- and 16-bit inputs");

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5;
    const uint64_t n = P.n;
    uint32_t *rows = sm.rows[wave];
    const TileSpan span = tile_span(P.reg, tile, kWaves * kChunkElems);
    const int cpw_t = (int)span.cpw;
    const uint64_t wave_base = span.base + (uint64_t)wave * cpw_t * kChunkElems;

    // segment starts before my span (position 0 of the vector is not counted): those before my tile (the table holds
    // them per tile, or, for long vectors, their prefix sums already) and those in the spans of the waves before mine.
    // Asked for ahead of the values (loads come back in the order they went out), added up when the first end needs them.
    uint32_t count_part = 0;
    if (P.count_is_prefix) {
        if (lane == 0) count_part = P.tile_count[tile];
    } else {
        for (uint32_t i = lane; i < tile; i += 64) count_part += P.tile_count[i];
    }
    if (lane < wave) count_part += P.span_count[(uint64_t)tile * kWaves + lane];
    __builtin_amdgcn_sched_barrier(0);
    SumSlot<TT> slot[kDepth];
#pragma unroll
    for (int i = 0; i < kDepth; ++i)
        if (i < cpw_t) sum_load_slot<TT>(P, wave_base + (uint64_t)i * kChunkElems, lane, slot[i]);
#if MMV_LOAD_PRIO
    __builtin_amdgcn_s_setprio(0);
#endif
    if (lane == 0) sm.late_on[wave] = 0;
    const uint32_t count_carry = wave_sum<uint32_t, true>(count_part);

    // ================= the chunks of my span =================
    A run_v = A(0);                 // value after the last flag of the chunks so far (their plain sum while run_f == 0)
    uint32_t run_f = 0, run_c = 0;  // whether they hold a flag; their segment starts
    bool head_flagged = false;      // the first position of my span starts a segment
#pragma unroll 1
    for (int c0 = 0; c0 < cpw_t; c0 += kDepth) {
#pragma unroll
        for (int i = 0; i < kDepth; ++i) {
            const int c = c0 + i;
            if (c < cpw_t) {
                const uint64_t cb = wave_base + (uint64_t)c * kChunkElems;
                const uint64_t row_start = cb + 32u * lane;
                v4u(&raw)[2 * K] = slot[i].raw;
                uint32_t F = slot[i].F;
                if (row_start + 32 > n) F = row_start < n ? (F & ((1u << (uint32_t)(n - row_start)) - 1u)) : 0u;   // bits beyond n do not count
                if (c == 0) head_flagged = (__builtin_amdgcn_readfirstlane(F) & 1u) != 0;
                if constexpr (K > 1) to_operand_layout<K>(raw, rows, lane);
                // total of the row I own: the two lanes that hold a row's halves sit 32 lanes apart, so one swap of the
                // half-waves of the two tiles' partial sums puts both halves of row `lane` into this lane
                const A part0 = TilePart<TT>::run(raw), part1 = TilePart<TT>::run(raw + K);
                const auto sw = __builtin_amdgcn_permlane32_swap(to_bits(part0), to_bits(part1), false, false);
                const A tot = from_bits<A>((uint32_t)sw[0]) + from_bits<A>((uint32_t)sw[1]);
                const uint32_t Fc = row_start == 0 ? (F & ~1u) : F;   // position 0 is not counted
                const uint32_t cnt = __popc(Fc);
                A inc_t;
                uint32_t inc_c;
                ScanPair<TT>::run(tot, cnt, inc_t, inc_c);
                const A ex_t = inc_t - tot;            // sum of the rows of the chunk before mine (speculative: flags ignored)
                const uint32_t ex_c = inc_c - cnt;     // segment starts in the rows of the chunk before mine
                const A chunk_total = read_lane(inc_t, 63);
                const uint64_t rows_flagged = __ballot(F != 0);
                A chunk_agg = chunk_total;
                if (rows_flagged) {
                    // what lies before the chunk's last flag: the rows before its row and the head of that row
                    const int r_star = 63 - __builtin_clzll((unsigned long long)rows_flagged);
                    const uint32_t f_star = (uint32_t)__builtin_amdgcn_readlane((int)F, r_star);
                    const int p_star = 31 - __builtin_clz(f_star);
                    A before = read_lane(ex_t, r_star);
                    if (p_star > 0) {
                        const A hp = (r_star >> 5) ? HeadPart<TT>::run(raw + K, p_star, h) : HeadPart<TT>::run(raw, p_star, h);
                        before = (before + read_lane(hp, r_star & 31)) + read_lane(hp, (r_star & 31) + 32);
                    }
                    chunk_agg = chunk_total - before;
                }

                // ---- the segment ends of the chunk.  End mask of my row: bit p set iff position p + 1 starts a
                // segment or p is the last element ----
                uint32_t E = (F >> 1) | ((slot[i].Fnext & 1u) << 31);
                if (row_start < n) {
                    if (row_start + 32 >= n) {
                        const uint32_t last = (uint32_t)(n - 1 - row_start);
                        E = (E & ((1u << last) - 1u)) | (1u << last);
                    }
                } else {
                    E = 0;
                }
                const uint64_t rows_with_ends = __ballot(E != 0);
                if (rows_with_ends) {
                    // row scans of the 32x32 tiles that hold an end, and of the first one also when an end of the
                    // second may belong to a segment that starts there
                    const bool need1 = (rows_with_ends >> 32) != 0;
                    const bool need0 = (uint32_t)rows_with_ends != 0 || (need1 && (uint32_t)rows_flagged != 0);
                    if (need0) {
                        A acc[16];
                        Spec::run(raw, lane, acc);
                        Rows::store(rows, 0, lane, acc);
                    }
                    if (need1) {
                        A acc[16];
                        Spec::run(raw + K, lane, acc);
                        Rows::store(rows, 1, lane, acc);
                    }
                    // a segment that ends in my row and has no flag there starts at the last flag of the last flagged
                    // row r2 before mine (if there is one): what lies between is the rows from r2 on minus the head of r2
                    const uint64_t rows_before = rows_flagged & ((1ull << lane) - 1ull);
                    const int r2 = rows_before ? 63 - __builtin_clzll((unsigned long long)rows_before) : lane;
                    const int st2 = 31 - __builtin_clz(__shfl(F, r2) | 1u);
                    A across = ex_t - from_bits<A>(__shfl(to_bits(ex_t), r2));
                    wave_lds_sync();
                    if (st2 > 0) across -= Rows::x_bar(rows, r2, st2 - 1);

                    const uint32_t count_base = count_carry + run_c + ex_c;
                    // what an end of my row adds when no flag of the row precedes it: the rows from the last flagged
                    // row before mine on, or, without such a row, the rows of the chunk before mine and what the
                    // chunks before carried in
                    const A open_add = rows_before ? across : run_v + ex_t;
                    // the one end whose segment began before my span (no flag of the span before it): the first end
                    // of the chunk, if it is that; put aside for the end of the tile
                    if (run_f == 0 && rows_before == 0 && E != 0) {
                        const int e = __builtin_ctz(E);
                        if ((F & ((2u << e) - 1u)) == 0) {
                            sm.late_v[wave] = to_bits(Rows::x_bar(rows, lane, e) + open_add);
                            sm.late_k[wave] = count_base;
                            sm.late_on[wave] = 1u;
                            E &= E - 1u;
                        }
                    }
                    while (E) {
                        const int e = __builtin_ctz(E);
                        E &= E - 1u;
                        const uint32_t upto = (2u << e) - 1u;
                        const uint32_t m = F & upto;                 // flags of my row at or before the end
                        const uint32_t k = count_base + __popc(Fc & upto);
                        const int st = 31 - __builtin_clz(m | 1u);   // where the segment starts, if in my row (0 also without a flag)
                        const A head = Rows::x_bar(rows, lane, st > 0 ? st - 1 : 0);
                        const A v = (Rows::x_bar(rows, lane, e) - (st > 0 ? head : A(0))) + (m ? A(0) : open_add);
                        if (k < P.out_cap) ((A *)P.out)[k] = v;
                    }
                    wave_lds_sync();  // the rows are read before the next chunk overwrites them
                }
                run_v = rows_flagged ? chunk_agg : run_v + chunk_total;
                run_f |= rows_flagged ? 1u : 0u;
                run_c += (uint32_t)__builtin_amdgcn_readlane((int)inc_c, 63);
            }
            // the registers of this chunk take the chunk that many ahead
            __builtin_amdgcn_sched_barrier(0);
            if (c + kDepth < cpw_t) sum_load_slot<TT>(P, wave_base + (uint64_t)(c + kDepth) * kChunkElems, lane, slot[i]);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    if (lane == 0) {
        sm.wave_v[wave] = to_bits(run_v);
        sm.wave_f[wave] = run_f;
    }
    // (short vectors: the number of segments is what the last wave of the last tile has counted)
    if (!P.count_is_prefix && tile == P.num_tiles - 1 && wave == kWaves - 1 && lane == 0)
        *P.nseg = (uint64_t)count_carry + run_c + 1u;
    __syncthreads();

    // ---- the waves of the tile ----
    A wex_v = A(0), tagg_v = A(0);
    uint32_t wex_f = 0, tagg_f = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        if (w == wave) {
            wex_v = tagg_v;
            wex_f = tagg_f;
        }
        const A wv = from_bits<A>(sm.wave_v[w]);
        const uint32_t wf = sm.wave_f[w];
        tagg_v = wf ? wv : tagg_v + wv;
        tagg_f |= wf;
    }
    wex_f = __builtin_amdgcn_readfirstlane(wex_f);
    const bool final_now = tile == 0 || tagg_f;  // carry out does not depend on predecessors
    if (tid == 0) desc_store(P.desc_v + tile, final_now ? kStatusPrefix : kStatusAggregate, to_bits(tagg_v));

    // ---- the output that was waiting for the sum carried into my span ----
    const bool waiting = __builtin_amdgcn_readfirstlane(sm.late_on[wave]) != 0;
    A span_carry = wex_v;
    if (!wex_f) {
        // carry of the predecessor tiles by decoupled look-back
        A tile_carry = A(0);
        if (wave == 0) {
            if (tile > 0 && !head_flagged) tile_carry = lookback<A, true>(P.desc_v, (int)tile, lane, P.hdr);
            if (lane == 0) {
                if (!final_now) desc_store(P.desc_v + tile, kStatusPrefix, to_bits(tile_carry + tagg_v));
                sm.carry_v = to_bits(tile_carry);
                __hip_atomic_store(&sm.ready, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        } else if (waiting) {
            while (__hip_atomic_load(&sm.ready, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) == 0)
                __builtin_amdgcn_s_sleep(1);
            tile_carry = from_bits<A>(sm.carry_v);
        }
        span_carry = tile_carry + wex_v;
    }
    if (waiting && lane == 0) {
        const uint32_t k = sm.late_k[wave];
        if (k < P.out_cap) ((A *)P.out)[k] = from_bits<A>(sm.late_v[wave]) + span_carry;
    }
}

}  // namespace
