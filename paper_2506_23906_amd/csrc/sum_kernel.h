// libmmvseg, part of the one translation unit mmvseg.hip (included there, in order).
// The tile body of the segmented sum for 8- and 16-bit inputs in the matrix-core variant.
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
// scans x-bar come from the matrix cores and are made only for 32x32 tiles that the ends of the chunk need.
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

// Sum of the elements a lane holds of one 32x32 tile that lie at positions below p of their row (p is the same
// for all lanes, so the masks of both half-waves are made on the scalar unit and a lane picks its own).
template <typename TT> struct HeadPart;
__device__ __forceinline__ uint32_t low_bytes(int count, uint32_t ones) {   // `ones` in the first `count` of 4 bytes
    const int nb = count < 0 ? 0 : (count > 4 ? 4 : count);
    return nb == 4 ? ones : (ones & ((1u << (8 * nb)) - 1u));
}
template <> struct HeadPart<TI8> {
    static __device__ __forceinline__ uint32_t run(const v4u *raw, int p, int h) {
        int s = 0;
#pragma unroll
        for (int d = 0; d < 4; ++d) {   // half h holds positions 16 h + 4 d .. + 3 in word d
            const uint32_t m0 = low_bytes(p - 4 * d, 0x01010101u), m1 = low_bytes(p - 16 - 4 * d, 0x01010101u);
            s = __builtin_amdgcn_sdot4((int)raw[0][d], (int)(h ? m1 : m0), s, false);
        }
        return (uint32_t)s;
    }
};
template <> struct HeadPart<TX8> {
    static __device__ __forceinline__ XorWord run(const v4u *raw, int p, int h) {
        uint32_t x = 0;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t m0 = low_bytes(p - 4 * d, 0xFFFFFFFFu), m1 = low_bytes(p - 16 - 4 * d, 0xFFFFFFFFu);
            x ^= raw[0][d] & (h ? m1 : m0);
        }
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
        float s = 0.0f;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int d = 0; d < 4; ++d) {   // word ks of half h holds positions 16 ks + 8 h + 2 d and + 1 in dword d
                const int q0 = 16 * ks + 2 * d, q1 = q0 + 8;
                const uint32_t m0 = (q0 < p ? kOne : 0u) | (q0 + 1 < p ? kOne << 16 : 0u);
                const uint32_t m1 = (q1 < p ? kOne : 0u) | (q1 + 1 < p ? kOne << 16 : 0u);
                const uint32_t mask = h ? m1 : m0;
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

// Chunks per wave of this tile body: a sum keeps little per chunk besides the loaded values, so its tiles can be
// longer than those of the scan (fewer tickets, and the fixed costs of a tile spread over more elements).
template <typename TT> constexpr int sum_cpw() { return sizeof(typename TT::in_t) == 1 ? MMV_SUM_CPW_I8 : MMV_SUM_CPW_F16; }
template <> constexpr int sum_cpw<TX8>() { return MMV_CPW_X8_MFMA; }   // (the bit-plane products of exclusive or need the registers)
template <typename TT, int kOp, bool kMfma> constexpr bool chunk_sum_kernel() {
    return MMV_CHUNK_SUM != 0 && kOp == kSum && kMfma && sizeof(typename TT::in_t) <= 2;
}

template <typename TT>
__device__ __forceinline__ void sum_tile(const Params &P, SegShared<TT::kWaves> &sm, const uint32_t tile) {
    typedef typename TT::acc_t A;
    typedef typename TT::in_t In;
    constexpr int kWaves = TT::kWaves;
    constexpr int kCpw = sum_cpw<TT>();
    constexpr int K = 16 / TT::kEpl;
    static_assert(K <= 2, "8- and 16-bit inputs");

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5;
    const uint64_t n = P.n;
    uint32_t *rows = sm.rows[wave];
    const TileSpan span = tile_span(P.reg, tile, kWaves * kChunkElems);
    const int cpw_t = (int)span.cpw;
    const uint64_t wave_base = span.base + (uint64_t)wave * cpw_t * kChunkElems;

    // ---- all inputs of my span: the flag word of my row per chunk first, then the values; and the flag word that
    // follows the span (its lowest bit says whether the span's last position ends a segment) ----
    uint32_t F[kCpw];
    v4u raw[kCpw][2 * K];
#pragma unroll
    for (int c = 0; c < kCpw; ++c) {
        F[c] = 0;
        const uint64_t rs = wave_base + (uint64_t)c * kChunkElems + 32u * lane;
        if (c < cpw_t && rs < n) F[c] = __builtin_nontemporal_load(P.fw + (rs >> 5));
    }
    uint32_t next_word = 0;
    const uint64_t span_end = wave_base + (uint64_t)cpw_t * kChunkElems;
    if (span_end < n) next_word = P.fw[span_end >> 5];
#pragma unroll
    for (int c = 0; c < kCpw; ++c)
        if (c < cpw_t) load_raw<TT, true>((const In *)P.x, wave_base + (uint64_t)c * kChunkElems, n, lane, raw[c]);
#if MMV_LOAD_PRIO
    __builtin_amdgcn_s_setprio(0);
#endif
    // bits beyond n do not count
#pragma unroll
    for (int c = 0; c < kCpw; ++c) {
        const uint64_t rs = wave_base + (uint64_t)c * kChunkElems + 32u * lane;
        if (rs + 32 > n) F[c] = rs < n ? (F[c] & ((1u << (uint32_t)(n - rs)) - 1u)) : 0u;
    }
    // number of segment starts before my tile, while the loads are in flight: either the table holds the prefix
    // sums already, or (few tiles) wave 1 adds up the counts of the tiles before
    if (wave == 1) {
        uint32_t c = 0;
        if (P.count_is_prefix) {
            c = P.tile_count[tile];
        } else {
            for (uint32_t i = lane; i < tile; i += 64) c += P.tile_count[i];
            c = wave_sum<uint32_t, true>(c);
        }
        if (lane == 0) sm.carry_c = c;
    }

    // ================= phase A: totals of the rows, their scans over the chunk, the chunk's aggregate =================
    A ex_t[kCpw];           // per row: sum of the rows of the chunk before mine (speculative: flags ignored)
    uint32_t ex_c[kCpw];    // per row: segment starts in the rows of the chunk before mine
    A pre_v[kCpw];          // per chunk (the same in every lane): value carried into the chunk by the chunks of my span before it,
    uint32_t pre_f[kCpw], pre_c[kCpw];   // whether one of them holds a flag, and their segment starts
    A run_v = A(0);
    uint32_t run_f = 0, run_c = 0;
#pragma unroll
    for (int c = 0; c < kCpw; ++c) {
        ex_t[c] = pre_v[c] = A(0);
        ex_c[c] = pre_f[c] = pre_c[c] = 0;
        if (c < cpw_t) {
            const uint64_t cb = wave_base + (uint64_t)c * kChunkElems;
            if constexpr (K > 1) to_operand_layout<K>(raw[c], rows, lane);
            // total of the row I own: the two lanes that hold a row's halves sit 32 lanes apart, so one swap of the
            // half-waves of the two tiles' partial sums puts both halves of row `lane` into this lane
            const A part0 = TilePart<TT>::run(raw[c]), part1 = TilePart<TT>::run(raw[c] + K);
            const auto sw = __builtin_amdgcn_permlane32_swap(to_bits(part0), to_bits(part1), false, false);
            const A tot = from_bits<A>((uint32_t)sw[0]) + from_bits<A>((uint32_t)sw[1]);
            const uint32_t cnt = __popc(cb + 32u * lane == 0 ? (F[c] & ~1u) : F[c]);   // position 0 is not counted
            const A inc_t = wave_inclusive_scan(tot);
            const uint32_t inc_c = wave_inclusive_scan(cnt);
            ex_t[c] = inc_t - tot;
            ex_c[c] = inc_c - cnt;
            const A chunk_total = read_lane(inc_t, 63);
            const uint64_t rows_flagged = __ballot(F[c] != 0);
            A chunk_agg = chunk_total;
            if (rows_flagged) {
                // what lies before the chunk's last flag: the rows before its row and the head of that row
                const int r_star = 63 - __builtin_clzll((unsigned long long)rows_flagged);
                const uint32_t f_star = (uint32_t)__builtin_amdgcn_readlane((int)F[c], r_star);
                const int p_star = 31 - __builtin_clz(f_star);
                A before = read_lane(ex_t[c], r_star);
                if (p_star > 0) {
                    const A hp = (r_star >> 5) ? HeadPart<TT>::run(raw[c] + K, p_star, h) : HeadPart<TT>::run(raw[c], p_star, h);
                    before = (before + read_lane(hp, r_star & 31)) + read_lane(hp, (r_star & 31) + 32);
                }
                chunk_agg = chunk_total - before;
            }
            pre_v[c] = run_v;
            pre_f[c] = run_f;
            pre_c[c] = run_c;
            run_v = rows_flagged ? chunk_agg : run_v + chunk_total;
            run_f |= rows_flagged ? 1u : 0u;
            run_c += (uint32_t)__builtin_amdgcn_readlane((int)inc_c, 63);
        }
    }
    const bool head_flagged = (__builtin_amdgcn_readfirstlane(F[0]) & 1u) != 0;
    if (lane == 0) {
        sm.wave_v[wave] = to_bits(run_v);
        sm.wave_f[wave] = run_f;
        sm.wave_c[wave] = run_c;
    }
    __syncthreads();

    // ---- the waves of the tile ----
    A wex_v = A(0), tagg_v = A(0);
    uint32_t wex_f = 0, wex_c = 0, tagg_f = 0, tagg_c = 0;
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
    if (!P.count_is_prefix && tile == P.num_tiles - 1 && tid == 0) *P.nseg = (uint64_t)sm.carry_c + tagg_c + 1u;

    const bool final_now = tile == 0 || tagg_f;  // carry out does not depend on predecessors
    if (tid == 0) desc_store(P.desc_v + tile, final_now ? kStatusPrefix : kStatusAggregate, to_bits(tagg_v));
    A span_carry = wex_v;
    const uint32_t count_carry = sm.carry_c;

    // ================= phase B: the segment ends =================
#pragma unroll 1
    for (int pass = 0; pass < 2; ++pass) {
        if (pass == 1) {
            // carry of the predecessor tiles by decoupled look-back
            A tile_carry = A(0);
            if (wave == 0) {
                if (tile > 0 && !head_flagged) tile_carry = lookback<A, true>(P.desc_v, (int)tile, lane, P.hdr);
                if (lane == 0) {
                    if (!final_now) desc_store(P.desc_v + tile, kStatusPrefix, to_bits(tile_carry + tagg_v));
                    sm.carry_v = to_bits(tile_carry);
                    __hip_atomic_store(&sm.ready, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
            }
            if (wave != 0 && !wex_f) {
                while (__hip_atomic_load(&sm.ready, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) == 0)
                    __builtin_amdgcn_s_sleep(1);
                tile_carry = from_bits<A>(sm.carry_v);
            }
            if (!wex_f) span_carry = tile_carry + wex_v;
        }
#pragma unroll
        for (int c = 0; c < kCpw; ++c) {
            // a chunk is "open" when no flag of the tile precedes it: its first segment needs the carry of the tiles before
            const bool behind_own_flag = __builtin_amdgcn_readfirstlane(pre_f[c]) != 0;
            const bool chunk_open = !(wex_f || behind_own_flag);
            if (c >= cpw_t || chunk_open != (pass == 1)) continue;
            const uint64_t cb = wave_base + (uint64_t)c * kChunkElems;
            const uint64_t row_start = cb + 32u * lane;
            // end mask of my row: bit p set iff position p + 1 starts a segment or p is the last element
            uint32_t next0 = dpp_or_zero<0x130, 0xF>(F[c]) & 1u;   // wave_shl 1: the word of the next row
            if (lane == 63)
                next0 = (c + 1 < kCpw && c + 1 < cpw_t ? (uint32_t)__builtin_amdgcn_readlane((int)F[c + 1 < kCpw ? c + 1 : c], 0) : next_word) & 1u;
            uint32_t E = (F[c] >> 1) | (next0 << 31);
            if (row_start < n) {
                if (row_start + 32 >= n) {
                    const uint32_t last = (uint32_t)(n - 1 - row_start);
                    E = (E & ((1u << last) - 1u)) | (1u << last);
                }
            } else {
                E = 0;
            }
            const uint64_t rows_with_ends = __ballot(E != 0);
            if (rows_with_ends == 0) continue;
            const uint64_t rows_flagged = __ballot(F[c] != 0);
            // row scans of the 32x32 tiles that hold an end, and of the first one also when an end of the second
            // may belong to a segment that starts there
            const bool need1 = (rows_with_ends >> 32) != 0;
            const bool need0 = (uint32_t)rows_with_ends != 0 || (need1 && (uint32_t)rows_flagged != 0);
            if (need0) {
                A acc[16];
                SpecMfma<TT>::run(raw[c], lane, acc);
                store_spec_rows(rows, 0, lane, acc);
            }
            if (need1) {
                A acc[16];
                SpecMfma<TT>::run(raw[c] + K, lane, acc);
                store_spec_rows(rows, 1, lane, acc);
            }
            rows[lane * kRowStride + kSlotF] = F[c];
            rows[lane * kRowStride + kSlotPrefix] = to_bits(ex_t[c]);
            wave_lds_sync();

            const A carry_chunk = behind_own_flag ? pre_v[c] : span_carry + pre_v[c];   // into the chunk's first segment
            const uint64_t count_base = (uint64_t)count_carry + wex_c + pre_c[c] + ex_c[c];
            const uint32_t Fc = row_start == 0 ? (F[c] & ~1u) : F[c];  // position 0 is not counted
            const uint64_t rows_before = rows_flagged & ((1ull << lane) - 1ull);   // flagged rows before mine
            const uint32_t *rp = rows + lane * kRowStride + kRowData;
            while (E) {
                const int e = __builtin_ctz(E);
                E &= E - 1u;
                const uint32_t m = F[c] & ((2u << e) - 1u);  // flags of my row at or before the end
                A v = from_bits<A>(rp[e]);
                if (m) {
                    const int st = 31 - __builtin_clz(m);
                    if (st > 0) v -= from_bits<A>(rp[st - 1]);   // x-bar(e) - x-bar(start - 1), both in my row
                } else if (rows_before) {
                    // the segment starts in an earlier row r2 of the chunk, at that row's last flag
                    const int r2 = 63 - __builtin_clzll((unsigned long long)rows_before);
                    const uint32_t *rq = rows + r2 * kRowStride;
                    const int st = 31 - __builtin_clz(rq[kSlotF]);
                    v += ex_t[c] - from_bits<A>(rq[kSlotPrefix]);
                    if (st > 0) v -= from_bits<A>(rq[kRowData + st - 1]);
                } else {
                    v += carry_chunk + ex_t[c];                   // the segment began before the chunk
                }
                const uint64_t k = count_base + __popc(Fc & ((2u << e) - 1u));
                if (k < P.out_cap) ((A *)P.out)[k] = v;
            }
            wave_lds_sync();  // the rows are read before the next chunk overwrites them
        }
    }
}

}  // namespace
