// libmmvseg, part of the one translation unit mmvseg.hip (included there, in order).
// The single-pass kernel: segmented scan, segmented sum, SpMV (COO and CSR) and the unsegmented scan.
#pragma once

namespace {

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
    uint32_t early_v[kWaves], early_f[kWaves];   // plain sum and any-flag of every wave's span, written as the loads land
    uint32_t tile, carry_v, carry_c, ready, arrived;
};

// One tile, from the loads on.  kLateVal (SpMV only): the values are loaded behind the gathers of
// x[col] instead of beside the columns.
template <typename TT, int kOp, bool kMfma, bool kLateVal>
__device__ __forceinline__ void seg_tile(const Params &P, const uint32_t *__restrict__ hints, SegShared<TT::kWaves> &sm,
                                         const uint32_t tile) {
    typedef typename TT::acc_t A;
    typedef typename TT::in_t In;
    constexpr int kWaves = TT::kWaves;
    constexpr int kCpw = chunks_per_wave<TT, kOp, kMfma>();   // most chunks a wave takes (register arrays)
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
    // A chunk in which every position starts a segment is its own result (Algorithm "Revert Speculative
    // Prefix Sums", the case of all flags set, taken here for 64 rows at once): with 32-bit inputs and one
    // chunk per wave the striped registers are stored as they are, straight after the load (all-flag
    // vectors 8 % faster).  Matrix-core variant only: in the other one the test cost 1 % on vectors without
    // such chunks and gained 2 % on those with.
    constexpr bool kDenseShortcut = MMV_DENSE_SHORTCUT != 0 && kOp == kScan && sizeof(In) == 4 && kKeepRows;
    // the count of the segments before the tile comes from a table of per-tile counts made by a
    // small kernel before this one, so that no chunk has to wait for it
    constexpr bool kProduct = kOp == kSpmv || kOp == kSpmvCsr;      // values are val * x[col]
    // A tile that holds no flag hands on a plain sum, and its successors cannot finish before they have it.  In the
    // scan kernels such a tile publishes that sum as soon as its loads have landed, ahead of the row scans of
    // phase A (which take several microseconds when all waves of a compute unit are at it): the wave whose loads
    // land last adds up the sums of all waves.  Without this a vector without flags ran 13 % slower than one
    // with a flag in every tile, each tile waiting 6 us for the slowest of the tiles before it.
    // Floats are not a group, so x-bar(j) - x-bar(j - 1) is not x(j) bit for bit.  With 32-bit inputs the striped
    // registers of the load hold exactly the four positions a lane stores, so a position that starts a segment
    // gets its input itself, and the positions behind it in the lane's four run on from there (the case of set
    // flags in Algorithm "Revert Speculative Prefix Sums", taken per element).  16-bit inputs do not need it: their
    // row prefixes are exact in fp32 unless the exponents of a row differ widely.
    constexpr bool kExactStarts = MMV_EXACT_STARTS != 0 && kOp == kScan && sizeof(In) == 4;
    constexpr int kEarlyMode = !kScanLike ? 0 : (sizeof(In) == 1 ? MMV_EARLY_I8 : (sizeof(In) == 2 ? MMV_EARLY_F16 : (kOp == kPlainScan ? MMV_EARLY_F32_SCAN : (kMfma ? MMV_EARLY_F32 : MMV_EARLY_F32_SHUFFLE))));
    constexpr bool kEarly = kEarlyMode != 0;
    constexpr bool kEarlyLookback = kEarlyMode == 2;
    // mode 3: that wave asks for the descriptors of the tiles before at the end of its phase A and looks at them after
    // the barrier (the look-back takes 3 to 4 us whatever has been published: the poll is under way meanwhile)
    constexpr bool kAsyncLookback = kEarlyMode == 3;

    // the wave index as a scalar: everything derived from it (the wave's span, chunk bases, the
    // "whole chunk inside the vector" tests, base addresses of loads and stores) then lives in scalar
    // registers and costs no vector instructions
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint64_t n = P.n;
    uint32_t *rows = sm.rows[wave];
    // tiles at both ends of a long vector are shorter (fewer chunks per wave)
    const TileSpan span = tile_span(P.reg, tile, kWaves * kChunkElems);
    const int cpw_t = (int)span.cpw;
    const uint64_t tile_base = span.base;
    const uint64_t wave_base = tile_base + (uint64_t)wave * cpw_t * kChunkElems;

    // ---- all inputs of my span: flag word of my row and raw values (and columns) per chunk ----
    uint32_t F[kCpw];
    v4u raw[kCpw][2 * K];
    v4u rawc[kProduct ? kCpw : 1][2 * K];  // column indices (spmv)
    v4u striped[kExactStarts && kKeepRows ? 2 * K : 1];   // the loaded words as they came, where phase A reorders raw[]
    // (the flag words go first: a wave knows whether its span holds a flag before the values have landed)
#pragma unroll
    for (int c = 0; c < kCpw; ++c) {
        F[c] = 0;
        if constexpr (kOp != kPlainScan) {
            const uint64_t rs = wave_base + (uint64_t)c * kChunkElems + 32u * lane;
            if (c < cpw_t && rs < n) F[c] = __builtin_nontemporal_load(P.fw + (rs >> 5));
        }
    }
#pragma unroll
    for (int c = 0; c < kCpw; ++c) {
        const uint64_t cb = wave_base + (uint64_t)c * kChunkElems;
        if (c < cpw_t) {
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
    // bits beyond n do not count
    if constexpr (kOp != kPlainScan) {
#pragma unroll
        for (int c = 0; c < kCpw; ++c) {
            const uint64_t rs = wave_base + (uint64_t)c * kChunkElems + 32u * lane;
            if (rs + 32 > n) F[c] = rs < n ? (F[c] & ((1u << (uint32_t)(n - rs)) - 1u)) : 0u;
        }
    }
    bool i_published = false;   // (kEarly) my wave has published the sum of a tile without flags
    if constexpr (kEarly) {
        uint32_t any = 0;
#pragma unroll
        for (int c = 0; c < kCpw; ++c) any |= F[c];
        if (tile == 0) any |= 1u;                       // nobody waits for the first tile's sum ahead of time
        const bool span_flagged = __ballot(any != 0) != 0;
        A s = A(0);
        if (!span_flagged) {
#pragma unroll
            for (int c = 0; c < kCpw; ++c)
                if (c < cpw_t) s += RawSum<TT>::run(raw[c]);
            s = wave_sum<A, kAluLanes>(s);
        }
        uint32_t before = 0;
        if (lane == 0) {
            sm.early_v[wave] = to_bits(s);
            sm.early_f[wave] = span_flagged ? 1u : 0u;
            before = __hip_atomic_fetch_add(&sm.arrived, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        if (__builtin_amdgcn_readfirstlane(before) == kWaves - 1) {   // my wave's loads landed last
            A total = A(0);
            uint32_t flagged = 0;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                total += from_bits<A>(sm.early_v[w]);
                flagged |= sm.early_f[w];
            }
            if (!flagged) {
                i_published = true;
                if (lane == 0) desc_store(P.desc_v + tile, kStatusAggregate, to_bits(total));
                if constexpr (kEarlyLookback) {
                    // ... and it looks back for the carry of the tiles before right away, so that the tile's own
                    // prefix is out for its successors a whole phase A earlier (the other waves go on meanwhile)
                    const A carry_in = lookback<A, kAluLanes>(P.desc_v, (int)tile, lane, P.hdr);
                    if (lane == 0) {
                        desc_store(P.desc_v + tile, kStatusPrefix, to_bits(carry_in + total));
                        sm.carry_v = to_bits(carry_in);
                        __hip_atomic_store(&sm.ready, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                    }
                }
            }
        }
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
    bool dense_chunk = false;   // (uniform) the wave's chunk was stored in phase A already

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
            if constexpr (kDenseShortcut) {
                // A chunk all of whose positions start segments: the striped registers are the result.  The row
                // scans are still made, for the aggregates; the test sits behind the first use of the loaded
                // values, and the 0 / 1 operands are made before that, as they are without the branch (a branch
                // ahead of the loads' first use, or operands made behind it: 1.5 to 3 % on vectors without such
                // chunks).
                typename SpecMfma<TT>::Operand op = SpecMfma<TT>::operand(lane);
                SpecMfma<TT>::pin(op);
                if constexpr (kExactStarts) {
#pragma unroll
                    for (int i = 0; i < 2 * K; ++i) striped[i] = raw[S][i];
                }
                operand_layout_write4(raw[S], rows, lane);
                dense_chunk = cb + kChunkElems <= n && __ballot(F[S] != 0xFFFFFFFFu) == 0;
                if (dense_chunk) {
#pragma unroll
                    for (int i = 0; i < 2 * K; ++i)
                        __builtin_nontemporal_store(
                            raw[S][i],
                            reinterpret_cast<v4u *>((A *)P.z + cb + 1024u * (i / K) + raw_offset<TT, kMfma>(i % K, lane)));
                }
                operand_layout_read4(raw[S], rows, lane);
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    A acc[16];
                    SpecMfma<TT>::run(raw[S] + t * K, lane, acc, op);
                    store_spec_rows(rows, t, lane, acc);
                }
            } else {
                if constexpr (kExactStarts) {
#pragma unroll
                    for (int i = 0; i < 2 * K; ++i) striped[i] = raw[S][i];
                }
                if constexpr (K > 1) to_operand_layout<K>(raw[S], rows, lane);
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    A acc[16];
                    SpecMfma<TT>::run(raw[S] + t * K, lane, acc);
                    store_spec_rows(rows, t, lane, acc);
                }
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
    // (wave 0) the tile's first element starts a segment: nothing of the tile takes a carry from the tiles before
    // (after the loop the register slots are back in place: slot 0 is the wave's first chunk)
    const bool head_flagged = (__builtin_amdgcn_readfirstlane(F[0]) & 1u) != 0;
    if (lane == 0) {
        sm.wave_v[wave] = to_bits(run_v);
        sm.wave_f[wave] = run_f;
        sm.wave_c[wave] = run_c;
    }
    uint64_t polled[MMV_POLL_WINDOWS] = {};
    if constexpr (kAsyncLookback) {
        if (i_published) lookback_poll(P.desc_v, (int)tile, lane, polled);
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
    // (a tile without any flag, other than tile 0, has published its aggregate already where kEarly is set)
    if (tid == 0 && (!kEarly || final_now))
        desc_store(P.desc_v + tile, final_now ? kStatusPrefix : kStatusAggregate, to_bits(tagg_v));

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
            // (a tile without flags, other than tile 0, has looked back already where kEarly is set)
            const bool looked_back = (kEarlyLookback || kAsyncLookback) && !final_now;
            if constexpr (kAsyncLookback) {
                if (i_published) {
                    tile_carry = lookback_from<A, kAluLanes, MMV_POLL_WINDOWS>(P.desc_v, (int)tile, lane, P.hdr, polled);
                    if (lane == 0) {
                        desc_store(P.desc_v + tile, kStatusPrefix, to_bits(tile_carry + tagg_v));
                        sm.carry_v = to_bits(tile_carry);
                        __hip_atomic_store(&sm.ready, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                    }
                }
            }
            if (wave == 0 && !looked_back) {
                if (tile > 0 && !head_flagged) tile_carry = lookback<A, kAluLanes>(P.desc_v, (int)tile, lane, P.hdr);
                if (lane == 0) {
                    if (!final_now) desc_store(P.desc_v + tile, kStatusPrefix, to_bits(tile_carry + tagg_v));
                    sm.carry_v = to_bits(tile_carry);
                    __hip_atomic_store(&sm.ready, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
            }
            if ((wave != 0 || looked_back) && !wex_f) {
                // my span starts inside a segment that began in an earlier tile: wait for wave 0
                while (__hip_atomic_load(&sm.ready, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) == 0)
                    __builtin_amdgcn_s_sleep(1);
                tile_carry = from_bits<A>(sm.carry_v);
            }
            if (!wex_f) span_carry = tile_carry + wex_v;
        }
#pragma unroll 1
        for (int c0 = 0; c0 < kCpw; c0 += kStep) {
#pragma unroll
          for (int u = 0; u < kStep; ++u) {
            const int c = c0 + u;
            const int S = kUnrollChunks ? c : u;
            // a chunk is "open" when no flag of the tile precedes it
            const bool chunk_open = !(wex_f || __builtin_amdgcn_readfirstlane(pre_f[S]));
            if (c < cpw_t && chunk_open == (pass == 1) && !(kDenseShortcut && dense_chunk)) {
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
                            if constexpr (kExactStarts) {
                                const v4u xr = kKeepRows ? striped[kKeepRows ? j : 0] : raw[S][j];   // my four inputs
                                bool restarted = ((Fr >> p0) & 1u) != 0;
                                if (restarted) o[0] = from_bits<A>(xr[0]);
#pragma unroll
                                for (int i = 1; i < 4; ++i) {
                                    const A x = from_bits<A>(xr[i]);
                                    if ((Fr >> (p0 + i)) & 1u) {
                                        o[i] = x;
                                        restarted = true;
                                    } else {
                                        o[i] = restarted ? o[i - 1] + x : from_bits<A>(xb[i]) - b;
                                    }
                                }
                            } else {
#pragma unroll
                                for (int i = 1; i < 4; ++i) {
                                    if ((Fr >> (p0 + i)) & 1u) b = from_bits<A>(xb[i - 1]);
                                    o[i] = from_bits<A>(xb[i]) - b;
                                }
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
}

}  // namespace
