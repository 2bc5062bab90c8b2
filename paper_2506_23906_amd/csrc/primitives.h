// libmmvseg, part of the one translation unit mmvseg.hip (included there, in order).
// The stand-alone primitives of Algorithms SCD and SSCR (Sec. 4.1): COMPRESS, DIFF, REVERT and their helpers.
#pragma once

namespace {

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
// A wave owns kGroups groups of 64 * kWords consecutive positions (kWords = 64 or 16): lane j < kWords
// holds the 64-bit mask word j of every group, and for every word the wave reads only the selected entries
// (one coalesced load, skipped when the word is empty) and writes them to consecutive output slots; a wave with
// few selected entries lets every lane walk its own words instead.  Short masks take the short
// spans: four times the waves, a quarter of the words each wave visits one after the other.  Long masks take
// two or four groups per wave: a tile costs a ticket (11 ns each, one after the other), a barrier and a look-back
// whatever its length, and with one group per wave the tickets alone took 93 us of the 111 us at n = 2^28
// and 0.1 % selected (now 0.048 ms; 30 % selected: 0.454 -> 0.415 ms).
// The workgroups that are resident from the start take the tile of their own index, as in the main kernel.
constexpr int kCompressWaves = 8;
constexpr uint64_t kCompressShortN = 1ull << 22;   // masks up to this length take 16 words per wave
// masks from 2^26 positions on take two groups of words per wave, from 2^28 on four: the mask has to be long enough
// for several rounds of workgroups (n = 2^26, 30 % selected: 0.125 ms with one group, 0.110 with two, 0.164 with four,
// which leaves two workgroups per compute unit; 0.1 % selected: 0.038, 0.015, 0.014 ms)
inline int compress_words(uint64_t n) { return n <= kCompressShortN ? 16 : 64; }
inline int compress_groups(uint64_t n) { return n >= (1ull << 28) ? 4 : n >= (1ull << 26) ? 2 : 1; }
inline uint64_t compress_tile(uint64_t n) { return (uint64_t)kCompressWaves * 64u * compress_words(n) * compress_groups(n); }

template <int kWords, int kGroups>
__global__ __launch_bounds__(kCompressWaves * 64, 8) void compress_kernel(
    const uint32_t *__restrict__ x, const uint32_t *__restrict__ mw, uint64_t n, uint32_t *__restrict__ out,
    uint64_t out_cap, uint64_t *__restrict__ count, uint32_t *hdr, uint64_t *desc, uint32_t num_tiles,
    const uint32_t *needed, uint32_t first_round) {
    __shared__ uint32_t s_tile, s_wave[kCompressWaves], s_carry;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (needed && *needed == 0) return;   // CSR SpMV without empty rows: nobody reads the row map
    const bool own_index = blockIdx.x < first_round;
    if (tid == 0 && !own_index)
        s_tile = first_round + __hip_atomic_fetch_add(hdr + kHdrTicket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const uint32_t tile = own_index ? blockIdx.x : s_tile;
    constexpr uint32_t kGroupSpan = 64u * kWords;                                   // positions of one group
    constexpr uint32_t kSpan = kGroupSpan * kGroups;                                // positions of a wave
    const uint64_t span = ((uint64_t)tile * kCompressWaves + wave) * kSpan;          // first position of my wave
    uint64_t m[kGroups];
    uint32_t before[kGroups];   // selected entries of my wave before my word of group g
    uint32_t wave_cnt = 0;
#pragma unroll
    for (int g = 0; g < kGroups; ++g) {
        const uint64_t p0 = span + (uint64_t)g * kGroupSpan + 64u * lane;            // first position of my word
        m[g] = 0;
        if (lane < kWords && p0 < n) {
            const uint64_t wi = p0 >> 5;
            m[g] = mw[wi];
            if (p0 + 32 < n) m[g] |= (uint64_t)mw[wi + 1] << 32;
            if (p0 + 64 > n) m[g] &= (1ull << (n - p0)) - 1ull;
        }
    }
#pragma unroll
    for (int g = 0; g < kGroups; ++g) {
        const uint32_t cnt = (uint32_t)__popcll((unsigned long long)m[g]);
        uint32_t inc = cnt;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t o = __shfl_up(inc, d);
            if (lane >= d) inc += o;
        }
        before[g] = wave_cnt + (inc - cnt);
        wave_cnt += (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
    }
    if (lane == 0) s_wave[wave] = wave_cnt;
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
    const uint64_t wave_base = (uint64_t)s_carry + wave_ex;   // output index of the first selected entry of my wave
    if (wave_cnt <= 4u * kWords * kGroups) {
        // few selected entries in my wave's positions: every lane walks the set bits of its own
        // words (a handful of independent loads per lane) instead of the wave visiting every word
        // Four entries of a word at a time, their loads all under way before the first store: one memory round trip
        // per four entries instead of one per entry.
#pragma unroll
        for (int g = 0; g < kGroups; ++g) {
            const uint64_t p0 = span + (uint64_t)g * kGroupSpan + 64u * lane;
            uint64_t mm = m[g], k = wave_base + before[g];
            while (mm) {
                uint64_t p[4];
                uint32_t v[4];
                bool on[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    on[i] = mm != 0;
                    p[i] = p0 + (on[i] ? (uint32_t)__builtin_ctzll((unsigned long long)mm) : 0u);
                    mm &= mm - 1;   // (0 stays 0)
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = !on[i] ? 0u : (x ? __builtin_nontemporal_load(x + p[i]) : (uint32_t)p[i]);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (on[i] && k + i < out_cap) out[k + i] = v[i];
                k += 4;
            }
        }
        return;
    }
    const uint64_t lane_below = (1ull << lane) - 1ull;
#pragma unroll
    for (int g = 0; g < kGroups; ++g) {
        const uint64_t word_base = wave_base + before[g];
        const uint32_t m_lo = (uint32_t)m[g], m_hi = (uint32_t)(m[g] >> 32);
        const uint32_t base_lo = (uint32_t)word_base, base_hi = (uint32_t)(word_base >> 32);
#pragma unroll 8
        for (int j = 0; j < kWords; ++j) {
            const uint64_t mj = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)m_hi, j) << 32) |
                                (uint32_t)__builtin_amdgcn_readlane((int)m_lo, j);
            const uint64_t bj = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)base_hi, j) << 32) |
                                (uint32_t)__builtin_amdgcn_readlane((int)base_lo, j);
            if ((mj >> lane) & 1ull) {
                const uint64_t p = span + (uint64_t)g * kGroupSpan + 64u * j + lane;
                const uint32_t v = x ? __builtin_nontemporal_load(x + p) : (uint32_t)p;
                const uint64_t k = bj + (uint32_t)__popcll((unsigned long long)(mj & lane_below));
                if (k < out_cap) out[k] = v;
            }
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
// left alone).  A count that points outside w subtracts nothing (there is no workspace to report it through;
// the compositions of this library only ever pass counts that COMPRESS has produced entries for).
template <typename A>
__global__ __launch_bounds__(256) void revert_kernel(const uint32_t *xhat, const int32_t *__restrict__ fhat,
                                                     const uint32_t *__restrict__ w, uint64_t n, uint64_t nw,
                                                     uint32_t *z) {
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
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        A v = from_bits<A>(xv[i]);
        const int64_t k = kv[i];
        if (k >= 2) {
            if ((uint64_t)(k - 2) < nw) v -= from_bits<A>(w[k - 2]);
        }
        o[i] = to_bits(v);
    }
    if (full) {
        __builtin_nontemporal_store(o, reinterpret_cast<v4u *>(z + e0));
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (e0 + i < n) z[e0 + i] = o[i];
    }
}

}  // namespace
