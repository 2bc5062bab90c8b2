// libmmvseg, part of the one translation unit mmvseg.hip (included there, in order).
// Lane-level helpers: bit casts, descriptor loads and stores, lane exchanges (DPP moves, permlane swap,
// shuffles), wave sums, the look-back over tile descriptors.
#pragma once

namespace {

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
// kPolled windows of 64 descriptors may have been loaded by the caller itself, some time ago (lookback_poll: lane l
// of window w holds the descriptor of tile  tile - 1 - 64 w - l); they are used as far as they suffice, then the loop
// polls as usual.
template <int kWindows>
__device__ __forceinline__ void lookback_poll(const uint64_t *desc, int tile, int lane, uint64_t (&polled)[kWindows]) {
#pragma unroll
    for (int w = 0; w < kWindows; ++w) {
        const int idx = tile - 1 - 64 * w - lane;
        polled[w] = idx >= 0 ? desc_load(desc + idx) : (kStatusPrefix << 62);
    }
}
template <typename T, bool kAlu, int kPolled>
__device__ T lookback_from(const uint64_t *desc, int tile, int lane, uint32_t *hdr, const uint64_t *polled) {
    T carry = T(0);
    int pos = tile - 1;
    uint32_t spins = 0;
    int window = 0;     // windows done
    bool fresh = true;  // the polled copy of this window has not been tried
    while (true) {
        const int idx = pos - lane;
        uint64_t d = 0;
        bool have = false;
#pragma unroll
        for (int w = 0; w < kPolled; ++w)
            if (fresh && window == w) {
                d = polled[w];
                have = true;
            }
        if (!have) d = idx >= 0 ? desc_load(desc + idx) : (kStatusPrefix << 62);
        fresh = false;
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
        ++window;
        fresh = true;
    }
    return carry;
}
template <typename T, bool kAlu = true>
__device__ T lookback(const uint64_t *desc, int tile, int lane, uint32_t *hdr) {
    return lookback_from<T, kAlu, 0>(desc, tile, lane, hdr, nullptr);
}

}  // namespace
