// libmmvseg, part of the one translation unit mmvseg.hip (included there, in order).
// The entry of the single-pass kernel: which tile a workgroup takes, and which tile body runs.
#pragma once

namespace {

// Tiles are handed out by an atomic ticket, so that a tile never waits for a predecessor that
// has not started.  The tickets of workgroups that start together are served one after the other
// (about 11 ns each: the 512 workgroups of the first round would get theirs spread over 6 us), so the
// workgroups that are resident at once from the start (all of them, if the grid fits the device) take
// the tile of their own index instead: they are started in index order, so the predecessors of such a
// tile are never behind it.  Tickets begin where those tiles end.
template <typename Shared> __device__ __forceinline__ uint32_t take_tile(const Params &P, Shared &sm) {
    const bool own_index = blockIdx.x < P.first_round;
    if (threadIdx.x == 0) {
        sm.ready = 0;
        sm.arrived = 0;
        if (blockIdx.x < P.stagger_wgs && P.stagger_ticks) {
            // low-discrepancy spread of the start times: fraction of blockIdx * golden ratio
            const uint32_t frac = blockIdx.x * 2654435769u;
            const uint64_t wait = ((uint64_t)frac * P.stagger_ticks) >> 32;
            const uint64_t t0 = wall_clock64();
            while (wall_clock64() - t0 < wait) __builtin_amdgcn_s_sleep(8);
        }
        if (!own_index)
            sm.tile = P.first_round +
                      __hip_atomic_fetch_add(P.hdr + kHdrTicket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    return __builtin_amdgcn_readfirstlane(own_index ? blockIdx.x : sm.tile);   // a scalar, like the wave index
}

template <typename TT, int kOp, bool kMfma>
__global__ __launch_bounds__(TT::kWaves * 64, MMV_MIN_WAVES_PER_SIMD) void seg_kernel(Params P, const uint32_t *__restrict__ hints) {
    __shared__ SegShared<TT::kWaves> sm;
    constexpr bool kProduct = kOp == kSpmv || kOp == kSpmvCsr;
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
    if constexpr (kProduct) {
        // SpMV in two steps: without the mark of the preparing call for this matrix the flags, counts and row map of
        // the workspace are not to be trusted (the reset launch has put that into the status word)
        if (P.prepared && hints[kHdrPrepared - kHdrHints] != P.prepared) return;
        late_val = hints[kHdrColumnRuns - kHdrHints] != 0;
    }
    const uint32_t tile = take_tile(P, sm);
    if (kProduct && late_val)
        seg_tile<TT, kOp, kMfma, kProduct>(P, hints, sm, tile);
    else
        seg_tile<TT, kOp, kMfma, false>(P, hints, sm, tile);
}

// The segmented sum of 8- and 16-bit inputs (speculation over whole chunks): its waves keep less in LDS and in
// registers than those of the scan, so more workgroups share a compute unit.
template <typename TT, bool kMfma>
__global__ __launch_bounds__(TT::kWaves * 64, sum_waves_per_simd<TT>()) void sum_kernel(Params P, const uint32_t *__restrict__) {
    __shared__ SumShared<TT> sm;
#if MMV_LOAD_PRIO
    __builtin_amdgcn_s_setprio(MMV_LOAD_PRIO);
#endif
    const uint32_t tile = take_tile(P, sm);
    sum_tile<TT, kMfma>(P, sm, tile);
}

}  // namespace
