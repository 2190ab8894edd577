// Device-side helpers shared by the kernels of the SIDCo library: wave primitives, the split of the
// vector into per-wave tile ranges, and the LDS-staged writer of per-wave survivor lists.
#ifndef SIDCO_DEVICE_H
#define SIDCO_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sidco_internal.h"

namespace sidco {

typedef float f4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;  // lane 0 holds the sum
}

__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;
}

// number of set bits of `mask` below this lane
__device__ __forceinline__ uint32_t lane_prefix(unsigned long long mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// first tile of wave w: tiles are split as evenly as possible over the waves
__device__ __forceinline__ uint32_t tile_begin(uint32_t w, uint32_t ntiles, uint32_t nwaves)
{
    return (uint32_t)(((unsigned long long)w * ntiles) / nwaves);
}

// A wave's survivor list under construction.  Entries are collected in LDS and written out in long
// contiguous runs: global stores complete in order with the wave's loads, so a store issued between
// two batches of streaming loads holds the next batch back by its own round trip; few, large,
// full-line stores cost a fraction of one small partial-line store per tile component (measured:
// 1.6 M entries out of 25.6 M elements add 9 us as they come and 3 us staged).
constexpr uint32_t kRingFlush = 512;                // staged entries that trigger a write-out
constexpr uint32_t kRingSize = kRingFlush + kTile;  // a whole tile can arrive between two checks
struct ListWriter {
    int2* __restrict__ list;  // the wave's list in global memory (room for every element of its tiles)
    int2* ring;               // the wave's staging area in LDS, kRingSize entries
    uint32_t run;             // entries already written to `list` (wave-uniform)
    uint32_t fill;            // entries staged in `ring` (wave-uniform, < kRingFlush after list_flush)
};

__device__ __forceinline__ void list_push(ListWriter& lw, bool keep, int32_t idx, float x, int lane)
{
    const unsigned long long mask = __ballot(keep);
    if (keep) lw.ring[lw.fill + lane_prefix(mask)] = make_int2(idx, __float_as_int(x));
    lw.fill += (uint32_t)__popcll(mask);
}

// After at most kTile pushes: writes out kRingFlush entries at a time while that many are staged.
__device__ __forceinline__ void list_flush(ListWriter& lw, int lane)
{
    if (lw.fill < kRingFlush) return;  // wave-uniform
    const uint32_t whole = lw.fill & ~(kRingFlush - 1);
#pragma unroll 1
    for (uint32_t c = 0; c < whole; c += 64) lw.list[lw.run + c + lane] = lw.ring[c + lane];
    // the leftover (fewer than kRingFlush entries) moves to the front; LDS accesses of a wave stay in order
    const uint32_t left = lw.fill - whole;
#pragma unroll 1
    for (uint32_t c = 0; c < left; c += 64)
        if (c + lane < left) lw.ring[c + lane] = lw.ring[whole + c + lane];  // source and destination are disjoint
    lw.run += whole;
    lw.fill = left;
}

// writes out what is still staged; returns the list's length
__device__ __forceinline__ uint32_t list_finish(ListWriter& lw, int lane)
{
#pragma unroll 1
    for (uint32_t c = 0; c < lw.fill; c += 64)
        if (c + lane < lw.fill) lw.list[lw.run + c + lane] = lw.ring[c + lane];
    lw.run += lw.fill;
    lw.fill = 0;
    return lw.run;
}

}  // namespace sidco
#endif
