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

// Four consecutive gradient elements as fp32, starting at element 4 * v: one 16-byte load of an fp32
// buffer, one 8-byte load of an fp16 / bf16 buffer (widening either type is exact).  STREAM: the
// buffer is read once per call, keep it out of the caches' way (a template parameter: as a run-time
// flag the two loads are merged and the non-temporal hint is lost).
template <int GT, bool STREAM>
__device__ __forceinline__ f4 load_grad4(const void* __restrict__ g, size_t v)
{
    if constexpr (GT == kGradF32) {
        const f4* g4 = reinterpret_cast<const f4*>(g);
        if constexpr (STREAM) return __builtin_nontemporal_load(g4 + v);
        else return g4[v];
    } else {
        const uint64_t* g8 = reinterpret_cast<const uint64_t*>(g);
        uint64_t w;
        if constexpr (STREAM) w = __builtin_nontemporal_load(g8 + v);
        else w = g8[v];
        const uint32_t w0 = (uint32_t)w, w1 = (uint32_t)(w >> 32);  // elements 0,1 and 2,3
        f4 c;
        if constexpr (GT == kGradBf16) {
            c.x = __uint_as_float(w0 << 16);
            c.y = __uint_as_float(w0 & 0xffff0000u);
            c.z = __uint_as_float(w1 << 16);
            c.w = __uint_as_float(w1 & 0xffff0000u);
        } else {
            typedef _Float16 h2 __attribute__((ext_vector_type(2)));
            const h2 lo = __builtin_bit_cast(h2, w0), hi = __builtin_bit_cast(h2, w1);
            c.x = (float)lo.x;
            c.y = (float)lo.y;
            c.z = (float)hi.x;
            c.w = (float)hi.y;
        }
        return c;
    }
}

// one gradient element as fp32
template <int GT>
__device__ __forceinline__ float load_grad1(const void* __restrict__ g, int64_t i)
{
    if constexpr (GT == kGradF32) return reinterpret_cast<const float*>(g)[i];
    else if constexpr (GT == kGradBf16)
        return __uint_as_float((uint32_t) reinterpret_cast<const uint16_t*>(g)[i] << 16);
    else return (float)reinterpret_cast<const _Float16*>(g)[i];
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
template <typename T>
struct ListWriterT {
    T* __restrict__ list;  // the wave's list in global memory (room for every element of its tiles)
    T* ring;               // the wave's staging area in LDS, kRingSize entries
    uint32_t run;          // entries already written to `list` (wave-uniform)
    uint32_t fill;         // entries staged in `ring` (wave-uniform, < kRingFlush after list_flush)
};
typedef ListWriterT<int2> ListWriter;  // (index, value bits) pairs

template <typename T>
__device__ __forceinline__ void list_push_entry(ListWriterT<T>& lw, bool keep, T e, int lane)
{
    const unsigned long long mask = __ballot(keep);
    if (keep) lw.ring[lw.fill + lane_prefix(mask)] = e;
    lw.fill += (uint32_t)__popcll(mask);
}

__device__ __forceinline__ void list_push(ListWriter& lw, bool keep, int32_t idx, float x, int lane)
{
    list_push_entry(lw, keep, make_int2(idx, __float_as_int(x)), lane);
}

// After at most kTile pushes: writes out kRingFlush entries at a time while that many are staged.
template <typename T>
__device__ __forceinline__ void list_flush(ListWriterT<T>& lw, int lane)
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
template <typename T>
__device__ __forceinline__ uint32_t list_finish(ListWriterT<T>& lw, int lane)
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
