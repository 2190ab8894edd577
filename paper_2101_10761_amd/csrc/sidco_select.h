// Radix-select building blocks shared by the exact Top-k comparator and the DGC comparator: the
// magnitude key of an fp32 value, the search of a digit histogram for the bin that holds the k-th
// largest key, the merge of a block's LDS histogram into the global one, and the split of the
// per-wave lists over a small grid.
#ifndef SIDCO_SELECT_H
#define SIDCO_SELECT_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sidco_internal.h"

namespace sidco {

__device__ __forceinline__ uint32_t mag_key(float x) { return (uint32_t)__float_as_int(x) & 0x7fffffffu; }

// Bin of `hist` (nb bins, nb = kBlock * PER) that holds the k-th largest entry, counted from the top
// bin downwards, and the rank the entry has inside that bin.  Every thread of the block returns the
// same pair.  Needs sum(hist) >= k >= 1.
template <int PER>
__device__ __forceinline__ void pick_bin(const uint32_t* __restrict__ hist, unsigned long long k, uint32_t* sh_scan,
                                         uint32_t* sh_out, uint32_t& bin, uint32_t& k_in_bin)
{
    const uint32_t t = threadIdx.x;
    uint32_t local[PER];
    uint32_t tsum = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        local[j] = hist[t * PER + j];
        tsum += local[j];
    }
    // inclusive suffix sums over the threads (counts are at most d < 2^31: no overflow)
    __syncthreads();  // protects sh_scan / sh_out against a previous use
    sh_scan[t] = tsum;
    if (t == 0) sh_out[0] = sh_out[1] = 0;  // only reached if the histogram holds fewer than k entries
    __syncthreads();
    uint32_t s = tsum;
    for (uint32_t o = 1; o < (uint32_t)kBlock; o <<= 1) {
        const uint32_t other = t + o < (uint32_t)kBlock ? sh_scan[t + o] : 0u;
        __syncthreads();
        s += other;
        sh_scan[t] = s;
        __syncthreads();
    }
    const unsigned long long above = (unsigned long long)s - tsum;  // entries in the bins of later threads
    if (above < k && k <= (unsigned long long)s) {                  // exactly one thread
        unsigned long long acc = above;
#pragma unroll
        for (int j = PER - 1; j >= 0; --j) {
            if (acc < k && k <= acc + local[j]) {
                sh_out[0] = t * PER + j;
                sh_out[1] = (uint32_t)(k - acc);
            }
            acc += local[j];
        }
    }
    __syncthreads();
    bin = sh_out[0];
    k_in_bin = sh_out[1];
}

// adds a block's LDS histogram to the global one
__device__ __forceinline__ void merge_hist(const uint32_t* sh_hist, uint32_t* __restrict__ hist, int nb)
{
    for (int i = threadIdx.x; i < nb; i += kBlock) {
        const uint32_t c = sh_hist[i];
        if (c) atomicAdd(&hist[i], c);
    }
}

// ---------------------------------------------------------------------------------------------
// the per-wave lists split over a small grid: a wave takes the lists first, first + 8, ... below last
// ---------------------------------------------------------------------------------------------
struct ListRange {
    uint32_t first, last;
};
__device__ __forceinline__ ListRange my_lists(uint32_t nwaves)
{
    const uint32_t per_block = (nwaves + gridDim.x - 1) / gridDim.x;
    ListRange r;
    r.first = blockIdx.x * per_block + (threadIdx.x >> 6);
    const uint32_t end = (blockIdx.x + 1) * per_block;
    r.last = end < nwaves ? end : nwaves;
    return r;
}

}  // namespace sidco
#endif
