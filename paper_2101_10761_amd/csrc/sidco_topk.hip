// Exact Top-k by magnitude on MI355X (gfx950): the comparator the paper measures its threshold
// estimators against (arXiv 2101.10761, Sec. 1: Top-k keeps the k entries of largest magnitude and is
// found on a GPU by a radix select that reads the vector once per digit; footnote of Sec. 2.3: the
// threshold operator C_eta equals Top-k at k = khat).
//
// Radix select on the 31 magnitude bits of the fp32 values (|x| as an unsigned integer orders like |x|
// itself; NaN patterns lie above infinity and therefore count as the largest entries), most
// significant digit first, digits of 11 + 10 + 10 bits.  Only the first digit needs the whole vector:
//
//   k_topk_zero      clears the three digit histograms and the output counters
//   k_topk_hist      acc = g + residual (App. B.2), stored back; histogram of digit 0 of |acc|
//                    (per-block histogram in LDS, merged into the global one with atomics on 2048
//                    distinct addresses)                                         [12 B / element]
//   k_topk_compact   prologue: every block finds the digit-0 bin b0 that holds the k-th largest key
//                    (suffix sums of the histogram).  Body: entries with digit 0 >= b0 go to per-wave
//                    lists; those with digit 0 == b0 are binned by digit 1       [4 B / element]
//   k_topk_refine    prologue: bin b1 of digit 1; body (lists only): digit-2 histogram of the entries
//                    that match b0 and b1
//   k_topk_final     prologue: bin b2, i.e. the exact k-th largest key kappa and the number of entries
//                    equal to it that are still needed.  Body (lists only): entries above kappa and
//                    the needed number of entries equal to kappa go to the output; residual update.
//
// The k-th largest magnitude, the set of selected entries above it and every value are deterministic.
// Which of the entries that EQUAL the k-th largest magnitude complete the set is decided by the
// order in which blocks reserve their share and may differ between runs.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sidco_internal.h"
#include "sidco_device.h"
#include "sidco_select.h"

namespace sidco {

__global__ __launch_bounds__(kBlock) void k_topk_zero(TopkParams p)
{
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    if (i < 3u * kTopkBins) p.hist[i] = 0;
    if (i == 0) {
        p.st->gt_ctr = 0;
        p.st->eq_ctr = 0;
        p.st->prefix[0] = p.st->prefix[1] = p.st->prefix[2] = 0;
        p.st->k_rem[0] = p.st->k_rem[1] = p.st->k_rem[2] = 0;
        p.st->kth_key = 0;
        p.st->k_eff = 0;
    }
}

// ---------------------------------------------------------------------------------------------
// k_topk_hist: error-compensation add + digit-0 histogram
// ---------------------------------------------------------------------------------------------
template <bool EC, int GT>
__global__ __launch_bounds__(kBlock) void k_topk_hist(TopkParams p)
{
    // a 16-bit gradient is widened as it is read, and acc is always stored then (every later kernel reads fp32)
    constexpr bool WRITE = EC || GT != kGradF32;
    __shared__ uint32_t sh_hist[kTopkBins];
    for (int i = threadIdx.x; i < kTopkBins; i += kBlock) sh_hist[i] = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    const uint32_t w = blockIdx.x * kWavesPerBlock + wib;
    if (w < p.nwaves) {
        const uint32_t t0 = tile_begin(w, p.ntiles, p.nwaves), t1 = tile_begin(w + 1, p.ntiles, p.nwaves);
        const uint32_t tf = t1 < p.nfull ? t1 : p.nfull;
        uint32_t t = t0;
        if (p.vec_ok) {
            f4* __restrict__ r4 = reinterpret_cast<f4*>(p.acc_w);
            constexpr int U = 4;
            for (; t + U <= tf; t += U) {
                f4 a[U], b[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const size_t i = (size_t)(t + u) * 64 + lane;
                    // read once per call when acc is stored elsewhere: keep it out of the caches' way
                    a[u] = load_grad4<GT, WRITE>(p.grad, i);
                    if (EC) b[u] = r4[i];
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    f4 c = a[u];
                    if (EC) c = a[u] + b[u];
                    if (WRITE) r4[(size_t)(t + u) * 64 + lane] = c;
                    atomicAdd(&sh_hist[mag_key(c.x) >> 20], 1u);
                    atomicAdd(&sh_hist[mag_key(c.y) >> 20], 1u);
                    atomicAdd(&sh_hist[mag_key(c.z) >> 20], 1u);
                    atomicAdd(&sh_hist[mag_key(c.w) >> 20], 1u);
                }
            }
            for (; t < tf; ++t) {
                const size_t i = (size_t)t * 64 + lane;
                f4 c = load_grad4<GT, false>(p.grad, i);
                if (EC) c = c + r4[i];
                if (WRITE) r4[i] = c;
                atomicAdd(&sh_hist[mag_key(c.x) >> 20], 1u);
                atomicAdd(&sh_hist[mag_key(c.y) >> 20], 1u);
                atomicAdd(&sh_hist[mag_key(c.z) >> 20], 1u);
                atomicAdd(&sh_hist[mag_key(c.w) >> 20], 1u);
            }
        }
        for (; t < t1; ++t) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t i = (int64_t)t * kTile + lane * 4 + j;
                if (i < p.d) {
                    float c = load_grad1<GT>(p.grad, i);
                    if (EC) c = c + p.acc_w[i];
                    if (WRITE) p.acc_w[i] = c;
                    atomicAdd(&sh_hist[mag_key(c) >> 20], 1u);
                }
            }
        }
    }
    __syncthreads();
    merge_hist(sh_hist, p.hist, kTopkBins);
}

// ---------------------------------------------------------------------------------------------
// k_topk_compact: dense pass.  Entries whose digit 0 is at least b0 go to the wave's list; digit-1
// histogram of those whose digit 0 equals b0.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void topk_emit(bool valid, float x, int32_t idx, uint32_t b0, ListWriter& lw, int lane,
                                          uint32_t* sh_hist)
{
    const uint32_t key = mag_key(x);
    const uint32_t d0 = key >> 20;
    list_push(lw, valid && d0 >= b0, idx, x, lane);
    if (valid && d0 == b0) atomicAdd(&sh_hist[(key >> 10) & 1023u], 1u);
}

__global__ __launch_bounds__(kBlock, 4) void k_topk_compact(TopkParams p)
{
    __shared__ uint32_t sh_hist[1024];
    __shared__ uint32_t sh_scan[kBlock];
    __shared__ uint32_t sh_out[2];
    __shared__ int2 ring[kWavesPerBlock][kRingSize];
    for (int i = threadIdx.x; i < 1024; i += kBlock) sh_hist[i] = 0;
    uint32_t b0, k1;
    pick_bin<kTopkBins / kBlock>(p.hist, (unsigned long long)p.k, sh_scan, sh_out, b0, k1);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        p.st->prefix[0] = b0;
        p.st->k_rem[0] = k1;
    }
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    const uint32_t w = blockIdx.x * kWavesPerBlock + wib;
    if (w < p.nwaves) {
        const uint32_t t0 = tile_begin(w, p.ntiles, p.nwaves), t1 = tile_begin(w + 1, p.ntiles, p.nwaves);
        const uint32_t tf = t1 < p.nfull ? t1 : p.nfull;
        ListWriter lw;
        lw.list = p.seg + (size_t)t0 * kTile;
        lw.ring = ring[wib];
        lw.run = lw.fill = 0;
        uint32_t ts = t0;
        if (p.vec_ok) {
            const f4* __restrict__ x4 = reinterpret_cast<const f4*>(p.acc);
            constexpr uint32_t U = 4;
            const uint32_t nb = (tf - t0) / U, rem = (tf - t0) - nb * U;
            // from the last tile to the first: k_topk_hist left the end of the wave's range in L2
#pragma unroll 1
            for (uint32_t kb = 0; kb < nb; ++kb) {
                const uint32_t t = tf - (kb + 1) * U;
                f4 a[U];
#pragma unroll
                for (uint32_t u = 0; u < U; ++u) a[u] = x4[(size_t)(t + u) * 64 + lane];
#pragma unroll
                for (uint32_t u = 0; u < U; ++u) {
                    const int32_t i0 = (int32_t)((t + u) * kTile + lane * 4);
                    topk_emit(true, a[u].x, i0 + 0, b0, lw, lane, sh_hist);
                    topk_emit(true, a[u].y, i0 + 1, b0, lw, lane, sh_hist);
                    topk_emit(true, a[u].z, i0 + 2, b0, lw, lane, sh_hist);
                    topk_emit(true, a[u].w, i0 + 3, b0, lw, lane, sh_hist);
                    list_flush(lw, lane);
                }
            }
            for (uint32_t t = t0; t < t0 + rem; ++t) {
                const f4 a = x4[(size_t)t * 64 + lane];
                const int32_t i0 = (int32_t)(t * kTile + lane * 4);
                topk_emit(true, a.x, i0 + 0, b0, lw, lane, sh_hist);
                topk_emit(true, a.y, i0 + 1, b0, lw, lane, sh_hist);
                topk_emit(true, a.z, i0 + 2, b0, lw, lane, sh_hist);
                topk_emit(true, a.w, i0 + 3, b0, lw, lane, sh_hist);
                list_flush(lw, lane);
            }
            ts = tf;
        }
        for (uint32_t t = ts; t < t1; ++t) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t i = (int64_t)t * kTile + lane * 4 + j;
                const bool valid = i < p.d;
                topk_emit(valid, valid ? p.acc[i] : 0.0f, (int32_t)i, b0, lw, lane, sh_hist);
            }
            list_flush(lw, lane);
        }
        const uint32_t n = list_finish(lw, lane);
        if (lane == 0) p.cnt[w] = n;
    }
    __syncthreads();
    merge_hist(sh_hist, p.hist + kTopkBins, 1024);
}

// k_topk_refine: digit-2 histogram of the list entries whose digits 0 and 1 are b0 and b1
__global__ __launch_bounds__(kBlock) void k_topk_refine(TopkParams p)
{
    __shared__ uint32_t sh_hist[1024];
    __shared__ uint32_t sh_scan[kBlock];
    __shared__ uint32_t sh_out[2];
    for (int i = threadIdx.x; i < 1024; i += kBlock) sh_hist[i] = 0;
    const uint32_t b0 = p.st->prefix[0];
    const uint32_t k1 = p.st->k_rem[0];
    uint32_t b1, k2;
    pick_bin<1024 / kBlock>(p.hist + kTopkBins, (unsigned long long)k1, sh_scan, sh_out, b1, k2);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        p.st->prefix[1] = b1;
        p.st->k_rem[1] = k2;
    }
    const int lane = threadIdx.x & 63;
    const uint32_t want = (b0 << 10) | b1;  // key >> 10
    const ListRange r = my_lists(p.nwaves);
    for (uint32_t sw = r.first; sw < r.last; sw += kWavesPerBlock) {
        const int2* __restrict__ list = p.seg + (size_t)tile_begin(sw, p.ntiles, p.nwaves) * kTile;
        const uint32_t n = p.cnt[sw];
        for (uint32_t c = lane; c < n; c += 64) {
            const uint32_t key = mag_key(__int_as_float(list[c].y));
            if ((key >> 10) == want) atomicAdd(&sh_hist[key & 1023u], 1u);
        }
    }
    __syncthreads();
    merge_hist(sh_hist, p.hist + 2 * kTopkBins, 1024);
}

// k_topk_final: the k-th largest key, the output and the residual update
__global__ __launch_bounds__(kBlock) void k_topk_final(TopkParams p)
{
    __shared__ uint32_t sh_scan[kBlock];
    __shared__ uint32_t sh_out[2];
    __shared__ uint32_t sh_gt[kWavesPerBlock], sh_eq[kWavesPerBlock];
    __shared__ unsigned long long sh_base[2];
    const uint32_t b0 = p.st->prefix[0], b1 = p.st->prefix[1];
    const uint32_t k2 = p.st->k_rem[1];
    uint32_t b2, need;
    pick_bin<1024 / kBlock>(p.hist + 2 * kTopkBins, (unsigned long long)k2, sh_scan, sh_out, b2, need);
    const uint32_t kappa = (b0 << 20) | (b1 << 10) | b2;
    const unsigned long long K = p.k_from_state ? (unsigned long long)p.st->k_eff : (unsigned long long)p.k;
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    const ListRange r = my_lists(p.nwaves);

    // pass A: entries above kappa and entries equal to it, per wave
    uint32_t n_gt = 0, n_eq = 0;
    for (uint32_t sw = r.first; sw < r.last; sw += kWavesPerBlock) {
        const int2* __restrict__ list = p.seg + (size_t)tile_begin(sw, p.ntiles, p.nwaves) * kTile;
        const uint32_t n = p.cnt[sw];
        for (uint32_t c = 0; c < n; c += 64) {
            const bool in = c + lane < n;
            const uint32_t key = in ? mag_key(__int_as_float(list[c + lane].y)) : 0u;
            n_gt += (uint32_t)__popcll(__ballot(in && key > kappa));
            n_eq += (uint32_t)__popcll(__ballot(in && key == kappa));
        }
    }
    if (lane == 0) {
        sh_gt[wib] = n_gt;
        sh_eq[wib] = n_eq;
    }
    __syncthreads();
    uint32_t off_gt = 0, off_eq = 0, tot_gt = 0, tot_eq = 0;
#pragma unroll
    for (int i = 0; i < kWavesPerBlock; ++i) {
        if (i < wib) {
            off_gt += sh_gt[i];
            off_eq += sh_eq[i];
        }
        tot_gt += sh_gt[i];
        tot_eq += sh_eq[i];
    }
    if (threadIdx.x == 0) {
        // one reservation per block and counter (same-address atomics are slow: keep them few)
        sh_base[0] = tot_gt ? atomicAdd(&p.st->gt_ctr, (unsigned long long)tot_gt) : 0ull;
        sh_base[1] = tot_eq ? atomicAdd(&p.st->eq_ctr, (unsigned long long)tot_eq) : 0ull;
        if (blockIdx.x == 0) {
            p.st->prefix[2] = b2;
            p.st->k_rem[2] = need;
            p.st->kth_key = kappa;
            *p.out_count = (int32_t)K;
            *p.out_kth = __int_as_float((int)kappa);
        }
    }
    __syncthreads();
    // the k - need entries above kappa fill the front of the output, the ties the last `need` places
    unsigned long long pos_gt = sh_base[0] + off_gt;
    unsigned long long pos_eq = sh_base[1] + off_eq;
    const unsigned long long tie_base = K - need;

    // pass B: same traversal, writing
    for (uint32_t sw = r.first; sw < r.last; sw += kWavesPerBlock) {
        const int2* __restrict__ list = p.seg + (size_t)tile_begin(sw, p.ntiles, p.nwaves) * kTile;
        const uint32_t n = p.cnt[sw];
        for (uint32_t c = 0; c < n; c += 64) {
            const bool in = c + lane < n;
            const int2 e = in ? list[c + lane] : make_int2(0, 0);
            const uint32_t key = mag_key(__int_as_float(e.y));
            const bool gt = in && key > kappa, eq = in && key == kappa;
            const unsigned long long m_gt = __ballot(gt), m_eq = __ballot(eq);
            unsigned long long at = 0;
            bool take = false;
            if (gt) {
                at = pos_gt + lane_prefix(m_gt);
                take = at < tie_base;  // always true; keeps a corrupted histogram from writing out of bounds
            } else if (eq) {
                const unsigned long long rank = pos_eq + lane_prefix(m_eq);
                take = rank < need;
                at = tie_base + rank;
            }
            if (take) {
                p.out_idx[at] = e.x;
                p.out_val[at] = __int_as_float(e.y);
                if (p.residual) p.residual[e.x] = 0.0f;
            }
            pos_gt += (unsigned long long)__popcll(m_gt);
            pos_eq += (unsigned long long)__popcll(m_eq);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
void launch_topk_zero(const TopkParams& p, hipStream_t s)
{
    hipLaunchKernelGGL(k_topk_zero, dim3((3 * kTopkBins + kBlock - 1) / kBlock), dim3(kBlock), 0, s, p);
}

template <int GT>
static void launch_topk_hist_type(const TopkParams& p, hipStream_t s)
{
    if (p.residual) hipLaunchKernelGGL((k_topk_hist<true, GT>), dim3(p.nblocks), dim3(kBlock), 0, s, p);
    else hipLaunchKernelGGL((k_topk_hist<false, GT>), dim3(p.nblocks), dim3(kBlock), 0, s, p);
}

void launch_topk_hist(const TopkParams& p, hipStream_t s)
{
    switch (p.gt) {
        case kGradF16: launch_topk_hist_type<kGradF16>(p, s); break;
        case kGradBf16: launch_topk_hist_type<kGradBf16>(p, s); break;
        default: launch_topk_hist_type<kGradF32>(p, s); break;
    }
}

void launch_topk_compact(const TopkParams& p, hipStream_t s)
{
    hipLaunchKernelGGL(k_topk_compact, dim3(p.nblocks), dim3(kBlock), 0, s, p);
}

void launch_topk_refine(const TopkParams& p, uint32_t grid, hipStream_t s)
{
    hipLaunchKernelGGL(k_topk_refine, dim3(grid), dim3(kBlock), 0, s, p);
}

void launch_topk_final(const TopkParams& p, uint32_t grid, hipStream_t s)
{
    hipLaunchKernelGGL(k_topk_final, dim3(grid), dim3(kBlock), 0, s, p);
}

}  // namespace sidco
