// DGC's sampling threshold on MI355X (gfx950): one of the threshold methods the paper compares itself
// with (arXiv 2101.10761, Sec. 1, related work and its footnote).  A random subset of the gradient
// (about 1 %) is drawn, Top-k of the subset at the target ratio gives a threshold, the threshold
// selects from the whole vector, and if it selects more than the target k a second Top-k trims the
// selection to k.
//
// Both Top-k steps are radix selects on the 31 magnitude bits (digits of 11 + 10 + 10 bits), as in
// the exact Top-k comparator; only the first pass reads the whole vector, and it does so once:
//
//   k_dgc_zero     clears the six digit histograms and the state
//   k_dgc_sample   draw j of the subset is element floor(u_j d / 2^32), u_j the upper half of output j
//                  of the splitmix64 sequence started at the caller's seed (counter based: every
//                  thread computes its own draws); acc = g + residual of the drawn elements, their
//                  magnitude keys stored, digit-0 histogram
//   k_dgc_digit<1> bin of digit 0 that holds the k_s-th largest key; digit-1 histogram of its keys
//   k_dgc_digit<2> bin of digit 1; digit-2 histogram
//   k_dgc_dense    prologue: bin of digit 2, i.e. the threshold eta.  Body: acc = g + residual
//                  (App. B.2), stored back; entries with |acc| > eta go to per-wave lists; digit-0
//                  histogram of those entries                                      [12 B / element]
//   k_dgc_lists    first-pass count S (the histogram's total), K = min(k, S); bin of digit 0 that
//                  holds the K-th largest listed key; digit-1 histogram (lists only)
//   k_topk_refine, k_topk_final (shared with the exact Top-k): digits 1 and 2, output of the K largest
//                  listed entries, residual update.  With S <= k that is every listed entry.
//
// No step depends on a host read-back: the device decides whether the trim is needed.
// Finishing the subset's select inside one kernel (the block that takes the last ticket resolves the
// remaining digits) was measured and dropped: the device-scope fence it needs writes the dirty part of
// L2 back, 43 us for a kernel that otherwise takes 6.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sidco_internal.h"
#include "sidco_device.h"
#include "sidco_select.h"

namespace sidco {

// output j (j = 0 first) of the splitmix64 sequence (Steele, Lea, Flood 2014) whose state starts at seed
__device__ __forceinline__ uint64_t splitmix64_at(uint64_t seed, uint64_t j)
{
    uint64_t z = seed + (j + 1u) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__global__ __launch_bounds__(kBlock) void k_dgc_zero(DgcParams p)
{
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    if (i < 3u * kTopkBins) {
        p.hist_s[i] = 0;
        p.hist_l[i] = 0;
    }
    if (i == 0) {
        DgcState z = {};
        *p.st = z;
    }
}

constexpr int kDrawsPerThread = 4;  // independent random accesses a thread has in flight

template <bool EC, int GT>
__global__ __launch_bounds__(kBlock) void k_dgc_sample(DgcParams p)
{
    __shared__ uint32_t sh_hist[kTopkBins];
    for (int i = threadIdx.x; i < kTopkBins; i += kBlock) sh_hist[i] = 0;
    __syncthreads();
    const uint32_t stride = gridDim.x * kBlock;
    for (uint32_t j0 = blockIdx.x * kBlock + threadIdx.x; j0 < p.n_s; j0 += stride * kDrawsPerThread) {
        float x[kDrawsPerThread], r[kDrawsPerThread];
#pragma unroll
        for (int q = 0; q < kDrawsPerThread; ++q) {  // all loads first: one round trip for the lot
            const uint32_t j = j0 + q * stride;
            const uint64_t u = splitmix64_at(p.seed, j) >> 32;
            const int64_t i = (int64_t)((u * (uint64_t)p.d) >> 32);
            x[q] = j < p.n_s ? load_grad1<GT>(p.grad, i) : 0.0f;
            r[q] = (EC && j < p.n_s) ? p.residual[i] : 0.0f;
        }
#pragma unroll
        for (int q = 0; q < kDrawsPerThread; ++q) {
            const uint32_t j = j0 + q * stride;
            if (j < p.n_s) {
                const uint32_t key = mag_key(EC ? x[q] + r[q] : x[q]);
                p.keys[j] = key;
                atomicAdd(&sh_hist[key >> 20], 1u);
            }
        }
    }
    __syncthreads();
    merge_hist(sh_hist, p.hist_s, kTopkBins);
}

// DIGIT 1: keys whose digit 0 is b0, binned by digit 1.  DIGIT 2: keys that match b0 and b1, binned by digit 2.
template <int DIGIT>
__global__ __launch_bounds__(kBlock) void k_dgc_digit(DgcParams p)
{
    __shared__ uint32_t sh_hist[1024];
    __shared__ uint32_t sh_scan[kBlock];
    __shared__ uint32_t sh_out[2];
    for (int i = threadIdx.x; i < 1024; i += kBlock) sh_hist[i] = 0;
    uint32_t want, rest;
    if (DIGIT == 1) {
        pick_bin<kTopkBins / kBlock>(p.hist_s, (unsigned long long)p.k_s, sh_scan, sh_out, want, rest);
    } else {
        const uint32_t b0 = p.st->sample.prefix[0];
        uint32_t b1;
        pick_bin<1024 / kBlock>(p.hist_s + kTopkBins, (unsigned long long)p.st->sample.k_rem[0], sh_scan, sh_out, b1,
                                rest);
        want = (b0 << 10) | b1;
        if (blockIdx.x == 0 && threadIdx.x == 0) p.st->sample.prefix[1] = b1;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (DIGIT == 1) p.st->sample.prefix[0] = want;
        p.st->sample.k_rem[DIGIT - 1] = rest;
    }
    constexpr int shift = DIGIT == 1 ? 20 : 10;
    for (uint32_t j = blockIdx.x * kBlock + threadIdx.x; j < p.n_s; j += gridDim.x * kBlock) {
        const uint32_t key = p.keys[j];
        if ((key >> shift) == want) atomicAdd(&sh_hist[(key >> (shift - 10)) & 1023u], 1u);
    }
    __syncthreads();
    merge_hist(sh_hist, p.hist_s + DIGIT * kTopkBins, 1024);
}

// ---------------------------------------------------------------------------------------------
// k_dgc_dense: the one pass over the vector
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void dgc_emit(bool valid, float x, int32_t idx, float eta, ListWriter& lw, int lane,
                                         uint32_t* sh_hist)
{
    // strict and fp32, as the threshold operator of Sec. 2.3; NaN on either side is false
    const bool keep = valid && (__builtin_fabsf(x) > eta);
    list_push(lw, keep, idx, x, lane);
    if (keep) atomicAdd(&sh_hist[mag_key(x) >> 20], 1u);
}

template <bool EC, int GT>
__global__ __launch_bounds__(kBlock, 4) void k_dgc_dense(DgcParams p)
{
    __shared__ uint32_t sh_hist[kTopkBins];
    __shared__ uint32_t sh_scan[kBlock];
    __shared__ uint32_t sh_out[2];
    __shared__ int2 ring[kWavesPerBlock][kRingSize];
    for (int i = threadIdx.x; i < kTopkBins; i += kBlock) sh_hist[i] = 0;
    uint32_t b2, ties;
    pick_bin<1024 / kBlock>(p.hist_s + 2 * kTopkBins, (unsigned long long)p.st->sample.k_rem[1], sh_scan, sh_out, b2,
                            ties);
    const uint32_t kappa = (p.st->sample.prefix[0] << 20) | (p.st->sample.prefix[1] << 10) | b2;
    const float eta = __int_as_float((int)kappa);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        p.st->sample.prefix[2] = b2;
        p.st->sample.k_rem[2] = ties;
        p.st->sample.kth_key = kappa;
        p.st->eta = eta;
        *p.out_eta = eta;
    }
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    const uint32_t w = blockIdx.x * kWavesPerBlock + wib;
    if (w < p.nwaves) {
        const uint32_t t0 = tile_begin(w, p.ntiles, p.nwaves), t1 = tile_begin(w + 1, p.ntiles, p.nwaves);
        const uint32_t tf = t1 < p.nfull ? t1 : p.nfull;  // tiles [t0,tf) are complete
        ListWriter lw;
        lw.list = p.seg + (size_t)t0 * kTile;
        lw.ring = ring[wib];
        lw.run = lw.fill = 0;
        uint32_t t = t0;
        if (p.vec_ok) {
            f4* __restrict__ r4 = reinterpret_cast<f4*>(p.residual);
            constexpr uint32_t U = 4;
#pragma unroll 1
            for (; t + U <= tf; t += U) {
                f4 a[U], b[U];
#pragma unroll
                for (uint32_t u = 0; u < U; ++u) {
                    const size_t i = (size_t)(t + u) * 64 + lane;
                    a[u] = load_grad4<GT, EC>(p.grad, i);
                    if (EC) b[u] = r4[i];
                }
#pragma unroll
                for (uint32_t u = 0; u < U; ++u) {
                    f4 c = a[u];
                    if (EC) {
                        c = a[u] + b[u];
                        r4[(size_t)(t + u) * 64 + lane] = c;
                    }
                    const int32_t i0 = (int32_t)((t + u) * kTile + lane * 4);
                    dgc_emit(true, c.x, i0 + 0, eta, lw, lane, sh_hist);
                    dgc_emit(true, c.y, i0 + 1, eta, lw, lane, sh_hist);
                    dgc_emit(true, c.z, i0 + 2, eta, lw, lane, sh_hist);
                    dgc_emit(true, c.w, i0 + 3, eta, lw, lane, sh_hist);
                    list_flush(lw, lane);
                }
            }
            for (; t < tf; ++t) {
                const size_t i = (size_t)t * 64 + lane;
                f4 c = load_grad4<GT, false>(p.grad, i);
                if (EC) {
                    c = c + r4[i];
                    r4[i] = c;
                }
                const int32_t i0 = (int32_t)(t * kTile + lane * 4);
                dgc_emit(true, c.x, i0 + 0, eta, lw, lane, sh_hist);
                dgc_emit(true, c.y, i0 + 1, eta, lw, lane, sh_hist);
                dgc_emit(true, c.z, i0 + 2, eta, lw, lane, sh_hist);
                dgc_emit(true, c.w, i0 + 3, eta, lw, lane, sh_hist);
                list_flush(lw, lane);
            }
        }
        // unaligned buffers and the ragged last tile: guarded scalar accesses
        for (; t < t1; ++t) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t i = (int64_t)t * kTile + lane * 4 + j;
                const bool valid = i < p.d;
                float c = 0.0f;
                if (valid) {
                    c = load_grad1<GT>(p.grad, i);
                    if (EC) {
                        c = c + p.residual[i];
                        p.residual[i] = c;
                    }
                }
                dgc_emit(valid, c, (int32_t)i, eta, lw, lane, sh_hist);
            }
            list_flush(lw, lane);
        }
        const uint32_t n = list_finish(lw, lane);
        if (lane == 0) p.cnt[w] = n;
    }
    __syncthreads();
    merge_hist(sh_hist, p.hist_l, kTopkBins);
}

// ---------------------------------------------------------------------------------------------
// k_dgc_lists: how many entries the first pass took, how many stay, and the first digit of the
// second select
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_dgc_lists(DgcParams p)
{
    __shared__ uint32_t sh_hist[1024];
    __shared__ uint32_t sh_scan[kBlock];
    __shared__ uint32_t sh_out[2];
    __shared__ unsigned long long sh_tot[kWavesPerBlock];
    for (int i = threadIdx.x; i < 1024; i += kBlock) sh_hist[i] = 0;
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    // S = total of the digit-0 histogram
    unsigned long long part = 0;
    for (int i = threadIdx.x; i < kTopkBins; i += kBlock) part += p.hist_l[i];
    part = wave_sum_u64(part);
    if (lane == 0) sh_tot[wib] = part;
    __syncthreads();
    unsigned long long S = 0;
#pragma unroll
    for (int i = 0; i < kWavesPerBlock; ++i) S += sh_tot[i];
    const unsigned long long K = S < (unsigned long long)p.k ? S : (unsigned long long)p.k;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        p.st->first_pass = S;
        p.st->lists.k_eff = (uint32_t)K;
    }
    if (K == 0) return;  // block-uniform: nothing listed; the kernels after this one find k_eff = 0
    uint32_t b0, k1;
    pick_bin<kTopkBins / kBlock>(p.hist_l, K, sh_scan, sh_out, b0, k1);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        p.st->lists.prefix[0] = b0;
        p.st->lists.k_rem[0] = k1;
    }
    const ListRange r = my_lists(p.nwaves);
    for (uint32_t sw = r.first; sw < r.last; sw += kWavesPerBlock) {
        const int2* __restrict__ list = p.seg + (size_t)tile_begin(sw, p.ntiles, p.nwaves) * kTile;
        const uint32_t n = p.cnt[sw];
        for (uint32_t c = lane; c < n; c += 64) {
            const uint32_t key = mag_key(__int_as_float(list[c].y));
            if ((key >> 20) == b0) atomicAdd(&sh_hist[(key >> 10) & 1023u], 1u);
        }
    }
    __syncthreads();
    merge_hist(sh_hist, p.hist_l + kTopkBins, 1024);
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
static uint32_t sample_grid(const DgcParams& p)
{
    uint32_t g = (p.n_s + kDrawsPerThread * kBlock - 1) / (kDrawsPerThread * kBlock);
    if (g > 256) g = 256;
    return g < 1 ? 1 : g;
}

void launch_dgc_zero(const DgcParams& p, hipStream_t s)
{
    hipLaunchKernelGGL(k_dgc_zero, dim3((3 * kTopkBins + kBlock - 1) / kBlock), dim3(kBlock), 0, s, p);
}

template <int GT>
static void launch_dgc_sample_type(const DgcParams& p, hipStream_t s)
{
    if (p.residual) hipLaunchKernelGGL((k_dgc_sample<true, GT>), dim3(sample_grid(p)), dim3(kBlock), 0, s, p);
    else hipLaunchKernelGGL((k_dgc_sample<false, GT>), dim3(sample_grid(p)), dim3(kBlock), 0, s, p);
}

void launch_dgc_sample(const DgcParams& p, hipStream_t s)
{
    switch (p.gt) {
        case kGradF16: launch_dgc_sample_type<kGradF16>(p, s); break;
        case kGradBf16: launch_dgc_sample_type<kGradBf16>(p, s); break;
        default: launch_dgc_sample_type<kGradF32>(p, s); break;
    }
}

void launch_dgc_digit(const DgcParams& p, int digit, hipStream_t s)
{
    uint32_t g = (p.n_s + 8 * kBlock - 1) / (8 * kBlock);  // the keys are contiguous: more per thread
    if (g > 128) g = 128;
    if (g < 1) g = 1;
    if (digit == 1) hipLaunchKernelGGL(k_dgc_digit<1>, dim3(g), dim3(kBlock), 0, s, p);
    else hipLaunchKernelGGL(k_dgc_digit<2>, dim3(g), dim3(kBlock), 0, s, p);
}

template <int GT>
static void launch_dgc_dense_type(const DgcParams& p, hipStream_t s)
{
    if (p.residual) hipLaunchKernelGGL((k_dgc_dense<true, GT>), dim3(p.nblocks), dim3(kBlock), 0, s, p);
    else hipLaunchKernelGGL((k_dgc_dense<false, GT>), dim3(p.nblocks), dim3(kBlock), 0, s, p);
}

void launch_dgc_dense(const DgcParams& p, hipStream_t s)
{
    switch (p.gt) {
        case kGradF16: launch_dgc_dense_type<kGradF16>(p, s); break;
        case kGradBf16: launch_dgc_dense_type<kGradBf16>(p, s); break;
        default: launch_dgc_dense_type<kGradF32>(p, s); break;
    }
}

void launch_dgc_lists(const DgcParams& p, uint32_t grid, hipStream_t s)
{
    hipLaunchKernelGGL(k_dgc_lists, dim3(grid), dim3(kBlock), 0, s, p);
}

}  // namespace sidco
