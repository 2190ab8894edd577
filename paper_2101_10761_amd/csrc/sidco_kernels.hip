// SIDCo gradient sparsifier for MI355X (gfx950): device kernels and their launchers.
//
// Pipeline of one call (arXiv 2101.10761; Algorithm 1 "Sparsify", Sec. 2.3-2.4, App. B.2-B.3):
//
//   k_fit        acc = g + residual, stored back to residual; per-block fp64 partial sums of
//                |acc|, acc^2, log2|acc| (whichever the chosen law needs)       [reads 8 B, writes 4 B / element]
//                Two launch shapes: every wave walks its own contiguous range (short vectors), or
//                k_fit_flat, one float4 per thread in address order, followed by k_fit_reduce, which
//                folds the per-block sums into the 512 slots the next kernel expects (long vectors,
//                whose operands come from HBM: that shape streams 15 % faster there).
//                The gradient may be fp16 / bf16; it is widened as it is read.
//   stage m      m = 1..M, one kernel each.  Prologue: every block reduces the previous kernel's partial
//                sums in a fixed order and its first wave evaluates the closed-form threshold eta_m in
//                fp64 (the same arithmetic, hence identical bits, in every block).
//                k_compact: the stage whose source is the dense acc (m = 1; also later stages while the
//                exceedances are still a large part of the vector).  It forms n and the sums of
//                (|x| - eta_m) and its square over the exceedances for the next stage's fit, and writes
//                per-wave lists of the entries above a candidate threshold at or above eta_m - high enough
//                that the lists stay short, low enough (judged from the fit and from where the previous
//                call's next threshold fell) that the next stage can select from them alone.  On long
//                vectors a wave requests tiles before its threshold is known and stays a batch ahead.
//                k_lists: a middle stage whose source is those lists (or, if they turn out not to reach
//                down to its threshold, the dense acc again): same sums, exact exceedance lists out.
//                k_final_lists: the last stage for M >= 2; it selects, writes the contiguous
//                (index, value) output and zeroes the residual at those indices in one kernel, each
//                block reserving its output range with one atomic.
//   k_gather     M = 1 only (last stage read the dense vector): exclusive prefix over the per-block
//                survivor counts, copy of the lists into the output, residual zeroing.
//
// Design rules, from measurement on this chip: same-address atomics serialise at ~11 ns each and a
// device-scope fence in a write-heavy kernel forces an L2 write-back, so the big kernels have
// neither.  Kernel boundaries are the only global synchronisation; every wave owns a contiguous
// range of 256-element tiles and a survivor list at the same offset, so list positions need no
// atomics, and thresholds, selected set and values are deterministic.
// The *_batched kernels run the same bodies for the vectors of a batch, each block on the vector that a
// table on the device assigns to it.
//
// All floating-point accumulation is fp64 (full rate on CDNA4 vector ALUs); comparisons are fp32
// against the fp32 threshold, so the decision |x| > eta is the same one an fp32 reference takes.
#include <hip/hip_runtime.h>
#include <float.h>
#include <math.h>
#include <stdint.h>

#include "sidco_internal.h"
#include "sidco_device.h"

namespace sidco {

// Sums of `v[q]` over the block, in a fixed order; every thread returns the same values.
template <int Q>
__device__ __forceinline__ void block_sum(double (&v)[Q], double (*sh)[4])
{
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
#pragma unroll
    for (int q = 0; q < Q; ++q) v[q] = wave_sum(v[q]);
    __syncthreads();  // protects sh against a previous use
    if (lane == 0) {
#pragma unroll
        for (int q = 0; q < Q; ++q) sh[wib][q] = v[q];
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        double t = 0.0;
#pragma unroll
        for (int i = 0; i < kWavesPerBlock; ++i) t += sh[i][q];
        v[q] = t;
    }
}

// ---------------------------------------------------------------------------------------------
// closed-form thresholds (fp64, evaluated redundantly by every thread of every block)
// ---------------------------------------------------------------------------------------------

// A fitted law, reduced to what its quantile above the stage's location needs:
//   linear : t(L) = s * L + c   exponential (eqs. (6), (10)-(11)): s = mean, c = 0
//                               gamma (Corollary 1.2): s = beta, c = -beta * log Gamma(alpha)
//                               degenerate fits: s = 0, c = the limit of the closed form
//   gpd    : t(L) = (b / a) * (exp(a L) - 1)   moment-matched GPD (eqs. (7)-(9); Corollary 1.3):
//                               a = (1 - mu^2/var) / 2, b = mu (mu^2/var + 1) / 2
// with L = log(1/ratio).  The parameters are computed once in fp64; the stage's own threshold is the
// fp64 quantile, the candidate threshold (any value at or above it would do) a cheaper fp32 one.
struct Fit {
    bool gpd;
    double s, c, a, b;
};

__device__ __forceinline__ Fit fit_linear(double s, double c)
{
    Fit f;
    f.gpd = false;
    f.s = s;
    f.c = c;
    f.a = f.b = 0.0;
    return f;
}

__device__ __forceinline__ Fit fit_gpd(double mu, double var, uint32_t& status)
{
    if (!(var > 0.0)) {  // all magnitudes equal: limit of the closed form as var -> 0+
        status |= kStVarZero;
        return fit_linear(0.0, mu);
    }
    const double q = (mu * mu) / var;
    Fit f;
    f.gpd = true;
    f.a = 0.5 * (1.0 - q);
    f.b = 0.5 * mu * (q + 1.0);
    f.s = f.c = 0.0;
    if (f.a == 0.0) return fit_linear(f.b, 0.0);  // the exponential limit
    return f;
}

// Stage-1 fit of the chosen law to |acc| (Corollary 1 / eq. (6); Corollaries 1.2, 1.3).
// `var` is only used for the GPD law, `mulog` only for the gamma law.
__device__ Fit stage1_fit(int dist, double mu, double var, double mulog, uint32_t& status)
{
    if (dist == kDistExp) return fit_linear(mu, 0.0);  // eq. (6)
    if (dist == kDistGpd) return fit_gpd(mu, var, status);
    // gamma law: closed-form shape from s = log(mean) - mean(log), threshold -beta (log delta + log Gamma(alpha))
    const double s = log(mu) - mulog;
    if (!(s > 0.0)) {  // the closed form tends to -infinity here and negative thresholds clamp to 0
        status |= kStGammaS;
        return fit_linear(0.0, 0.0);
    }
    const double a = (3.0 - s + sqrt((s - 3.0) * (s - 3.0) + 24.0 * s)) / (12.0 * s);
    const double b = mu / a;
    return fit_linear(b, -b * lgamma(a));
}

// Stage m >= 2 fit of the exceedances over eta_{m-1}
// (Lemma 2 / eqs. (7)-(9) for the GPD chains, Corollary 2 / eqs. (10)-(11) for the exponential chain).
__device__ Fit pot_fit(int dist, double ybar, double yvar, uint32_t& status)
{
    if (dist == kDistExp) return fit_linear(ybar, 0.0);
    return fit_gpd(ybar, yvar, status);
}

// the stage's threshold above its location, fp64
__device__ __forceinline__ double fit_quantile(const Fit& f, double L)
{
    return f.gpd ? (f.b / f.a) * expm1(f.a * L) : f.s * L + f.c;
}

// a candidate threshold above the location, fp32 arithmetic (its accuracy does not matter)
__device__ __forceinline__ float fit_quantile_fast(const Fit& f, double L)
{
    if (!f.gpd) return (float)(f.s * L + f.c);
    return (float)(f.b / f.a) * expm1f((float)(f.a * L));
}

// log(1/delta_i) of stage i+1.  A chain of selects rather than an index: the arguments of a batched launch
// are assembled in registers, and an indexed array there would be spilled to scratch memory.
__device__ __forceinline__ double stage_L(const Params& p, int i)
{
    double v = 0.0;
#pragma unroll
    for (int j = 0; j < SIDCO_MAX_STAGES; ++j)
        if (j == i) v = p.L[j];
    return v;
}

// What the prologue of a stage's kernel hands to its body.
struct StageEta {
    float eta;      // eta_m: the stage's threshold (statistics of the next fit; selection in the last stage)
    float eta_w;    // the lists this kernel writes hold every entry above eta_w (eta_w >= eta)
    bool lists_ok;  // the producer's lists hold every entry above eta: they can stand in for the dense vector
};

// Prologue of every stage kernel: reduce the producer's per-block partial sums (fixed order) and
// evaluate eta for stage p.stage.  Returns the same values in every thread of every block.
// Block 0 records the stage in the diagnostics.
//
// Speculative candidate lists.  A stage that reads the dense vector and keeps a large fraction
// (delta_1 = 0.25) would have to write a quarter of it as 8-byte pairs, or make the next stage read the
// dense vector again.  Instead it evaluates the SAME fitted law a second time at a smaller ratio,
// log(1/ratio) = L_m + theta * L_{m+1}, and writes only the entries above that candidate threshold
// eta_w.  theta is the host's setting (0.5: halfway between this stage's target and the next one's) or,
// when the previous call on the device had the same shape, the place where that call's next
// threshold really fell, less a margin (and not so low that the lists would outgrow what the host
// planned for: theta_min).  The next stage's eta is computed from the exact statistics as
// always; if it lands at or above eta_w the candidate lists contain every entry it can select and
// replace the dense vector, else that kernel falls back to the dense vector.  Either way the result is
// the same: only the time depends on the guess.
//
// What a stage's prologue reads from memory: issued as early as possible, and BEFORE any bulk loads of
// the kernel's body - the wave's memory counter retires in order, so a wait for these few values would
// otherwise also wait for every load issued ahead of them.
struct PrologueLoads {
    double v[3];        // this thread's share of the producer's partial sums (and counts)
    float eta_prev;     // eta_{m-1}
    uint32_t status;    // status bits accumulated up to stage m-1
    bool frozen;        // an empty exceedance set has stopped the refinement
    float list_eta;     // the producer's lists hold every entry above this
    float seen;         // where the next stage's threshold fell last time (hint), NaN if unknown
    FitRecord prev_fit; // the producer's candidate fit (block 0, thread 0 only)
};

__device__ __forceinline__ PrologueLoads prologue_load(const Params& p, Blk b, bool auto_src)
{
    const int m = p.stage;  // 1-based
    const uint32_t t = threadIdx.x;
    const bool have = t < p.nblocks;  // one thread per block of the kernel that produced the partial sums
    PrologueLoads g;
    g.seen = (p.theta > 0.0f && p.use_hint) ? p.st->theta_seen[m] : __builtin_nanf("");
    g.prev_fit.gpd = 0;
    g.prev_fit.loc = 0.0f;
    g.prev_fit.s = g.prev_fit.c = g.prev_fit.a = g.prev_fit.b = 0.0;
    if (auto_src && p.prev_cand && b.id == 0 && t == 0) g.prev_fit = p.st->cand_fit[m - 1];
    g.list_eta = auto_src ? p.st->list_eta[m - 1] : 0.0f;
    g.eta_prev = 0.0f;
    g.status = 0;
    g.frozen = false;
    if (m == 1) {
        g.v[0] = have ? p.part_in[0 * kMaxBlocks + t] : 0.0;
        g.v[1] = (have && p.dist == kDistGpd) ? p.part_in[1 * kMaxBlocks + t] : 0.0;
        g.v[2] = (have && p.dist == kDistGamma) ? p.part_in[2 * kMaxBlocks + t] : 0.0;
    } else {
        g.v[0] = have ? p.part_in[0 * kMaxBlocks + t] : 0.0;
        g.v[1] = (have && p.dist != kDistExp) ? p.part_in[1 * kMaxBlocks + t] : 0.0;
        g.v[2] = have ? (double)p.blk_in[t] : 0.0;  // counts < 2^31: exact in fp64
        g.eta_prev = p.st->diag.eta[m - 2];
        g.status = p.st->status_after[m - 1];
        g.frozen = p.st->frozen_after[m - 1] != 0;
    }
    return g;
}

// Reduces the partial sums (fixed order) and evaluates eta for stage p.stage.  Returns the same values
// in every thread of every block.  Block 0 records the stage in the diagnostics.
__device__ StageEta prologue_finish(const Params& p, Blk b, bool auto_src, PrologueLoads& g, double (*sh)[4])
{
    const int m = p.stage;  // 1-based
    const uint32_t t = threadIdx.x;
    const double L = stage_L(p, m - 1);
    // candidate threshold of this kernel's lists: log-ratio Lw > L, or none
    double Lw = 0.0;
    if (p.theta > 0.0f) {
        float theta = p.theta;
        if (g.seen == g.seen) theta = fminf(fmaxf(g.seen - kHintMargin, p.theta_min), kHintMax);
        Lw = L + (double)theta * stage_L(p, m);
    }
    const FitRecord prev_fit = g.prev_fit;
    Fit fit = fit_linear(0.0, 0.0);
    float loc = 0.0f;
    uint32_t status = g.status;
    double stats[3] = {0.0, 0.0, 0.0};
    StageEta r;
    bool frozen = g.frozen;
    unsigned long long n;
    block_sum<3>(g.v, sh);
    r.eta = r.eta_w = 0.0f;
    r.lists_ok = false;
    // One wave per block evaluates the closed form - a few hundred dependent fp64 instructions, more for
    // the gamma law - and the others wait: with every wave at it, four per SIMD take turns on the same
    // arithmetic and the prologue lasts that much longer (measured).
    if (t < 64) {
        if (m == 1) {
            n = (unsigned long long)p.d;
            const double d = (double)p.d;
            const double mu = g.v[0] / d;
            double var = 0.0, mulog = 0.0;
            bool finite = isfinite(mu);
            if (p.dist == kDistGpd) {
                var = g.v[1] / d - mu * mu;
                finite = finite && isfinite(var);
            } else if (p.dist == kDistGamma) {
                mulog = (g.v[2] / d) * 0.6931471805599453094;  // log2 -> natural log
                finite = finite && isfinite(mulog);
            }
            stats[0] = mu;
            stats[1] = var;
            stats[2] = mulog;
            if (!finite) {
                status |= kStNonfinite;
                r.eta = r.eta_w = __builtin_nanf("");
            } else {
                fit = stage1_fit(p.dist, mu, var, mulog, status);
                double tq = fit_quantile(fit, L);
                if (tq < 0.0) {  // only the gamma form can be negative: delta_1 * Gamma(alpha) > 1
                    status |= kStGammaClamp;
                    tq = 0.0;
                }
                r.eta = r.eta_w = (float)tq;
                if (Lw > L) {
                    const float c = fit_quantile_fast(fit, Lw);
                    if (c > r.eta) r.eta_w = c;
                }
            }
        } else {
            const float eta_prev = g.eta_prev;
            n = (unsigned long long)g.v[2];
            r.eta = r.eta_w = eta_prev;
            if (!frozen) {
                if (n == 0) {  // nothing exceeds eta_prev: keep it for all later stages
                    frozen = true;
                    status |= kStStopped;
                } else {
                    const double ybar = g.v[0] / (double)n;
                    const double yvar = p.dist == kDistExp ? 0.0 : g.v[1] / (double)n - ybar * ybar;
                    stats[0] = ybar;
                    stats[1] = yvar;
                    fit = pot_fit(p.dist, ybar, yvar, status);
                    loc = eta_prev;
                    r.eta = r.eta_w = (float)((double)eta_prev + fit_quantile(fit, L));
                    if (Lw > L) {
                        const float c = eta_prev + fit_quantile_fast(fit, Lw);
                        if (c > r.eta) r.eta_w = c;
                    }
                }
            }
        }
        r.lists_ok = auto_src && (r.eta >= g.list_eta);  // false for a NaN threshold, which selects nothing anyway
        if (auto_src && !r.lists_ok) status |= kStFallback;
        if (b.id == 0 && t == 0) {
            p.st->diag.eta[m - 1] = r.eta;
            p.st->diag.n[m - 1] = (int64_t)n;
            p.st->diag.stats[m - 1][0] = stats[0];
            p.st->diag.stats[m - 1][1] = stats[1];
            p.st->diag.stats[m - 1][2] = stats[2];
            p.st->status_after[m] = status;
            p.st->frozen_after[m] = frozen ? 1u : 0u;
            p.st->list_eta[m] = r.eta_w;
            if (p.theta > 0.0f) {
                FitRecord rec;
                rec.gpd = fit.gpd ? 1 : 0;
                rec.loc = loc;
                rec.s = fit.s;
                rec.c = fit.c;
                rec.a = fit.a;
                rec.b = fit.b;
                p.st->cand_fit[m] = rec;
            }
            if (auto_src && p.prev_cand) {
                // invert the producer's quantile function at this stage's threshold:
                // eta = loc + Q(L_{m-1} + theta * L_m)  ->  theta
                const double tq = (double)r.eta - (double)prev_fit.loc;
                const double Lq = prev_fit.gpd ? log1p(tq * prev_fit.a / prev_fit.b) / prev_fit.a : (tq - prev_fit.c) / prev_fit.s;
                const float seen = (float)((Lq - stage_L(p, m - 2)) / L);
                p.st->theta_seen[m - 1] = (frozen || !(fabsf(seen) < 1.0e6f)) ? __builtin_nanf("") : seen;
            }
        }
    }
    __syncthreads();  // every thread has left block_sum: sh is free
    if (t == 0) {
        float* out = reinterpret_cast<float*>(&sh[0][0]);
        out[0] = r.eta;
        out[1] = r.eta_w;
        out[2] = r.lists_ok ? 1.0f : 0.0f;
    }
    __syncthreads();
    {
        const float* in = reinterpret_cast<const float*>(&sh[0][0]);
        r.eta = in[0];
        r.eta_w = in[1];
        r.lists_ok = in[2] != 0.0f;
    }
    return r;
}

// both halves back to back, for kernels whose body loads little before the threshold is known
__device__ __forceinline__ StageEta stage_prologue(const Params& p, Blk b, bool auto_src, double (*sh)[4])
{
    PrologueLoads g = prologue_load(p, b, auto_src);
    return prologue_finish(p, b, auto_src, g, sh);
}

// ---------------------------------------------------------------------------------------------
// k_fit: error-compensation add (App. B.2) fused with the sums of the stage-1 fit
// ---------------------------------------------------------------------------------------------
template <int DIST>
__device__ __forceinline__ void fit_accum(float x, double& s1, double& s2, double& sl, int& se)
{
    const float a = __builtin_fabsf(x);
    const double da = (double)a;
    s1 += da;
    if constexpr (DIST == kDistGpd) s2 = __builtin_fma(da, da, s2);  // a*a is exact in fp64
    if constexpr (DIST == kDistGamma) {
        // log2 max(|x|, 2^-126) = exponent + log2(mantissa in [0.5,1)): the exponents are summed
        // exactly as integers, the hardware log2 only sees [0.5,1) where its error is <= 1 ulp of a
        // value in [-1,0).  NaN compares false and is replaced by 2^-126 here; s1 carries the NaN.
        const float c = __builtin_fmaxf(a, FLT_MIN);
        se += __builtin_amdgcn_frexp_expf(c);
        sl += (double)__builtin_amdgcn_logf(__builtin_amdgcn_frexp_mantf(c));
    }
}

// U complete tiles starting at tile t, 4-element accesses.  EC: acc = g + residual, stored back.  A
// 16-bit gradient is widened to fp32 first and acc is always stored (into the residual, or, without
// one, into the workspace's own buffer), because every later kernel reads an fp32 vector.
template <int DIST, bool EC, int GT, int U>
__device__ __forceinline__ void fit_tiles(const void* __restrict__ g, f4* __restrict__ a4, uint32_t t, int lane,
                                          double& s1, double& s2, double& sl, int& se)
{
    constexpr bool WRITE = EC || GT != kGradF32;
    f4 a[U], b[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const size_t i = (size_t)(t + u) * 64 + lane;
        // the gradient is read once per call when acc is re-materialised elsewhere
        a[u] = load_grad4<GT, WRITE>(g, i);
        if (EC) b[u] = a4[i];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        f4 c = a[u];
        if (EC) c = a[u] + b[u];
        if (WRITE) a4[(size_t)(t + u) * 64 + lane] = c;
        fit_accum<DIST>(c.x, s1, s2, sl, se);
        fit_accum<DIST>(c.y, s1, s2, sl, se);
        fit_accum<DIST>(c.z, s1, s2, sl, se);
        fit_accum<DIST>(c.w, s1, s2, sl, se);
    }
}

// start of a call: per-call device state, by one thread
__device__ __forceinline__ void fit_reset_state(const Params& p)
{
    p.st->status_after[0] = 0;
    p.st->frozen_after[0] = 0;
    p.st->diag.stages = p.M;
    // Adapt_Stages bookkeeping: the pairs the previous call reported join the running count
    const unsigned long long prev_sel = p.st->selected_ctr;
    const unsigned long long prev_cap = (unsigned long long)p.st->prev_cap;
    p.st->khat_sum = p.acc_reset ? 0ull : p.st->khat_sum + (prev_sel < prev_cap ? prev_sel : prev_cap);
    // a window of a controller's count is only its own if every call since its start was that controller's
    if (p.acc_reset) p.st->disturbed = 0;
    else if (p.st->owner != p.owner) p.st->disturbed = 1;
    p.st->owner = p.owner;
    p.st->prev_cap = (long long)p.out_cap;
    p.st->selected_ctr = 0;
    p.st->overflow = 0;
    if (p.out_count) *p.out_count = 0;
    if (p.status_out) *p.status_out = 0;
}

// one element through the guarded scalar path
template <int DIST, bool EC, int GT>
__device__ __forceinline__ float fit_one(const Params& p, int64_t i, double& s1, double& s2, double& sl, int& se)
{
    float c = load_grad1<GT>(p.grad, i);
    if (EC) c = c + p.acc_w[i];
    if (EC || GT != kGradF32) p.acc_w[i] = c;
    fit_accum<DIST>(c, s1, s2, sl, se);
    return c;
}

// One wave's tiles.
template <int DIST, bool EC, int GT>
__device__ __forceinline__ void fit_wave(const Params& p, uint32_t w, int lane, double& s1, double& s2, double& sl,
                                         int& se)
{
    const uint32_t t0 = tile_begin(w, p.ntiles, p.nwaves), t1 = tile_begin(w + 1, p.ntiles, p.nwaves);
    const uint32_t tf = t1 < p.nfull ? t1 : p.nfull;  // tiles [t0,tf) are complete
    uint32_t t = t0;
    if (p.vec_ok) {
        f4* a4 = reinterpret_cast<f4*>(p.acc_w);
        // no second register buffer: with 16 waves per CU in flight it gained nothing (measured)
#pragma unroll 1
        for (; t + 4 <= tf; t += 4) fit_tiles<DIST, EC, GT, 4>(p.grad, a4, t, lane, s1, s2, sl, se);
#pragma unroll 1
        for (; t < tf; ++t) fit_tiles<DIST, EC, GT, 1>(p.grad, a4, t, lane, s1, s2, sl, se);
    }
    // unaligned buffers and the ragged last tile: guarded scalar accesses
    for (; t < t1; ++t) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t i = (int64_t)t * kTile + lane * 4 + j;
            if (i < p.d) fit_one<DIST, EC, GT>(p, i, s1, s2, sl, se);
        }
    }
}

template <int DIST, bool EC, int GT>
__device__ __forceinline__ void fit_body(const Params& p, Blk b)
{
    __shared__ double sh[kWavesPerBlock][4];
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    const uint32_t w = b.id * kWavesPerBlock + wib;
    double s1 = 0.0, s2 = 0.0, sl = 0.0;
    int se = 0;
    if (w < p.nwaves) fit_wave<DIST, EC, GT>(p, w, lane, s1, s2, sl, se);
    double v[3] = {s1, s2, sl + (double)se};
    v[0] = wave_sum(v[0]);
    v[1] = wave_sum(v[1]);
    v[2] = wave_sum(v[2]);
    if (lane == 0) {
        sh[wib][0] = v[0];
        sh[wib][1] = v[1];
        sh[wib][2] = v[2];
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        double tot = 0.0;
#pragma unroll
        for (int i = 0; i < kWavesPerBlock; ++i) tot += sh[i][threadIdx.x];
        p.part_out[threadIdx.x * kMaxBlocks + b.id] = tot;
    }
    if (b.id == 0 && threadIdx.x == 0) fit_reset_state(p);
}

// ---------------------------------------------------------------------------------------------
// k_fit_flat + k_fit_reduce: the same pass for large vectors.  One float4 per thread and a grid that
// covers the vector in address order: the blocks in flight at any time touch one narrow window of each
// buffer, which DRAM serves better than the 3 x 4096 separate streams of the per-wave ranges when
// the operands come from HBM (measured with a gradient and a residual that no cache holds: 52.9 us
// against 62.5 us at d = 25.6 M, 129 us against 156 us at 66 M, i.e. what a plain in-place add reaches;
// with a residual that is still in the memory-side cache from the previous call the per-wave shape is
// the faster one up to 66 M, but no training loop leaves it there).
// The price is one partial sum per 256-thread block - far too many for every block of the next
// kernel to add up - so a second, small kernel folds them into the usual 512 slots, in a fixed order.
// ---------------------------------------------------------------------------------------------
template <int DIST, bool EC, int GT>
__global__ __launch_bounds__(kFlatBlock) void k_fit_flat(Params p, double* __restrict__ flat_part, uint32_t nflat)
{
    __shared__ double sh[kFlatBlock / 64][4];
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    const size_t nvec = (size_t)(p.d / 4);
    const size_t i = (size_t)blockIdx.x * kFlatBlock + threadIdx.x;
    double s1 = 0.0, s2 = 0.0, sl = 0.0;
    int se = 0;
    if (i < nvec) {
        constexpr bool WRITE = EC || GT != kGradF32;
        f4* a4 = reinterpret_cast<f4*>(p.acc_w);
        f4 c = load_grad4<GT, WRITE>(p.grad, i);
        if (EC) c = c + a4[i];
        if (WRITE) a4[i] = c;
        fit_accum<DIST>(c.x, s1, s2, sl, se);
        fit_accum<DIST>(c.y, s1, s2, sl, se);
        fit_accum<DIST>(c.z, s1, s2, sl, se);
        fit_accum<DIST>(c.w, s1, s2, sl, se);
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {  // the last d % 4 elements
        for (int64_t j = (int64_t)nvec * 4; j < p.d; ++j) fit_one<DIST, EC, GT>(p, j, s1, s2, sl, se);
    }
    double v[3] = {s1, s2, sl + (double)se};
    v[0] = wave_sum(v[0]);
    v[1] = wave_sum(v[1]);
    v[2] = wave_sum(v[2]);
    if (lane == 0) {
        sh[wib][0] = v[0];
        sh[wib][1] = v[1];
        sh[wib][2] = v[2];
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        double tot = 0.0;
#pragma unroll
        for (int w = 0; w < kFlatBlock / 64; ++w) tot += sh[w][threadIdx.x];
        flat_part[(size_t)threadIdx.x * nflat + blockIdx.x] = tot;
    }
}

// Slot s of the 512 receives the partial sums of the flat blocks [s * per, (s + 1) * per): one wave
// per slot, every lane adds its share in order, then the lanes are combined in a fixed order.
__global__ __launch_bounds__(kBlock) void k_fit_reduce(Params p, const double* __restrict__ flat_part, uint32_t nflat,
                                                       uint32_t per)
{
    const int lane = threadIdx.x & 63;
    const uint32_t slot = blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    const uint32_t b0 = slot * per, b1 = b0 + per < nflat ? b0 + per : nflat;
    double v[3] = {0.0, 0.0, 0.0};
    for (uint32_t b = b0 + lane; b < b1; b += 64) {
        v[0] += flat_part[b];
        if (p.dist == kDistGpd) v[1] += flat_part[(size_t)nflat + b];
        if (p.dist == kDistGamma) v[2] += flat_part[2 * (size_t)nflat + b];
    }
    v[0] = wave_sum(v[0]);
    v[1] = wave_sum(v[1]);
    v[2] = wave_sum(v[2]);
    if (lane == 0 && slot < (uint32_t)kMaxBlocks) {
        p.part_out[0 * kMaxBlocks + slot] = v[0];
        p.part_out[1 * kMaxBlocks + slot] = v[1];
        p.part_out[2 * kMaxBlocks + slot] = v[2];
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) fit_reset_state(p);
}

// ---------------------------------------------------------------------------------------------
// k_compact: statistics of the exceedances of eta_m for the next fit, and per-wave survivor lists
// ---------------------------------------------------------------------------------------------

// One component of a tile (64 candidates, one per lane).  Entries above eta_w go to the wave's list;
// entries above eta_s are counted (`ns`, wave-uniform) and enter the sums of y = |x| - eta_s.
// Comparisons are strict and fp32; NaN on either side is false.
template <bool STATS, bool WRITE>
__device__ __forceinline__ void emit(bool valid, float x, int32_t idx, float eta_s, float eta_w, ListWriter& lw,
                                     int lane, uint32_t& ns, double& sy, double& syy)
{
    const float a = __builtin_fabsf(x);
    if (WRITE) list_push(lw, valid && (a > eta_w), idx, x, lane);
    if (STATS) {
        // y = |x| - eta_s over the selected entries, exactly, and 0 elsewhere (eta_s - eta_s)
        const bool sel = valid && (a > eta_s);
        ns += (uint32_t)__popcll(__ballot(sel));
        const double y = (double)(sel ? a : eta_s) - (double)eta_s;
        sy += y;
        syy = __builtin_fma(y, y, syy);
    }
}

// U complete tiles of the dense vector, already loaded
template <bool STATS, bool WRITE, int U>
__device__ __forceinline__ void compact_loaded(const f4* a, uint32_t t, int lane, float eta_s, float eta_w,
                                               ListWriter& lw, uint32_t& ns, double& sy, double& syy)
{
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int32_t i0 = (int32_t)((t + u) * kTile + lane * 4);
        emit<STATS, WRITE>(true, a[u].x, i0 + 0, eta_s, eta_w, lw, lane, ns, sy, syy);
        emit<STATS, WRITE>(true, a[u].y, i0 + 1, eta_s, eta_w, lw, lane, ns, sy, syy);
        emit<STATS, WRITE>(true, a[u].z, i0 + 2, eta_s, eta_w, lw, lane, ns, sy, syy);
        emit<STATS, WRITE>(true, a[u].w, i0 + 3, eta_s, eta_w, lw, lane, ns, sy, syy);
        if (WRITE) list_flush(lw, lane);
    }
}

// Plain (L2-allocating) loads: the next pass over the dense vector, if any, starts with what this one read last.
template <int U>
__device__ __forceinline__ void load_tiles(f4 (&a)[U], const f4* __restrict__ x4, uint32_t t, int lane)
{
#pragma unroll
    for (int u = 0; u < U; ++u) a[u] = x4[(size_t)(t + u) * 64 + lane];
}

// Tiles [t0, t1) of the dense vector (complete below tf).  p.reverse walks them from the last to the
// first: the kernel before this one left the end of what it touched last in L2 (32 MB over the chip),
// and the host alternates the direction from pass to pass so that each pass starts where the one
// before it stopped (measured: 15.5 us instead of 18.3 us for 102 MB right after k_fit).
// Batches of U tiles.  The caller has loaded the first PRE batches already, into a[0 .. PRE*U), while it
// still waited for its threshold: a stage kernel's prologue is a cold round trip for the partial sums
// plus a few hundred dependent fp64 instructions, 4-5 us in which the memory pipes would otherwise run
// dry after the first batch.  PRE is a template parameter and the caller's loads are unconditional:
// loads under a run-time condition come with copies that the compiler waits for on the spot.
// After them the wave stays PRE batches ahead: the request for batch k + PRE goes out
// before batch k is processed, into the last register batch, and the batches move up by register copies
// once batch k is done - one copy of the loop body (two inlined copies cost more in code size and
// registers than they gained).  Measured against load-then-process steps with two prefetched batches:
// 1-2 us less per dense stage at 14.7 M to 66 M elements, nothing at 138 M, where the stage is bound by
// what the memory system still has to write back for the pass before it.
__device__ __forceinline__ uint32_t dense_batch_tile(const Params& p, uint32_t t0, uint32_t tf, uint32_t U, uint32_t k)
{
    return p.reverse ? tf - (k + 1) * U : t0 + k * U;
}

// register batches a wave holds: the PRE prefetched ones and the one in flight behind them
constexpr int dense_batches(int PRE) { return PRE > 0 ? PRE + 1 : 1; }

template <bool STATS, bool WRITE, int U, int PRE>
__device__ __forceinline__ void compact_dense(const Params& p, f4 (&a)[dense_batches(PRE) * U], uint32_t t0, uint32_t t1,
                                              uint32_t tf, int lane, float eta_s, float eta_w, ListWriter& lw,
                                              uint32_t& ns, double& sy, double& syy)
{
    const f4* __restrict__ x4 = reinterpret_cast<const f4*>(p.acc);
    uint32_t ts = t0;  // tiles [ts, t1) take guarded scalar loads: unaligned buffers, the ragged last tile
    if (p.vec_ok) {
        const uint32_t nb = (tf - t0) / U, rem = (tf - t0) - nb * U;
#pragma unroll 1  // unrolled, the batches' loads pile up in registers and halve the occupancy
        for (uint32_t k = 0; k < nb; ++k) {
            const uint32_t t = dense_batch_tile(p, t0, tf, U, k);
            if constexpr (PRE > 0) {
                // Batch k + PRE is requested before batch k is processed, so the wave keeps a batch in flight
                // while it computes (per-wave time max(latency, arithmetic) instead of their sum).  The load is
                // unconditional - the last batches are requested again, from L2, instead of a load under a
                // condition - and lands in the last register batch; the batches move up once batch k is done.
                const uint32_t kn = k + PRE < nb ? k + PRE : nb - 1;
                const uint32_t tn = dense_batch_tile(p, t0, tf, U, kn);
#pragma unroll
                for (int u = 0; u < U; ++u) a[PRE * U + u] = x4[(size_t)(tn + u) * 64 + lane];
                compact_loaded<STATS, WRITE, U>(a, t, lane, eta_s, eta_w, lw, ns, sy, syy);
#pragma unroll
                for (int u = 0; u < PRE * U; ++u) a[u] = a[u + U];
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) a[u] = x4[(size_t)(t + u) * 64 + lane];
                compact_loaded<STATS, WRITE, U>(a, t, lane, eta_s, eta_w, lw, ns, sy, syy);
            }
        }
        const uint32_t tr = p.reverse ? t0 : t0 + nb * U;
        for (uint32_t t = tr; t < tr + rem; ++t) {
            f4 one[1];
            load_tiles<1>(one, x4, t, lane);
            compact_loaded<STATS, WRITE, 1>(one, t, lane, eta_s, eta_w, lw, ns, sy, syy);
        }
        ts = tf;
    }
    for (uint32_t t = ts; t < t1; ++t) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t i = (int64_t)t * kTile + lane * 4 + j;
            const bool valid = i < p.d;
            const float v = valid ? p.acc[i] : 0.0f;
            emit<STATS, WRITE>(valid, v, (int32_t)i, eta_s, eta_w, lw, lane, ns, sy, syy);
        }
        if (WRITE) list_flush(lw, lane);
    }
}

// Two list entries per lane and load (16 B): slot i of a wave's list holds entries 2i and 2i+1.
// `cap2` is the number of slots the wave's segment has room for; slots past the list's end hold
// stale data and are masked by `n_in`.
template <int U>
__device__ __forceinline__ void load_slots(int4 (&q)[U], const int4* __restrict__ src4, uint32_t c, uint32_t cap2,
                                           int lane)
{
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t i = c + u * 64 + lane;
        q[u] = i < cap2 ? src4[i] : make_int4(0, 0, 0, 0);
    }
}

template <bool STATS, int U>
__device__ __forceinline__ void compact_slots(const int4 (&q)[U], uint32_t c, uint32_t n_in, int lane, float eta,
                                              ListWriter& lw, uint32_t& ns, double& sy, double& syy)
{
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t e = 2 * (c + u * 64 + lane);
        emit<STATS, true>(e < n_in, __int_as_float(q[u].y), q[u].x, eta, eta, lw, lane, ns, sy, syy);
        emit<STATS, true>(e + 1 < n_in, __int_as_float(q[u].w), q[u].z, eta, eta, lw, lane, ns, sy, syy);
        if (u & 1) list_flush(lw, lane);  // every 4 components = at most kTile entries
    }
    static_assert(U % 2 == 0, "flush check after every second slot group");
}

// End of a stage kernel: per block, the number of exceedances of eta_m (the n of the next fit) - or,
// without statistics (dense last stage), the number of list entries (k_gather's prefix) - and the
// block's partial sums of y and y^2, each in its fixed slot.
template <bool STATS>
__device__ __forceinline__ void stage_epilogue(const Params& p, Blk b, int lane, int wib, uint32_t count, double sy,
                                               double syy, double (*sh)[4], uint32_t* sh_cnt)
{
    if (lane == 0) sh_cnt[wib] = count;
    if (STATS) {
        sy = wave_sum(sy);
        syy = wave_sum(syy);
        __syncthreads();  // the prologue's reads of sh are done
        if (lane == 0) {
            sh[wib][0] = sy;
            sh[wib][1] = syy;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t tot = 0;
#pragma unroll
        for (int i = 0; i < kWavesPerBlock; ++i) tot += sh_cnt[i];
        p.blk_out[b.id] = tot;
    }
    if (STATS && threadIdx.x < 2) {
        double tot = 0.0;
#pragma unroll
        for (int i = 0; i < kWavesPerBlock; ++i) tot += sh[i][threadIdx.x];
        p.part_out[threadIdx.x * kMaxBlocks + b.id] = tot;
    }
}

// k_compact: a stage that reads the dense vector.  STATS: form the sums for the next stage's fit.
// WRITE: append the entries above eta_w to this stage's lists (eta_w = eta_m, or a candidate threshold
// above it); a stage whose candidates would still be a large fraction only counts and sums.
// PRE: batches of U tiles that every wave loads before the prologue; the host picks PRE > 0 only when the
// vector is aligned for 4-element accesses and every wave owns at least PRE * U complete tiles.
template <bool STATS, bool WRITE, int PRE>
__device__ __forceinline__ void compact_body(const Params& p, Blk b)
{
    __shared__ double sh[kWavesPerBlock][4];
    __shared__ uint32_t sh_cnt[kWavesPerBlock];
    __shared__ int2 ring[WRITE ? kWavesPerBlock : 1][kRingSize];
    constexpr int U = 4;
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    const uint32_t w = b.id * kWavesPerBlock + wib;
    const bool active = w < p.nwaves;
    const uint32_t t0 = active ? tile_begin(w, p.ntiles, p.nwaves) : 0;
    const uint32_t t1 = active ? tile_begin(w + 1, p.ntiles, p.nwaves) : 0;
    const uint32_t tf = t1 < p.nfull ? t1 : p.nfull;  // tiles [t0,tf) are complete

    // Neither the prologue's own loads nor the first loads of the body depend on the threshold.  The
    // prologue's go first (the memory counter retires in order: behind the tiles they would wait for
    // them), then the first batches of tiles, so that the stream runs while the partial sums are reduced
    // and the closed form is evaluated.
    PrologueLoads g = prologue_load(p, b, false);
    f4 a0[dense_batches(PRE) * U];
    if constexpr (PRE > 0) {
        const f4* __restrict__ x4 = reinterpret_cast<const f4*>(p.acc);
#pragma unroll
        for (int k = 0; k < PRE; ++k) {
            const uint32_t t = dense_batch_tile(p, t0, tf, U, k);
#pragma unroll
            for (int u = 0; u < U; ++u) a0[k * U + u] = x4[(size_t)(t + u) * 64 + lane];
        }
    }

    const StageEta se = prologue_finish(p, b, false, g, sh);

    uint32_t run = 0, ns = 0;
    double sy = 0.0, syy = 0.0;
    if (active) {
        ListWriter lw;
        lw.list = p.seg_out + (size_t)t0 * kTile;  // room for every element of the wave's tiles
        lw.ring = ring[WRITE ? wib : 0];
        lw.run = lw.fill = 0;
        compact_dense<STATS, WRITE, U, PRE>(p, a0, t0, t1, tf, lane, se.eta, se.eta_w, lw, ns, sy, syy);
        if (WRITE) run = list_finish(lw, lane);
        if (lane == 0) p.cnt_out[w] = run;
    }
    stage_epilogue<STATS>(p, b, lane, wib, STATS ? ns : run, sy, syy, sh, sh_cnt);
}

// ---------------------------------------------------------------------------------------------
// k_lists: a stage m < M whose source is the producer's survivor lists, or, if those are candidate
// lists that do not reach down to this stage's threshold (see stage_prologue), the dense vector.
// The lists are short (a few per cent of the vector at most) and the kernel is bound by latency and
// by the launch itself, so the host sizes the grid to the expected list volume: block b takes the
// source lists [b * per_block, (b + 1) * per_block), wave i of it every 8th of those, and writes one
// output list per source list, in the same per-wave segments.  The first 128 entries of a wave's
// first kListGroup lists are loaded before the prologue.
// ---------------------------------------------------------------------------------------------
constexpr int kListGroup = 4;

__device__ __forceinline__ void lists_body(const Params& p, Blk b)
{
    __shared__ double sh[kWavesPerBlock][4];
    __shared__ uint32_t sh_cnt[kWavesPerBlock];
    __shared__ int2 ring[kWavesPerBlock][kRingSize];
    constexpr int K = kListGroup, U = 4;
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    const uint32_t per_block = (p.nwaves + b.n - 1) / b.n;
    const uint32_t first = b.id * per_block + wib;
    const uint32_t last = min(p.nwaves, (b.id + 1) * per_block);

    uint32_t n0[K];
    int4 q0[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t sw = first + k * kWavesPerBlock;
        const bool valid = sw < last;
        const uint32_t t0 = valid ? tile_begin(sw, p.ntiles, p.nwaves) : 0;
        const uint32_t t1 = valid ? tile_begin(sw + 1, p.ntiles, p.nwaves) : 0;
        n0[k] = valid ? p.cnt_in[sw] : 0u;
        q0[k] = (uint32_t)lane < (t1 - t0) * (kTile / 2)
                    ? reinterpret_cast<const int4*>(p.seg_in + (size_t)t0 * kTile)[lane]
                    : make_int4(0, 0, 0, 0);
    }

    const StageEta se = stage_prologue(p, b, true, sh);
    const float eta = se.eta;

    uint32_t ns = 0;
    double sy = 0.0, syy = 0.0;
    for (uint32_t g = first, grp = 0; g < last; g += K * kWavesPerBlock, ++grp) {
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const uint32_t sw = g + k * kWavesPerBlock;
            if (sw >= last) break;  // wave-uniform
            const uint32_t t0 = tile_begin(sw, p.ntiles, p.nwaves), t1 = tile_begin(sw + 1, p.ntiles, p.nwaves);
            ListWriter lw;
            lw.list = p.seg_out + (size_t)t0 * kTile;
            lw.ring = ring[wib];
            lw.run = lw.fill = 0;
            if (!se.lists_ok) {
                // this stage's exceedances straight from the dense vector
                f4 unused[U];
                const uint32_t tf = t1 < p.nfull ? t1 : p.nfull;
                compact_dense<true, true, U, 0>(p, unused, t0, t1, tf, lane, eta, eta, lw, ns, sy, syy);
            } else {
                const int4* __restrict__ src4 = reinterpret_cast<const int4*>(p.seg_in + (size_t)t0 * kTile);
                const uint32_t cap2 = (t1 - t0) * (kTile / 2);
                const uint32_t n_in = __builtin_amdgcn_readfirstlane(grp == 0 ? n0[k] : p.cnt_in[sw]);
                const uint32_t nslot = (n_in + 1) / 2;
                // slots [0, 64): prefetched for the first group
                {
                    int4 q = q0[k];
                    if (grp != 0) q = (uint32_t)lane < cap2 ? src4[lane] : make_int4(0, 0, 0, 0);
                    const uint32_t e = 2 * lane;
                    emit<true, true>(e < n_in, __int_as_float(q.y), q.x, eta, eta, lw, lane, ns, sy, syy);
                    emit<true, true>(e + 1 < n_in, __int_as_float(q.w), q.z, eta, eta, lw, lane, ns, sy, syy);
                }
                // the rest, 256 slots per step
                for (uint32_t c = 64; c < nslot; c += 64 * U) {
                    int4 q[U];
                    load_slots<U>(q, src4, c, cap2, lane);
                    compact_slots<true, U>(q, c, n_in, lane, eta, lw, ns, sy, syy);
                }
            }
            const uint32_t n_out = list_finish(lw, lane);
            if (lane == 0) p.cnt_out[sw] = n_out;
        }
    }
    stage_epilogue<true>(p, b, lane, wib, ns, sy, syy, sh, sh_cnt);
}

// ---------------------------------------------------------------------------------------------
// k_final_lists: last stage when its source is a set of survivor lists (M >= 2).
// Threshold eta_M, selection, contiguous output and residual update in one kernel.  If the lists are
// candidate lists that turn out not to reach down to eta_M (see stage_prologue), the same two passes
// run over the dense vector instead: slower, same result.  The lists are
// short by now and the kernel is bound by memory latency, not bandwidth: every wave takes up to
// kFinalGroup lists at a time and issues all their loads together, before the prologue, so that the
// whole kernel is a few dependent round trips.  Each block reserves its output range with ONE atomic
// add on the pair counter (same-address atomics cost ~11 ns each on this chip: a hundred of them are
// cheaper than another kernel boundary).  The set of pairs is deterministic; the order of the
// blocks' ranges in the output is not.
// ---------------------------------------------------------------------------------------------
constexpr int kFinalGroup = 4;

struct FinalList {
    const int4* src4;  // the list, two entries per slot
    uint32_t cap2;     // slots the segment has room for
    uint32_t n;        // entries
};

__device__ __forceinline__ FinalList final_list(const Params& p, uint32_t sw, bool valid)
{
    FinalList l;
    const uint32_t t0 = valid ? tile_begin(sw, p.ntiles, p.nwaves) : 0;
    const uint32_t t1 = valid ? tile_begin(sw + 1, p.ntiles, p.nwaves) : 0;
    l.src4 = reinterpret_cast<const int4*>(p.seg_in + (size_t)t0 * kTile);
    l.cap2 = (t1 - t0) * (kTile / 2);
    l.n = valid ? p.cnt_in[sw] : 0u;
    return l;
}

// exceedances among the two entries of this lane's slot `slot` (wave-wide count)
__device__ __forceinline__ uint32_t final_count(int4 q, uint32_t slot, uint32_t n, float eta)
{
    const uint32_t e = 2 * slot;
    const bool s0 = e < n && __builtin_fabsf(__int_as_float(q.y)) > eta;
    const bool s1 = e + 1 < n && __builtin_fabsf(__int_as_float(q.w)) > eta;
    return (uint32_t)__popcll(__ballot(s0)) + (uint32_t)__popcll(__ballot(s1));
}

// writes the exceedances of this lane's slot at the wave's running position `pos`
__device__ __forceinline__ void final_emit(const Params& p, int4 q, uint32_t slot, uint32_t n, float eta,
                                           unsigned long long cap, unsigned long long& pos)
{
    const uint32_t e = 2 * slot;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int32_t idx = h ? q.z : q.x;
        const float x = __int_as_float(h ? q.w : q.y);
        const bool sel = e + h < n && __builtin_fabsf(x) > eta;
        const unsigned long long mask = __ballot(sel);
        const unsigned long long at = pos + lane_prefix(mask);
        if (sel && at < cap) {  // pairs beyond the capacity stay in the residual
            p.out_idx[at] = idx;
            p.out_val[at] = x;
            if (p.residual) p.residual[idx] = 0.0f;
        }
        pos += (unsigned long long)__popcll(mask);
    }
}

// Dense fallback of the two passes: the elements of source wave sw's tiles, 64 consecutive ones per step.
__device__ __forceinline__ uint32_t final_count_dense(const Params& p, uint32_t sw, int lane, float eta)
{
    const int64_t b0 = (int64_t)tile_begin(sw, p.ntiles, p.nwaves) * kTile;
    const int64_t b1 = (int64_t)tile_begin(sw + 1, p.ntiles, p.nwaves) * kTile;
    uint32_t c = 0;
    for (int64_t b = b0; b < b1 && b < p.d; b += 64) {
        const int64_t i = b + lane;
        const bool sel = i < p.d && __builtin_fabsf(p.acc[i < p.d ? i : 0]) > eta;
        c += (uint32_t)__popcll(__ballot(sel));
    }
    return c;
}

__device__ __forceinline__ void final_emit_dense(const Params& p, uint32_t sw, int lane, float eta,
                                                 unsigned long long cap, unsigned long long& pos)
{
    const int64_t b0 = (int64_t)tile_begin(sw, p.ntiles, p.nwaves) * kTile;
    const int64_t b1 = (int64_t)tile_begin(sw + 1, p.ntiles, p.nwaves) * kTile;
    for (int64_t b = b0; b < b1 && b < p.d; b += 64) {
        const int64_t i = b + lane;
        const float x = i < p.d ? p.acc[i] : 0.0f;
        const bool sel = i < p.d && __builtin_fabsf(x) > eta;
        const unsigned long long mask = __ballot(sel);
        const unsigned long long at = pos + lane_prefix(mask);
        if (sel && at < cap) {  // pairs beyond the capacity stay in the residual
            p.out_idx[at] = (int32_t)i;
            p.out_val[at] = x;
            if (p.residual) p.residual[i] = 0.0f;
        }
        pos += (unsigned long long)__popcll(mask);
    }
}

__device__ __forceinline__ void final_body(const Params& p, Blk b)
{
    __shared__ double sh[kWavesPerBlock][4];
    __shared__ uint32_t sh_cnt[kWavesPerBlock];
    __shared__ unsigned long long sh_base;
    constexpr int K = kFinalGroup;
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    // source lists of this wave: first, first + 8, first + 16, first + 24 (below last): the launchers give a
    // block at most kFinalGroup * 8 = 32 source lists, so one group of loads covers them all
    const uint32_t per_block = (p.nwaves + b.n - 1) / b.n;
    const uint32_t first = b.id * per_block + wib;
    const uint32_t last = min(p.nwaves, (b.id + 1) * per_block);

    // first group of lists: counts and first 64 slots of each, all loads issued together and before
    // the prologue (none depends on the threshold)
    FinalList l0[K];
    int4 q0[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t sw = first + k * kWavesPerBlock;
        l0[k] = final_list(p, sw, sw < last);
        q0[k] = (uint32_t)lane < l0[k].cap2 ? l0[k].src4[lane] : make_int4(0, 0, 0, 0);
    }

    const StageEta se = stage_prologue(p, b, true, sh);
    const float eta = se.eta;

    // pass A: count
    uint32_t mine = 0;
    if (!se.lists_ok) {
        for (uint32_t sw = first; sw < last; sw += kWavesPerBlock) mine += final_count_dense(p, sw, lane, eta);
    } else {
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t n = __builtin_amdgcn_readfirstlane(l0[k].n);
        mine += final_count(q0[k], lane, n, eta);
        for (uint32_t c = 64; c < (n + 1) / 2; c += 64) {
            const uint32_t i = c + lane;
            const int4 q = i < l0[k].cap2 ? l0[k].src4[i] : make_int4(0, 0, 0, 0);
            mine += final_count(q, i, n, eta);
        }
    }
    }
    if (lane == 0) sh_cnt[wib] = mine;
    __syncthreads();
    uint32_t off = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < kWavesPerBlock; ++i) {
        if (i < wib) off += sh_cnt[i];
        tot += sh_cnt[i];
    }
    const unsigned long long cap = (unsigned long long)p.out_cap;
    if (threadIdx.x == 0) {
        const unsigned long long base = atomicAdd(&p.st->selected_ctr, (unsigned long long)tot);
        sh_base = base;
        const unsigned long long end = base + tot;
        atomicMax(p.out_count, (int32_t)(end < cap ? end : cap));
        if (end > cap) {
            p.st->overflow = 1u;  // every writer stores the same value
            if (p.status_out) atomicOr(p.status_out, kStOverflow);
        }
        if (b.id == 0) {
            *p.out_eta = eta;
            const uint32_t status = p.st->status_after[p.M];  // written by this thread in the prologue
            p.st->diag.status = status;
            if (p.status_out && status) atomicOr(p.status_out, status);
        }
    }
    __syncthreads();
    unsigned long long pos = sh_base + off;

    // pass B: same traversal, now writing; the first group is still in registers
    if (!se.lists_ok) {
        for (uint32_t sw = first; sw < last; sw += kWavesPerBlock) final_emit_dense(p, sw, lane, eta, cap, pos);
        return;
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t n = __builtin_amdgcn_readfirstlane(l0[k].n);
        final_emit(p, q0[k], lane, n, eta, cap, pos);
        for (uint32_t c = 64; c < (n + 1) / 2; c += 64) {
            const uint32_t i = c + lane;
            const int4 q = i < l0[k].cap2 ? l0[k].src4[i] : make_int4(0, 0, 0, 0);
            final_emit(p, q, i, n, eta, cap, pos);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// k_gather: survivor lists of the last stage -> contiguous (index, value) output; residual update.
// Used when the last stage read the dense vector (M = 1): no atomics, output order is fixed.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void gather_body(const Params& p, Blk b)
{
    __shared__ unsigned long long sh_u[kWavesPerBlock][2];
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    const uint32_t t = threadIdx.x;
    const uint32_t w = b.id * kWavesPerBlock + wib;
    const uint32_t w0 = b.id * kWavesPerBlock;
    const bool active = w < p.nwaves;
    // independent loads first: block counts, the block's wave counts, this wave's count and first entries
    const unsigned long long c = t < p.nblocks ? (unsigned long long)p.blk_in[t] : 0ull;
    uint32_t mine = (lane < wib && w0 + lane < p.nwaves) ? p.cnt_in[w0 + lane] : 0u;
    uint32_t n_in = active ? p.cnt_in[w] : 0u;
    const int2* __restrict__ src = p.seg_in + (size_t)(active ? tile_begin(w, p.ntiles, p.nwaves) : 0) * kTile;
    const uint32_t cap_w = active ? (tile_begin(w + 1, p.ntiles, p.nwaves) - tile_begin(w, p.ntiles, p.nwaves)) * kTile : 0;
    int2 first = make_int2(0, 0);
    if ((uint32_t)lane < cap_w) first = src[lane];

    // exclusive prefix of the per-block counts at this block, and their total
    unsigned long long below = wave_sum_u64(t < b.id ? c : 0ull);
    unsigned long long total = wave_sum_u64(c);
    if (lane == 0) {
        sh_u[wib][0] = below;
        sh_u[wib][1] = total;
    }
    __syncthreads();
    below = 0;
    total = 0;
#pragma unroll
    for (int i = 0; i < kWavesPerBlock; ++i) {
        below += sh_u[i][0];
        total += sh_u[i][1];
    }
    const unsigned long long cap = (unsigned long long)p.out_cap;
    if (b.id == 0 && t == 0) {
        *p.out_count = (int32_t)(total > cap ? cap : total);
        *p.out_eta = p.st->diag.eta[p.M - 1];
        p.st->selected_ctr = total;
        p.st->overflow = total > cap ? 1u : 0u;
        const uint32_t status = p.st->status_after[p.M];
        p.st->diag.status = status;
        if (p.status_out) *p.status_out = status | (total > cap ? kStOverflow : 0u);
    }
    if (!active) return;
    // offset of this wave inside the block: counts of the block's earlier waves
#pragma unroll
    for (int o = 4; o > 0; o >>= 1) mine += __shfl_down(mine, o, 64);  // lanes 0..7 only carry data
    const unsigned long long base = below + __builtin_amdgcn_readfirstlane(mine);
    n_in = __builtin_amdgcn_readfirstlane(n_in);
    for (uint32_t i = lane; i < n_in; i += 64) {
        const unsigned long long pos = base + i;
        if (pos < cap) {  // pairs beyond the capacity stay in the residual
            const int2 q = i < 64 ? first : src[i];
            p.out_idx[pos] = q.x;
            p.out_val[pos] = __int_as_float(q.y);
            if (p.residual) p.residual[q.x] = 0.0f;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// k_scatter_add: the step after the sparsifier in Algorithm 2 - a worker's (index, value) pairs are
// added into the dense aggregate, dense[idx[i]] += scale * val[i].  The indices of one list are
// distinct, so plain read-modify-write needs no atomics and the result is deterministic; lists of
// several workers are added by consecutive launches.  Two roundings per element (product, then sum),
// as a plain fp32 loop does.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_scatter_add(float* __restrict__ dense, int64_t d, const int32_t* __restrict__ idx,
                                                        const float* __restrict__ val, const int32_t* __restrict__ count,
                                                        int64_t capacity, float scale, uint32_t* __restrict__ bad)
{
    int64_t n = (int64_t)*count;
    if (n > capacity) n = capacity;
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) {
        const int64_t j = (int64_t)idx[i];
        if (j < 0 || j >= d) {  // never written; reported
            atomicOr(bad, 1u);
            continue;
        }
        dense[j] = __fadd_rn(dense[j], __fmul_rn(scale, val[i]));
    }
}

__global__ void k_clear_u32(uint32_t* p) { *p = 0; }

// a fill kernel rather than a memset: callers may record the stream into a HIP graph
void launch_clear_u32(uint32_t* p, hipStream_t s) { hipLaunchKernelGGL(k_clear_u32, dim3(1), dim3(1), 0, s, p); }

void launch_scatter_add(float* dense, int64_t d, const int32_t* idx, const float* val, const int32_t* count,
                        int64_t capacity, float scale, uint32_t* bad, hipStream_t s)
{
    // the list length is only known on the device: a grid for the capacity, capped; idle blocks exit at once
    int64_t blocks = (capacity + 4 * kBlock - 1) / (4 * kBlock);
    if (blocks < 1) blocks = 1;
    if (blocks > 2 * kMaxBlocks) blocks = 2 * kMaxBlocks;
    hipLaunchKernelGGL(k_scatter_add, dim3((uint32_t)blocks), dim3(kBlock), 0, s, dense, d, idx, val, count, capacity,
                       scale, bad);
}

// ---------------------------------------------------------------------------------------------
// kernels: one call on one vector (the grid is the vector's), or a batch of vectors in one launch
// (every block belongs to one vector and finds that vector's arguments in a table on the device)
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ Blk whole_grid() { return Blk{blockIdx.x, gridDim.x}; }

// Arguments of this block's vector in a batched launch.  final_grid: the launch uses the last stage's
// (smaller) grid.
__device__ __forceinline__ Params batch_params(const BatchArgs& a, bool final_grid, Blk& b, uint32_t gb = blockIdx.x)
{
    const uint32_t t = __builtin_amdgcn_readfirstlane((uint32_t)(final_grid ? a.tb->fmap[gb] : a.tb->map[gb]));
    const TensorDesc& ds = a.tb->desc[t];
    Params p = {};
    p.grad = reinterpret_cast<const char*>(a.grad) + ds.offset * (a.gt == kGradF32 ? 4 : 2);
    p.gt = a.gt;
    p.residual = a.residual ? a.residual + ds.offset : nullptr;
    p.acc_w = p.residual ? p.residual : (a.acc_own ? a.acc_own + ds.offset : nullptr);
    p.acc = p.acc_w ? p.acc_w : reinterpret_cast<const float*>(p.grad);
    p.d = ds.d;
    p.ntiles = (uint32_t)((ds.d + kTile - 1) / kTile);
    p.nfull = (uint32_t)(ds.d / kTile);
    p.nwaves = ds.nblocks * kWavesPerBlock < p.ntiles ? ds.nblocks * kWavesPerBlock : p.ntiles;
    p.nblocks = ds.nblocks;
    p.vec_ok = ((uintptr_t)p.grad & (a.gt == kGradF32 ? 15u : 7u)) == 0 && ((uintptr_t)p.acc_w & 15u) == 0;
    p.reverse = a.reverse;
    p.acc_reset = 1;
    p.dist = a.dist;
    p.M = a.M;
    p.stage = a.stage;
#pragma unroll
    for (int m = 0; m < SIDCO_MAX_STAGES; ++m) p.L[m] = a.L[m];
    p.theta = a.theta;
    p.theta_min = a.theta_min;
    p.use_hint = a.use_hint;
    p.prev_cand = a.prev_cand;
    p.st = &a.tb->st[t];
    p.part_in = a.part[a.in] + ds.first_block;
    p.part_out = a.part[a.out] + ds.first_block;
    p.cnt_in = a.cnt[a.in] + ds.first_block * kWavesPerBlock;
    p.cnt_out = a.cnt[a.out] + ds.first_block * kWavesPerBlock;
    p.blk_in = a.blk[a.in] + ds.first_block;
    p.blk_out = a.blk[a.out] + ds.first_block;
    p.seg_in = a.seg[a.in] + ds.seg_off;
    p.seg_out = a.seg[a.out] + ds.seg_off;
    p.out_idx = a.out_idx + ds.out_offset;
    p.out_val = a.out_val + ds.out_offset;
    p.out_count = a.out_counts + ds.index;
    p.out_eta = a.out_etas + ds.index;
    p.out_cap = ds.out_cap;
    b.id = gb - (final_grid ? ds.first_final : ds.first_block);
    b.n = final_grid ? ds.nfinal : ds.nblocks;
    return p;
}

// Tiles of block b of a vector's dense grid: those of its (at most) kWavesPerBlock waves.
__device__ __forceinline__ void block_tiles(const Params& p, Blk b, uint32_t& T0, uint32_t& T1)
{
    const uint32_t w0 = b.id * kWavesPerBlock;
    const uint32_t w1 = w0 + kWavesPerBlock < p.nwaves ? w0 + kWavesPerBlock : p.nwaves;
    T0 = w0 < p.nwaves ? tile_begin(w0, p.ntiles, p.nwaves) : 0;
    T1 = w0 < p.nwaves ? tile_begin(w1, p.ntiles, p.nwaves) : 0;
}

template <int DIST, bool EC, int GT>
__global__ __launch_bounds__(kBlock, 4) void k_fit(Params p) { fit_body<DIST, EC, GT>(p, whole_grid()); }
template <bool STATS, bool WRITE, int PRE>
__global__ __launch_bounds__(kBlock, 4) void k_compact(Params p) { compact_body<STATS, WRITE, PRE>(p, whole_grid()); }
__global__ __launch_bounds__(kBlock, 4) void k_lists(Params p) { lists_body(p, whole_grid()); }
__global__ __launch_bounds__(kBlock) void k_final_lists(Params p) { final_body(p, whole_grid()); }
__global__ __launch_bounds__(kBlock) void k_gather(Params p) { gather_body(p, whole_grid()); }

template <int DIST, bool EC, int GT>
__global__ __launch_bounds__(kBlock) void k_fit_batched(BatchArgs a)
{
    Blk b;
    const Params p = batch_params(a, false, b);
    fit_body<DIST, EC, GT>(p, b);
}
// The first pass of a batch in the flat shape (see k_fit_flat): blockIdx.y is a block of the batch's dense grid
// - it names the vector and, within it, the tiles that block's waves own - and blockIdx.x a chunk of
// kFlatBlock / 64 = 4 of those tiles, one tile per wave.  Blocks run in the order x first, then y: address
// order.  Chunks past the end of a y's tiles exit at once (the host launches the flat shape only when few
// are).  A vector that does not start on a 16-byte boundary (8 for a 16-bit gradient) takes guarded scalar
// accesses, like the incomplete last tile.
template <int DIST, bool EC, int GT>
__global__ __launch_bounds__(kFlatBlock) void k_fit_flat_batched(BatchArgs a, double* __restrict__ flat_part,
                                                                  uint32_t stride)
{
    __shared__ double sh[kFlatBlock / 64][4];
    Blk b;
    const Params p = batch_params(a, false, b, blockIdx.y);
    uint32_t T0, T1;
    block_tiles(p, b, T0, T1);
    const uint32_t first = T0 + blockIdx.x * (kFlatBlock / 64);
    if (first >= T1) return;  // the whole block
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    const uint32_t t = first + wib;
    double s1 = 0.0, s2 = 0.0, sl = 0.0;
    int se = 0;
    if (t < T1) {
        if (p.vec_ok && t < p.nfull) {
            fit_tiles<DIST, EC, GT, 1>(p.grad, reinterpret_cast<f4*>(p.acc_w), t, lane, s1, s2, sl, se);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t i = (int64_t)t * kTile + lane * 4 + j;
                if (i < p.d) fit_one<DIST, EC, GT>(p, i, s1, s2, sl, se);
            }
        }
    }
    double v[3] = {s1, s2, sl + (double)se};
    v[0] = wave_sum(v[0]);
    v[1] = wave_sum(v[1]);
    v[2] = wave_sum(v[2]);
    if (lane == 0) {
        sh[wib][0] = v[0];
        sh[wib][1] = v[1];
        sh[wib][2] = v[2];
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        double tot = 0.0;
#pragma unroll
        for (int w = 0; w < kFlatBlock / 64; ++w) tot += sh[w][threadIdx.x];
        flat_part[(size_t)threadIdx.x * stride + (size_t)blockIdx.y * gridDim.x + blockIdx.x] = tot;
    }
}

// Folds the chunks' partial sums of every block y of the batch's dense grid into that block's slot, in a
// fixed order: one wave per y.  `gx` is the x extent of k_fit_flat_batched's grid, `nb` its y extent.
__global__ __launch_bounds__(kBlock) void k_fit_reduce_batched(BatchArgs a, const double* __restrict__ flat_part,
                                                               uint32_t gx, uint32_t nb)
{
    const int lane = threadIdx.x & 63;
    const uint32_t y = blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    if (y >= nb) return;  // the whole wave; no block-wide synchronisation below
    Blk b;
    const Params p = batch_params(a, false, b, y);
    uint32_t T0, T1;
    block_tiles(p, b, T0, T1);
    const uint32_t nchunk = (T1 - T0 + kFlatBlock / 64 - 1) / (kFlatBlock / 64);
    const size_t stride = (size_t)gx * nb, base = (size_t)y * gx;
    double v[3] = {0.0, 0.0, 0.0};
    for (uint32_t c = lane; c < nchunk; c += 64) {
        v[0] += flat_part[base + c];
        if (p.dist == kDistGpd) v[1] += flat_part[stride + base + c];
        if (p.dist == kDistGamma) v[2] += flat_part[2 * stride + base + c];
    }
    v[0] = wave_sum(v[0]);
    v[1] = wave_sum(v[1]);
    v[2] = wave_sum(v[2]);
    if (lane == 0) {
        p.part_out[0 * kMaxBlocks + b.id] = v[0];
        p.part_out[1 * kMaxBlocks + b.id] = v[1];
        p.part_out[2 * kMaxBlocks + b.id] = v[2];
        if (b.id == 0) fit_reset_state(p);
    }
}

template <bool STATS, bool WRITE, int PRE>
__global__ __launch_bounds__(kBlock, 4) void k_compact_batched(BatchArgs a)
{
    Blk b;
    const Params p = batch_params(a, false, b);
    compact_body<STATS, WRITE, PRE>(p, b);
}
__global__ __launch_bounds__(kBlock, 4) void k_lists_batched(BatchArgs a)
{
    Blk b;
    const Params p = batch_params(a, false, b);
    lists_body(p, b);
}
__global__ __launch_bounds__(kBlock) void k_final_lists_batched(BatchArgs a)
{
    Blk b;
    const Params p = batch_params(a, true, b);
    final_body(p, b);
}
__global__ __launch_bounds__(kBlock) void k_gather_batched(BatchArgs a)
{
    Blk b;
    const Params p = batch_params(a, false, b);
    gather_body(p, b);
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
template <bool EC, int GT>
static void launch_fit_as(const Params& p, hipStream_t s)
{
    const dim3 grid(p.nblocks), block(kBlock);
    switch (p.dist) {
        case kDistExp: hipLaunchKernelGGL((k_fit<kDistExp, EC, GT>), grid, block, 0, s, p); break;
        case kDistGamma: hipLaunchKernelGGL((k_fit<kDistGamma, EC, GT>), grid, block, 0, s, p); break;
        default: hipLaunchKernelGGL((k_fit<kDistGpd, EC, GT>), grid, block, 0, s, p); break;
    }
}

template <bool EC, int GT>
static void launch_fit_flat_as(const Params& p, double* flat_part, uint32_t nflat, hipStream_t s)
{
    const dim3 grid(nflat), block(kFlatBlock);
    switch (p.dist) {
        case kDistExp:
            hipLaunchKernelGGL((k_fit_flat<kDistExp, EC, GT>), grid, block, 0, s, p, flat_part, nflat);
            break;
        case kDistGamma:
            hipLaunchKernelGGL((k_fit_flat<kDistGamma, EC, GT>), grid, block, 0, s, p, flat_part, nflat);
            break;
        default: hipLaunchKernelGGL((k_fit_flat<kDistGpd, EC, GT>), grid, block, 0, s, p, flat_part, nflat); break;
    }
}

template <bool EC, int GT>
static void launch_fit_shape(const Params& p, double* scratch, hipStream_t s)
{
    if (fit_uses_flat(p.d, p.vec_ok != 0)) {
        const uint32_t nflat = fit_flat_blocks(p.d);
        launch_fit_flat_as<EC, GT>(p, scratch, nflat, s);
        const uint32_t per = (nflat + kMaxBlocks - 1) / kMaxBlocks;
        hipLaunchKernelGGL(k_fit_reduce, dim3(kMaxBlocks / kWavesPerBlock), dim3(kBlock), 0, s, p, scratch, nflat, per);
        return;
    }
    launch_fit_as<EC, GT>(p, s);
}

template <int GT>
static void launch_fit_type(const Params& p, double* scratch, hipStream_t s)
{
    if (p.residual) launch_fit_shape<true, GT>(p, scratch, s);
    else launch_fit_shape<false, GT>(p, scratch, s);
}

// `scratch`: device memory for 3 * fit_flat_blocks(d) doubles when the flat shape is used (else unused)
void launch_fit(const Params& p, double* scratch, hipStream_t s)
{
    switch (p.gt) {
        case kGradF16: launch_fit_type<kGradF16>(p, scratch, s); break;
        case kGradBf16: launch_fit_type<kGradBf16>(p, scratch, s); break;
        default: launch_fit_type<kGradF32>(p, scratch, s); break;
    }
}

template <int PRE>
static void launch_compact_pre(const Params& p, bool stats, bool write, hipStream_t s)
{
    const dim3 grid(p.nblocks), block(kBlock);
    if (stats && write) hipLaunchKernelGGL((k_compact<true, true, PRE>), grid, block, 0, s, p);
    else if (stats) hipLaunchKernelGGL((k_compact<true, false, PRE>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((k_compact<false, true, PRE>), grid, block, 0, s, p);
}

void launch_compact(const Params& p, bool stats, bool write, hipStream_t s)
{
    // Prefetch before the prologue only where every wave has that many complete tiles to itself: a wave owns
    // at least floor(nfull / nwaves) tiles, and the last wave's last tile may be the incomplete one, which a
    // whole-tile load must not touch - hence one tile more than the prefetched batches hold.
    const uint32_t per_wave = p.nwaves ? p.nfull / p.nwaves : 0;
    if (p.vec_ok && p.nwaves == (uint32_t)kMaxWaves && per_wave >= (uint32_t)(kCompactPrefetch * 4 + 1))
        launch_compact_pre<kCompactPrefetch>(p, stats, write, s);
    else
        launch_compact_pre<0>(p, stats, write, s);
}

void launch_lists(const Params& p, uint32_t grid_blocks, hipStream_t s)
{
    hipLaunchKernelGGL(k_lists, dim3(grid_blocks), dim3(kBlock), 0, s, p);
}

void launch_final_lists(const Params& p, uint32_t grid_blocks, hipStream_t s)
{
    // a block reads at most kFinalGroup lists per wave (see final_body)
    const uint32_t least = (p.nwaves + kFinalGroup * kWavesPerBlock - 1) / (kFinalGroup * kWavesPerBlock);
    if (grid_blocks < least) grid_blocks = least;
    hipLaunchKernelGGL(k_final_lists, dim3(grid_blocks), dim3(kBlock), 0, s, p);
}

void launch_gather(const Params& p, hipStream_t s)
{
    hipLaunchKernelGGL(k_gather, dim3(p.nblocks), dim3(kBlock), 0, s, p);
}

// batched: `blocks` is the sum of the vectors' grids (the last stage's own, smaller sum for launch_final).
// `flat_gx` > 0: the first pass in the flat shape, `flat_gx` chunks of 4 tiles per block of the dense grid, with
// `scratch` holding 3 * flat_gx * blocks doubles; a second kernel folds them.
template <bool EC, int GT>
static void launch_fit_batched_as(const BatchArgs& a, uint32_t blocks, uint32_t flat_gx, double* scratch, hipStream_t s)
{
    if (flat_gx > 0) {
        const dim3 grid(flat_gx, blocks), block(kFlatBlock);
        const uint32_t stride = flat_gx * blocks;
        switch (a.dist) {
            case kDistExp:
                hipLaunchKernelGGL((k_fit_flat_batched<kDistExp, EC, GT>), grid, block, 0, s, a, scratch, stride);
                break;
            case kDistGamma:
                hipLaunchKernelGGL((k_fit_flat_batched<kDistGamma, EC, GT>), grid, block, 0, s, a, scratch, stride);
                break;
            default:
                hipLaunchKernelGGL((k_fit_flat_batched<kDistGpd, EC, GT>), grid, block, 0, s, a, scratch, stride);
                break;
        }
        hipLaunchKernelGGL(k_fit_reduce_batched, dim3((blocks + kWavesPerBlock - 1) / kWavesPerBlock), dim3(kBlock), 0, s,
                           a, scratch, flat_gx, blocks);
        return;
    }
    const dim3 grid(blocks), block(kBlock);
    switch (a.dist) {
        case kDistExp: hipLaunchKernelGGL((k_fit_batched<kDistExp, EC, GT>), grid, block, 0, s, a); break;
        case kDistGamma: hipLaunchKernelGGL((k_fit_batched<kDistGamma, EC, GT>), grid, block, 0, s, a); break;
        default: hipLaunchKernelGGL((k_fit_batched<kDistGpd, EC, GT>), grid, block, 0, s, a); break;
    }
}

template <int GT>
static void launch_fit_batched_type(const BatchArgs& a, bool ec, uint32_t blocks, uint32_t flat_gx, double* scratch,
                                    hipStream_t s)
{
    if (ec) launch_fit_batched_as<true, GT>(a, blocks, flat_gx, scratch, s);
    else launch_fit_batched_as<false, GT>(a, blocks, flat_gx, scratch, s);
}

void launch_fit_batched(const BatchArgs& a, bool ec, uint32_t blocks, uint32_t flat_gx, double* scratch, hipStream_t s)
{
    switch (a.gt) {
        case kGradF16: launch_fit_batched_type<kGradF16>(a, ec, blocks, flat_gx, scratch, s); break;
        case kGradBf16: launch_fit_batched_type<kGradBf16>(a, ec, blocks, flat_gx, scratch, s); break;
        default: launch_fit_batched_type<kGradF32>(a, ec, blocks, flat_gx, scratch, s); break;
    }
}

template <int PRE>
static void launch_compact_batched_pre(const BatchArgs& a, bool stats, bool write, uint32_t blocks, hipStream_t s)
{
    const dim3 grid(blocks), block(kBlock);
    if (stats && write) hipLaunchKernelGGL((k_compact_batched<true, true, PRE>), grid, block, 0, s, a);
    else if (stats) hipLaunchKernelGGL((k_compact_batched<true, false, PRE>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((k_compact_batched<false, true, PRE>), grid, block, 0, s, a);
}

// `prefetch`: every vector of the batch meets launch_compact's condition (aligned, all waves of its blocks in
// use, enough complete tiles per wave), so the dense stage may request tiles before its threshold is known
void launch_compact_batched(const BatchArgs& a, bool stats, bool write, bool prefetch, uint32_t blocks, hipStream_t s)
{
    if (prefetch) launch_compact_batched_pre<kCompactPrefetch>(a, stats, write, blocks, s);
    else launch_compact_batched_pre<0>(a, stats, write, blocks, s);
}

void launch_lists_batched(const BatchArgs& a, uint32_t blocks, hipStream_t s)
{
    hipLaunchKernelGGL(k_lists_batched, dim3(blocks), dim3(kBlock), 0, s, a);
}

void launch_final_lists_batched(const BatchArgs& a, uint32_t final_blocks, hipStream_t s)
{
    hipLaunchKernelGGL(k_final_lists_batched, dim3(final_blocks), dim3(kBlock), 0, s, a);
}

void launch_gather_batched(const BatchArgs& a, uint32_t blocks, hipStream_t s)
{
    hipLaunchKernelGGL(k_gather_batched, dim3(blocks), dim3(kBlock), 0, s, a);
}

}  // namespace sidco
