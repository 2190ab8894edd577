/*
 * CPU oracle for the SIDCo gradient sparsifier (arXiv 2101.10761).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of
 * what the sparsifier computes, written from the paper.  Only the test-suite,
 * the smoke check and the benchmark's CPU-baseline leg may call it; the GPU
 * library never does, and the two share no source, header, table or helper.
 *
 * Everything is a straight loop in double precision, single threaded, with no
 * blocking, fusion or reordering beyond what the paper's statement implies:
 *
 *   - error-compensation add ............ App. B.2 (memory-based compression)
 *   - first-stage fits and thresholds ... Corollary 1 / eq. (6); Corollaries 1.2
 *                                         and 1.3 (App. B.3); Algorithm 1,
 *                                         function Thresh_Estimation
 *   - peak-over-threshold refinement .... Sec. 2.4, Lemma 2 / eqs. (7)-(9),
 *                                         Corollary 2 / eqs. (10)-(11)
 *   - threshold operator C_eta .......... Sec. 2.3 ("Gradient compression
 *                                         through thresholding")
 *   - stage loop ........................ Algorithm 1, function Sparsify
 *   - number of stages .................. Algorithm 1, function Adapt_Stages; Sec. 3
 *   - aggregation of sparse gradients ... Algorithm 2 (App. A)
 *
 * Readings taken where the paper is silent or inconsistent (each is a reading,
 * not a quotation; they are listed again in the design notes of the build):
 *   R1  thresholds are absolute: eta_m = eta_{m-1} + increment (Lemma 2 and
 *       Corollary 2 are followed, not the shifted-temp bookkeeping of the
 *       pseudo-code), and eta_M is applied to |acc|.
 *   R2  stage m >= 2 statistics run over the exceedances only (n = khat_{m-1}).
 *   R3  the GPD scale estimator uses mu^2/sigma^2 (the pseudo-code drops the
 *       square; eqs. (8)-(9) and App. B.3 keep it).
 *   R4  "sample variance" is the population (1/n) variance of a moment match.
 *   R5  selection is strict: |x| > eta, compared in fp32 against the fp32
 *       threshold (an all-zero gradient then selects nothing).
 *   R6  delta_1 is given; delta_m = (delta/delta_1)^(1/(M-1)) for m = 2..M;
 *       M = 1 or delta_1 <= delta collapses to a single stage at delta.
 *   R7  log|x| is taken of max(|x|, 2^-126) in the log-mean only.
 *   R8  each eta_m is rounded once to fp32; that value is used for the
 *       comparison and for the next stage's shift.
 *   R9  degenerate fits take the limit of the closed form, so that rounding
 *       noise in a sum cannot flip the outcome: non-finite sums -> eta = NaN,
 *       nothing selected; variance <= 0 in a GPD fit (all magnitudes equal)
 *       -> increment = mean (the closed form's limit as variance -> 0+);
 *       s <= 0 in the gamma fit -> threshold 0 (the closed form tends to
 *       -infinity there and negative thresholds are clamped to 0); an empty
 *       exceedance set stops refining (eta_M = eta_{m-1}).
 *   R10 residual' = acc with zeros at the selected positions.
 *   R16 the stage controller averages all Q counts of a window (the pseudo-code
 *       leaves the adapting iteration's count out of the sum yet divides by Q;
 *       Sec. 3 says "average ... over the past training steps Q"); this lives in
 *       the Python driver oracle.adaptive_run, the C function is Adapt_Stages as
 *       printed.
 *
 * Pins (tests/test_oracle_*.py, run without a GPU): hand-worked examples in
 * tests/golden/, scipy quantile functions of the three distributions, exact
 * quantile grids of exponential / GPD / gamma laws, the exact gamma MLE
 * equation, brute-force sort on tiny inputs, binomial count band, nesting and
 * monotonicity invariants, planted ties, residual conservation.
 * Parity unpinned by the paper itself: R4, R5 and R6 (no printed value
 * distinguishes them); they are pinned only as readings.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_MAX_STAGES 8

/* dist argument: which first-stage law, and therefore which chain (Sec. 2.4,
 * last paragraph): 0 exponential->exponential, 1 gamma->GPD, 2 GPD->GPD. */
enum { DIST_EXP = 0, DIST_GAMMA_GPD = 1, DIST_GPD = 2 };

/* status bits (oracle's own numbering is part of the tested interface) */
enum {
    ST_NONFINITE   = 1u << 0, /* a stage-1 sum was NaN/Inf (R9) */
    ST_VAR_ZERO    = 1u << 1, /* a GPD fit had variance <= 0: increment = mean */
    ST_GAMMA_S     = 1u << 2, /* gamma fit had s <= 0: threshold 0 */
    ST_GAMMA_CLAMP = 1u << 3, /* gamma closed form was negative, clamped to 0 */
    ST_STOPPED     = 1u << 4  /* refinement stopped early (empty exceedance set) */
};

/* ------------------------------------------------------------------------ */
/* App. B.2: the error of the previous iteration is added to the gradient
 * before compression.  One IEEE fp32 addition per element (the paper's
 * tensors are fp32). r == NULL is the memoryless variant: acc = g.           */
void sidco_oracle_ec_add(const float *g, const float *r, int64_t d, float *acc)
{
    for (int64_t j = 0; j < d; ++j) {
        if (r) {
            volatile float s = g[j] + r[j]; /* volatile: no excess precision, no fusing */
            acc[j] = s;
        } else {
            acc[j] = g[j];
        }
    }
}

/* R6: split of delta over the stages.  Returns the effective number of stages
 * and writes that many ratios, whose product is delta.                       */
int sidco_oracle_schedule(double delta, int stages, double delta1, double *ratios)
{
    if (stages <= 1 || !(delta1 > delta) || !(delta1 < 1.0)) {
        ratios[0] = delta;
        return 1;
    }
    if (stages > ORACLE_MAX_STAGES) stages = ORACLE_MAX_STAGES;
    ratios[0] = delta1;
    double rest = pow(delta / delta1, 1.0 / (double)(stages - 1));
    for (int m = 1; m < stages; ++m) ratios[m] = rest;
    return stages;
}

/* ------------------------------------------------------------------------ */
/* Sample moments of |acc| over all d entries: mean, population variance and
 * mean of log (Corollary 1; Corollaries 1.2, 1.3).                           */
void sidco_oracle_moments_all(const float *acc, int64_t d,
                              double *mu, double *var, double *mulog)
{
    const double tiny = ldexp(1.0, -126); /* R7 */
    double s1 = 0.0, s2 = 0.0, sl = 0.0;
    for (int64_t j = 0; j < d; ++j) {
        double x = fabs((double)acc[j]);
        s1 += x;
        s2 += x * x;
        sl += log(x > tiny ? x : tiny);
    }
    double m = s1 / (double)d;
    *mu = m;
    *var = s2 / (double)d - m * m;
    *mulog = sl / (double)d;
}

/* Sample mean and population variance of y = |x| - eta_prev over the
 * exceedances {|x| > eta_prev} (Lemma 2: "sample mean and variance of
 * |g_bar_m| - eta_{m-1}").  Returns their number.                            */
int64_t sidco_oracle_moments_pot(const float *acc, int64_t d, float eta_prev,
                                 double *ybar, double *yvar)
{
    double s1 = 0.0, s2 = 0.0;
    int64_t n = 0;
    for (int64_t j = 0; j < d; ++j) {
        float a = fabsf(acc[j]);
        if (a > eta_prev) { /* R5: fp32 comparison */
            double y = (double)a - (double)eta_prev;
            s1 += y;
            s2 += y * y;
            ++n;
        }
    }
    if (n == 0) {
        *ybar = 0.0;
        *yvar = 0.0;
        return 0;
    }
    double m = s1 / (double)n;
    *ybar = m;
    *yvar = s2 / (double)n - m * m;
    return n;
}

/* ------------------------------------------------------------------------ */
/* Closed-form thresholds.  Each returns the distance above the stage's
 * location (0 for stage 1, eta_{m-1} afterwards).                            */

/* eq. (6) / eq. (10): beta_hat * log(1/delta), beta_hat the sample mean.      */
double sidco_oracle_eta_exp(double mu, double delta)
{
    return mu * log(1.0 / delta);
}

/* eqs. (8)-(9) and Corollary 1.3: moment-matched GPD shape and scale.         */
void sidco_oracle_gpd_fit(double mu, double var, double *alpha, double *beta)
{
    double q = (mu * mu) / var;
    *alpha = 0.5 * (1.0 - q);
    *beta = 0.5 * mu * (q + 1.0);
}

/* eq. (7) without the location term: (beta/alpha) (exp(-alpha log delta) - 1).
 * exp(z)-1 is evaluated as expm1(z); alpha == 0 is the exponential limit
 * noted in the footnote of App. B.3.2.                                        */
double sidco_oracle_eta_gpd(double mu, double var, double delta)
{
    double a, b;
    sidco_oracle_gpd_fit(mu, var, &a, &b);
    if (a == 0.0) return b * log(1.0 / delta);
    return (b / a) * expm1(-a * log(delta));
}

/* Corollary 1.2: closed-form approximation of the gamma MLE shape.            */
double sidco_oracle_gamma_shape(double s)
{
    return (3.0 - s + sqrt((s - 3.0) * (s - 3.0) + 24.0 * s)) / (12.0 * s);
}

/* Corollary 1.2: eta ~= -beta_hat [log delta + log Gamma(alpha_hat)].         */
double sidco_oracle_eta_gamma(double mu, double mulog, double delta)
{
    double s = log(mu) - mulog;
    double a = sidco_oracle_gamma_shape(s);
    double b = mu / a;
    return -b * (log(delta) + lgamma(a));
}

/* ------------------------------------------------------------------------ */
/* Threshold operator C_eta (Sec. 2.3) with R5, plus the residual update R10.
 * idx/val may be NULL (count only).  residual, if given, must already hold
 * acc; the selected positions are zeroed.  Output is in ascending index.     */
int64_t sidco_oracle_select(const float *acc, int64_t d, float eta,
                            int32_t *idx, float *val, float *residual)
{
    int64_t k = 0;
    for (int64_t j = 0; j < d; ++j) {
        if (fabsf(acc[j]) > eta) {
            if (idx) idx[k] = (int32_t)j;
            if (val) val[k] = acc[j];
            if (residual) residual[j] = 0.0f;
            ++k;
        }
    }
    return k;
}

/* ------------------------------------------------------------------------ */
/* First-stage threshold for a given law (Algorithm 1, Thresh_Estimation),
 * with the degenerate cases of R9.  stats[0..2] = mu, var, mulog.            */
static double stage1_threshold(int dist, const double *stats, double delta1,
                               uint32_t *status)
{
    double mu = stats[0], var = stats[1], mulog = stats[2];
    if (!isfinite(mu) || !isfinite(var) || (dist == DIST_GAMMA_GPD && !isfinite(mulog))) {
        *status |= ST_NONFINITE;
        return NAN;
    }
    if (dist == DIST_EXP) return sidco_oracle_eta_exp(mu, delta1);
    if (dist == DIST_GPD) {
        if (!(var > 0.0)) {
            *status |= ST_VAR_ZERO;
            return mu;
        }
        return sidco_oracle_eta_gpd(mu, var, delta1);
    }
    /* gamma first stage (an all-zero vector has log(mu) = -inf and lands in the s <= 0 case) */
    double s = log(mu) - mulog;
    if (!(s > 0.0)) {
        *status |= ST_GAMMA_S;
        return 0.0;
    }
    double t = sidco_oracle_eta_gamma(mu, mulog, delta1);
    if (t < 0.0) {
        *status |= ST_GAMMA_CLAMP;
        t = 0.0;
    }
    return t;
}

/*
 * The whole sparsifier (Algorithm 1, function Sparsify, with readings R1-R10).
 *
 *  g, d            gradient (fp32)
 *  r               residual, in/out, or NULL for the memoryless variant
 *  dist            DIST_*
 *  M, ratios       stage ratios delta_1..delta_M (product = target delta)
 *  eta_inject      NULL, or M fp32 thresholds: after stage m has produced its
 *                  own eta_m (reported in etas_own[m-1]) the injected value
 *                  replaces it for the selection and for the next stage's
 *                  location.  NaN entries are ignored.  Used to compare a
 *                  second implementation stage by stage.
 *  idx, val        outputs, capacity d (ascending index order)
 *  count           khat
 *  etas_own[M]     thresholds this routine computed at each stage
 *  etas_used[M]    thresholds that were applied (own or injected)
 *  n_stage[M]      n_stage[m-1] = number of elements the stage-m fit ran over
 *  stats[3*M]      per stage: mean, variance, log-mean (stage 1) or
 *                  ybar, yvar, 0 (stages >= 2)
 *  status          OR of ST_* bits
 * Returns 0, or -1 on allocation failure.
 */
int sidco_oracle_compress(const float *g, float *r, int64_t d, int dist,
                          int M, const double *ratios, const float *eta_inject,
                          int32_t *idx, float *val, int64_t *count,
                          float *etas_own, float *etas_used, int64_t *n_stage,
                          double *stats, uint32_t *status)
{
    float *acc_own = NULL;
    float *acc;
    uint32_t st = 0;

    /* step 0: error compensation */
    if (r) {
        sidco_oracle_ec_add(g, r, d, r);
        acc = r;
    } else {
        acc_own = (float *)malloc((size_t)(d > 0 ? d : 1) * sizeof(float));
        if (!acc_own) return -1;
        sidco_oracle_ec_add(g, NULL, d, acc_own);
        acc = acc_own;
    }

    for (int m = 0; m < M; ++m) {
        etas_own[m] = etas_used[m] = 0.0f;
        n_stage[m] = 0;
        stats[3 * m] = stats[3 * m + 1] = stats[3 * m + 2] = 0.0;
    }

    /* stage 1: fit all of |acc| */
    sidco_oracle_moments_all(acc, d, &stats[0], &stats[1], &stats[2]);
    n_stage[0] = d;
    float eta = (float)stage1_threshold(dist, stats, ratios[0], &st); /* R8 */
    etas_own[0] = eta;
    if (eta_inject && !isnan(eta_inject[0])) eta = eta_inject[0];
    etas_used[0] = eta;

    /* stages 2..M: fit the exceedances over eta_{m-1} */
    int stopped = 0;
    for (int m = 1; m < M; ++m) {
        float eta_prev = eta;
        if (!stopped) {
            double ybar, yvar;
            int64_t n = sidco_oracle_moments_pot(acc, d, eta_prev, &ybar, &yvar);
            n_stage[m] = n;
            stats[3 * m] = ybar;
            stats[3 * m + 1] = yvar;
            if (n == 0) {
                stopped = 1;
            } else if (dist == DIST_EXP) {
                eta = (float)((double)eta_prev + sidco_oracle_eta_exp(ybar, ratios[m]));
            } else if (!(yvar > 0.0)) {
                st |= ST_VAR_ZERO;
                eta = (float)((double)eta_prev + ybar);
            } else {
                eta = (float)((double)eta_prev + sidco_oracle_eta_gpd(ybar, yvar, ratios[m]));
            }
            if (stopped) st |= ST_STOPPED;
        }
        etas_own[m] = eta;
        if (eta_inject && !isnan(eta_inject[m])) eta = eta_inject[m];
        etas_used[m] = eta;
    }

    /* final: C_eta on acc, residual update */
    *count = sidco_oracle_select(acc, d, eta, idx, val, r);
    *status = st;
    free(acc_own);
    return 0;
}

/* Algorithm 2, aggregation of the workers' sparsified gradients: one worker's
 * (index, value) pairs are added into the dense sum, scaled (1/N for the
 * average).  fp32, two roundings per element: product, then sum.  Returns the
 * number of pairs whose index is outside [0, d) (they are skipped).          */
int64_t sidco_oracle_scatter_add(float *dense, int64_t d, const int32_t *idx,
                                 const float *val, int64_t n, float scale)
{
    int64_t bad = 0;
    for (int64_t i = 0; i < n; ++i) {
        int64_t j = idx[i];
        if (j < 0 || j >= d) {
            ++bad;
            continue;
        }
        volatile float prod = scale * val[i]; /* volatile: no fused multiply-add */
        volatile float sum = dense[j] + prod;
        dense[j] = sum;
    }
    return bad;
}

/* Algorithm 1, function Adapt_Stages (and Sec. 3): one stage fewer when the
 * average number of selected elements is above k (1 + eps_H), one more when it
 * is below k (1 - eps_L), and the result clamped to [1, M_max].               */
int sidco_oracle_adapt_stages(int M, double khat_avg, double k, double eps_h,
                              double eps_l, int M_max)
{
    if (khat_avg > k * (1.0 + eps_h)) M = M - 1;
    if (khat_avg < k * (1.0 - eps_l)) M = M + 1;
    if (M < 1) M = 1;
    if (M > M_max) M = M_max;
    return M;
}

/* Exact Top-k by magnitude, for tiny cross-checks (footnote of Sec. 2.3:
 * C_eta equals Top-k at k = khat).  O(d log d) sort; ties broken by lower
 * index.  Writes k indices in ascending index order. Returns k or -1.        */
typedef struct { float a; int32_t j; } mag_t;
static int mag_cmp(const void *p, const void *q)
{
    const mag_t *x = (const mag_t *)p, *y = (const mag_t *)q;
    if (x->a > y->a) return -1;
    if (x->a < y->a) return 1;
    return (x->j > y->j) - (x->j < y->j);
}
static int i32_cmp(const void *p, const void *q)
{
    int32_t x = *(const int32_t *)p, y = *(const int32_t *)q;
    return (x > y) - (x < y);
}
int64_t sidco_oracle_topk(const float *acc, int64_t d, int64_t k, int32_t *idx)
{
    if (k > d) k = d;
    if (k <= 0) return 0;
    mag_t *m = (mag_t *)malloc((size_t)d * sizeof(mag_t));
    if (!m) return -1;
    for (int64_t j = 0; j < d; ++j) {
        m[j].a = fabsf(acc[j]);
        m[j].j = (int32_t)j;
    }
    qsort(m, (size_t)d, sizeof(mag_t), mag_cmp);
    for (int64_t i = 0; i < k; ++i) idx[i] = m[i].j;
    qsort(idx, (size_t)k, sizeof(int32_t), i32_cmp);
    free(m);
    return k;
}

/* ------------------------------------------------------------------------ */
/* DGC's sampling threshold, the comparator the paper describes in Sec. 1
 * (related work, with its footnote): draw a random subset of the gradient
 * (about 1 %), take Top-k of that subset at the same ratio to obtain a
 * threshold, select with the threshold, and - if that selects more than the
 * target k - run Top-k once more on the selected entries.
 *
 * Readings (the paper gives no more than the sentence above):
 *   R18 the subset is n_s draws WITH replacement; draw j is element
 *       floor(u_j * d / 2^32), u_j = the upper 32 bits of output j of the
 *       splitmix64 sequence started at `seed` (a counter-based generator, so
 *       the draws can be made in any order);
 *   R19 k_s = ceil(delta * n_s) (at least 1); the threshold is the k_s-th
 *       largest magnitude of the subset, bit patterns ordered as unsigned
 *       integers (a NaN sorts above infinity);
 *   R20 the first pass selects |acc| > threshold, strictly, in fp32, as C_eta;
 *   R21 k = ceil(delta * d); with more than k selected the k of largest
 *       magnitude stay (ties: lower index first here; any choice is valid);
 *       with k or fewer selected they all stay - no second threshold search.
 */
static uint64_t splitmix64_at(uint64_t seed, uint64_t j)
{
    /* output j (j = 0 is the first) of the sequence whose state starts at seed */
    uint64_t z = seed + (j + 1u) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
uint64_t sidco_oracle_splitmix64(uint64_t seed, uint64_t j) { return splitmix64_at(seed, j); }

int64_t sidco_oracle_dgc_sample_index(uint64_t seed, uint64_t j, int64_t d)
{
    uint64_t u = splitmix64_at(seed, j) >> 32;
    return (int64_t)((u * (uint64_t)d) >> 32);
}

static int u32_desc(const void *p, const void *q)
{
    uint32_t x = *(const uint32_t *)p, y = *(const uint32_t *)q;
    return (x < y) - (x > y);
}
static uint32_t mag_bits(float x)
{
    uint32_t b;
    memcpy(&b, &x, 4);
    return b & 0x7fffffffu;
}

static int dgc_above(float x, float eta) { return fabsf(x) > eta; } /* R20 */

/* g, r as in sidco_oracle_compress (r in/out, may be NULL).  idx/val have room
 * for k = ceil(delta*d) pairs; idx is written in ascending order.  Returns 0,
 * or -1 when out of memory.                                                  */
int sidco_oracle_dgc(const float *g, float *r, int64_t d, double delta, int64_t n_s,
                     uint64_t seed, int32_t *idx, float *val, int64_t *count,
                     float *eta_out, int64_t *first_pass)
{
    float *acc_own = NULL, *acc = r;
    if (!r) {
        acc_own = (float *)malloc((size_t)d * sizeof(float));
        if (!acc_own) return -1;
        acc = acc_own;
    }
    sidco_oracle_ec_add(g, r, d, acc);

    /* threshold from the subset */
    uint32_t *keys = (uint32_t *)malloc((size_t)n_s * sizeof(uint32_t));
    if (!keys) { free(acc_own); return -1; }
    for (int64_t j = 0; j < n_s; ++j)
        keys[j] = mag_bits(acc[sidco_oracle_dgc_sample_index(seed, (uint64_t)j, d)]);
    qsort(keys, (size_t)n_s, sizeof(uint32_t), u32_desc);
    int64_t k_s = (int64_t)ceil(delta * (double)n_s);
    if (k_s < 1) k_s = 1;
    if (k_s > n_s) k_s = n_s;
    uint32_t kappa = keys[k_s - 1];
    free(keys);
    float eta;
    memcpy(&eta, &kappa, 4);
    *eta_out = eta;

    /* first pass: everything above the threshold */
    int64_t k = (int64_t)ceil(delta * (double)d);
    if (k < 1) k = 1;
    if (k > d) k = d;
    int64_t n_sel = 0;
    for (int64_t j = 0; j < d; ++j)
        if (dgc_above(acc[j], eta)) ++n_sel;
    *first_pass = n_sel;

    mag_t *m = (mag_t *)malloc((size_t)(n_sel > 0 ? n_sel : 1) * sizeof(mag_t));
    if (!m) { free(acc_own); return -1; }
    int64_t n = 0;
    for (int64_t j = 0; j < d; ++j)
        if (dgc_above(acc[j], eta)) {
            m[n].a = fabsf(acc[j]);
            m[n].j = (int32_t)j;
            ++n;
        }
    /* second pass only if the first one selected too many */
    int64_t keep = n_sel;
    if (n_sel > k) {
        qsort(m, (size_t)n_sel, sizeof(mag_t), mag_cmp);
        keep = k;
    }
    for (int64_t i = 0; i < keep; ++i) idx[i] = m[i].j;
    free(m);
    qsort(idx, (size_t)keep, sizeof(int32_t), i32_cmp);
    for (int64_t i = 0; i < keep; ++i) {
        val[i] = acc[idx[i]];
        if (r) r[idx[i]] = 0.0f;
    }
    *count = keep;
    free(acc_own);
    return 0;
}
