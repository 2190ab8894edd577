/* Runs the CPU oracle's entry points on small inputs, built together with oracle/sidco_oracle.c under
 * -fsanitize=address,undefined: out-of-bounds accesses, leaks and undefined arithmetic abort the run. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int sidco_oracle_schedule(double delta, int stages, double delta1, double *ratios);
int sidco_oracle_compress(const float *g, float *r, int64_t d, int dist, int M, const double *ratios,
                          const float *eta_inject, int32_t *idx, float *val, int64_t *count, float *etas_own,
                          float *etas_used, int64_t *n_stage, double *stats, uint32_t *status);
int64_t sidco_oracle_topk(const float *acc, int64_t d, int64_t k, int32_t *idx);
int sidco_oracle_adapt_stages(int M, double khat_avg, double k, double eps_h, double eps_l, int M_max);
int64_t sidco_oracle_scatter_add(float *dense, int64_t d, const int32_t *idx, const float *val, int64_t n, float scale);
int sidco_oracle_dgc(const float *g, float *r, int64_t d, double delta, int64_t n_s, uint64_t seed, int32_t *idx,
                     float *val, int64_t *count, float *eta_out, int64_t *first_pass);

static uint64_t state = 88172645463325252ull;
static double uniform(void)
{
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return (double)(state >> 11) / 9007199254740992.0;
}

int main(void)
{
    const int64_t sizes[] = {1, 2, 63, 257, 5000, 70001};
    int failures = 0;
    for (unsigned s = 0; s < sizeof sizes / sizeof sizes[0]; ++s) {
        const int64_t d = sizes[s];
        float *g = malloc((size_t)d * sizeof *g), *r = malloc((size_t)d * sizeof *r);
        float *acc = malloc((size_t)d * sizeof *acc), *res = malloc((size_t)d * sizeof *res);
        float *r0 = malloc((size_t)d * sizeof *r0);
        int32_t *idx = malloc((size_t)d * sizeof *idx);
        float *val = malloc((size_t)d * sizeof *val);
        for (int64_t j = 0; j < d; ++j) {
            const double u = uniform() - 0.5;
            g[j] = (float)((u < 0 ? 1.0 : -1.0) * 1e-3 * log(1.0 - 2.0 * fabs(u) + 1e-300));
            r0[j] = (float)(1e-4 * (uniform() - 0.5));
        }
        if (d > 10) {
            g[3] = 0.0f;
            g[7] = -0.0f;
        }
        for (int dist = 0; dist < 3; ++dist) {
            for (int stages = 1; stages <= 8; stages += 2) {
                double ratios[8];
                const int M = sidco_oracle_schedule(0.01, stages, 0.25, ratios);
                if (M < 1) {
                    ++failures;
                    continue;
                }
                float etas[8], etas_own[8];
                int64_t n_stage[8], count = -1;
                double stats[8 * 3];
                uint32_t status = 0;
                for (int64_t j = 0; j < d; ++j) r[j] = r0[j];   /* the residual is updated in place */
                const int rc = sidco_oracle_compress(g, (stages & 2) ? r : NULL, d, dist, M, ratios, NULL, idx, val, &count,
                                                     etas_own, etas, n_stage, stats, &status);
                if (rc != 0 || count < 0 || count > d) ++failures;
                for (int64_t i = 0; i < count; ++i)
                    if (idx[i] < 0 || idx[i] >= d || !(fabsf(val[i]) > etas[M - 1])) ++failures;
            }
        }
        const int64_t k = d / 3 + 1;
        if (sidco_oracle_topk(g, d, k, idx) != (k < d ? k : d)) ++failures;
        for (int64_t j = 0; j < d; ++j) acc[j] = 0.0f;
        if (sidco_oracle_scatter_add(acc, d, idx, g, 1, 0.5f) != 0) ++failures;
        {
            int64_t count = -1, first = -1;
            float eta = 0.0f;
            const int64_t n_s = d / 10 + 1;
            for (int64_t j = 0; j < d; ++j) r[j] = r0[j];
            if (sidco_oracle_dgc(g, r, d, 0.05, n_s, 42u, idx, val, &count, &eta, &first) != 0 || count < 0 || count > d) ++failures;
        }
        free(r0);
        free(g);
        free(r);
        free(acc);
        free(res);
        free(idx);
        free(val);
    }
    if (sidco_oracle_adapt_stages(2, 130.0, 100.0, 0.2, 0.2, 8) != 1) ++failures;
    if (sidco_oracle_adapt_stages(2, 70.0, 100.0, 0.2, 0.2, 8) != 3) ++failures;
    printf("oracle under sanitizers: %d failures\n", failures);
    return failures ? 1 : 0;
}
