"""CPU oracle of the SIDCo sparsifier: test infrastructure only.

Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may
import this package.  The GPU library never does.
"""
from .binding import (  # noqa: F401
    DIST_EXP,
    DIST_GAMMA_GPD,
    DIST_GPD,
    ST_NONFINITE,
    ST_VAR_ZERO,
    ST_GAMMA_S,
    ST_GAMMA_CLAMP,
    ST_STOPPED,
    DgcResult,
    OracleResult,
    adapt_stages,
    adaptive_run,
    build,
    compress,
    dgc,
    dgc_sample_indices,
    dgc_sizes,
    ec_add,
    eta_exp,
    eta_gamma,
    eta_gpd,
    gamma_shape,
    gpd_fit,
    moments_all,
    moments_pot,
    scatter_add,
    schedule,
    select,
    splitmix64,
    topk,
)
