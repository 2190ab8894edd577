"""ctypes binding of oracle/sidco_oracle.c (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import math
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sidco_oracle.c")
_LIB = os.path.join(_HERE, "libsidco_oracle.so")
# The mutation test points this at deliberately broken builds to show that the pins catch them.
_LIB_OVERRIDE = os.environ.get("SIDCO_ORACLE_LIB")

DIST_EXP, DIST_GAMMA_GPD, DIST_GPD = 0, 1, 2
ST_NONFINITE, ST_VAR_ZERO, ST_GAMMA_S, ST_GAMMA_CLAMP, ST_STOPPED = 1, 2, 4, 8, 16
MAX_STAGES = 8


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C99, -O2, no fast-math, no FMA contraction)."""
    if _LIB_OVERRIDE:
        return _LIB_OVERRIDE
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        f32p, f64p = C.POINTER(C.c_float), C.POINTER(C.c_double)
        i32p, i64p, u32p = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_uint32)
        lib.sidco_oracle_ec_add.argtypes = [f32p, f32p, C.c_int64, f32p]
        lib.sidco_oracle_ec_add.restype = None
        lib.sidco_oracle_schedule.argtypes = [C.c_double, C.c_int, C.c_double, f64p]
        lib.sidco_oracle_schedule.restype = C.c_int
        lib.sidco_oracle_moments_all.argtypes = [f32p, C.c_int64, f64p, f64p, f64p]
        lib.sidco_oracle_moments_all.restype = None
        lib.sidco_oracle_moments_pot.argtypes = [f32p, C.c_int64, C.c_float, f64p, f64p]
        lib.sidco_oracle_moments_pot.restype = C.c_int64
        lib.sidco_oracle_eta_exp.argtypes = [C.c_double, C.c_double]
        lib.sidco_oracle_eta_exp.restype = C.c_double
        lib.sidco_oracle_gpd_fit.argtypes = [C.c_double, C.c_double, f64p, f64p]
        lib.sidco_oracle_gpd_fit.restype = None
        lib.sidco_oracle_eta_gpd.argtypes = [C.c_double, C.c_double, C.c_double]
        lib.sidco_oracle_eta_gpd.restype = C.c_double
        lib.sidco_oracle_gamma_shape.argtypes = [C.c_double]
        lib.sidco_oracle_gamma_shape.restype = C.c_double
        lib.sidco_oracle_eta_gamma.argtypes = [C.c_double, C.c_double, C.c_double]
        lib.sidco_oracle_eta_gamma.restype = C.c_double
        lib.sidco_oracle_select.argtypes = [f32p, C.c_int64, C.c_float, i32p, f32p, f32p]
        lib.sidco_oracle_select.restype = C.c_int64
        lib.sidco_oracle_compress.argtypes = [f32p, f32p, C.c_int64, C.c_int, C.c_int, f64p, f32p,
                                              i32p, f32p, i64p, f32p, f32p, i64p, f64p, u32p]
        lib.sidco_oracle_compress.restype = C.c_int
        lib.sidco_oracle_adapt_stages.argtypes = [C.c_int, C.c_double, C.c_double, C.c_double, C.c_double, C.c_int]
        lib.sidco_oracle_adapt_stages.restype = C.c_int
        lib.sidco_oracle_scatter_add.argtypes = [f32p, C.c_int64, i32p, f32p, C.c_int64, C.c_float]
        lib.sidco_oracle_scatter_add.restype = C.c_int64
        lib.sidco_oracle_topk.argtypes = [f32p, C.c_int64, C.c_int64, i32p]
        lib.sidco_oracle_topk.restype = C.c_int64
        lib.sidco_oracle_splitmix64.argtypes = [C.c_uint64, C.c_uint64]
        lib.sidco_oracle_splitmix64.restype = C.c_uint64
        lib.sidco_oracle_dgc_sample_index.argtypes = [C.c_uint64, C.c_uint64, C.c_int64]
        lib.sidco_oracle_dgc_sample_index.restype = C.c_int64
        lib.sidco_oracle_dgc.argtypes = [f32p, f32p, C.c_int64, C.c_double, C.c_int64, C.c_uint64, i32p, f32p, i64p,
                                         f32p, i64p]
        lib.sidco_oracle_dgc.restype = C.c_int
        _lib = lib
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(C.POINTER(C.c_float))


def ec_add(g, r=None):
    g, gp = _f32(g)
    acc = np.empty_like(g)
    rp = None
    if r is not None:
        r, rp = _f32(r)
    _load().sidco_oracle_ec_add(gp, rp, g.size, acc.ctypes.data_as(C.POINTER(C.c_float)))
    return acc


def schedule(delta, stages, delta1=0.25):
    out = (C.c_double * MAX_STAGES)()
    m = _load().sidco_oracle_schedule(delta, stages, delta1, out)
    return [out[i] for i in range(m)]


def moments_all(acc):
    acc, p = _f32(acc)
    mu, var, ml = C.c_double(), C.c_double(), C.c_double()
    _load().sidco_oracle_moments_all(p, acc.size, C.byref(mu), C.byref(var), C.byref(ml))
    return mu.value, var.value, ml.value


def moments_pot(acc, eta_prev):
    acc, p = _f32(acc)
    yb, yv = C.c_double(), C.c_double()
    n = _load().sidco_oracle_moments_pot(p, acc.size, np.float32(eta_prev), C.byref(yb), C.byref(yv))
    return int(n), yb.value, yv.value


def eta_exp(mu, delta):
    return _load().sidco_oracle_eta_exp(mu, delta)


def gpd_fit(mu, var):
    a, b = C.c_double(), C.c_double()
    _load().sidco_oracle_gpd_fit(mu, var, C.byref(a), C.byref(b))
    return a.value, b.value


def eta_gpd(mu, var, delta):
    return _load().sidco_oracle_eta_gpd(mu, var, delta)


def gamma_shape(s):
    return _load().sidco_oracle_gamma_shape(s)


def eta_gamma(mu, mulog, delta):
    return _load().sidco_oracle_eta_gamma(mu, mulog, delta)


def select(acc, eta, residual=None):
    """C_eta on acc.  Returns (idx, val); zeroes `residual` (a float32 array holding acc) in place."""
    acc, p = _f32(acc)
    idx = np.empty(acc.size, dtype=np.int32)
    val = np.empty(acc.size, dtype=np.float32)
    rp = None
    if residual is not None:
        assert residual.dtype == np.float32 and residual.flags.c_contiguous
        rp = residual.ctypes.data_as(C.POINTER(C.c_float))
    k = _load().sidco_oracle_select(p, acc.size, np.float32(eta),
                                    idx.ctypes.data_as(C.POINTER(C.c_int32)),
                                    val.ctypes.data_as(C.POINTER(C.c_float)), rp)
    return idx[:k].copy(), val[:k].copy()


@dataclass
class OracleResult:
    idx: np.ndarray          # int32, ascending
    val: np.ndarray          # float32
    count: int
    eta: float               # threshold applied (eta_M)
    etas_own: np.ndarray     # float32[M], thresholds the oracle computed
    etas_used: np.ndarray    # float32[M], thresholds applied (own or injected)
    n_stage: np.ndarray      # int64[M], elements each stage's fit ran over
    stats: np.ndarray        # float64[M,3]
    status: int
    residual: np.ndarray | None  # updated residual (None when memoryless)


def compress(g, residual=None, *, ratios, dist=DIST_EXP, eta_inject=None) -> OracleResult:
    """Whole sparsifier.  `residual` is not modified; the updated copy is returned."""
    g, gp = _f32(g)
    d = g.size
    M = len(ratios)
    assert 1 <= M <= MAX_STAGES
    r = rp = None
    if residual is not None:
        r = np.array(residual, dtype=np.float32, copy=True)
        rp = r.ctypes.data_as(C.POINTER(C.c_float))
    rat = (C.c_double * M)(*ratios)
    inj = None
    if eta_inject is not None:
        inj_arr = np.ascontiguousarray(eta_inject, dtype=np.float32)
        assert inj_arr.size == M
        inj = inj_arr.ctypes.data_as(C.POINTER(C.c_float))
    idx = np.empty(max(d, 1), dtype=np.int32)
    val = np.empty(max(d, 1), dtype=np.float32)
    count = C.c_int64()
    own = np.zeros(M, dtype=np.float32)
    used = np.zeros(M, dtype=np.float32)
    ns = np.zeros(M, dtype=np.int64)
    stats = np.zeros((M, 3), dtype=np.float64)
    status = C.c_uint32()
    rc = _load().sidco_oracle_compress(
        gp, rp, d, dist, M, rat, inj,
        idx.ctypes.data_as(C.POINTER(C.c_int32)), val.ctypes.data_as(C.POINTER(C.c_float)),
        C.byref(count), own.ctypes.data_as(C.POINTER(C.c_float)),
        used.ctypes.data_as(C.POINTER(C.c_float)), ns.ctypes.data_as(C.POINTER(C.c_int64)),
        stats.ctypes.data_as(C.POINTER(C.c_double)), C.byref(status))
    if rc != 0:
        raise MemoryError("sidco_oracle_compress failed")
    k = count.value
    return OracleResult(idx[:k].copy(), val[:k].copy(), k, float(used[M - 1]), own, used, ns,
                        stats, status.value, r)


def topk(acc, k):
    acc, p = _f32(acc)
    idx = np.empty(max(min(k, acc.size), 1), dtype=np.int32)
    n = _load().sidco_oracle_topk(p, acc.size, k, idx.ctypes.data_as(C.POINTER(C.c_int32)))
    return idx[:n].copy()


def adapt_stages(M, khat_avg, k, eps_h=0.2, eps_l=0.2, M_max=MAX_STAGES):
    return _load().sidco_oracle_adapt_stages(M, khat_avg, k, eps_h, eps_l, M_max)


def adaptive_run(grads, residual, *, delta, dist, stages, max_stages=MAX_STAGES, Q=5, eps_h=0.2, eps_l=0.2,
                 delta1=0.25):
    """Algorithm 1 over consecutive iterations: compress with the current number of stages, carry the residual,
    and after every Q-th iteration adapt the number of stages from the average count of the window (R16).
    `grads` is an iterable of gradients.  Returns a list of (stages used, OracleResult) per iteration."""
    out = []
    M = stages
    acc = 0
    r = None if residual is None else np.array(residual, dtype=np.float32, copy=True)
    for i, g in enumerate(grads, start=1):
        res = compress(g, r, ratios=schedule(delta, M, delta1), dist=dist)
        out.append((M, res))
        if r is not None:
            r = res.residual
        acc += res.count
        if i % Q == 0:
            M = adapt_stages(M, acc / Q, delta * g.size, eps_h, eps_l, max_stages)
            acc = 0
    return out


def scatter_add(dense, idx, val, scale=1.0):
    """dense[idx] += scale * val in place (float32 array); returns the number of out-of-range indices skipped."""
    assert dense.dtype == np.float32 and dense.flags.c_contiguous
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    val = np.ascontiguousarray(val, dtype=np.float32)
    assert idx.size == val.size
    return int(_load().sidco_oracle_scatter_add(
        dense.ctypes.data_as(C.POINTER(C.c_float)), dense.size, idx.ctypes.data_as(C.POINTER(C.c_int32)),
        val.ctypes.data_as(C.POINTER(C.c_float)), idx.size, np.float32(scale)))


def splitmix64(seed, j):
    return int(_load().sidco_oracle_splitmix64(seed, j))


def dgc_sample_indices(seed, n_s, d):
    lib = _load()
    return np.array([lib.sidco_oracle_dgc_sample_index(seed, j, d) for j in range(n_s)], dtype=np.int64)


def dgc_sizes(d, delta, sample_ratio):
    """(n_s, k_s, k) of the DGC comparator (readings R18, R19, R21)."""
    n_s = min(max(int(math.ceil(sample_ratio * float(d))), 1), d)
    k_s = min(max(int(math.ceil(delta * float(n_s))), 1), n_s)
    k = min(max(int(math.ceil(delta * float(d))), 1), d)
    return n_s, k_s, k


@dataclass
class DgcResult:
    idx: np.ndarray          # ascending
    val: np.ndarray
    count: int
    eta: np.float32          # threshold from the subset
    first_pass: int          # entries above it, before the trim to k
    residual: np.ndarray | None


def dgc(g, residual=None, *, delta, sample_ratio=0.01, seed=0) -> DgcResult:
    """DGC's sampling threshold with the hierarchical trim (Sec. 1, related work and its footnote)."""
    g, gp = _f32(g)
    d = g.size
    n_s, _, k = dgc_sizes(d, delta, sample_ratio)
    r = rp = None
    if residual is not None:
        r = np.array(residual, dtype=np.float32, copy=True)
        rp = r.ctypes.data_as(C.POINTER(C.c_float))
    idx = np.empty(k, dtype=np.int32)
    val = np.empty(k, dtype=np.float32)
    count, first = C.c_int64(0), C.c_int64(0)
    eta = C.c_float(0)
    rc = _load().sidco_oracle_dgc(gp, rp, d, delta, n_s, seed, idx.ctypes.data_as(C.POINTER(C.c_int32)),
                                  val.ctypes.data_as(C.POINTER(C.c_float)), C.byref(count), C.byref(eta),
                                  C.byref(first))
    if rc != 0:
        raise MemoryError("sidco_oracle_dgc failed")
    n = count.value
    return DgcResult(idx[:n].copy(), val[:n].copy(), n, np.float32(eta.value), first.value, r)
