"""Thin ctypes binding of libsidco.so: argument marshalling only.

Function names and argument order follow include/sidco.h.  Tensors are torch tensors on the GPU
(torch is used for device memory and streams, nothing else); every step of the sparsifier runs in
the library's HIP kernels.  There is no fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsidco.so")

MAX_STAGES = 8
DIST_EXP, DIST_GAMMA_GPD, DIST_GPD = 0, 1, 2
ST_NONFINITE, ST_VAR_ZERO, ST_GAMMA_S, ST_GAMMA_CLAMP, ST_STOPPED, ST_OVERFLOW, ST_FALLBACK = 1, 2, 4, 8, 16, 32, 64

EXPORTS = [
    "sidco_compress", "sidco_compress_static", "sidco_static_max_elements", "sidco_static_init", "sidco_compress_typed", "sidco_workspace_bytes_typed",
    "sidco_compress_batched_typed", "sidco_workspace_bytes_batched_typed", "sidco_controller_compress_typed", "sidco_topk_typed",
    "sidco_dgc_typed", "sidco_compress_ex", "sidco_compress_batched", "sidco_batched_out_offsets",
    "sidco_workspace_bytes_batched", "sidco_read_diag_batched", "sidco_topk", "sidco_dgc", "sidco_dgc_sizes", "sidco_dgc_result", "sidco_adapt_stages", "sidco_controller_create",
    "sidco_controller_destroy", "sidco_controller_stages", "sidco_controller_iteration",
    "sidco_controller_last_average", "sidco_controller_compress", "sidco_scatter_add", "sidco_scatter_check",
    "sidco_fit", "sidco_fit_typed", "sidco_fit_result", "sidco_stage_ratios", "sidco_out_capacity",
    "sidco_workspace_bytes", "sidco_set_workspace", "sidco_reserve", "sidco_release", "sidco_set_status_word",
    "sidco_set_delta1", "sidco_get_diag", "sidco_controller_disturbed",
    "sidco_set_speculation", "sidco_read_diag", "sidco_set_profiling",
    "sidco_get_profile", "sidco_strerror", "sidco_last_hip_error", "sidco_version", "sidco_shutdown",
]


class Diag(C.Structure):
    """Mirror of struct sidco_diag."""
    _fields_ = [
        ("eta", C.c_float * MAX_STAGES),
        ("n", C.c_int64 * MAX_STAGES),
        ("stats", (C.c_double * 3) * MAX_STAGES),
        ("selected", C.c_int64),
        ("count", C.c_int32),
        ("stages", C.c_int32),
        ("status", C.c_uint32),
        ("reserved", C.c_uint32),
    ]


class SidcoError(RuntimeError):
    def __init__(self, code: int, where: str):
        lib = load()
        msg = lib.sidco_strerror(code).decode()
        detail = lib.sidco_last_hip_error().decode()
        if code == -7 or (code == -2 and detail.startswith("sidco_compress_static")):
            msg += " (" + detail + ")"
        super().__init__(f"{where}: error {code}: {msg}")
        self.code = code


_lib = None


def load() -> C.CDLL:
    """Loads libsidco.so; raises if it has not been built (python -m paper_2101_10761_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2101_10761_amd.build` "
            "(there is no CPU or PyTorch fallback for the sparsifier)")
    # One HIP runtime per process: libsidco.so needs libamdhip64.so.7, and so does torch, which ships
    # its own copy.  Loading torch's first makes the dynamic linker resolve ours to the same object;
    # two runtimes in one process cannot both open the device.
    import torch
    bundled = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
    if os.path.exists(bundled):
        C.CDLL(bundled, mode=C.RTLD_GLOBAL)
    lib = C.CDLL(LIB_PATH)
    vp, f32p, i32p, f64p = C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_double)
    lib.sidco_compress.argtypes = [vp, f32p, f32p, C.c_int64, C.c_double, C.c_int, C.c_int, i32p, f32p, i32p, f32p]
    lib.sidco_compress.restype = C.c_int
    lib.sidco_compress_static.argtypes = [vp, f32p, f32p, C.c_int64, C.c_double, C.c_int, C.c_int, i32p, f32p, i32p, f32p]
    lib.sidco_compress_static.restype = C.c_int
    lib.sidco_static_init.argtypes = []
    lib.sidco_static_init.restype = C.c_int
    lib.sidco_static_max_elements.argtypes = []
    lib.sidco_static_max_elements.restype = C.c_int64
    lib.sidco_compress_ex.argtypes = [vp, f32p, f32p, C.c_int64, C.c_int, f64p, C.c_int, i32p, f32p, C.c_int64,
                                      i32p, f32p]
    lib.sidco_compress_ex.restype = C.c_int
    lib.sidco_compress_typed.argtypes = [vp, vp, C.c_int, f32p, C.c_int64, C.c_double, C.c_int, C.c_int, i32p, f32p,
                                         i32p, f32p]
    lib.sidco_compress_typed.restype = C.c_int
    lib.sidco_workspace_bytes_typed.argtypes = [C.c_int64, C.c_int, C.c_int]
    lib.sidco_workspace_bytes_typed.restype = C.c_size_t
    lib.sidco_topk.argtypes = [vp, f32p, f32p, C.c_int64, C.c_int64, i32p, f32p, i32p, f32p]
    lib.sidco_topk.restype = C.c_int
    lib.sidco_topk_typed.argtypes = [vp, vp, C.c_int, f32p, C.c_int64, C.c_int64, i32p, f32p, i32p, f32p]
    lib.sidco_topk_typed.restype = C.c_int
    i64p = C.POINTER(C.c_int64)
    lib.sidco_dgc.argtypes = [vp, f32p, f32p, C.c_int64, C.c_double, C.c_double, C.c_uint64, i32p, f32p, i32p, f32p]
    lib.sidco_dgc.restype = C.c_int
    lib.sidco_dgc_typed.argtypes = [vp, vp, C.c_int, f32p, C.c_int64, C.c_double, C.c_double, C.c_uint64, i32p, f32p, i32p,
                                    f32p]
    lib.sidco_dgc_typed.restype = C.c_int
    lib.sidco_compress_batched_typed.argtypes = [vp, vp, C.c_int, f32p, i64p, C.c_int, C.c_double, C.c_int, C.c_int, i32p,
                                                 f32p, i64p, i32p, f32p]
    lib.sidco_compress_batched_typed.restype = C.c_int
    lib.sidco_workspace_bytes_batched_typed.argtypes = [i64p, C.c_int, C.c_int, C.c_int]
    lib.sidco_workspace_bytes_batched_typed.restype = C.c_size_t
    lib.sidco_controller_compress_typed.argtypes = [C.c_void_p, vp, vp, C.c_int, f32p, C.c_int64, i32p, f32p, i32p, f32p]
    lib.sidco_controller_compress_typed.restype = C.c_int
    lib.sidco_dgc_sizes.argtypes = [C.c_int64, C.c_double, C.c_double, i64p]
    lib.sidco_dgc_sizes.restype = C.c_int
    lib.sidco_dgc_result.argtypes = [vp, i64p]
    lib.sidco_dgc_result.restype = C.c_int
    lib.sidco_compress_batched.argtypes = [vp, f32p, f32p, i64p, C.c_int, C.c_double, C.c_int, C.c_int, i32p, f32p,
                                           i64p, i32p, f32p]
    lib.sidco_compress_batched.restype = C.c_int
    lib.sidco_batched_out_offsets.argtypes = [i64p, C.c_int, C.c_double, i64p]
    lib.sidco_batched_out_offsets.restype = C.c_int
    lib.sidco_workspace_bytes_batched.argtypes = [i64p, C.c_int]
    lib.sidco_workspace_bytes_batched.restype = C.c_size_t
    lib.sidco_read_diag_batched.argtypes = [vp, C.c_int, C.POINTER(Diag)]
    lib.sidco_read_diag_batched.restype = C.c_int
    lib.sidco_adapt_stages.argtypes = [C.c_int, C.c_double, C.c_double, C.c_double, C.c_double, C.c_int]
    lib.sidco_adapt_stages.restype = C.c_int
    lib.sidco_controller_create.argtypes = [C.POINTER(C.c_void_p), C.c_double, C.c_int, C.c_int, C.c_int, C.c_int,
                                            C.c_double, C.c_double, C.c_double]
    lib.sidco_controller_create.restype = C.c_int
    lib.sidco_controller_destroy.argtypes = [C.c_void_p]
    lib.sidco_controller_destroy.restype = None
    lib.sidco_controller_stages.argtypes = [C.c_void_p]
    lib.sidco_controller_stages.restype = C.c_int
    lib.sidco_controller_iteration.argtypes = [C.c_void_p]
    lib.sidco_controller_iteration.restype = C.c_int64
    lib.sidco_controller_last_average.argtypes = [C.c_void_p]
    lib.sidco_controller_last_average.restype = C.c_double
    lib.sidco_controller_compress.argtypes = [C.c_void_p, vp, f32p, f32p, C.c_int64, i32p, f32p, i32p, f32p]
    lib.sidco_controller_compress.restype = C.c_int
    lib.sidco_scatter_add.argtypes = [vp, f32p, C.c_int64, i32p, f32p, i32p, C.c_int64, C.c_float]
    lib.sidco_scatter_add.restype = C.c_int
    lib.sidco_scatter_check.argtypes = [vp]
    lib.sidco_scatter_check.restype = C.c_int
    lib.sidco_fit.argtypes = [vp, f32p, f32p, C.c_int64, C.c_int]
    lib.sidco_fit.restype = C.c_int
    lib.sidco_fit_typed.argtypes = [vp, vp, C.c_int, f32p, C.c_int64, C.c_int]
    lib.sidco_fit_typed.restype = C.c_int
    lib.sidco_fit_result.argtypes = [vp, f64p]
    lib.sidco_fit_result.restype = C.c_int
    lib.sidco_stage_ratios.argtypes = [C.c_double, C.c_int, C.c_double, f64p]
    lib.sidco_stage_ratios.restype = C.c_int
    lib.sidco_out_capacity.argtypes = [C.c_int64, C.c_double]
    lib.sidco_out_capacity.restype = C.c_int64
    lib.sidco_workspace_bytes.argtypes = [C.c_int64]
    lib.sidco_workspace_bytes.restype = C.c_size_t
    lib.sidco_set_workspace.argtypes = [vp, C.c_size_t]
    lib.sidco_set_workspace.restype = C.c_int
    lib.sidco_reserve.argtypes = [vp, C.c_size_t]
    lib.sidco_reserve.restype = C.c_int
    lib.sidco_release.argtypes = [vp]
    lib.sidco_release.restype = C.c_int
    lib.sidco_set_status_word.argtypes = [vp, vp]
    lib.sidco_set_status_word.restype = C.c_int
    lib.sidco_set_delta1.argtypes = [C.c_double]
    lib.sidco_set_delta1.restype = C.c_int
    lib.sidco_get_diag.argtypes = [vp, C.POINTER(Diag)]
    lib.sidco_get_diag.restype = C.c_int
    lib.sidco_controller_disturbed.argtypes = [C.c_void_p]
    lib.sidco_controller_disturbed.restype = C.c_int64
    lib.sidco_set_speculation.argtypes = [C.c_double]
    lib.sidco_set_speculation.restype = C.c_int
    lib.sidco_read_diag.argtypes = [vp, C.POINTER(Diag)]
    lib.sidco_read_diag.restype = C.c_int
    lib.sidco_set_profiling.argtypes = [C.c_int]
    lib.sidco_set_profiling.restype = C.c_int
    lib.sidco_get_profile.argtypes = [C.POINTER(C.c_float), C.POINTER(C.c_char_p), C.c_int]
    lib.sidco_get_profile.restype = C.c_int
    lib.sidco_strerror.argtypes = [C.c_int]
    lib.sidco_strerror.restype = C.c_char_p
    lib.sidco_last_hip_error.argtypes = []
    lib.sidco_last_hip_error.restype = C.c_char_p
    lib.sidco_version.argtypes = []
    lib.sidco_version.restype = C.c_int
    lib.sidco_shutdown.argtypes = []
    lib.sidco_shutdown.restype = None
    _lib = lib
    return lib


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise SidcoError(rc, where)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream_handle(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _check_tensor(t, dtype, name, n=None):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous CUDA tensor of dtype {dtype}")
    if n is not None and t.numel() < n:
        raise ValueError(f"{name} has {t.numel()} elements, needs {n}")


def sidco_stage_ratios(delta: float, stages: int, delta1: float = 0.25) -> list[float]:
    out = (C.c_double * MAX_STAGES)()
    m = load().sidco_stage_ratios(delta, stages, delta1, out)
    if m < 1:
        raise SidcoError(m, "sidco_stage_ratios")
    return [out[i] for i in range(m)]


def sidco_out_capacity(d: int, delta: float) -> int:
    cap = load().sidco_out_capacity(d, delta)
    if cap < 0:
        raise SidcoError(int(cap), "sidco_out_capacity")
    return int(cap)


def sidco_workspace_bytes(d: int) -> int:
    return int(load().sidco_workspace_bytes(d))


def sidco_workspace_bytes_typed(d: int, grad_dtype: int, has_residual: bool) -> int:
    return int(load().sidco_workspace_bytes_typed(d, grad_dtype, 1 if has_residual else 0))


def sidco_set_workspace(buf) -> None:
    """buf: a CUDA uint8 tensor the caller keeps alive, or None to return to library allocation."""
    if buf is None:
        _check(load().sidco_set_workspace(None, 0), "sidco_set_workspace")
    else:
        _check(load().sidco_set_workspace(C.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size()),
               "sidco_set_workspace")


def sidco_reserve(nbytes: int, stream=None) -> None:
    """Grows the library's own workspace of `stream` to at least nbytes (see sidco_workspace_bytes)."""
    _check(load().sidco_reserve(_stream_handle(stream), int(nbytes)), "sidco_reserve")


def sidco_release(stream=None) -> None:
    _check(load().sidco_release(_stream_handle(stream)), "sidco_release")


def sidco_set_status_word(word, stream=None) -> None:
    """word: a CUDA uint32/int32 tensor of one element that receives the status bits of every call on
    `stream`, or None to switch that off."""
    _check(load().sidco_set_status_word(_stream_handle(stream), _ptr(word)), "sidco_set_status_word")


def sidco_set_delta1(delta1: float) -> None:
    _check(load().sidco_set_delta1(float(delta1)), "sidco_set_delta1")


def sidco_compress(grad, residual, delta: float, dist: int, stages: int, out_idx, out_val, out_count, out_eta,
                   stream=None) -> None:
    """Enqueues one sparsifier call; see include/sidco.h.  `residual` may be None."""
    import torch
    d = grad.numel()
    _check_tensor(grad, torch.float32, "grad")
    if residual is not None:
        _check_tensor(residual, torch.float32, "residual", d)
    cap = sidco_out_capacity(d, delta)
    _check_tensor(out_idx, torch.int32, "out_idx", cap)
    _check_tensor(out_val, torch.float32, "out_val", cap)
    _check_tensor(out_count, torch.int32, "out_count", 1)
    _check_tensor(out_eta, torch.float32, "out_eta", 1)
    _check(load().sidco_compress(_stream_handle(stream), _ptr(grad), _ptr(residual), d, delta, dist, stages,
                                 _ptr(out_idx), _ptr(out_val), _ptr(out_count), _ptr(out_eta)), "sidco_compress")


def sidco_compress_static(grad, residual, delta: float, dist: int, stages: int, out_idx, out_val, out_count, out_eta,
                          stream=None) -> None:
    """sidco_compress in the library's static scratch: no device allocation; d <= sidco_static_max_elements()."""
    import torch
    d = grad.numel()
    _check_tensor(grad, torch.float32, "grad")
    if residual is not None:
        _check_tensor(residual, torch.float32, "residual", d)
    cap = sidco_out_capacity(d, delta)
    _check_tensor(out_idx, torch.int32, "out_idx", cap)
    _check_tensor(out_val, torch.float32, "out_val", cap)
    _check_tensor(out_count, torch.int32, "out_count", 1)
    _check_tensor(out_eta, torch.float32, "out_eta", 1)
    _check(load().sidco_compress_static(_stream_handle(stream), _ptr(grad), _ptr(residual), d, delta, dist, stages,
                                        _ptr(out_idx), _ptr(out_val), _ptr(out_count), _ptr(out_eta)),
           "sidco_compress_static")


def sidco_static_init() -> None:
    _check(load().sidco_static_init(), "sidco_static_init")


def sidco_static_max_elements() -> int:
    return int(load().sidco_static_max_elements())


GRAD_F32, GRAD_F16, GRAD_BF16 = 0, 1, 2


def sidco_compress_typed(grad, residual, delta: float, dist: int, stages: int, out_idx, out_val, out_count, out_eta,
                         stream=None) -> None:
    """sidco_compress on a gradient tensor of dtype float32, float16 or bfloat16 (the residual stays float32)."""
    import torch
    codes = {torch.float32: GRAD_F32, torch.float16: GRAD_F16, torch.bfloat16: GRAD_BF16}
    if not isinstance(grad, torch.Tensor) or grad.dtype not in codes:
        raise TypeError("grad must be a CUDA tensor of dtype float32, float16 or bfloat16")
    d = grad.numel()
    _check_tensor(grad, grad.dtype, "grad")
    if residual is not None:
        _check_tensor(residual, torch.float32, "residual", d)
    cap = sidco_out_capacity(d, delta)
    _check_tensor(out_idx, torch.int32, "out_idx", cap)
    _check_tensor(out_val, torch.float32, "out_val", cap)
    _check_tensor(out_count, torch.int32, "out_count", 1)
    _check_tensor(out_eta, torch.float32, "out_eta", 1)
    _check(load().sidco_compress_typed(_stream_handle(stream), _ptr(grad), codes[grad.dtype], _ptr(residual), d, delta,
                                       dist, stages, _ptr(out_idx), _ptr(out_val), _ptr(out_count), _ptr(out_eta)),
           "sidco_compress_typed")


def sidco_compress_ex(grad, residual, dist: int, ratios, out_idx, out_val, out_count, out_eta, stream=None) -> None:
    """Explicit stage ratios; the output capacity is min(len(out_idx), len(out_val))."""
    import torch
    d = grad.numel()
    _check_tensor(grad, torch.float32, "grad")
    if residual is not None:
        _check_tensor(residual, torch.float32, "residual", d)
    _check_tensor(out_idx, torch.int32, "out_idx", 1)
    _check_tensor(out_val, torch.float32, "out_val", 1)
    _check_tensor(out_count, torch.int32, "out_count", 1)
    _check_tensor(out_eta, torch.float32, "out_eta", 1)
    cap = min(out_idx.numel(), out_val.numel())
    r = (C.c_double * len(ratios))(*ratios)
    _check(load().sidco_compress_ex(_stream_handle(stream), _ptr(grad), _ptr(residual), d, dist, r, len(ratios),
                                    _ptr(out_idx), _ptr(out_val), cap, _ptr(out_count), _ptr(out_eta)),
           "sidco_compress_ex")


def _i64_array(values):
    return (C.c_int64 * len(values))(*[int(v) for v in values])


def sidco_batched_out_offsets(offsets, delta: float) -> list[int]:
    """Default placement of the tensors' outputs: sidco_out_capacity pairs each, back to back."""
    n = len(offsets) - 1
    out = (C.c_int64 * (n + 1))()
    _check(load().sidco_batched_out_offsets(_i64_array(offsets), n, delta, out), "sidco_batched_out_offsets")
    return [out[i] for i in range(n + 1)]


def sidco_workspace_bytes_batched(offsets) -> int:
    return int(load().sidco_workspace_bytes_batched(_i64_array(offsets), len(offsets) - 1))


def sidco_compress_batched(grad, residual, offsets, delta: float, dist: int, stages: int, out_idx, out_val, out_offsets,
                           out_counts, out_etas, stream=None) -> None:
    """Enqueues one sparsifier call per tensor of the flat buffer, all in one launch sequence; see include/sidco.h."""
    import torch
    n = len(offsets) - 1
    _check_tensor(grad, torch.float32, "grad", offsets[-1])
    if residual is not None:
        _check_tensor(residual, torch.float32, "residual", offsets[-1])
    _check_tensor(out_idx, torch.int32, "out_idx", out_offsets[-1])
    _check_tensor(out_val, torch.float32, "out_val", out_offsets[-1])
    _check_tensor(out_counts, torch.int32, "out_counts", n)
    _check_tensor(out_etas, torch.float32, "out_etas", n)
    _check(load().sidco_compress_batched(_stream_handle(stream), _ptr(grad), _ptr(residual), _i64_array(offsets), n, delta,
                                         dist, stages, _ptr(out_idx), _ptr(out_val), _i64_array(out_offsets),
                                         _ptr(out_counts), _ptr(out_etas)), "sidco_compress_batched")


def sidco_read_diag_batched(t: int, stream=None) -> Diag:
    diag = Diag()
    _check(load().sidco_read_diag_batched(_stream_handle(stream), t, C.byref(diag)), "sidco_read_diag_batched")
    return diag


def sidco_topk(grad, residual, k: int, out_idx, out_val, out_count, out_kth, stream=None) -> None:
    """Enqueues the exact Top-k comparator; see include/sidco.h.  `residual` may be None."""
    import torch
    d = grad.numel()
    _check_tensor(grad, torch.float32, "grad")
    if residual is not None:
        _check_tensor(residual, torch.float32, "residual", d)
    _check_tensor(out_idx, torch.int32, "out_idx", k)
    _check_tensor(out_val, torch.float32, "out_val", k)
    _check_tensor(out_count, torch.int32, "out_count", 1)
    _check_tensor(out_kth, torch.float32, "out_kth", 1)
    _check(load().sidco_topk(_stream_handle(stream), _ptr(grad), _ptr(residual), d, k, _ptr(out_idx), _ptr(out_val),
                             _ptr(out_count), _ptr(out_kth)), "sidco_topk")


def sidco_dgc_sizes(d: int, delta: float, sample_ratio: float = 0.01):
    """(n_s, k_s, k) of the DGC comparator for a vector of d elements."""
    sizes = (C.c_int64 * 3)()
    _check(load().sidco_dgc_sizes(d, delta, sample_ratio, sizes), "sidco_dgc_sizes")
    return int(sizes[0]), int(sizes[1]), int(sizes[2])


def sidco_dgc(grad, residual, delta: float, sample_ratio: float, seed: int, out_idx, out_val, out_count, out_eta,
              stream=None) -> None:
    """Enqueues the DGC comparator; see include/sidco.h.  `residual` may be None."""
    import torch
    d = grad.numel()
    _check_tensor(grad, torch.float32, "grad")
    if residual is not None:
        _check_tensor(residual, torch.float32, "residual", d)
    k = sidco_dgc_sizes(d, delta, sample_ratio)[2]
    _check_tensor(out_idx, torch.int32, "out_idx", k)
    _check_tensor(out_val, torch.float32, "out_val", k)
    _check_tensor(out_count, torch.int32, "out_count", 1)
    _check_tensor(out_eta, torch.float32, "out_eta", 1)
    _check(load().sidco_dgc(_stream_handle(stream), _ptr(grad), _ptr(residual), d, delta, sample_ratio, seed,
                            _ptr(out_idx), _ptr(out_val), _ptr(out_count), _ptr(out_eta)), "sidco_dgc")


def _grad_code(grad):
    """SIDCO_GRAD_* of a gradient tensor (float32, float16 or bfloat16)."""
    import torch
    codes = {torch.float32: GRAD_F32, torch.float16: GRAD_F16, torch.bfloat16: GRAD_BF16}
    if not isinstance(grad, torch.Tensor) or grad.dtype not in codes:
        raise TypeError("grad must be a CUDA tensor of dtype float32, float16 or bfloat16")
    _check_tensor(grad, grad.dtype, "grad")
    return codes[grad.dtype]


def sidco_topk_typed(grad, residual, k: int, out_idx, out_val, out_count, out_kth, stream=None) -> None:
    """sidco_topk on a gradient tensor of dtype float32, float16 or bfloat16 (the residual stays float32)."""
    import torch
    code = _grad_code(grad)
    d = grad.numel()
    if residual is not None:
        _check_tensor(residual, torch.float32, "residual", d)
    _check_tensor(out_idx, torch.int32, "out_idx", k)
    _check_tensor(out_val, torch.float32, "out_val", k)
    _check_tensor(out_count, torch.int32, "out_count", 1)
    _check_tensor(out_kth, torch.float32, "out_kth", 1)
    _check(load().sidco_topk_typed(_stream_handle(stream), _ptr(grad), code, _ptr(residual), d, k, _ptr(out_idx),
                                   _ptr(out_val), _ptr(out_count), _ptr(out_kth)), "sidco_topk_typed")


def sidco_dgc_typed(grad, residual, delta: float, sample_ratio: float, seed: int, out_idx, out_val, out_count, out_eta,
                    stream=None) -> None:
    """sidco_dgc on a gradient tensor of dtype float32, float16 or bfloat16 (the residual stays float32)."""
    import torch
    code = _grad_code(grad)
    d = grad.numel()
    if residual is not None:
        _check_tensor(residual, torch.float32, "residual", d)
    k = sidco_dgc_sizes(d, delta, sample_ratio)[2]
    _check_tensor(out_idx, torch.int32, "out_idx", k)
    _check_tensor(out_val, torch.float32, "out_val", k)
    _check_tensor(out_count, torch.int32, "out_count", 1)
    _check_tensor(out_eta, torch.float32, "out_eta", 1)
    _check(load().sidco_dgc_typed(_stream_handle(stream), _ptr(grad), code, _ptr(residual), d, delta, sample_ratio, seed,
                                  _ptr(out_idx), _ptr(out_val), _ptr(out_count), _ptr(out_eta)), "sidco_dgc_typed")


def sidco_compress_batched_typed(grad, residual, offsets, delta: float, dist: int, stages: int, out_idx, out_val,
                                 out_offsets, out_counts, out_etas, stream=None) -> None:
    """sidco_compress_batched on a gradient buffer of dtype float32, float16 or bfloat16."""
    import torch
    code = _grad_code(grad)
    n = len(offsets) - 1
    if grad.numel() < offsets[-1]:
        raise ValueError(f"grad has {grad.numel()} elements, needs {offsets[-1]}")
    if residual is not None:
        _check_tensor(residual, torch.float32, "residual", offsets[-1])
    _check_tensor(out_idx, torch.int32, "out_idx", out_offsets[-1])
    _check_tensor(out_val, torch.float32, "out_val", out_offsets[-1])
    _check_tensor(out_counts, torch.int32, "out_counts", n)
    _check_tensor(out_etas, torch.float32, "out_etas", n)
    _check(load().sidco_compress_batched_typed(_stream_handle(stream), _ptr(grad), code, _ptr(residual),
                                               _i64_array(offsets), n, delta, dist, stages, _ptr(out_idx), _ptr(out_val),
                                               _i64_array(out_offsets), _ptr(out_counts), _ptr(out_etas)),
           "sidco_compress_batched_typed")


def sidco_workspace_bytes_batched_typed(offsets, grad_dtype: int, has_residual: bool) -> int:
    return int(load().sidco_workspace_bytes_batched_typed(_i64_array(offsets), len(offsets) - 1, grad_dtype,
                                                          1 if has_residual else 0))


def sidco_dgc_result(stream=None):
    """(n_s, k_s, first-pass count, entries written) of the last sidco_dgc; synchronises the stream."""
    out = (C.c_int64 * 4)()
    _check(load().sidco_dgc_result(_stream_handle(stream), out), "sidco_dgc_result")
    return tuple(int(v) for v in out)


def sidco_adapt_stages(stages: int, khat_avg: float, k: float, eps_high: float = 0.2, eps_low: float = 0.2,
                       max_stages: int = MAX_STAGES) -> int:
    m = load().sidco_adapt_stages(stages, khat_avg, k, eps_high, eps_low, max_stages)
    if m < 1:
        raise SidcoError(m, "sidco_adapt_stages")
    return m


class Controller:
    """Handle of a sidco_controller (the sparsifier with its stage controller); see include/sidco.h."""

    def __init__(self, delta: float, dist: int, stages: int = 1, max_stages: int = MAX_STAGES, Q: int = 5,
                 eps_high: float = 0.2, eps_low: float = 0.2, delta1: float = 0.25):
        self._h = C.c_void_p()
        _check(load().sidco_controller_create(C.byref(self._h), delta, dist, stages, max_stages, Q, eps_high, eps_low,
                                              delta1), "sidco_controller_create")
        self.delta = delta

    def close(self):
        if self._h:
            load().sidco_controller_destroy(self._h)
            self._h = C.c_void_p()

    __del__ = close

    @property
    def stages(self) -> int:
        return load().sidco_controller_stages(self._h)

    @property
    def iteration(self) -> int:
        return load().sidco_controller_iteration(self._h)

    @property
    def last_average(self) -> float:
        return load().sidco_controller_last_average(self._h)

    @property
    def disturbed(self) -> int:
        """Windows whose count another caller of the same workspace broke (the stages were left as they were)."""
        return int(load().sidco_controller_disturbed(self._h))

    def compress(self, grad, residual, out_idx, out_val, out_count, out_eta, stream=None) -> None:
        """One iteration; `grad` may be float32 (sidco_controller_compress) or float16 / bfloat16
        (sidco_controller_compress_typed)."""
        import torch
        d = grad.numel()
        code = _grad_code(grad)
        if residual is not None:
            _check_tensor(residual, torch.float32, "residual", d)
        cap = sidco_out_capacity(d, self.delta)
        _check_tensor(out_idx, torch.int32, "out_idx", cap)
        _check_tensor(out_val, torch.float32, "out_val", cap)
        _check_tensor(out_count, torch.int32, "out_count", 1)
        _check_tensor(out_eta, torch.float32, "out_eta", 1)
        if code == GRAD_F32:
            _check(load().sidco_controller_compress(self._h, _stream_handle(stream), _ptr(grad), _ptr(residual), d,
                                                    _ptr(out_idx), _ptr(out_val), _ptr(out_count), _ptr(out_eta)),
                   "sidco_controller_compress")
        else:
            _check(load().sidco_controller_compress_typed(self._h, _stream_handle(stream), _ptr(grad), code,
                                                          _ptr(residual), d, _ptr(out_idx), _ptr(out_val),
                                                          _ptr(out_count), _ptr(out_eta)),
                   "sidco_controller_compress_typed")


def sidco_scatter_add(dense, idx, val, count, scale: float = 1.0, stream=None) -> None:
    """dense[idx[i]] += scale * val[i] for i < count (a device scalar); see include/sidco.h."""
    import torch
    _check_tensor(dense, torch.float32, "dense")
    _check_tensor(idx, torch.int32, "idx", 1)
    _check_tensor(val, torch.float32, "val", 1)
    _check_tensor(count, torch.int32, "count", 1)
    cap = min(idx.numel(), val.numel())
    _check(load().sidco_scatter_add(_stream_handle(stream), _ptr(dense), dense.numel(), _ptr(idx), _ptr(val), _ptr(count),
                                    cap, scale), "sidco_scatter_add")


def sidco_scatter_check(stream=None) -> bool:
    rc = load().sidco_scatter_check(_stream_handle(stream))
    if rc < 0:
        raise SidcoError(rc, "sidco_scatter_check")
    return bool(rc)


def sidco_fit(grad, residual, dist: int, stream=None) -> None:
    """Enqueues steps 1-2 alone (error-compensation add fused with the stage-1 sums); the gradient may be
    float32, float16 or bfloat16."""
    import torch
    codes = {torch.float32: GRAD_F32, torch.float16: GRAD_F16, torch.bfloat16: GRAD_BF16}
    if not isinstance(grad, torch.Tensor) or grad.dtype not in codes:
        raise TypeError("grad must be a CUDA tensor of dtype float32, float16 or bfloat16")
    _check_tensor(grad, grad.dtype, "grad")
    if residual is not None:
        _check_tensor(residual, torch.float32, "residual", grad.numel())
    _check(load().sidco_fit_typed(_stream_handle(stream), _ptr(grad), codes[grad.dtype], _ptr(residual), grad.numel(),
                                  dist), "sidco_fit")


def sidco_fit_result(stream=None) -> tuple[float, float, float, float]:
    """(sum|acc|, sum acc^2, sum log|acc|, d) of the last sidco_fit; synchronises."""
    out = (C.c_double * 4)()
    _check(load().sidco_fit_result(_stream_handle(stream), out), "sidco_fit_result")
    return out[0], out[1], out[2], out[3]


def sidco_set_speculation(theta: float) -> None:
    """Position of a dense stage's candidate threshold (0 = lists of all exceedances); see include/sidco.h."""
    _check(load().sidco_set_speculation(float(theta)), "sidco_set_speculation")


def sidco_read_diag(stream=None) -> Diag:
    diag = Diag()
    _check(load().sidco_read_diag(_stream_handle(stream), C.byref(diag)), "sidco_read_diag")
    return diag


def sidco_get_diag(stream=None) -> Diag:
    """The same call under its other exported name."""
    diag = Diag()
    _check(load().sidco_get_diag(_stream_handle(stream), C.byref(diag)), "sidco_get_diag")
    return diag


def sidco_set_profiling(enable: bool) -> None:
    _check(load().sidco_set_profiling(int(bool(enable))), "sidco_set_profiling")


def sidco_get_profile() -> list[tuple[str, float]]:
    """Per-kernel (name, milliseconds) of the last profiled call on the current device."""
    ms = (C.c_float * 16)()
    names = (C.c_char_p * 16)()
    n = load().sidco_get_profile(ms, names, 16)
    if n < 0:
        raise SidcoError(n, "sidco_get_profile")
    return [(names[i].decode(), float(ms[i])) for i in range(n)]


def sidco_version() -> int:
    return load().sidco_version()


def sidco_shutdown() -> None:
    load().sidco_shutdown()
