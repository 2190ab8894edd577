"""Host-side checks of the C-ABI library that need no GPU: it loads, exports what the header declares,
rejects bad arguments before touching HIP, and its host helpers agree with the oracle's schedule."""
import ctypes as C
import math
import os
import re
import subprocess

import pytest

import paper_2101_10761_amd as sidco
from paper_2101_10761_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sidco.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2101_10761_amd import build
        build.build()
    return sidco.load()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sidco_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert "sidco_compress" in names and len(names) >= 10
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/sidco.h but not exported"
    assert sorted(binding.EXPORTS) == names


def test_diag_struct_layout_matches_header(tmp_path):
    src = tmp_path / "layout.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "sidco.h"\n'
                   'int main(void){printf("%zu %zu %zu %zu %zu %zu %zu\\n", sizeof(sidco_diag),'
                   'offsetof(sidco_diag,n), offsetof(sidco_diag,stats), offsetof(sidco_diag,selected),'
                   'offsetof(sidco_diag,count), offsetof(sidco_diag,stages), offsetof(sidco_diag,status));return 0;}\n')
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(src)], check=True)
    got = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    D = binding.Diag
    assert got == [C.sizeof(D), D.n.offset, D.stats.offset, D.selected.offset, D.count.offset, D.stages.offset,
                   D.status.offset]


def test_argument_errors_are_caught_on_the_host(lib):
    ok = C.c_void_p(256)   # never dereferenced: every call below must fail before any HIP call
    f = lib.sidco_compress
    base = dict(stream=None, grad=ok, residual=None, d=1000, delta=0.01, dist=0, stages=2,
                out_idx=ok, out_val=ok, out_count=ok, out_eta=ok)

    def call(**kw):
        a = dict(base, **kw)
        return f(a["stream"], a["grad"], a["residual"], a["d"], a["delta"], a["dist"], a["stages"],
                 a["out_idx"], a["out_val"], a["out_count"], a["out_eta"])

    assert call(grad=None) == -1
    assert call(out_idx=None) == -1 and call(out_val=None) == -1
    assert call(out_count=None) == -1 and call(out_eta=None) == -1
    assert call(d=0) == -2 and call(d=-5) == -2 and call(d=2 ** 31) == -2
    for bad in (0.0, 1.0, -0.1, 1.5, math.nan):
        assert call(delta=bad) == -3
    assert call(stages=0) == -4 and call(stages=9) == -4
    assert call(dist=3) == -5 and call(dist=-1) == -5
    assert call(grad=C.c_void_p(258)) == -8 and call(residual=C.c_void_p(1026)) == -8
    assert call(residual=ok) == -9          # residual aliases grad
    g = lib.sidco_compress_ex
    r2 = (C.c_double * 2)(0.25, 0.04)
    assert g(None, ok, None, 1000, 0, None, 2, ok, ok, 100, ok, ok) == -1
    assert g(None, ok, None, 1000, 0, r2, 0, ok, ok, 100, ok, ok) == -4
    assert g(None, ok, None, 1000, 0, r2, 9, ok, ok, 100, ok, ok) == -4
    assert g(None, ok, None, 1000, 0, r2, 2, ok, ok, 0, ok, ok) == -2
    assert g(None, ok, None, 1000, 0, (C.c_double * 2)(0.25, 1.0), 2, ok, ok, 100, ok, ok) == -3
    t = lib.sidco_topk
    assert t(None, None, None, 1000, 10, ok, ok, ok, ok) == -1
    assert t(None, ok, None, 1000, 10, ok, ok, ok, None) == -1
    assert t(None, ok, None, 0, 10, ok, ok, ok, ok) == -2
    assert t(None, ok, None, 1000, 0, ok, ok, ok, ok) == -2 and t(None, ok, None, 1000, 1001, ok, ok, ok, ok) == -2
    assert t(None, C.c_void_p(258), None, 1000, 10, ok, ok, ok, ok) == -8
    assert t(None, ok, ok, 1000, 10, ok, ok, ok, ok) == -9
    assert lib.sidco_set_workspace(C.c_void_p(100), 1 << 20) == -6      # misaligned
    assert lib.sidco_set_workspace(C.c_void_p(256), 16) == -6           # too small
    assert lib.sidco_read_diag(None, None) == -1
    for bad in (-0.1, 1.5, math.nan):
        assert lib.sidco_set_speculation(C.c_double(bad)) == -9
    assert lib.sidco_set_speculation(C.c_double(0.5)) == 0
    for code in range(-9, 1):
        assert lib.sidco_strerror(code)
    assert lib.sidco_version() >= 100


def test_host_helpers(lib, oracle):
    for delta, stages, d1 in ((0.001, 3, 0.25), (0.001, 2, 0.05), (0.1, 3, 0.25), (0.3, 4, 0.25), (1e-4, 8, 0.25),
                              (0.01, 1, 0.25)):
        assert sidco.sidco_stage_ratios(delta, stages, d1) == pytest.approx(oracle.schedule(delta, stages, d1),
                                                                           rel=1e-15)
    with pytest.raises(sidco.SidcoError):
        sidco.sidco_stage_ratios(0.0, 2)
    with pytest.raises(sidco.SidcoError):
        sidco.sidco_stage_ratios(0.01, 0)
    assert sidco.sidco_out_capacity(25_557_032, 0.001) == 4 * 25_558 + 4096
    assert sidco.sidco_out_capacity(1000, 0.5) == 1000
    with pytest.raises(sidco.SidcoError):
        sidco.sidco_out_capacity(0, 0.5)
    assert sidco.sidco_workspace_bytes(0) == 0
    w = sidco.sidco_workspace_bytes(25_557_032)
    assert w % 256 == 0 and w >= 2 * 8 * 25_557_032


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libsidco.so"))
    with pytest.raises(FileNotFoundError):
        binding.load()


def test_controller_argument_errors(lib):
    h = C.c_void_p()
    f = lib.sidco_controller_create
    assert f(None, 0.01, 0, 1, 8, 5, 0.2, 0.2, 0.25) == -1
    assert f(C.byref(h), 0.0, 0, 1, 8, 5, 0.2, 0.2, 0.25) == -3
    assert f(C.byref(h), 0.01, 7, 1, 8, 5, 0.2, 0.2, 0.25) == -5
    assert f(C.byref(h), 0.01, 0, 9, 8, 5, 0.2, 0.2, 0.25) == -4
    assert f(C.byref(h), 0.01, 0, 1, 8, 0, 0.2, 0.2, 0.25) == -9
    assert f(C.byref(h), 0.01, 0, 1, 8, 5, -0.2, 0.2, 0.25) == -9
    assert not h.value


def test_adapt_stages_matches_the_oracle(lib, oracle):
    for M in (1, 2, 5, 8):
        for avg in (0.0, 10.0, 799.0, 800.0, 1000.0, 1200.0, 1201.0, 1e6):
            for eh, el, mmax in ((0.2, 0.2, 8), (0.1, 0.3, 8), (0.2, 0.2, 5)):
                if M > mmax:
                    continue
                assert sidco.sidco_adapt_stages(M, avg, 1000.0, eh, el, mmax) == oracle.adapt_stages(M, avg, 1000.0, eh, el, mmax)
    assert lib.sidco_adapt_stages(0, 1.0, 1.0, 0.2, 0.2, 8) == -4
    assert lib.sidco_adapt_stages(1, 1.0, 0.0, 0.2, 0.2, 8) == -9
    assert lib.sidco_adapt_stages(1, 1.0, 1.0, 0.2, 1.0, 8) == -9


def test_batched_argument_errors_and_helpers(lib):
    ok = C.c_void_p(256)
    off = (C.c_int64 * 3)(0, 1000, 3000)
    oo = (C.c_int64 * 3)(0, 100, 300)
    f = lib.sidco_compress_batched
    assert f(None, None, None, off, 2, 0.01, 0, 2, ok, ok, oo, ok, ok) == -1
    assert f(None, ok, None, None, 2, 0.01, 0, 2, ok, ok, oo, ok, ok) == -1
    assert f(None, ok, None, off, 0, 0.01, 0, 2, ok, ok, oo, ok, ok) == -2
    assert f(None, ok, None, off, 513, 0.01, 0, 2, ok, ok, oo, ok, ok) == -2
    assert f(None, ok, None, (C.c_int64 * 3)(0, 1000, 1000), 2, 0.01, 0, 2, ok, ok, oo, ok, ok) == -2   # empty tensor
    assert f(None, ok, None, off, 2, 0.01, 0, 2, ok, ok, (C.c_int64 * 3)(0, 100, 100), ok, ok) == -2    # no room
    assert f(None, ok, None, off, 2, 1.0, 0, 2, ok, ok, oo, ok, ok) == -3
    assert f(None, ok, None, off, 2, 0.01, 5, 2, ok, ok, oo, ok, ok) == -5
    assert f(None, ok, None, off, 2, 0.01, 0, 0, ok, ok, oo, ok, ok) == -4
    assert f(None, ok, ok, off, 2, 0.01, 0, 2, ok, ok, oo, ok, ok) == -9
    offs = [0, 1000, 3000, 3001]
    got = sidco.sidco_batched_out_offsets(offs, 0.01)
    caps = [sidco.sidco_out_capacity(b - a, 0.01) for a, b in zip(offs, offs[1:])]
    assert got == [0, caps[0], caps[0] + caps[1], sum(caps)]
    assert sidco.sidco_workspace_bytes_batched(offs) >= 2 * 8 * (1024 + 2048 + 256)
    assert lib.sidco_read_diag_batched(None, 0, None) == -1


def test_dgc_argument_errors_and_sizes(lib, oracle):
    ok = C.c_void_p(256)
    f = lib.sidco_dgc
    assert f(None, None, None, 1000, 0.01, 0.01, 1, ok, ok, ok, ok) == -1
    assert f(None, ok, None, 1000, 0.01, 0.01, 1, ok, ok, ok, None) == -1
    assert f(None, ok, None, 0, 0.01, 0.01, 1, ok, ok, ok, ok) == -2
    assert f(None, ok, None, 2 ** 31, 0.01, 0.01, 1, ok, ok, ok, ok) == -2
    for bad in (0.0, 1.0, -1.0, math.nan):
        assert f(None, ok, None, 1000, bad, 0.01, 1, ok, ok, ok, ok) == -3
    for bad in (0.0, 1.5, -0.1, math.nan):
        assert f(None, ok, None, 1000, 0.01, bad, 1, ok, ok, ok, ok) == -3
    assert f(None, C.c_void_p(258), None, 1000, 0.01, 0.01, 1, ok, ok, ok, ok) == -8
    assert f(None, ok, ok, 1000, 0.01, 0.01, 1, ok, ok, ok, ok) == -9
    assert lib.sidco_dgc_sizes(1000, 0.01, 0.01, None) == -1
    assert lib.sidco_dgc_result(None, None) == -1
    for d, delta, rho in ((1_000_000, 0.001, 0.01), (269_722, 0.01, 0.01), (10, 0.001, 0.01), (25_557_032, 0.001, 0.01),
                          (138_357_544, 0.1, 0.01), (1, 0.5, 1.0), (12345, 0.3, 0.7)):
        assert sidco.sidco_dgc_sizes(d, delta, rho) == oracle.dgc_sizes(d, delta, rho)


def test_typed_argument_errors(lib):
    ok = C.c_void_p(256)
    f = lib.sidco_compress_typed
    assert f(None, ok, 3, None, 1000, 0.01, 0, 1, ok, ok, ok, ok) == -9        # unknown element type
    assert f(None, ok, -1, None, 1000, 0.01, 0, 1, ok, ok, ok, ok) == -9
    for code in (1, 2):
        assert f(None, None, code, None, 1000, 0.01, 0, 1, ok, ok, ok, ok) == -1
        assert f(None, ok, code, None, 1000, 0.01, 0, 1, ok, ok, ok, None) == -1
        assert f(None, ok, code, None, 0, 0.01, 0, 1, ok, ok, ok, ok) == -2
        assert f(None, ok, code, None, 1000, 0.0, 0, 1, ok, ok, ok, ok) == -3
        assert f(None, ok, code, None, 1000, 0.01, 0, 0, ok, ok, ok, ok) == -4
        assert f(None, ok, code, None, 1000, 0.01, 5, 1, ok, ok, ok, ok) == -5
        assert f(None, C.c_void_p(257), code, None, 1000, 0.01, 0, 1, ok, ok, ok, ok) == -8   # odd address
        assert f(None, ok, code, ok, 1000, 0.01, 0, 1, C.c_void_p(512), C.c_void_p(512), ok, ok) == -9   # aliasing
    assert f(None, None, 0, None, 1000, 0.01, 0, 1, ok, ok, ok, ok) == -1       # fp32 code: the plain call's checks
    w = lib.sidco_workspace_bytes_typed
    base = lib.sidco_workspace_bytes(1_000_000)
    assert w(1_000_000, 0, 0) == base and w(1_000_000, 1, 1) == base and w(1_000_000, 2, 1) == base
    assert w(1_000_000, 1, 0) == w(1_000_000, 2, 0) >= base + 4 * 1_000_000
    assert w(0, 1, 0) == 0 and w(1000, 7, 0) == 0


def test_typed_variants_of_the_other_calls_reject_bad_arguments(lib):
    """Each *_typed variant refuses an unknown element type and a misaligned gradient before touching the GPU;
    its other checks are the plain call's."""
    ok, odd, half = C.c_void_p(256), C.c_void_p(257), C.c_void_p(258)
    off = (C.c_int64 * 3)(0, 1000, 3000)
    oo = (C.c_int64 * 3)(0, 100, 300)
    tk, dg, bt = lib.sidco_topk_typed, lib.sidco_dgc_typed, lib.sidco_compress_batched_typed
    for bad in (3, -1):
        assert tk(None, ok, bad, None, 1000, 10, ok, ok, ok, ok) == -9
        assert dg(None, ok, bad, None, 1000, 0.01, 0.01, 0, ok, ok, ok, ok) == -9
        assert bt(None, ok, bad, None, off, 2, 0.01, 0, 2, ok, ok, oo, ok, ok) == -9
    for code in (0, 1, 2):
        assert tk(None, None, code, None, 1000, 10, ok, ok, ok, ok) == -1
        assert tk(None, ok, code, None, 1000, 0, ok, ok, ok, ok) == -2
        assert tk(None, ok, code, None, 1000, 1001, ok, ok, ok, ok) == -2
        assert tk(None, odd, code, None, 1000, 10, ok, ok, ok, ok) == -8
        assert tk(None, ok, code, ok, 1000, 10, ok, ok, ok, ok) == -9          # residual aliases the gradient
        assert dg(None, None, code, None, 1000, 0.01, 0.01, 0, ok, ok, ok, ok) == -1
        assert dg(None, odd, code, None, 1000, 0.01, 0.01, 0, ok, ok, ok, ok) == -8
        assert dg(None, ok, code, None, 1000, 1.5, 0.01, 0, ok, ok, ok, ok) == -3
        assert bt(None, None, code, None, off, 2, 0.01, 0, 2, ok, ok, oo, ok, ok) == -1
        assert bt(None, odd, code, None, off, 2, 0.01, 0, 2, ok, ok, oo, ok, ok) == -8
        assert bt(None, ok, code, None, off, 2, 0.01, 5, 2, ok, ok, oo, ok, ok) == -5
        assert bt(None, ok, code, None, off, 513, 0.01, 0, 2, ok, ok, oo, ok, ok) == -2
    # an address that is a multiple of 2 but not of 4 suits a 16-bit gradient only
    assert tk(None, half, 0, None, 1000, 10, ok, ok, ok, ok) == -8
    assert dg(None, half, 0, None, 1000, 0.01, 0.01, 0, ok, ok, ok, ok) == -8
    assert bt(None, half, 0, None, off, 2, 0.01, 0, 2, ok, ok, oo, ok, ok) == -8
    assert lib.sidco_controller_compress_typed(None, None, ok, 1, None, 1000, ok, ok, ok, ok) == -1
    w = lib.sidco_workspace_bytes_batched_typed
    base = lib.sidco_workspace_bytes_batched(off, 2)
    assert w(off, 2, 0, 0) == base and w(off, 2, 1, 1) == base and w(off, 2, 2, 1) == base
    assert w(off, 2, 1, 0) == w(off, 2, 2, 0) >= base + 4 * 3000
    assert w(off, 2, 9, 0) == 0 and w(None, 2, 1, 0) == 0


def test_new_setters_reject_bad_arguments(lib):
    assert lib.sidco_set_delta1(0.0) == -3 and lib.sidco_set_delta1(1.0) == -3 and lib.sidco_set_delta1(float("nan")) == -3
    assert lib.sidco_controller_disturbed(None) == -1
