"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before launching anything."""
import ctypes as C
import os
import re

import pytest

import paper_2601_07396_amd as pkg
from paper_2601_07396_amd.binding import Shape, FitParams

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(pkg.lib_path()):
        from paper_2601_07396_amd import build
        build.build()
    return pkg.load_library()


def test_header_symbols_are_exported(lib):
    header = open(os.path.join(ROOT, "include", "svdcache.h")).read()
    declared = set(re.findall(r"\b(svdcache_\w+)\s*\(", header))
    assert {"svdcache_fit_basis", "svdcache_full_step", "svdcache_forecast"} <= declared
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in the header but not exported"
    assert declared == set(pkg.exported_symbols())


def test_version_and_strerror(lib):
    assert pkg.svdcache_version() >= 100
    assert pkg.svdcache_strerror(0) == "ok"
    for code in range(-7, 0):
        assert pkg.svdcache_strerror(code) not in ("ok", "unknown status")
    assert pkg.svdcache_strerror(-99) == "unknown status"


def _shape(**kw):
    d = dict(B=1, N=64, D=64, k=8, ldf=64, block_stride=64 * 64, dtype=0, precision=0)
    d.update(kw)
    return Shape(**d)


@pytest.mark.parametrize("kw,code", [
    (dict(dtype=7), -3), (dict(precision=2), -5), (dict(B=0), -2), (dict(k=0), -2), (dict(k=65), -2), (dict(N=4, k=8), -2),
    (dict(ldf=32), -2), (dict(block_stride=100), -2), (dict(D=66, ldf=66, block_stride=66 * 64), -4),
    (dict(dtype=1, D=68, ldf=68, block_stride=68 * 64), -4),
    (dict(ldf=1 << 60, block_stride=(1 << 63) - 64), -2), (dict(B=4096, block_stride=1 << 40), -2),   # offsets would leave int64 / 2^48
])
def test_bad_shapes_are_rejected_on_the_host(lib, kw, code):
    s = _shape(**kw)
    dummy = C.c_void_p(256)   # never dereferenced: validation fails first
    rc = lib.svdcache_full_step(C.byref(s), dummy, dummy, None, dummy, dummy, None, 0.5, 1, None)
    assert rc == code
    rc = lib.svdcache_forecast(C.byref(s), dummy, dummy, None, dummy, dummy, None)
    assert rc == code
    assert lib.svdcache_fit_workspace_bytes(C.byref(s), None) == 0


def test_null_alpha_alignment_workspace(lib):
    s = _shape()
    p = C.c_void_p(256)
    assert lib.svdcache_full_step(None, p, p, None, p, p, None, 0.5, 1, None) == -1
    assert lib.svdcache_full_step(C.byref(s), None, p, None, p, p, None, 0.5, 1, None) == -1
    assert lib.svdcache_full_step(C.byref(s), p, p, None, p, None, None, 0.5, 1, None) == -1
    for bad in (0.0, -0.1, 1.5, float("nan")):
        assert lib.svdcache_full_step(C.byref(s), p, p, None, p, p, None, bad, 1, None) == -5
    assert lib.svdcache_full_step(C.byref(s), C.c_void_p(260), p, None, p, p, None, 0.5, 1, None) == -4
    assert lib.svdcache_forecast(C.byref(s), p, p, None, None, p, None) == -1
    need = lib.svdcache_fit_workspace_bytes(C.byref(s), None)
    assert need > 0
    assert lib.svdcache_fit_basis(C.byref(s), None, p, p, p, None, p, need - 1, None) == -6
    assert lib.svdcache_fit_basis(C.byref(s), None, p, p, p, None, None, need, None) == -1
    fp = FitParams(-5, 0, 0)
    assert lib.svdcache_fit_basis(C.byref(s), C.byref(fp), p, p, p, None, p, need, None) == -5


def test_workspace_grows_with_sketch_width(lib):
    s = _shape(N=512, D=256, k=16, ldf=256, block_stride=512 * 256)
    a = pkg.svdcache_fit_workspace_bytes(s, p=-1)
    b = pkg.svdcache_fit_workspace_bytes(s, p=16)
    c = pkg.svdcache_fit_workspace_bytes(s, p=48)
    assert 0 < a < b < c


def test_calls_refuse_cpu_tensors():
    import torch
    F = torch.zeros(1, 64, 64)
    s = pkg.make_shape(F, 8)
    with pytest.raises(RuntimeError, match="GPU"):
        pkg.svdcache_forecast(s, torch.zeros(1, 64, 8), torch.zeros(1, 64, 8), None, F, F)


def test_extrapolation_weights_is_a_host_function(lib):
    """No GPU work behind it: callable anywhere; checked against the oracle's rational-arithmetic version."""
    import numpy as np
    from oracle import ref_extrapolation_weights
    for order in range(4):
        for off, itv in [(1, 6), (5, 6), (2.5, 3), (0, 4), (-4, 4), (7, 2)]:
            got = pkg.svdcache_extrapolation_weights(order, off, itv)
            want = ref_extrapolation_weights(order, off, itv).astype(np.float32)
            assert np.allclose(got, want, rtol=2e-7, atol=1e-7), (order, off, itv)
    w = (C.c_float * 4)()
    assert lib.svdcache_extrapolation_weights(1, 1.0, 6.0, None) == -1
    assert lib.svdcache_extrapolation_weights(4, 1.0, 6.0, w) == -5      # more states than SVDC_MAX_STATES
    assert lib.svdcache_extrapolation_weights(-1, 1.0, 6.0, w) == -5
    assert lib.svdcache_extrapolation_weights(1, 1.0, 0.0, w) == -5


def test_widened_entry_points_validate_on_the_host(lib):
    s = Shape(1, 16, 64, 4, 64, 16 * 64, 0, 0)
    fake = C.c_void_p(256)
    assert lib.svdcache_select_rank(1, 4, None, fake, 0.85, fake, None, None) == -1
    assert lib.svdcache_select_rank(0, 4, fake, fake, 0.85, fake, None, None) == -2
    assert lib.svdcache_select_rank(1, 4, fake, fake, 0.0, fake, None, None) == -5
    assert lib.svdcache_truncate_basis(C.byref(s), None, None, fake, None) == -1
    ptrs = (C.c_void_p * 1)(256)
    w = (C.c_float * 1)(1.0)
    assert lib.svdcache_forecast_combine(C.byref(s), 0, ptrs, w, fake, None, fake, None, fake, None) == -5
    assert lib.svdcache_forecast_combine(C.byref(s), 1, None, w, fake, None, fake, None, fake, None) == -1
    bad = (C.c_void_p * 1)(260)                                           # not 16-byte aligned
    assert lib.svdcache_forecast_combine(C.byref(s), 1, bad, w, fake, None, fake, None, fake, None) == -4


def test_basis_file_round_trip(tmp_path):
    """The offline basis file holds plain arrays and comes back bit for bit (file IO only, no GPU)."""
    import torch
    g = torch.Generator().manual_seed(1)
    V, sigma, fro2 = torch.randn(3, 40, 6, generator=g), torch.rand(3, 6, generator=g), torch.rand(3, generator=g)
    path = str(tmp_path / "basis.npz")
    pkg.save_basis(path, V, sigma, fro2)
    V2, s2, f2 = pkg.load_basis(path, device="cpu")
    assert torch.equal(V, V2) and torch.equal(sigma, s2) and torch.equal(fro2, f2)
    pkg.save_basis(path, V, sigma)
    assert pkg.load_basis(path, device="cpu")[2] is None
    import numpy as np
    np.savez(path, V=np.zeros((2, 3)), sigma=np.zeros(3))
    with pytest.raises(ValueError):
        pkg.load_basis(path, device="cpu")


def test_residual_ema_validates_on_the_host(lib):
    s = Shape(1, 16, 64, 4, 64, 16 * 64, 0, 0)
    f, r, v, st = C.c_void_p(256), C.c_void_p(512), C.c_void_p(1024), C.c_void_p(2048)
    call = lib.svdcache_full_step_residual_ema
    assert call(C.byref(s), f, v, None, None, r, st, None, 0.5, 0.5, 0, None) == -1     # R_prev needed
    assert call(C.byref(s), f, v, None, f, r, st, None, 0.5, 0.5, 0, None) == -5        # R_prev is F
    assert call(C.byref(s), f, v, None, r, r, st, None, 0.5, 0.0, 0, None) == -5        # alpha_r out of range
    assert call(C.byref(s), None, v, None, r, r, st, None, 0.5, 0.5, 0, None) == -1


def test_binding_refuses_mismatched_layouts():
    """The C ABI has one (ldf, block_stride, dtype) for F, R, Fhat, X and R_prev and takes V, S, C as dense
    float32: the binding refuses tensors whose own layout differs before anything is launched (CPU tensors here;
    a refusal comes before the check for device memory)."""
    import torch
    B, N, D, k, ldf = 2, 32, 128, 8, 160
    buf = torch.zeros(B, N, ldf)
    F = buf[:, :, :D]                                   # row-strided view
    s = pkg.make_shape(F, k)
    assert s.ldf == ldf
    V, S = torch.zeros(B, D, k), torch.zeros(B, N, k)
    with pytest.raises(ValueError, match="strides"):    # empty_like of a gapped view is contiguous
        pkg.svdcache_full_step(s, F, V, None, torch.empty_like(F), S, None, 0.5, True)
    with pytest.raises(ValueError, match="dtype"):
        pkg.svdcache_full_step(s, F, V, None, buf.bfloat16()[:, :, :D], S, None, 0.5, True)
    with pytest.raises(ValueError, match="shape"):
        pkg.svdcache_forecast(s, S, V, None, F, buf[:, :N - 1, :D])
    with pytest.raises(ValueError, match="V"):
        pkg.svdcache_full_step(s, F, V.double(), None, F, S, None, 0.5, True)
    with pytest.raises(ValueError, match="V"):
        pkg.svdcache_forecast(s, S, torch.zeros(B, k, D).transpose(1, 2), None, F, F)
    with pytest.raises(ValueError, match="S"):
        pkg.svdcache_full_step(s, F, V, None, F, torch.zeros(B, N, k + 1), None, 0.5, True)
    with pytest.raises(ValueError, match="C"):
        pkg.svdcache_full_step(s, F, V, None, F, S, torch.zeros(B, N, 2 * k)[:, :, :k], 0.5, True)
    with pytest.raises(ValueError, match=r"S_list\[1\]"):
        pkg.svdcache_forecast_combine(s, [S, S[:1]], [1.0, 0.0], V, None, F, None, F)
    with pytest.raises(ValueError, match="X"):
        pkg.svdcache_forecast_combine(s, [S], [1.0], V, None, F, torch.zeros(B, N, D), F)
    with pytest.raises(ValueError, match="R_prev"):
        pkg.svdcache_full_step_residual_ema(s, F, V, None, torch.zeros(B, N, D), F, S, None, 0.5, 0.5, False)
    # a packed basis of another rank is too small (or of a shape without a matrix-core path: not accepted at all)
    Fm = torch.zeros(1, 64, 256, dtype=torch.bfloat16)
    s64, s32 = pkg.make_shape(Fm, 64), pkg.make_shape(Fm, 32)
    small = torch.zeros(pkg.svdcache_packed_basis_bytes(s32), dtype=torch.uint8)
    with pytest.raises(ValueError, match="packed"):
        pkg.svdcache_forecast(s64, torch.zeros(1, 64, 64), torch.zeros(1, 256, 64), small, Fm, Fm)
    with pytest.raises(ValueError, match="packed"):
        pkg.svdcache_forecast(s, S, V, small, F, F)
    # the fit: sigma and fro2 sized by the shape
    with pytest.raises(ValueError, match="sigma"):
        pkg.svdcache_fit_basis(s, F, V, torch.zeros(B, k + 1), None, torch.zeros(16, dtype=torch.uint8))
    # matching layouts pass the checks and stop at the device check
    with pytest.raises(RuntimeError, match="GPU"):
        pkg.svdcache_full_step(s, F, V, None, torch.zeros(B, N, ldf)[:, :, :D], S, None, 0.5, True)


def test_probe_library_exports_its_header():
    """libsvdcache_probes.so (memory-system probes for the benchmark) loads and exports what its header declares."""
    from paper_2601_07396_amd import probes
    header = open(os.path.join(ROOT, "include", "svdcache_probes.h")).read()
    declared = set(re.findall(r"\b(svdc_probe_\w+)\s*\(", header))
    assert declared and declared == set(probes.EXPORTS)
    lib = probes.load_library()
    for name in declared:
        assert hasattr(lib, name)
    # bad arguments are refused on the host
    assert lib.svdc_probe_copy(None, None, 16, None) == -1
    assert lib.svdc_probe_burst_copy(C.c_void_p(256), C.c_void_p(512), 100, 40, None) == -1


def test_bench_reads_its_traffic_figure_from_the_tracked_profile():
    """roofline.traffic is not a constant in bench.py: it is the figure the tracked rocprofv3 summary holds."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    text = open(bench.TRAFFIC_PROFILE).read()
    for kernel in ("forecast_mfma_kernel", "full_step_mfma_kernel"):
        got = bench.traffic_from_profile(kernel)
        assert got is not None and got > 3_000_000_000
        row = [l for l in text.splitlines() if l.startswith("| " + kernel)][0]
        assert row.rstrip(" |").endswith(str(got))
    assert bench.traffic_from_profile("no_such_kernel") is None
    assert "MEASURED_TRAFFIC" not in open(os.path.join(ROOT, "bench.py")).read()
