"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.
`assert_close` bounds the error of every element (one unit in the last place of the storage type plus the
accumulated arithmetic error, scaled by the row), of every row and of the whole block."""
import numpy as np
import pytest
import torch

import paper_2601_07396_amd as pkg
from oracle import ref_fit_basis, ref_full_step, ref_forecast
from synth import WORKLOADS, FeatureStream, is_full_step, torch_dtype
from util import TOL, to_np, rel_err, assert_close, principal_sines

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _rand_problem(B, N, D, k, dtype, seed, ldf=None):
    g = torch.Generator().manual_seed(seed)
    ldf = D if ldf is None else ldf
    buf = torch.zeros(B, N, ldf, dtype=dtype)
    buf[:, :, :D] = torch.randn(B, N, D, generator=g).to(dtype)
    V = torch.linalg.qr(torch.randn(B, D, k, generator=g, dtype=torch.float64))[0].float().contiguous()
    S = torch.randn(B, N, k, generator=g)
    return buf, V, S


def _run_full(Fbuf, D, V, S, alpha, init, want_C=True, inplace=False, packed="auto"):
    F = Fbuf.to(DEV)
    Fv = F[:, :, :D]
    shape = pkg.make_shape(Fv, V.shape[2])
    Vd, Sd = V.to(DEV), S.clone().to(DEV)
    pk = pkg.pack_basis(shape, Vd) if packed == "auto" else None
    R = F if inplace else torch.full_like(F, 7.0)
    Cd = torch.empty_like(Sd) if want_C else None
    pkg.svdcache_full_step(shape, Fv, Vd, pk, R[:, :, :D], Sd, Cd, alpha, init)
    torch.cuda.synchronize()
    return R, Sd, Cd, shape, pk


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("B,N,D,k", [(2, 256, 64, 8), (1, 37, 72, 5), (3, 130, 200, 17), (1, 1, 8, 1),
                                     (1, 20, 16, 16), (2, 67, 264, 40)])
def test_full_step_and_forecast_general_shapes(dtype, B, N, D, k):
    store = "f32" if dtype == torch.float32 else "bf16"
    Fbuf, V, S0 = _rand_problem(B, N, D, k, dtype, seed=B * 1000 + N)
    for init in (True, False):
        R, S, Cc, shape, pk = _run_full(Fbuf, D, V, S0, 0.3, init)
        Fh = torch.empty_like(R)
        pkg.svdcache_forecast(shape, S, V.to(DEV), pk, R, Fh)
        torch.cuda.synchronize()
        for b in range(B):
            Rr, Sr, Cr = ref_full_step(to_np(Fbuf[b]), to_np(V[b]), to_np(S0[b]), 0.3, init, store)
            assert_close(to_np(R[b]), Rr, store, f"R[{b}]", floor_of=to_np(Fbuf[b]))
            assert_close(to_np(S[b]), Sr, "f32", f"S[{b}]")
            assert_close(to_np(Cc[b]), Cr, "f32", f"C[{b}]")
            # the oracle forecasts from its OWN state: nothing computed on the GPU is fed to it
            Fr = ref_forecast(Sr, to_np(V[b]), Rr, store)
            assert_close(to_np(Fh[b]), Fr, store, f"Fhat[{b}]", scale_of=to_np(Fbuf[b]), ulp_of=Rr)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_strided_rows_inplace_and_null_C(dtype):
    store = "f32" if dtype == torch.float32 else "bf16"
    B, N, D, k, ldf = 2, 50, 64, 8, 96
    Fbuf, V, S0 = _rand_problem(B, N, D, k, dtype, seed=5, ldf=ldf)
    R, S, Cc, shape, pk = _run_full(Fbuf, D, V, S0, 0.5, False, want_C=False, inplace=True)
    assert Cc is None and shape.ldf == ldf
    state = []
    for b in range(B):
        Rr, Sr, _ = ref_full_step(to_np(Fbuf[b, :, :D]), to_np(V[b]), to_np(S0[b]), 0.5, False, store)
        assert_close(to_np(R[b, :, :D]), Rr, store, "R in place")
        assert_close(to_np(S[b]), Sr, "f32", "S")
        state.append((Rr, Sr))
    # the padding columns beyond D are not touched
    assert torch.equal(R[:, :, D:].cpu(), Fbuf[:, :, D:])
    # forecast in place (Fhat aliases R); the oracle continues from its own state
    pkg.svdcache_forecast(shape, S, V.to(DEV), pk, R[:, :, :D], R[:, :, :D])
    torch.cuda.synchronize()
    for b in range(B):
        Fr = ref_forecast(state[b][1], to_np(V[b]), state[b][0], store)
        assert_close(to_np(R[b, :, :D]), Fr, store, "Fhat in place", scale_of=to_np(Fbuf[b, :, :D]), ulp_of=state[b][0])


def test_forecast_after_init_reproduces_F_exactly_in_fp32_tolerance():
    B, N, D, k = 1, 64, 128, 16
    Fbuf, V, S0 = _rand_problem(B, N, D, k, torch.float32, seed=9)
    R, S, Cc, shape, pk = _run_full(Fbuf, D, V, S0, 0.5, True)
    assert torch.equal(S, Cc)
    Fh = torch.empty_like(R)
    pkg.svdcache_forecast(shape, S, V.to(DEV), pk, R, Fh)
    torch.cuda.synchronize()
    assert rel_err(to_np(Fh), to_np(Fbuf)) <= 1e-6


def _fit_checks(F_cpu, V, sigma, fro2, k, store, lead=None):
    """Compare a fitted basis with the exact truncated SVD.  Several bases are correct (signs,
    rotations inside clusters of close singular values), so compare what is unique: singular values,
    captured energy, orthonormality, and the leading subspace scaled by its spectral gap."""
    tol = TOL[store]
    Fd = to_np(F_cpu)
    n_all = min(Fd.shape)
    _, s_all, _ = ref_fit_basis(Fd, n_all) if n_all <= 512 else (None, None, None)
    Vr, sr, fr = ref_fit_basis(Fd, k)
    Vg = to_np(V)
    assert np.abs(Vg.T @ Vg - np.eye(k)).max() <= 1e-5
    sg = to_np(sigma)
    assert np.all(np.diff(sg) <= 1e-6 * sg[0])
    assert np.abs(sg / sr - 1).max() <= tol, f"sigma rel err {np.abs(sg / sr - 1).max():.2e}"
    assert abs(float(fro2) / fr - 1) <= 1e-5
    captured = np.sum((Fd @ Vg) ** 2)
    assert 1 - captured / np.sum(sr ** 2) <= tol
    # sigma reported must be the norms of F v_j
    assert np.abs(np.linalg.norm(Fd @ Vg, axis=0) / sg - 1).max() <= max(tol, 1e-4)
    if s_all is not None:
        lead = lead or max(1, k // 2)
        gap = s_all[lead - 1] / (s_all[lead - 1] - s_all[lead])
        sines = principal_sines(Vg[:, :lead], Vr[:, :lead])
        assert sines.max() <= tol * gap + 2e-4 * gap, f"leading subspace off: {sines.max():.2e} (gap factor {gap:.1f})"


def test_fit_basis_tiny_config():
    wl = WORKLOADS["tiny"]
    F = torch.stack([FeatureStream(wl, b).at(0) for b in range(wl.B)])
    V, sigma, fro2 = pkg.fit_basis(F.to(DEV), wl.k)
    torch.cuda.synchronize()
    for b in range(wl.B):
        _fit_checks(F[b], V[b], sigma[b], fro2[b], wl.k, "f32")


@pytest.mark.parametrize("dtype,N,D,k", [(torch.float32, 300, 96, 12), (torch.bfloat16, 500, 160, 16),
                                          (torch.float32, 40, 64, 40), (torch.bfloat16, 129, 72, 3)])
def test_fit_basis_power_law_inputs(dtype, N, D, k):
    store = "f32" if dtype == torch.float32 else "bf16"
    wl = WORKLOADS["flux1"].with_(N=N, D=D, k=k, dtype=store, signal_rank=min(48, D, N), rho=0.05)
    F = FeatureStream(wl, 0).at(0).unsqueeze(0)
    V, sigma, fro2 = pkg.fit_basis(F.to(DEV), k, q=6 if store == "f32" else 0)
    torch.cuda.synchronize()
    _fit_checks(F[0], V[0], sigma[0], fro2[0], k, store)


@pytest.mark.parametrize("alpha,interval", [(None, None), (0.3, 5), (0.7, 8), (0.1, 3), (1.0, 2)],
                         ids=["config", "a0.3-N5", "a0.7-N8", "a0.1-N3", "reuse-N2"])
def test_tiny_trajectory_matches_oracle_step_by_step(alpha, interval):
    """Config 1: 2 blocks, 256 x 64, k = 8, fp32, 10 steps, every 3rd a full step, alpha = 0.5; then the EMA
    weights and caching intervals of the sweep configuration (alpha = 0.1 is the paper's beta = 0.9, alpha = 1
    plain reuse).  Both sides use the same basis: the generator's leading directions."""
    wl = WORKLOADS["tiny"]
    if alpha is not None:
        wl = wl.with_(alpha=alpha, interval=interval, T=17)
    streams = [FeatureStream(wl, b) for b in range(wl.B)]
    feats = [torch.stack([s.at(t) for s in streams]) for t in range(wl.T)]
    F0 = feats[0].to(DEV)
    shape = pkg.make_shape(F0, wl.k)
    # the basis both sides use is the generator's own set of leading directions (nothing fitted on the GPU is
    # handed to the oracle; the fit has its own tests)
    V = torch.stack([s.V[:, :wl.k].float() for s in streams]).contiguous().to(DEV)
    pk = pkg.pack_basis(shape, V)
    R = torch.empty_like(F0)
    S = torch.empty(wl.B, wl.N, wl.k, device=DEV)
    Fh = torch.empty_like(F0)
    Vn = [to_np(V[b]) for b in range(wl.B)]
    Rr = [None] * wl.B
    Sr = [None] * wl.B
    first = True
    for t in range(wl.T):
        if is_full_step(t, wl.interval):
            pkg.svdcache_full_step(shape, feats[t].to(DEV), V, pk, R, S, None, wl.alpha, first)
            torch.cuda.synchronize()
            for b in range(wl.B):
                Rr[b], Sr[b], _ = ref_full_step(to_np(feats[t][b]), Vn[b], Sr[b], wl.alpha, first, "f32")
                assert_close(to_np(R[b]), Rr[b], "f32", f"t={t} R[{b}]")
                assert_close(to_np(S[b]), Sr[b], "f32", f"t={t} S[{b}]")
            first = False
        else:
            pkg.svdcache_forecast(shape, S, V, pk, R, Fh)
            torch.cuda.synchronize()
            for b in range(wl.B):
                assert_close(to_np(Fh[b]), ref_forecast(Sr[b], Vn[b], Rr[b], "f32"), "f32", f"t={t} Fhat[{b}]")


def test_checkpoint_split_is_bit_identical():
    """The state is (V, S, R) in caller-owned tensors: 10 steps in one go equal 5 + restore + 5."""
    wl = WORKLOADS["tiny"]
    feats = [torch.stack([FeatureStream(wl, b).at(t) for b in range(wl.B)]).to(DEV) for t in range(wl.T)]
    shape = pkg.make_shape(feats[0], wl.k)
    V, _, _ = pkg.fit_basis(feats[0], wl.k)

    def run(t0, t1, R, S, outs):
        for t in range(t0, t1):
            if is_full_step(t, wl.interval):
                pkg.svdcache_full_step(shape, feats[t], V, None, R, S, None, wl.alpha, t == 0)
                outs.append(R.clone())
            else:
                Fh = torch.empty_like(R)
                pkg.svdcache_forecast(shape, S, V, None, R, Fh)
                outs.append(Fh)
        torch.cuda.synchronize()

    R1, S1, o1 = torch.zeros_like(feats[0]), torch.zeros(wl.B, wl.N, wl.k, device=DEV), []
    run(0, wl.T, R1, S1, o1)
    R2, S2, o2 = torch.zeros_like(feats[0]), torch.zeros(wl.B, wl.N, wl.k, device=DEV), []
    run(0, 5, R2, S2, o2)
    saved = (R2.cpu(), S2.cpu())
    R3, S3 = saved[0].to(DEV), saved[1].to(DEV)
    run(5, wl.T, R3, S3, o2)
    assert all(torch.equal(a, b) for a, b in zip(o1, o2))


def test_errors_reported_through_the_binding():
    F = torch.zeros(1, 16, 16, device=DEV)
    shape = pkg.make_shape(F, 4)
    V = torch.zeros(1, 16, 4, device=DEV)
    S = torch.zeros(1, 16, 4, device=DEV)
    with pytest.raises(pkg.SvdcError) as e:
        pkg.svdcache_full_step(shape, F, V, None, F, S, None, 0.0, True)
    assert e.value.code == -5
    with pytest.raises(pkg.SvdcError) as e:
        pkg.svdcache_fit_basis(shape, F, V, torch.zeros(1, 4, device=DEV), None,
                               torch.zeros(16, device=DEV, dtype=torch.uint8))
    assert e.value.code == -6


# ---------------------------------------------------------------------------------------------
# matrix-core (MFMA) path for bf16 features
# ---------------------------------------------------------------------------------------------

def _lowrank_problem(B, N, D, k, seed, rho=0.05):
    """bf16 features with most energy in span(V) (like the real workload) plus a 5 % residual,
    so that R is a small difference of large terms."""
    g = torch.Generator().manual_seed(seed)
    V = torch.linalg.qr(torch.randn(B, D, k, generator=g, dtype=torch.float64))[0]
    Cc = torch.randn(B, N, k, generator=g, dtype=torch.float64) * (torch.arange(1, k + 1) ** -0.6)
    sig = Cc @ V.transpose(1, 2)
    noise = torch.randn(B, N, D, generator=g, dtype=torch.float64)
    noise *= (rho / (1 - rho)) ** 0.5 * sig.norm() / noise.norm()
    F = (sig + noise) * (D ** 0.5 / (sig.norm() / (B * N) ** 0.5))
    S = Cc.float() * float(F.abs().mean() / sig.abs().mean())
    return F.to(torch.bfloat16), V.float().contiguous(), S.contiguous()


@pytest.mark.parametrize("B,N,D,k", [(2, 200, 256, 32), (1, 77, 512, 8), (3, 64, 256, 64), (1, 131, 512, 128),
                                     (2, 49, 256, 20), (1, 150, 3072, 32), (2, 70, 3072, 64), (1, 140, 3072, 128),
                                     (1, 33, 3072, 16), (1, 80, 1024, 32), (1, 70, 1536, 64), (1, 50, 2048, 16),
                                     (1, 130, 2048, 128), (1, 45, 4096, 32), (1, 66, 4096, 64),
                                     (1, 70, 1152, 32), (2, 70, 1152, 64), (1, 90, 1920, 16), (1, 140, 1920, 128),
                                     (1, 75, 2560, 32), (1, 80, 2560, 64), (1, 60, 5120, 32), (1, 130, 5120, 128)])
def test_mfma_full_step_and_forecast(B, N, D, k):
    F, V, S0 = _lowrank_problem(B, N, D, k, seed=N * 7 + k)
    shape = pkg.make_shape(F, k)
    assert pkg.svdcache_has_mfma_path(shape)
    for init in (True, False):
        R, S, Cc, shape, pk = _run_full(F, D, V, S0, 0.5, init)
        assert pk is not None
        Fh = torch.empty_like(R)
        pkg.svdcache_forecast(shape, S, V.to(DEV), pk, R, Fh)
        torch.cuda.synchronize()
        for b in range(B):
            Rr, Sr, Cr = ref_full_step(to_np(F[b]), to_np(V[b]), to_np(S0[b]), 0.5, init, "bf16")
            assert_close(to_np(R[b]), Rr, "bf16", f"R[{b}]", floor_of=to_np(F[b]))
            assert_close(to_np(S[b]), Sr, "f32", f"S[{b}]")
            assert_close(to_np(Cc[b]), Cr, "f32", f"C[{b}]")
            Fr = ref_forecast(Sr, to_np(V[b]), Rr, "bf16")      # the oracle's own state
            assert_close(to_np(Fh[b]), Fr, "bf16", f"Fhat[{b}]", scale_of=to_np(F[b]), ulp_of=Rr)
            # the split-operand arithmetic is far inside the bf16 budget: the error is the output rounding
            assert rel_err(to_np(R[b]), Rr) <= 3e-3 and rel_err(to_np(Fh[b]), Fr) <= 3e-3


def test_mfma_and_general_paths_agree():
    """Same inputs through the packed (MFMA) and the unpacked (general) kernels."""
    B, N, D, k = 2, 100, 512, 32
    F, V, S0 = _lowrank_problem(B, N, D, k, seed=3)
    Ra, Sa, Ca, shape, pk = _run_full(F, D, V, S0, 0.3, False)
    Rb, Sb, Cb, _, none = _run_full(F, D, V, S0, 0.3, False, packed=None)
    assert pk is not None and none is None
    assert rel_err(to_np(Sa), to_np(Sb)) <= 1e-5 and rel_err(to_np(Ca), to_np(Cb)) <= 1e-5
    assert rel_err(to_np(Ra), to_np(Rb)) <= 3e-3
    Fa, Fb = torch.empty_like(Ra), torch.empty_like(Ra)
    pkg.svdcache_forecast(shape, Sa, V.to(DEV), pk, Ra, Fa)
    pkg.svdcache_forecast(shape, Sa, V.to(DEV), None, Ra, Fb)
    torch.cuda.synchronize()
    assert rel_err(to_np(Fa), to_np(Fb)) <= 3e-3


@pytest.mark.parametrize("k", [32, 64, 128])
def test_mfma_inplace_and_strided(k):
    """In-place residual (R aliases F), padded row stride, no coefficient output."""
    B, N, D, ldf = 2, 150, 256, 384
    F, V, S0 = _lowrank_problem(B, N, D, k, seed=11)
    buf = torch.zeros(B, N, ldf, dtype=torch.bfloat16)
    buf[:, :, :D] = F
    for init in (True, False):
        R, S, _, shape, pk = _run_full(buf, D, V, S0, 0.5, init, want_C=False, inplace=True)
        assert pk is not None and shape.ldf == ldf
        state = []
        for b in range(B):
            Rr, Sr, _ = ref_full_step(to_np(F[b]), to_np(V[b]), to_np(S0[b]), 0.5, init, "bf16")
            assert_close(to_np(R[b, :, :D]), Rr, "bf16", "R in place", floor_of=to_np(F[b]))
            assert_close(to_np(S[b]), Sr, "f32", "S")
            state.append((Rr, Sr))
        assert torch.equal(R[:, :, D:].cpu(), buf[:, :, D:])
    pkg.svdcache_forecast(shape, S, V.to(DEV), pk, R[:, :, :D], R[:, :, :D])
    torch.cuda.synchronize()
    for b in range(B):
        assert_close(to_np(R[b, :, :D]), ref_forecast(state[b][1], to_np(V[b]), state[b][0], "bf16"),
                     "bf16", "Fhat in place", scale_of=to_np(F[b]), ulp_of=state[b][0])


@pytest.mark.parametrize("dtype,B,N,D,k,mode", [
    (torch.bfloat16, 2, 200, 256, 32, 0), (torch.bfloat16, 1, 77, 512, 8, 0), (torch.bfloat16, 3, 130, 3072, 64, 0),
    (torch.bfloat16, 1, 145, 3072, 128, 0), (torch.bfloat16, 2, 333, 3072, 20, 1), (torch.bfloat16, 1, 90, 1024, 64, 1),
    (torch.float32, 1, 131, 512, 32, 0), (torch.float32, 1, 70, 3072, 64, 0)])
def test_packed_state_full_step_and_cached_step(dtype, B, N, D, k, mode):
    """The state handed over in the cached step's operand format: svdcache_full_step_packed writes it next to the
    float32 state, svdcache_pack_state makes it from a float32 state, svdcache_forecast_packed reads it.  Against the
    oracle at the usual bars, and bit for bit against the float32-state calls (same arithmetic, fewer conversions)."""
    store = "f32" if dtype == torch.float32 else "bf16"
    Fb, V, S0 = _lowrank_problem(B, N, D, k, seed=N + 3 * k)
    F = Fb.to(dtype)
    Fd, Vd = F.to(DEV), V.to(DEV)
    shape = pkg.make_shape(Fd, k, precision=mode)
    pk = pkg.pack_basis(shape, Vd)
    fast = mode == pkg.SVDC_FAST
    coef = "bf16" if fast else "f32"
    for init in (True, False):
        Sa, Sb = S0.clone().to(DEV), S0.clone().to(DEV)
        Ra, Rb = torch.empty_like(Fd), torch.empty_like(Fd)
        Ca, Cb = torch.empty_like(Sa), torch.empty_like(Sa)
        Sp = pkg.alloc_packed_state(shape, DEV)
        Sp.fill_(0xAB)
        pkg.svdcache_full_step(shape, Fd, Vd, pk, Ra, Sa, Ca, 0.4, init)
        pkg.svdcache_full_step_packed(shape, Fd, Vd, pk, Rb, Sb, Cb, Sp, 0.4, init)
        Fa, Fb2, Fc = torch.empty_like(Fd), torch.empty_like(Fd), torch.empty_like(Fd)
        pkg.svdcache_forecast(shape, Sa, Vd, pk, Ra, Fa)
        pkg.svdcache_forecast_packed(shape, Sp, pk, Rb, Fb2)
        Sp2 = torch.empty_like(Sp)
        pkg.svdcache_pack_state(shape, Sa, Sp2)
        pkg.svdcache_forecast_packed(shape, Sp2, pk, Ra, Fc)
        torch.cuda.synchronize()
        assert torch.equal(Ra, Rb) and torch.equal(Sa, Sb) and torch.equal(Ca, Cb)
        assert torch.equal(Sp, Sp2), "the full step's packed state differs from the packed float32 state"
        assert torch.equal(Fa, Fb2) and torch.equal(Fa, Fc)
        for b in range(B):
            Rr, Sr, _ = ref_full_step(to_np(F[b]), to_np(V[b]), to_np(S0[b]), 0.4, init, store)
            assert_close(to_np(Sb[b]), Sr, coef, f"S[{b}]", fast=fast)
            assert_close(to_np(Fb2[b]), ref_forecast(Sr, to_np(V[b]), Rr, store), store, f"Fhat[{b}] from packed state",
                         fast=fast, scale_of=to_np(F[b]), ulp_of=Rr)
    # a shape without a matrix-core path has no packed state
    odd = pkg.make_shape(torch.zeros(1, 16, 72, device=DEV), 4)
    assert pkg.svdcache_packed_state_bytes(odd) == 0


# ---------------------------------------------------------------------------------------------
# basis fit with the products on the matrix cores (bf16 features, D % 128 == 0, k + p <= 128)
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("N,D,k", [(300, 256, 16), (1000, 512, 32), (600, 3072, 32), (333, 384, 8), (700, 768, 64),
                                   (200, 128, 4), (20, 128, 4), (33, 128, 8), (65, 256, 40), (97, 128, 64)])
def test_fit_basis_mfma_path(N, D, k):
    wl = WORKLOADS["flux1"].with_(N=N, D=D, k=k, signal_rank=min(96, D, N))
    F = torch.stack([FeatureStream(wl, b).at(0) for b in range(2)])
    # at these small sizes the trailing singular values sit in the noise bulk (sigma_{l+1} / sigma_k close
    # to 1), where subspace iteration converges slowly: use more power iterations than the default
    V, sigma, fro2 = pkg.fit_basis(F.to(DEV), k, q=10)
    torch.cuda.synchronize()
    for b in range(2):
        _fit_checks(F[b], V[b], sigma[b], fro2[b], k, "bf16")


@pytest.mark.parametrize("dtype,k,p,rank", [(torch.float32, 50, 50, 55), (torch.float32, 60, 64, 124),
                                             (torch.bfloat16, 56, 56, 60)], ids=["f32-l100", "f32-l124", "bf16-l112"])
def test_fit_basis_wide_sketch_low_rank_features(dtype, k, p, rank):
    """Sketch widths 98..128: the small SVD keeps only one l x l matrix on chip and recovers the right vectors
    from the Cholesky factor at the end.  Features of exact rank < l (float32) make that factor as ill conditioned
    as the diagonal shift allows; the leading k directions must still come out orthonormal and exact."""
    store = "f32" if dtype == torch.float32 else "bf16"
    g = torch.Generator().manual_seed(k * 100 + rank)
    N, D = 400, 256
    left = torch.linalg.qr(torch.randn(N, rank, generator=g, dtype=torch.float64))[0]
    right = torch.linalg.qr(torch.randn(D, rank, generator=g, dtype=torch.float64))[0]
    spec = 10.0 * torch.arange(1, rank + 1, dtype=torch.float64) ** -0.8
    F = ((left * spec) @ right.T).to(dtype).unsqueeze(0).contiguous()
    V, sigma, fro2 = pkg.fit_basis(F.to(DEV), k, p=p, q=4)
    torch.cuda.synchronize()
    _fit_checks(F[0], V[0], sigma[0], fro2[0], k, store)


@pytest.mark.parametrize("dtype,N,D,k,p", [(torch.bfloat16, 600, 512, 96, 0), (torch.float32, 600, 512, 96, 0),
                                            (torch.bfloat16, 700, 384, 128, 0), (torch.float32, 520, 256, 128, 0),
                                            (torch.bfloat16, 450, 640, 100, 29), (torch.float32, 300, 320, 65, 64),
                                            (torch.bfloat16, 300, 256, 50, 50), (torch.float32, 300, 200, 40, 37),
                                            (torch.float32, 260, 384, 65, 65), (torch.bfloat16, 420, 256, 75, 75),
                                            (torch.bfloat16, 139, 256, 70, 70), (torch.float32, 400, 512, 100, 100),
                                            (torch.bfloat16, 500, 384, 110, 113)],
                         ids=["bf16-l192", "f32-l192", "bf16-l256", "f32-l256", "bf16-l129", "f32-l129",
                              "bf16-l100", "f32-l77-general", "f32-l130", "bf16-l150", "bf16-l139", "f32-l200",
                              "bf16-l223"])
def test_fit_basis_sketch_widths_65_to_256(dtype, N, D, k, p):
    """Sketch widths 65..256 (the default oversampling p = k puts every rank 33..128 there, config 5's k = 128
    at l = 256): singular values, captured energy, orthonormality and the leading subspace against the exact
    truncated SVD, for both storage types.  The widths are chosen to hit every branch of the l x l chain: a ragged
    last column block of the Cholesky factorisation and of its application (100 = 64 + 36, 130 = 2 x 64 + 2,
    200 = 3 x 64 + 8), the widest matrix that the single-workgroup Jacobi takes (129..138), and, for the Jacobi by
    column blocks, an odd number of blocks (139 and 150: five, 200 and 223: seven -- one block sits out per step)
    as well as an even one (192: six, 256: eight)."""
    store = "f32" if dtype == torch.float32 else "bf16"
    # full power-law spectrum sigma_i = 10 / i over all min(N, D) directions: no flat noise bulk at rank k, so a
    # few power iterations converge (sigma_{l+1} / sigma_k is about k / l)
    g = torch.Generator().manual_seed(N + D + k)
    r = min(N, D)
    spec = 10.0 / torch.arange(1, r + 1, dtype=torch.float64)
    blocks = []
    for _ in range(2):
        left = torch.linalg.qr(torch.randn(N, r, generator=g, dtype=torch.float64))[0]
        right = torch.linalg.qr(torch.randn(D, r, generator=g, dtype=torch.float64))[0]
        blocks.append(((left * spec) @ right.T).to(dtype))
    F = torch.stack(blocks).contiguous()
    V, sigma, fro2 = pkg.fit_basis(F.to(DEV), k, p=p, q=8)
    torch.cuda.synchronize()
    for b in range(2):
        _fit_checks(F[b], V[b], sigma[b], fro2[b], k, store)


@pytest.mark.parametrize("dtype,N,D,k,p", [(torch.float32, 300, 128, 12, 20), (torch.bfloat16, 400, 256, 24, 40),
                                            (torch.bfloat16, 500, 256, 70, 90)], ids=["f32", "bf16-mfma", "bf16-l160"])
def test_fit_basis_without_power_iterations(dtype, N, D, k, p):
    """q = -1: the orthonormalised Gaussian test matrix goes straight into the Rayleigh-Ritz step.  On features of
    exact rank <= l the sketch then already spans the whole row space, so the result must be the exact decomposition
    (a plain randomized range finder is exact for rank-deficient inputs)."""
    store = "f32" if dtype == torch.float32 else "bf16"
    rank = k + p // 2
    g = torch.Generator().manual_seed(N + k)
    left = torch.linalg.qr(torch.randn(N, rank, generator=g, dtype=torch.float64))[0]
    right = torch.linalg.qr(torch.randn(D, rank, generator=g, dtype=torch.float64))[0]
    spec = 10.0 * torch.arange(1, rank + 1, dtype=torch.float64) ** -0.7
    Fx = (left * spec) @ right.T
    if store == "bf16":
        # bf16 rounding adds a full-rank perturbation of relative size 2^-9: its effect on the leading k values and
        # on the energy they capture is far inside the bf16 bar
        Fx = Fx.to(torch.bfloat16)
    F = Fx.to(dtype).unsqueeze(0).contiguous()
    V, sigma, fro2 = pkg.fit_basis(F.to(DEV), k, p=p, q=-1)
    torch.cuda.synchronize()
    _fit_checks(F[0], V[0], sigma[0], fro2[0], k, store, lead=max(1, k // 4))


def test_fit_status_words():
    """Per-block status of the fit, read from the workspace: 0 for well-conditioned features; the rank-deficiency
    flag for features of exact rank < l (the fitted basis still passes every check); the sweep-cap flag when the
    host allows the small SVD a single sweep (every kernel still runs to its normal end)."""
    g = torch.Generator().manual_seed(77)
    N, D, k = 400, 256, 24
    r_all = min(N, D)                                           # full power-law spectrum: well conditioned
    good = (torch.linalg.qr(torch.randn(N, r_all, generator=g, dtype=torch.float64))[0]
            * (10.0 / torch.arange(1, r_all + 1, dtype=torch.float64))) \
        @ torch.linalg.qr(torch.randn(D, r_all, generator=g, dtype=torch.float64))[0].T
    rank = 30                                                   # < l = 48
    left = torch.linalg.qr(torch.randn(N, rank, generator=g, dtype=torch.float64))[0]
    right = torch.linalg.qr(torch.randn(D, rank, generator=g, dtype=torch.float64))[0]
    low = ((left * (10.0 * torch.arange(1, rank + 1, dtype=torch.float64) ** -0.8)) @ right.T)
    for dtype, store in ((torch.bfloat16, "bf16"), (torch.float32, "f32")):
        # bf16 rounding would make the low-rank block full rank at the 2^-9 level: keep it exactly low rank by
        # building it from bf16-representable factors only in the float32 case
        F = torch.stack([good.to(dtype), low.to(dtype)]).contiguous()
        V, sigma, fro2, status = pkg.fit_basis(F.to(DEV), k, q=6, return_status=True)
        torch.cuda.synchronize()
        status = status.cpu().tolist()
        assert status[0] == 0, f"{store}: well-conditioned block reports {status[0]}"
        _fit_checks(F[0], V[0], sigma[0], fro2[0], k, store)
        if store == "f32":
            assert status[1] == pkg.SVDC_FIT_RANK_DEFICIENT, f"rank-deficient block reports {status[1]}"
            _fit_checks(F[1], V[1], sigma[1], fro2[1], k, store)
        # one sweep is never enough for a 48 x 48 factor: flagged, and nothing else changes for the other flag
        _, _, _, capped = pkg.fit_basis(F.to(DEV), k, q=6, max_sweeps=1, return_status=True)
        torch.cuda.synchronize()
        capped = capped.cpu().tolist()
        assert capped[0] == pkg.SVDC_FIT_JACOBI_CAPPED
        assert capped[1] & pkg.SVDC_FIT_JACOBI_CAPPED
    shape = pkg.make_shape(F.to(DEV), k)
    assert pkg.svdcache_workspace_bytes(shape) == pkg.svdcache_fit_workspace_bytes(shape) > 0
    assert 0 < pkg.svdcache_fit_status_offset(shape) < pkg.svdcache_workspace_bytes(shape)


def test_fit_status_words_column_block_jacobi():
    """The sweep-cap flag of the Jacobi by column blocks (sketch widths above 138), whose convergence is tracked in
    three rotating counters on the device: caps of 1, 2 and 3 sweeps end on each of the three counters and are all
    too few for a 192 x 192 factor (flag set, the call still succeeds and V is orthonormal); the default cap converges
    (no flag) and gives the basis of the exact decomposition."""
    g = torch.Generator().manual_seed(78)
    N, D, k = 500, 256, 96
    r_all = min(N, D)
    blocks = []
    for _ in range(2):
        left = torch.linalg.qr(torch.randn(N, r_all, generator=g, dtype=torch.float64))[0]
        right = torch.linalg.qr(torch.randn(D, r_all, generator=g, dtype=torch.float64))[0]
        blocks.append(((left * (10.0 / torch.arange(1, r_all + 1, dtype=torch.float64))) @ right.T).to(torch.bfloat16))
    F = torch.stack(blocks).contiguous()
    for cap in (1, 2, 3):
        V, _, _, status = pkg.fit_basis(F.to(DEV), k, q=8, max_sweeps=cap, return_status=True)
        torch.cuda.synchronize()
        assert status.cpu().tolist() == [pkg.SVDC_FIT_JACOBI_CAPPED] * 2, f"cap {cap}: {status.cpu().tolist()}"
        Vd = V.double().cpu()
        for b in range(2):
            # columns of L after any number of rotations, normalised: unit norm, but not yet orthogonal
            assert (Vd[b].norm(dim=0) - 1).abs().max() < 1e-3
    V, sigma, fro2, status = pkg.fit_basis(F.to(DEV), k, q=8, return_status=True)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0, 0]
    for b in range(2):
        _fit_checks(F[b], V[b], sigma[b], fro2[b], k, "bf16")


def test_fit_basis_flux_block_full_size():
    """One FLUX-shaped block (4608 x 3072 bf16, k = 32) at full size against the exact decomposition."""
    wl = WORKLOADS["flux1"]
    F = FeatureStream(wl, 0, work=torch.float32).at(0).unsqueeze(0)
    V, sigma, fro2 = pkg.fit_basis(F.to(DEV), wl.k)
    torch.cuda.synchronize()
    _fit_checks(F[0], V[0], sigma[0], fro2[0], wl.k, "bf16")


@pytest.mark.parametrize("B,N,D,k", [(2, 200, 256, 32), (1, 150, 3072, 32), (1, 100, 3072, 64), (1, 140, 512, 128)])
def test_mfma_fast_precision_mode_is_within_the_bf16_tolerance(B, N, D, k):
    """SVDC_FAST: single bf16 operands.  Same parity bar (2e-2 for bf16 storage), larger error than
    the default mode."""
    F, V, S0 = _lowrank_problem(B, N, D, k, seed=N + k)
    Fd, Vd = F.to(DEV), V.to(DEV)
    errs = {}
    for mode in (pkg.SVDC_PRECISE, pkg.SVDC_FAST):
        shape = pkg.make_shape(Fd, k, precision=mode)
        pk = pkg.pack_basis(shape, Vd)
        R, S, Cc, Fh = torch.empty_like(Fd), S0.clone().to(DEV), torch.empty(B, N, k, device=DEV), torch.empty_like(Fd)
        pkg.svdcache_full_step(shape, Fd, Vd, pk, R, S, Cc, 0.5, False)
        pkg.svdcache_forecast(shape, S, Vd, pk, R, Fh)
        torch.cuda.synchronize()
        worst = 0.0
        fast = mode == pkg.SVDC_FAST
        for b in range(B):
            Rr, Sr, Cr = ref_full_step(to_np(F[b]), to_np(V[b]), to_np(S0[b]), 0.5, False, "bf16")
            assert_close(to_np(R[b]), Rr, "bf16", f"R[{b}] mode {mode}", floor_of=to_np(F[b]), fast=fast)
            assert_close(to_np(S[b]), Sr, "bf16", f"S[{b}] mode {mode}", fast=fast)
            assert_close(to_np(Cc[b]), Cr, "bf16", f"C[{b}] mode {mode}", fast=fast)
            assert_close(to_np(Fh[b]), ref_forecast(Sr, to_np(V[b]), Rr, "bf16"), "bf16", f"Fhat[{b}] mode {mode}",
                         fast=fast, scale_of=to_np(F[b]), ulp_of=Rr)
            worst = max(worst, rel_err(to_np(R[b]), Rr))
        errs[mode] = worst
    assert errs[pkg.SVDC_PRECISE] <= 3e-3 and errs[pkg.SVDC_FAST] <= 1.5e-2


@pytest.mark.parametrize("B,N,k", [(4, 4090, 32), (4, 3060, 64), (2, 4090, 128)])
def test_full_step_tiles_with_a_row_tile_in_lds(B, N, k):
    """3072 channels and one round of 256 or more workgroup tiles, each block ending in a partly filled tile.  At
    rank 64 these are the launches that keep the third row tile of a workgroup tile in LDS (both operand modes);
    ranks 32 and 128 run the register-only tiles at the same sizes.  Every element is compared, out of place and
    in place (R aliases F), with and without the coefficient output."""
    D = 3072
    F, V, S0 = _lowrank_problem(B, N, D, k, seed=N + k)
    ref = [ref_full_step(to_np(F[b]), to_np(V[b]), to_np(S0[b]), 0.3, False, "bf16") for b in range(B)]
    Vd = V.to(DEV)
    for mode in (pkg.SVDC_PRECISE, pkg.SVDC_FAST):
        coef = "f32" if mode == pkg.SVDC_PRECISE else "bf16"
        fast = mode == pkg.SVDC_FAST
        for inplace in (False, True):
            Fd = F.to(DEV)
            shape = pkg.make_shape(Fd, k, precision=mode)
            pk = pkg.pack_basis(shape, Vd)
            R = Fd if inplace else torch.full_like(Fd, 7.0)
            S = S0.clone().to(DEV)
            Cc = None if inplace else torch.empty(B, N, k, device=DEV)
            pkg.svdcache_full_step(shape, Fd, Vd, pk, R, S, Cc, 0.3, False)
            torch.cuda.synchronize()
            for b in range(B):
                Rr, Sr, Cr = ref[b]
                assert_close(to_np(R[b]), Rr, "bf16", f"R[{b}] mode {mode} inplace {inplace}", floor_of=to_np(F[b]),
                             fast=fast)
                assert_close(to_np(S[b]), Sr, coef, f"S[{b}] mode {mode}", fast=fast)
                if Cc is not None:
                    assert_close(to_np(Cc[b]), Cr, coef, f"C[{b}] mode {mode}", fast=fast)
                assert rel_err(to_np(R[b]), Rr) <= (3e-3 if mode == pkg.SVDC_PRECISE else 1.5e-2)


# ---------------------------------------------------------------------------------------------
# full-size launches (the configurations bench.py times), checked on sampled rows
# ---------------------------------------------------------------------------------------------

def _full_size_fit_check(F_block, V_b, sigma_b, fro2_b, k, store):
    """The fitted basis of one full-size block against the exact truncated SVD (Sec. 3.2, Eq. 4-5; the oracle takes
    the Gram route at these sizes): singular values, the energy the fitted directions capture relative to the
    optimum, and that the reported sigma_j are the norms of F v_j.  Unlike "the cached step right after the first
    full step returns F", which holds for any orthonormal V, these say WHICH subspace was found.

    Subspace iteration with a sketch of width l and q applications of F^T F finds sigma_j to a relative error of
    about (sigma_{l+1} / sigma_j)^(2 (2q + 1)): the values above the flat bulk of the synthetic residual are compared
    at the parity bar, those inside it (where sigma_{l+1} / sigma_j is close to one and no number of iterations
    separates them: rank 64 of the FLUX-shaped stream) by what still holds there -- a Rayleigh-Ritz value never
    exceeds the exact one, and the energy captured by all k directions is within 1e-3 of the optimum."""
    tol = TOL[store]
    Fd = to_np(F_block)
    l = min(2 * k, min(Fd.shape), 256)                  # the fit's defaults: p = k, q = 3 (bf16) / 5 (f32)
    q = 3 if store == "bf16" else 5
    _, s_more, fr = ref_fit_basis(Fd, min(l + 1, min(Fd.shape)))
    sr = s_more[:k]
    Vg, sg = to_np(V_b), to_np(sigma_b)
    assert np.abs(Vg.T @ Vg - np.eye(k)).max() <= 1e-5
    conv = (s_more[-1] / sr) ** (2 * (2 * q + 1)) if l + 1 <= min(Fd.shape) else np.zeros(k)
    err = np.abs(sg / sr - 1)
    resolved = 30 * conv <= tol
    assert resolved[: max(1, k // 2)].all(), "the leading half of the spectrum must be resolvable at the default q"
    assert err[resolved].max() <= tol, f"sigma rel err {err[resolved].max():.2e} on the resolved values"
    assert np.all(sg <= sr * (1 + 1e-5)) and np.all(sg >= 0.8 * sr), f"sigma outside [0.8, 1] x exact: {err.max():.2e}"
    assert abs(float(fro2_b) / fr - 1) <= 1e-5
    proj = Fd @ Vg
    deficit = 1 - np.sum(proj ** 2) / np.sum(sr ** 2)
    assert deficit <= 1e-3, f"captured-energy deficit {deficit:.2e}"      # measured: a few 1e-6 at the default q
    assert np.abs(np.linalg.norm(proj, axis=0) / sg - 1).max() <= 1e-4


def _sampled_row_parity(wl, B, blocks_to_check, n_rows, precision=0, fit_check_block=None):
    """Run fit + pack + two full steps + one cached step at full size on GPU-generated features and
    recompute sampled token rows with the oracle (rows are independent given V and S).  Nothing the GPU
    computed is handed to the oracle: it gets the generated features, the generator's basis and its own state."""
    store = wl.dtype
    feats = [torch.empty(B, wl.N, wl.D, device=DEV, dtype=torch_dtype(store)) for _ in range(2)]
    Vgen = torch.empty(B, wl.D, wl.k, device=DEV)
    for b in range(B):
        fs = FeatureStream(wl, b, device=DEV)
        feats[0][b], feats[1][b] = fs.at(0), fs.at(wl.interval)
        Vgen[b] = fs.V[:, :wl.k].float()          # the generator's leading directions: the basis of both sides
        del fs
    shape = pkg.make_shape(feats[0], wl.k, precision=precision)
    assert pkg.svdcache_has_mfma_path(shape)
    R = torch.empty_like(feats[0])
    S = torch.empty(B, wl.N, wl.k, device=DEV)
    Cc = torch.empty_like(S)
    Fh = torch.empty_like(R)
    # fit + pack + step with the FITTED basis, checked by an identity that needs no oracle: right after the
    # first full step the cached step gives the feature back (up to the rounding of R and Fhat)
    V, sigma, fro2 = pkg.fit_basis(feats[0], wl.k)
    pk = pkg.pack_basis(shape, V)
    pkg.svdcache_full_step(shape, feats[0], V, pk, R, S, None, wl.alpha, True)
    pkg.svdcache_forecast(shape, S, V, pk, R, Fh)
    torch.cuda.synchronize()
    back = 1e-5 if store == "f32" else (6e-3 if precision == 0 else 2e-2)
    for b in blocks_to_check:
        Vb = to_np(V[b])
        assert np.abs(Vb.T @ Vb - np.eye(wl.k)).max() <= 1e-5
        assert rel_err(to_np(Fh[b][:512]), to_np(feats[0][b][:512])) <= back
    if fit_check_block is not None:
        b = fit_check_block
        _full_size_fit_check(feats[0][b], V[b], sigma[b], fro2[b], wl.k, store)
    # parity of the steps against the oracle, both sides on the generator's basis
    pk = pkg.pack_basis(shape, Vgen)
    pkg.svdcache_full_step(shape, feats[0], Vgen, pk, R, S, None, wl.alpha, True)
    S0 = S.clone()
    pkg.svdcache_full_step(shape, feats[1], Vgen, pk, R, S, Cc, wl.alpha, False)
    pkg.svdcache_forecast(shape, S, Vgen, pk, R, Fh)
    # the same two calls with the state handed over in packed form: identical results at full size
    Sp = pkg.alloc_packed_state(shape, DEV)
    S2, R2, Fh2 = S0.clone(), torch.empty_like(R), torch.empty_like(R)
    pkg.svdcache_full_step_packed(shape, feats[1], Vgen, pk, R2, S2, None, Sp, wl.alpha, False)
    pkg.svdcache_forecast_packed(shape, Sp, pk, R2, Fh2)
    torch.cuda.synchronize()
    for b in blocks_to_check:
        assert torch.equal(S2[b], S[b]) and torch.equal(R2[b], R[b]) and torch.equal(Fh2[b], Fh[b])
    del S2, R2, Fh2, Sp
    g = torch.Generator().manual_seed(wl.config_id)
    fast = precision != 0
    for b in blocks_to_check:
        assert torch.isfinite(R[b].float()).all() and torch.isfinite(Fh[b].float()).all() and torch.isfinite(S[b]).all()
        rows = torch.cat([torch.tensor([0, 1, 15, 16, 31, 32, wl.N - 17, wl.N - 16, wl.N - 1]),
                          torch.randint(0, wl.N, (n_rows,), generator=g)]).unique()
        Vb = to_np(Vgen[b])
        F0r, F1r = to_np(feats[0][b][rows]), to_np(feats[1][b][rows])
        _, S0r, _ = ref_full_step(F0r, Vb, None, wl.alpha, True, store)
        coef_store = "f32" if precision == 0 else "bf16"   # SVDC_FAST rounds V to bf16 in the projection
        assert_close(to_np(S0[b][rows]), S0r, coef_store, f"S after init, block {b}", fast=fast)
        Rr, S1r, C1r = ref_full_step(F1r, Vb, S0r, wl.alpha, False, store)       # the oracle's own state
        assert_close(to_np(R[b][rows]), Rr, store, f"R block {b}", floor_of=F1r, fast=fast)
        assert_close(to_np(S[b][rows]), S1r, coef_store, f"S block {b}", fast=fast)
        assert_close(to_np(Cc[b][rows]), C1r, coef_store, f"C block {b}", fast=fast)
        Fr = ref_forecast(S1r, Vb, Rr, store)
        assert_close(to_np(Fh[b][rows]), Fr, store, f"Fhat block {b}", fast=fast, scale_of=F1r, ulp_of=Rr)
    return sigma, fro2, feats


def test_flux57_full_size_launch_sampled_rows():
    """Config 3 as bench.py launches it: 57 blocks x 4608 x 3072 bf16, k = 32, one launch per kernel."""
    wl = WORKLOADS["flux57"]
    sigma, fro2, feats = _sampled_row_parity(wl, wl.B, blocks_to_check=[0, 28, 56], n_rows=96)
    # the fitted singular values of one block against the exact ones
    _, sr, fr = ref_fit_basis(to_np(feats[0][56]), wl.k)
    assert np.abs(to_np(sigma[56]) / sr - 1).max() <= TOL["bf16"]
    assert abs(float(fro2[56]) / fr - 1) <= 1e-5


@pytest.mark.parametrize("k", [16, 64])
def test_flux57_full_size_launch_other_ranks(k):
    """Config 3 lists the ranks 16, 32 and 64: the same 57-block launches at the other two ranks (rank 64 runs the
    full step with 48-row tiles whose third row tile sits in LDS, over 22 rounds of the persistent grid)."""
    wl = WORKLOADS["flux57"].with_(k=k)
    _sampled_row_parity(wl, wl.B, blocks_to_check=[0, 31, 56], n_rows=64, fit_check_block=31)


def test_flux57_full_size_launch_fast_mode():
    wl = WORKLOADS["flux57"].with_(B=8)
    _sampled_row_parity(wl, wl.B, blocks_to_check=[0, 7], n_rows=64, precision=pkg.SVDC_FAST)


def test_hunyuan_shape_offsets_beyond_2_to_31_sampled_rows():
    """Config 4 shape (119056 tokens x 3072, k = 64) on 7 of its 60 blocks: the last block starts 2.19e9 elements
    (4.4e9 bytes) into the tensors, beyond what 32-bit element or byte offsets reach.  First and last block are
    compared with the oracle on sampled rows; the fitted basis of the last block against the exact decomposition."""
    wl = WORKLOADS["hyv60"]
    assert 6 * wl.N * wl.D > 2 ** 31
    _sampled_row_parity(wl, 7, blocks_to_check=[0, 6], n_rows=96, fit_check_block=6)


def test_hunyuan_60_block_launch_first_middle_and_last_block():
    """Config 4 at its real size, the launch bench.py times: 60 blocks x 119056 x 3072 bf16 (43.9 GB per tensor),
    k = 64.  Blocks 0 and 59 hold generated features; to keep the generation short the blocks between hold copies
    of them (even blocks of block 0, odd ones of block 59) with the matching basis.  Sampled rows of the first
    and last block are recomputed by the oracle; a middle block must equal, bit for bit, the block it copies (every
    element of it is thereby compared with a block whose rows were sampled against the oracle)."""
    wl = WORKLOADS["hyv60"]
    B, N, D, k = wl.B, wl.N, wl.D, wl.k
    F = torch.empty(B, N, D, device=DEV, dtype=torch.bfloat16)
    Vgen = torch.empty(B, D, k, device=DEV)
    for b in (0, B - 1):
        fs = FeatureStream(wl, b, device=DEV)
        F[b] = fs.at(0)
        Vgen[b] = fs.V[:, :k].float()
        del fs
    for b in range(1, B - 1):
        src = 0 if b % 2 == 0 else B - 1
        F[b].copy_(F[src])
        Vgen[b].copy_(Vgen[src])
    shape = pkg.make_shape(F, k)
    pk = pkg.pack_basis(shape, Vgen)
    R = torch.empty_like(F)
    S = torch.empty(B, N, k, device=DEV)
    pkg.svdcache_full_step(shape, F, Vgen, pk, R, S, None, wl.alpha, True)
    torch.cuda.synchronize()
    mid = 30
    assert torch.equal(R[mid], R[0]) and torch.equal(S[mid], S[0])
    assert torch.equal(R[mid + 1], R[B - 1]) and torch.equal(S[mid + 1], S[B - 1])
    g = torch.Generator().manual_seed(wl.config_id + 60)
    ref = {}
    for b in (0, B - 1):
        rows = torch.cat([torch.tensor([0, 15, 16, 47, 48, N - 17, N - 1]),
                          torch.randint(0, N, (64,), generator=g)]).unique()
        Fr = to_np(F[b][rows])
        Rr, Sr, _ = ref_full_step(Fr, to_np(Vgen[b]), None, wl.alpha, True, "bf16")
        assert_close(to_np(R[b][rows]), Rr, "bf16", f"R block {b}", floor_of=Fr)
        assert_close(to_np(S[b][rows]), Sr, "f32", f"S block {b}")
        ref[b] = (rows, Fr, Rr, Sr)
    # the cached step in place (Fhat takes the buffer of R), same launch size
    pkg.svdcache_forecast(shape, S, Vgen, pk, R, R)
    torch.cuda.synchronize()
    assert torch.equal(R[mid], R[0]) and torch.equal(R[mid + 1], R[B - 1])
    for b in (0, B - 1):
        rows, Fr, Rr, Sr = ref[b]
        assert_close(to_np(R[b][rows]), ref_forecast(Sr, to_np(Vgen[b]), Rr, "bf16"), "bf16", f"Fhat block {b}",
                     scale_of=Fr, ulp_of=Rr)


def test_rank_sweep_at_stacked_prompt_shape():
    """Config 5 shape: 4 prompts stacked along N with one shared basis, k in {16, 64, 128}."""
    for k in (16, 64, 128):
        wl = WORKLOADS["sweep"].with_(k=k)
        _sampled_row_parity(wl, 1, blocks_to_check=[0], n_rows=64)


@pytest.mark.parametrize("k", [8, 32, 128])
def test_rank_sweep_float32_at_stacked_prompt_shape(k):
    """The float32 half of config 5 at its real size (18432 x 3072): the matrix-core kernels with float32 features
    split into bf16 high + low parts on the fly, sampled rows against the oracle at the float32 bar."""
    wl = WORKLOADS["sweep"].with_(k=k, dtype="f32")
    _sampled_row_parity(wl, 1, blocks_to_check=[0], n_rows=64, fit_check_block=0 if k == 32 else None)


# ---------------------------------------------------------------------------------------------
# float32 features on the matrix cores (operands split into bf16 high + low parts)
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("B,N,D,k", [(2, 200, 256, 32), (1, 77, 512, 8), (1, 131, 512, 128), (1, 150, 3072, 32),
                                     (1, 70, 3072, 64), (2, 49, 256, 20), (1, 60, 1024, 32), (1, 50, 1536, 16),
                                     (1, 70, 2048, 64), (1, 40, 4096, 32), (1, 50, 1152, 32), (1, 70, 1920, 64),
                                     (1, 40, 2560, 16), (1, 36, 5120, 32), (1, 129, 5120, 128)])
def test_mfma_float32_features(B, N, D, k):
    Fb, V, S0 = _lowrank_problem(B, N, D, k, seed=N * 3 + k)
    g = torch.Generator().manual_seed(N)
    F = Fb.float() + 1e-3 * torch.randn(B, N, D, generator=g)      # not bf16-representable
    shape = pkg.make_shape(F, k)
    assert pkg.svdcache_has_mfma_path(shape)
    for init in (True, False):
        R, S, Cc, shape, pk = _run_full(F, D, V, S0, 0.5, init)
        assert pk is not None
        Fh = torch.empty_like(R)
        pkg.svdcache_forecast(shape, S, V.to(DEV), pk, R, Fh)
        torch.cuda.synchronize()
        for b in range(B):
            Rr, Sr, Cr = ref_full_step(to_np(F[b]), to_np(V[b]), to_np(S0[b]), 0.5, init, "f32")
            assert_close(to_np(R[b]), Rr, "f32", f"R[{b}]", floor_of=to_np(F[b]))
            assert_close(to_np(S[b]), Sr, "f32", f"S[{b}]")
            assert_close(to_np(Cc[b]), Cr, "f32", f"C[{b}]")
            Fr = ref_forecast(Sr, to_np(V[b]), Rr, "f32")       # the oracle's own state
            assert_close(to_np(Fh[b]), Fr, "f32", f"Fhat[{b}]", scale_of=to_np(F[b]))


def test_step_kernels_are_bitwise_deterministic():
    """No atomics on the output path of the step kernels: two runs on the same inputs give the same bits
    (matrix-core path at FLUX width and the general path)."""
    for (B, N, D, k) in [(3, 300, 3072, 32), (2, 130, 200, 17)]:
        Fbuf, V, S0 = _rand_problem(B, N, D, k, torch.bfloat16, seed=N)
        runs = []
        for _ in range(2):
            R, S, Cc, shape, pk = _run_full(Fbuf, D, V, S0, 0.4, False)
            Fh = torch.empty_like(R)
            pkg.svdcache_forecast(shape, S, V.to(DEV), pk, R, Fh)
            torch.cuda.synchronize()
            runs.append((R.clone(), S.clone(), Cc.clone(), Fh.clone()))
        for a, b in zip(*runs):
            assert torch.equal(a, b)


def test_flux57_fit_is_bitwise_reproducible():
    """At the batch size of the benchmark no step of the fit sums in an order that depends on scheduling
    (back-projection with one row group per block, Gram matrices from ordered partial sums): two fits of the
    same features give the same basis, bit for bit."""
    wl = WORKLOADS["flux57"]
    F = torch.empty(wl.B, wl.N, wl.D, device=DEV, dtype=torch.bfloat16)
    for b in range(wl.B):
        F[b] = FeatureStream(wl, b, device=DEV).at(0)
    V1, s1, _ = pkg.fit_basis(F, wl.k)
    V2, s2, _ = pkg.fit_basis(F, wl.k)
    torch.cuda.synchronize()
    assert torch.equal(V1, V2) and torch.equal(s1, s2)


def test_flux_block_trajectory_against_a_free_running_oracle():
    """Config 2 (one FLUX-sized block, bf16, k = 32, full step every 5) over 16 timesteps on the matrix-core
    path.  The oracle keeps its OWN state on 80 sampled token rows (rows are independent given V), so errors of
    the GPU path would have to stay small over four EMA updates, not just within one call."""
    wl = WORKLOADS["flux1"].with_(T=16)
    fs = FeatureStream(wl, 0, device=DEV)
    F0 = fs.at(0).unsqueeze(0).contiguous()
    shape = pkg.make_shape(F0, wl.k)
    V = fs.V[:, :wl.k].float().unsqueeze(0).contiguous()          # the generator's leading directions
    pk = pkg.pack_basis(shape, V)
    assert pk is not None
    Vn = to_np(V[0])
    rows = torch.cat([torch.tensor([0, 15, 16, 47, 48, wl.N - 1]),
                      torch.randint(0, wl.N, (74,), generator=torch.Generator().manual_seed(4))]).unique()
    R = torch.empty_like(F0)
    S = torch.empty(1, wl.N, wl.k, device=DEV)
    Fh = torch.empty_like(F0)
    Rr = Sr = None
    for t in range(wl.T):
        if is_full_step(t, wl.interval):
            Ft = fs.at(t).unsqueeze(0).contiguous()
            pkg.svdcache_full_step(shape, Ft, V, pk, R, S, None, wl.alpha, t == 0)
            torch.cuda.synchronize()
            Frows = to_np(Ft[0][rows])
            Rr, Sr, _ = ref_full_step(Frows, Vn, Sr, wl.alpha, t == 0, "bf16")
            assert_close(to_np(R[0][rows]), Rr, "bf16", f"t={t} R", floor_of=Frows)
            assert_close(to_np(S[0][rows]), Sr, "f32", f"t={t} S")
        else:
            pkg.svdcache_forecast(shape, S, V, pk, R, Fh)
            torch.cuda.synchronize()
            assert_close(to_np(Fh[0][rows]), ref_forecast(Sr, Vn, Rr, "bf16"), "bf16", f"t={t} Fhat", scale_of=Frows,
                         ulp_of=Rr)
