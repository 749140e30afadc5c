"""GPU parity of the entry points beyond the three basic ones: rank selection by retained energy,
per-block rank truncation, and cached steps with forecasters that are linear in stored states."""
import numpy as np
import pytest
import torch

import paper_2601_07396_amd as pkg
from oracle import (ref_full_step, ref_select_rank, ref_truncate_basis, ref_forecast_combine,
                    ref_extrapolation_weights, ref_fit_basis)
from synth import WORKLOADS, FeatureStream
from util import TOL, to_np, assert_close, principal_sines

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _problem(B, N, D, k, dtype, seed, nstates=1):
    g = torch.Generator().manual_seed(seed)
    R = torch.randn(B, N, D, generator=g).to(dtype)
    X = torch.randn(B, N, D, generator=g).to(dtype)
    V = torch.linalg.qr(torch.randn(B, D, k, generator=g, dtype=torch.float64))[0].float().contiguous()
    S = [3.0 * torch.randn(B, N, k, generator=g) for _ in range(nstates)]
    return R, X, V, S


# ------------------------------------------------------------------ rank selection (Eq. 6)

def test_select_rank_matches_oracle_exactly():
    g = torch.Generator().manual_seed(3)
    B, k = 57, 32
    sig = torch.sort(torch.rand(B, k, generator=g) * 4 + 0.01, dim=1, descending=True)[0]
    energy = (sig.double() ** 2).sum(1)
    fro2 = (energy * (1.0 + 0.4 * torch.rand(B, generator=g).double())).float()     # part of the energy is outside
    fro2[::7] = energy[::7].float()                                                  # ... or none of it
    ks = torch.empty(B, dtype=torch.int32, device=DEV)
    ok = torch.empty(B, dtype=torch.int32, device=DEV)
    for tau in (0.05, 0.5, 0.85, 0.95, 1.0):
        pkg.svdcache_select_rank(sig.to(DEV), fro2.to(DEV), tau, ks, ok)
        torch.cuda.synchronize()
        for b in range(B):
            want = ref_select_rank(sig[b].numpy(), float(fro2[b]), tau)
            assert (int(ks[b]), bool(ok[b])) == want, (tau, b)
    # the flag is optional
    pkg.svdcache_select_rank(sig.to(DEV), fro2.to(DEV), 0.85, ks, None)
    torch.cuda.synchronize()
    assert all(int(ks[b]) == ref_select_rank(sig[b].numpy(), float(fro2[b]), 0.85)[0] for b in range(B))


def test_select_rank_on_a_fitted_basis():
    """tau-rule on the GPU fit of the tiny configuration against the rule applied to the exact spectrum."""
    wl = WORKLOADS["tiny"]
    F = torch.stack([FeatureStream(wl, b).at(0) for b in range(wl.B)])
    k = 32
    V, sigma, fro2 = pkg.fit_basis(F.to(DEV), k, q=8)
    ks = torch.empty(wl.B, dtype=torch.int32, device=DEV)
    ok = torch.empty(wl.B, dtype=torch.int32, device=DEV)
    for tau in (0.5, 0.85, 0.99):
        pkg.svdcache_select_rank(sigma, fro2, tau, ks, ok)
        torch.cuda.synchronize()
        for b in range(wl.B):
            _, s_exact, fr = ref_fit_basis(to_np(F[b]), k)
            want = ref_select_rank(s_exact.astype(np.float32), fr, tau)
            frac = np.cumsum(s_exact ** 2) / fr
            if np.min(np.abs(frac - tau)) > 1e-4:        # away from a tie the decision is unique
                assert (int(ks[b]), bool(ok[b])) == want, (tau, b)


def test_select_rank_and_truncate_reject_bad_arguments():
    sig = torch.ones(2, 4, device=DEV)
    fro = torch.ones(2, device=DEV)
    ks = torch.empty(2, dtype=torch.int32, device=DEV)
    for tau in (0.0, -1.0, 1.5, float("nan")):
        with pytest.raises(pkg.SvdcError) as e:
            pkg.svdcache_select_rank(sig, fro, tau, ks, None)
        assert e.value.code == -5
    with pytest.raises(pkg.SvdcError) as e:
        pkg.svdcache_select_rank(sig, fro, 0.5, None, None)
    assert e.value.code == -1


# ------------------------------------------------------------------ per-block ranks in one launch

@pytest.mark.parametrize("dtype,D", [(torch.float32, 64), (torch.bfloat16, 72), (torch.bfloat16, 256),
                                     (torch.float32, 256)], ids=["f32-general", "bf16-general", "bf16-mfma", "f32-mfma"])
def test_truncated_basis_gives_per_block_rank(dtype, D):
    store = "f32" if dtype == torch.float32 else "bf16"
    B, N, k = 3, 100, 16
    g = torch.Generator().manual_seed(D)
    F = torch.randn(B, N, D, generator=g).to(dtype)
    V = torch.linalg.qr(torch.randn(B, D, k, generator=g, dtype=torch.float64))[0].float().contiguous()
    sigma = torch.arange(k, 0, -1).float().repeat(B, 1)
    k_star = torch.tensor([16, 5, 1], dtype=torch.int32)
    Vd, sd = V.to(DEV), sigma.to(DEV)
    shape = pkg.make_shape(F, k)
    pkg.svdcache_truncate_basis(shape, Vd, sd, k_star.to(DEV))
    torch.cuda.synchronize()
    for b in range(B):
        Vt, st = ref_truncate_basis(to_np(V[b]), to_np(sigma[b]), int(k_star[b]))
        assert np.array_equal(to_np(Vd[b]), Vt) and np.array_equal(to_np(sd[b]), st)
    pk = pkg.pack_basis(shape, Vd)
    assert (pk is not None) == (D == 256)
    Fd = F.to(DEV)
    R = torch.empty_like(Fd)
    S = torch.empty(B, N, k, device=DEV)
    Cc = torch.empty_like(S)
    pkg.svdcache_full_step(shape, Fd, Vd, pk, R, S, Cc, 0.5, True)
    torch.cuda.synchronize()
    for b in range(B):
        ks = int(k_star[b])
        Rr, Sr, Cr = ref_full_step(to_np(F[b]), to_np(V[b][:, :ks]), None, 0.5, True, store)   # the rank-k* step
        assert_close(to_np(R[b]), Rr, store, f"R[{b}]", floor_of=to_np(F[b]))
        # few columns (k* may be 1): scale the element-wise allowance by the feature rows, not by the coefficients
        assert_close(to_np(Cc[b][:, :ks]), Cr, "f32", f"C[{b}]", scale_of=to_np(F[b]))
        assert not to_np(Cc[b][:, ks:]).any() and not to_np(S[b][:, ks:]).any()
    # sigma is optional
    pkg.svdcache_truncate_basis(shape, Vd, None, torch.zeros(B, dtype=torch.int32, device=DEV))
    torch.cuda.synchronize()
    assert not Vd.any()


# ------------------------------------------------------------------ forecasters linear in stored states

def test_extrapolation_weights_host_function():
    for order in range(4):
        for off, itv in [(1, 6), (5, 6), (2.5, 3), (0, 4), (-4, 4)]:
            got = pkg.svdcache_extrapolation_weights(order, off, itv)
            want = ref_extrapolation_weights(order, off, itv)
            assert np.allclose(got, want.astype(np.float32), rtol=2e-7, atol=1e-7), (order, off, itv)
    for bad in [(-1, 1, 6), (4, 1, 6), (1, 1, 0)]:
        with pytest.raises(pkg.SvdcError) as e:
            pkg.svdcache_extrapolation_weights(*bad)
        assert e.value.code == -5


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("B,N,D,k", [(2, 67, 72, 5), (1, 130, 200, 17),                       # general kernels
                                     (2, 150, 256, 32), (1, 77, 512, 8), (1, 140, 512, 128),   # matrix-core kernels
                                     (1, 150, 3072, 32), (1, 70, 3072, 64), (1, 33, 1024, 20)])
def test_forecast_combine(dtype, B, N, D, k):
    store = "f32" if dtype == torch.float32 else "bf16"
    R, X, V, S = _problem(B, N, D, k, dtype, seed=N + D + k, nstates=4)
    shape = pkg.make_shape(R, k)
    Rd, Xd, Vd, Sd = R.to(DEV), X.to(DEV), V.to(DEV), [s.to(DEV) for s in S]
    pk = pkg.pack_basis(shape, Vd)
    cases = [(1, [1.0], False), (2, [1.5, -0.5], False), (3, [1.875, -1.25, 0.375], True),
             (4, [0.25, -2.0, 3.0, 0.125], True), (1, [0.75], True)]
    for m, w, use_x in cases:
        out = torch.full_like(Rd, 7.0)
        pkg.svdcache_forecast_combine(shape, Sd[:m], w, Vd, pk, Rd, Xd if use_x else None, out)
        torch.cuda.synchronize()
        for b in range(B):
            want = ref_forecast_combine([to_np(s[b]) for s in S[:m]], w, to_np(V[b]), to_np(R[b]),
                                        to_np(X[b]) if use_x else None, store)
            assert_close(to_np(out[b]), want, store, f"combine m={m} x={use_x} block {b}")
    # one state with weight one is the basic cached step, bit for bit
    a, b_ = torch.empty_like(Rd), torch.empty_like(Rd)
    pkg.svdcache_forecast(shape, Sd[0], Vd, pk, Rd, a)
    pkg.svdcache_forecast_combine(shape, Sd[:1], [1.0], Vd, pk, Rd, None, b_)
    torch.cuda.synchronize()
    assert torch.equal(a, b_)
    # in place: the output may be the residual buffer or the added tensor
    want = torch.empty_like(Rd)
    pkg.svdcache_forecast_combine(shape, Sd[:2], [1.5, -0.5], Vd, pk, Rd, Xd, want)
    r2, x2 = Rd.clone(), Xd.clone()
    pkg.svdcache_forecast_combine(shape, Sd[:2], [1.5, -0.5], Vd, pk, r2, Xd, r2)
    pkg.svdcache_forecast_combine(shape, Sd[:2], [1.5, -0.5], Vd, pk, Rd, x2, x2)
    torch.cuda.synchronize()
    assert torch.equal(r2, want) and torch.equal(x2, want)


def test_forecast_combine_rejects_bad_arguments():
    R, X, V, S = _problem(1, 16, 64, 4, torch.float32, seed=1, nstates=5)
    shape = pkg.make_shape(R, 4)
    Rd, Vd, Sd = R.to(DEV), V.to(DEV), [s.to(DEV) for s in S]
    out = torch.empty_like(Rd)
    for m in (0, 5):
        with pytest.raises(pkg.SvdcError) as e:
            pkg.svdcache_forecast_combine(shape, Sd[:m], [1.0] * m, Vd, None, Rd, None, out)
        assert e.value.code == -5
    with pytest.raises(pkg.SvdcError) as e:
        pkg.svdcache_forecast_combine(shape, Sd[:2], [1.0, float("nan")], Vd, None, Rd, None, out)
    assert e.value.code == -5


def test_linear_trend_forecast_tracks_a_drifting_feature():
    """A feature whose principal coefficients drift linearly in time, observed at two full steps: the order-1
    weights on the two stored coefficient sets forecast the later feature; plain reuse of the last one does not."""
    B, N, D, k = 1, 200, 256, 32
    g = torch.Generator().manual_seed(11)
    V = torch.linalg.qr(torch.randn(B, D, k, generator=g, dtype=torch.float64))[0].float().contiguous()
    C0, dC = 4 * torch.randn(B, N, k, generator=g), 0.3 * torch.randn(B, N, k, generator=g)
    E = 0.05 * torch.randn(B, N, D, generator=g)
    E = E - (E @ V) @ V.transpose(1, 2)                       # residual part, orthogonal to the basis
    feat = lambda t: ((C0 + t * dC) @ V.transpose(1, 2) + E).to(torch.bfloat16)
    shape = pkg.make_shape(feat(0), k)
    Vd = V.to(DEV)
    pk = pkg.pack_basis(shape, Vd)
    R = torch.empty(B, N, D, device=DEV, dtype=torch.bfloat16)
    S = torch.empty(B, N, k, device=DEV)
    Cs = [torch.empty_like(S), torch.empty_like(S)]
    pkg.svdcache_full_step(shape, feat(0).to(DEV), Vd, pk, R, S, Cs[0], 1.0, True)
    pkg.svdcache_full_step(shape, feat(6).to(DEV), Vd, pk, R, S, Cs[1], 1.0, False)
    w = pkg.svdcache_extrapolation_weights(1, 3, 6)
    trend, reuse = torch.empty_like(R), torch.empty_like(R)
    pkg.svdcache_forecast_combine(shape, [Cs[1], Cs[0]], w, Vd, pk, R, None, trend)
    pkg.svdcache_forecast(shape, Cs[1], Vd, pk, R, reuse)
    torch.cuda.synchronize()
    target = feat(9).float()
    err = lambda x: float((x.float().cpu() - target).norm() / target.norm())
    assert err(trend) <= 1e-2 and err(reuse) >= 5 * err(trend)


def test_flux57_full_size_combine_sampled_rows():
    """The extended cached step in the launch configuration of the benchmark (57 x 4608 x 3072 bf16, k = 32):
    two states, an added tensor, sampled rows against the oracle."""
    wl = WORKLOADS["flux57"]
    B = wl.B
    R = torch.empty(B, wl.N, wl.D, device=DEV, dtype=torch.bfloat16)
    for b in range(B):
        R[b] = FeatureStream(wl, b, device=DEV).at(0)
    X = R.roll(1, dims=0).contiguous()
    g = torch.Generator(device=DEV).manual_seed(5)
    S = [torch.randn(B, wl.N, wl.k, device=DEV, generator=g) for _ in range(2)]
    V = torch.linalg.qr(torch.randn(B, wl.D, wl.k, device=DEV, generator=g))[0].contiguous()
    shape = pkg.make_shape(R, wl.k)
    pk = pkg.pack_basis(shape, V)
    out = torch.empty_like(R)
    w = [1.5, -0.5]
    pkg.svdcache_forecast_combine(shape, S, w, V, pk, R, X, out)
    torch.cuda.synchronize()
    gc = torch.Generator().manual_seed(6)
    for b in (0, 31, 56):
        rows = torch.cat([torch.tensor([0, 15, 16, wl.N - 1]), torch.randint(0, wl.N, (64,), generator=gc)]).unique()
        want = ref_forecast_combine([to_np(s[b][rows]) for s in S], w, to_np(V[b]), to_np(R[b][rows]),
                                    to_np(X[b][rows]), "bf16")
        assert_close(to_np(out[b][rows]), want, "bf16", f"combine block {b}")


# ------------------------------------------------------------------ basis reuse and re-basing (Sec. 3.3)

@pytest.mark.parametrize("B,N,D,k", [(2, 70, 200, 17), (1, 130, 3072, 32), (2, 130, 256, 128), (1, 9, 8, 1),
                                     (3, 257, 512, 64)])
def test_basis_overlap_and_rebase(B, N, D, k):
    from oracle import ref_basis_overlap, ref_rebase_state, ref_forecast
    g = torch.Generator().manual_seed(D + k)
    Vo = torch.linalg.qr(torch.randn(B, D, k, generator=g, dtype=torch.float64))[0].float().contiguous()
    # new basis: mostly a rotation of the old one, tilted a little out of its subspace
    Q = torch.linalg.qr(torch.randn(B, k, k, generator=g, dtype=torch.float64))[0]
    Vn = torch.linalg.qr(Vo.double() @ Q + 0.05 * torch.randn(B, D, k, generator=g, dtype=torch.float64))[0]
    Vn = Vn.float().contiguous()
    S = 3 * torch.randn(B, N, k, generator=g)
    R = torch.randn(B, N, D, generator=g)
    shape = pkg.make_shape(R, k)
    M = torch.empty(B, k, k, device=DEV)
    Sn = torch.empty(B, N, k, device=DEV)
    pkg.svdcache_basis_overlap(shape, Vo.to(DEV), Vn.to(DEV), M)
    pkg.svdcache_rebase_state(shape, M, S.to(DEV), Sn)
    Sip = S.clone().to(DEV)
    pkg.svdcache_rebase_state(shape, M, Sip, Sip)                      # in place
    torch.cuda.synchronize()
    assert torch.equal(Sip, Sn)
    for b in range(B):
        Mr = ref_basis_overlap(to_np(Vo[b]), to_np(Vn[b]))
        assert np.abs(to_np(M[b]) - Mr).max() <= 5e-6          # float32 sums over D products of unit vectors
        assert_close(to_np(Sn[b]), ref_rebase_state(to_np(S[b]), Mr, "f32"), "f32", f"rebase block {b}")
    # exact carry-over inside the same subspace: the cached step gives the same feature before and after
    Vrot = (Vo.double() @ Q).float().contiguous()
    pkg.svdcache_basis_overlap(shape, Vo.to(DEV), Vrot.to(DEV), M)
    pkg.svdcache_rebase_state(shape, M, S.to(DEV), Sn)
    a, c = torch.empty(B, N, D, device=DEV), torch.empty(B, N, D, device=DEV)
    pkg.svdcache_forecast(shape, S.to(DEV), Vo.to(DEV), None, R.to(DEV), a)
    pkg.svdcache_forecast(shape, Sn, Vrot.to(DEV), None, R.to(DEV), c)
    torch.cuda.synchronize()
    assert float((a - c).norm() / a.norm()) <= 2e-6


def test_refit_on_a_drifted_feature_keeps_the_state_useful():
    """Full step in the basis of F_0, refit on a later feature whose subspace has drifted, carry the EMA state
    over and continue.  The two bases are the oracle's exact fits (handed to the GPU, never the other way round)
    and the oracle runs the same chain on its own state."""
    from oracle import ref_basis_overlap, ref_rebase_state, ref_forecast
    wl = WORKLOADS["flux1"].with_(N=512)
    fs = FeatureStream(wl, 0, device=DEV)
    F0, F1 = fs.at(0).unsqueeze(0).contiguous(), fs.at(wl.interval).unsqueeze(0).contiguous()
    k = wl.k
    shape = pkg.make_shape(F0, k)
    V0r = ref_fit_basis(to_np(F0[0]), k)[0].astype(np.float32).astype(np.float64)
    V1r = ref_fit_basis(to_np(F1[0]), k)[0].astype(np.float32).astype(np.float64)
    V0 = torch.from_numpy(V0r).float().unsqueeze(0).contiguous().to(DEV)
    V1 = torch.from_numpy(V1r).float().unsqueeze(0).contiguous().to(DEV)
    pk0, pk1 = pkg.pack_basis(shape, V0), pkg.pack_basis(shape, V1)
    R = torch.empty_like(F0)
    S = torch.empty(1, wl.N, k, device=DEV)
    pkg.svdcache_full_step(shape, F0, V0, pk0, R, S, None, 0.5, True)
    M = torch.empty(1, k, k, device=DEV)
    pkg.svdcache_basis_overlap(shape, V0, V1, M)
    S1 = torch.empty_like(S)
    pkg.svdcache_rebase_state(shape, M, S, S1)
    pkg.svdcache_full_step(shape, F1, V1, pk1, R, S1, None, 0.5, False)     # EMA continues in the new basis
    Fh = torch.empty_like(F0)
    pkg.svdcache_forecast(shape, S1, V1, pk1, R, Fh)
    torch.cuda.synchronize()
    _, S0r, _ = ref_full_step(to_np(F0[0]), V0r, None, 0.5, True, "bf16")
    Mr = ref_basis_overlap(V0r, V1r)
    assert np.abs(to_np(M[0]) - Mr).max() <= 5e-6
    Rr, Sr, _ = ref_full_step(to_np(F1[0]), V1r, ref_rebase_state(S0r, Mr, "f32"), 0.5, False, "bf16")
    assert_close(to_np(S1[0]), Sr, "f32", "EMA state after re-basing")
    assert_close(to_np(Fh[0]), ref_forecast(Sr, V1r, Rr, "bf16"), "bf16", "Fhat", ulp_of=Rr)
    # the synthetic stream keeps its subspace: the GPU's own fits of the two features stay similar (Fig. 1(b))
    Vg0, s0, _ = pkg.fit_basis(F0, k)
    Vg1, s1, _ = pkg.fit_basis(F1, k)
    sim_dir = torch.empty(1, k, device=DEV)
    sim_sig = torch.empty(1, device=DEV)
    pkg.svdcache_basis_similarity(shape, Vg0, s0, Vg1, s1, sim_dir, sim_sig)
    torch.cuda.synchronize()
    assert float(sim_sig) > 0.8 and float(sim_dir[0, 0]) > 0.8


@pytest.mark.parametrize("B,D,k", [(2, 200, 17), (1, 3072, 32), (3, 64, 8)])
def test_basis_similarity(B, D, k):
    from oracle import ref_basis_similarity
    g = torch.Generator().manual_seed(D * 7 + k)
    Va = torch.linalg.qr(torch.randn(B, D, k, generator=g, dtype=torch.float64))[0].float().contiguous()
    Vb = (Va + 0.3 * torch.randn(B, D, k, generator=g) / D ** 0.5).contiguous()
    Vb[:, :, 0] *= -1.0                      # sign flip: no effect
    Vb[:, :, k - 1] = 0.0                    # a zero direction scores zero
    sa = torch.sort(torch.rand(B, k, generator=g) * 5 + 0.1, descending=True)[0]
    sb = (sa * (1 + 0.2 * torch.randn(B, k, generator=g))).abs() * 0.7
    shape = pkg.make_shape(torch.empty(B, max(k, 4), D), k)
    sd = torch.empty(B, k, device=DEV)
    ss = torch.empty(B, device=DEV)
    pkg.svdcache_basis_similarity(shape, Va.to(DEV), sa.to(DEV), Vb.to(DEV), sb.to(DEV), sd, ss)
    torch.cuda.synchronize()
    for b in range(B):
        wd, ws = ref_basis_similarity(to_np(Va[b]), to_np(sa[b]), to_np(Vb[b]), to_np(sb[b]))
        assert np.abs(to_np(sd[b]) - wd).max() <= 1e-6 and abs(float(ss[b]) - ws) <= 1e-6
    sd2 = torch.empty(B, k, device=DEV)
    pkg.svdcache_basis_similarity(shape, Va.to(DEV), None, Vb.to(DEV), None, sd2, None)   # spectrum part optional
    torch.cuda.synchronize()
    assert torch.equal(sd, sd2)


def test_rebase_rejects_ranks_beyond_its_limit():
    shape = pkg.make_shape(torch.empty(1, 200, 256), 160)
    t = torch.empty(1, 256, 160, device=DEV)
    with pytest.raises(pkg.SvdcError) as e:
        pkg.svdcache_basis_overlap(shape, t, t, torch.empty(1, 160, 160, device=DEV))
    assert e.value.code == -2


# ------------------------------------------------------------------ residual smoothed too (Sec. 4.5 ablation)

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("B,N,D,k", [(2, 67, 72, 5), (1, 130, 200, 17), (2, 150, 256, 32), (1, 140, 512, 128),
                                     (1, 150, 3072, 32), (1, 100, 3072, 64), (1, 50, 1024, 20)])
def test_full_step_residual_ema(dtype, B, N, D, k):
    from oracle import ref_full_step_residual_ema
    store = "f32" if dtype == torch.float32 else "bf16"
    g = torch.Generator().manual_seed(N * 5 + D + k)
    F = torch.randn(B, N, D, generator=g).to(dtype)
    Rp = torch.randn(B, N, D, generator=g).to(dtype)
    V = torch.linalg.qr(torch.randn(B, D, k, generator=g, dtype=torch.float64))[0].float().contiguous()
    S0 = torch.randn(B, N, k, generator=g)
    shape = pkg.make_shape(F, k)
    Fd, Vd = F.to(DEV), V.to(DEV)
    pk = pkg.pack_basis(shape, Vd)
    for init, a_r in [(False, 0.25), (True, 0.25), (False, 1.0)]:
        R = Rp.clone().to(DEV)                       # in place: the state buffer is both R_prev and R
        S = S0.clone().to(DEV)
        Cc = torch.empty_like(S)
        pkg.svdcache_full_step_residual_ema(shape, Fd, Vd, pk, R, R, S, Cc, 0.3, a_r, init)
        R2 = torch.full_like(R, 7.0)                 # out of place gives the same bits
        S2 = S0.clone().to(DEV)
        pkg.svdcache_full_step_residual_ema(shape, Fd, Vd, pk, Rp.to(DEV), R2, S2, None, 0.3, a_r, init)
        torch.cuda.synchronize()
        assert torch.equal(R, R2) and torch.equal(S, S2)
        for b in range(B):
            Rr, Sr, Cr = ref_full_step_residual_ema(to_np(F[b]), to_np(V[b]), to_np(S0[b]), to_np(Rp[b]), 0.3, a_r,
                                                    init, store)
            assert_close(to_np(R[b]), Rr, store, f"R[{b}] init={init} a_r={a_r}", floor_of=to_np(F[b]))
            assert_close(to_np(S[b]), Sr, "f32", f"S[{b}]")
            assert_close(to_np(Cc[b]), Cr, "f32", f"C[{b}]")
    # alpha_r = 1 is the paper's full step, bit for bit, and then R_prev is not needed
    Ra, Rb = torch.empty_like(Fd), torch.empty_like(Fd)
    Sa, Sb = S0.clone().to(DEV), S0.clone().to(DEV)
    pkg.svdcache_full_step(shape, Fd, Vd, pk, Ra, Sa, None, 0.3, False)
    pkg.svdcache_full_step_residual_ema(shape, Fd, Vd, pk, None, Rb, Sb, None, 0.3, 1.0, False)
    torch.cuda.synchronize()
    assert torch.equal(Ra, Rb) and torch.equal(Sa, Sb)


def test_full_step_residual_ema_rejects_bad_arguments():
    F = torch.randn(1, 16, 64, device=DEV)
    V = torch.linalg.qr(torch.randn(1, 64, 4, device=DEV))[0].contiguous()
    S = torch.zeros(1, 16, 4, device=DEV)
    R = torch.empty_like(F)
    shape = pkg.make_shape(F, 4)
    for a_r in (0.0, 1.5, float("nan")):
        with pytest.raises(pkg.SvdcError) as e:
            pkg.svdcache_full_step_residual_ema(shape, F, V, None, R, R, S, None, 0.5, a_r, False)
        assert e.value.code == -5
    with pytest.raises(pkg.SvdcError) as e:          # previous residual needed but missing
        pkg.svdcache_full_step_residual_ema(shape, F, V, None, None, R, S, None, 0.5, 0.5, False)
    assert e.value.code == -1
    with pytest.raises(pkg.SvdcError) as e:          # the previous residual cannot be the feature buffer
        pkg.svdcache_full_step_residual_ema(shape, F, V, None, F, R, S, None, 0.5, 0.5, False)
    assert e.value.code == -5


def test_flux57_full_size_residual_ema_sampled_rows():
    from oracle import ref_full_step_residual_ema
    wl = WORKLOADS["flux57"]
    B = wl.B
    F = torch.empty(B, wl.N, wl.D, device=DEV, dtype=torch.bfloat16)
    for b in range(B):
        F[b] = FeatureStream(wl, b, device=DEV).at(wl.interval)
    R = F.roll(3, dims=0).contiguous()
    Rp = R.clone()
    g = torch.Generator(device=DEV).manual_seed(9)
    S0 = torch.randn(B, wl.N, wl.k, device=DEV, generator=g)
    S = S0.clone()
    V = torch.linalg.qr(torch.randn(B, wl.D, wl.k, device=DEV, generator=g))[0].contiguous()
    shape = pkg.make_shape(F, wl.k)
    pk = pkg.pack_basis(shape, V)
    pkg.svdcache_full_step_residual_ema(shape, F, V, pk, R, R, S, None, wl.alpha, 0.5, False)
    torch.cuda.synchronize()
    gc = torch.Generator().manual_seed(10)
    for b in (0, 30, 56):
        rows = torch.cat([torch.tensor([0, 31, 32, 47, 48, wl.N - 1]), torch.randint(0, wl.N, (64,), generator=gc)]).unique()
        Rr, Sr, _ = ref_full_step_residual_ema(to_np(F[b][rows]), to_np(V[b]), to_np(S0[b][rows]), to_np(Rp[b][rows]),
                                               wl.alpha, 0.5, False, "bf16")
        assert_close(to_np(R[b][rows]), Rr, "bf16", f"R block {b}", floor_of=to_np(F[b][rows]))
        assert_close(to_np(S[b][rows]), Sr, "f32", f"S block {b}")


def test_fit_basis_for_energy_grows_the_rank_until_tau_is_reached():
    """Constructed spectra: block 0 needs 5 directions for 85 % of its energy, block 1 needs 22, so a first fit
    with rank 8 is too small for block 1 and the rank is doubled (8 -> 16 -> 32)."""
    B, N, D, m = 2, 600, 256, 40
    g = torch.Generator().manual_seed(77)
    U = torch.linalg.qr(torch.randn(B, N, m, generator=g, dtype=torch.float64))[0]
    W = torch.linalg.qr(torch.randn(B, D, m, generator=g, dtype=torch.float64))[0]
    s = torch.zeros(B, m, dtype=torch.float64)
    s[0] = torch.tensor([10.0, 8.0, 6.0] + [1.0] * (m - 3))
    s[1] = torch.tensor([3.0] * 24 + [1.0] * (m - 24))
    F = (U * s.unsqueeze(1)) @ W.transpose(1, 2)
    Fd = F.float().to(DEV)
    V, sigma, fro2, k_star, reached = pkg.fit_basis_for_energy(Fd, tau=0.85, k_init=8, k_max=64, q=6)
    torch.cuda.synchronize()
    assert V.shape[2] == 32 and bool(reached.all())
    want = []
    for b in range(B):
        e = np.cumsum(to_np(s[b]) ** 2) / float((s[b] ** 2).sum())
        want.append(int(np.searchsorted(e, 0.85) + 1))
    assert [int(x) for x in k_star] == want == [5, 22]
    for b in range(B):
        ks = int(k_star[b])
        assert not to_np(V[b][:, ks:]).any() and not to_np(sigma[b][ks:]).any()
        assert np.abs(to_np(sigma[b][:ks]) / to_np(s[b][:ks]) - 1).max() <= 1e-4
        # the kept directions span the leading right singular vectors
        P = to_np(V[b][:, :ks])
        assert np.abs(P.T @ P - np.eye(ks)).max() <= 1e-5
        # the directions above the flat tail lie in the span of the true leading singular vectors (inside a
        # cluster of equal sigma any rotation is a correct answer)
        lead, cols = (3, 3) if b == 0 else (24, ks)
        Wl = to_np(W[b][:, :lead])
        assert np.linalg.norm(P[:, :cols] - Wl @ (Wl.T @ P[:, :cols])) <= 1e-3 * np.sqrt(cols)
    # the rank cannot grow beyond k_max: the answer saturates and says so
    V2, s2, f2, ks2, r2 = pkg.fit_basis_for_energy(Fd, tau=0.85, k_init=8, k_max=16, q=6)
    torch.cuda.synchronize()
    assert V2.shape[2] == 16 and [int(x) for x in r2] == [1, 0] and int(ks2[1]) == 16


def test_extended_kernels_with_strided_rows():
    """Row stride larger than D on the matrix-core path: the combined cached step (3 states + added tensor) and
    the residual-smoothing full step touch nothing beyond column D."""
    from oracle import ref_full_step_residual_ema
    B, N, D, k, ldf = 2, 150, 3072, 32, 3072 + 64
    g = torch.Generator().manual_seed(3)

    def strided(x):
        buf = torch.zeros(B, N, ldf, dtype=torch.bfloat16)
        buf[:, :, :D] = x
        return buf.to(DEV)
    F, Rp, X = [torch.randn(B, N, D, generator=g).to(torch.bfloat16) for _ in range(3)]
    V = torch.linalg.qr(torch.randn(B, D, k, generator=g, dtype=torch.float64))[0].float().contiguous()
    S = [torch.randn(B, N, k, generator=g) for _ in range(3)]
    Fb, Rb, Xb, Ob = strided(F), strided(Rp), strided(X), strided(torch.zeros(B, N, D))
    shape = pkg.make_shape(Fb[:, :, :D], k)
    assert shape.ldf == ldf
    Vd = V.to(DEV)
    pk = pkg.pack_basis(shape, Vd)
    assert pk is not None
    w = [0.5, 1.25, -0.75]
    pkg.svdcache_forecast_combine(shape, [s.to(DEV) for s in S], w, Vd, pk, Rb[:, :, :D], Xb[:, :, :D], Ob[:, :, :D])
    S1 = S[0].clone().to(DEV)
    Rs = Rb.clone()
    pkg.svdcache_full_step_residual_ema(shape, Fb[:, :, :D], Vd, pk, Rs[:, :, :D], Rs[:, :, :D], S1, None, 0.3, 0.4,
                                        False)
    torch.cuda.synchronize()
    for b in range(B):
        want = ref_forecast_combine([to_np(s[b]) for s in S], w, to_np(V[b]), to_np(Rp[b]), to_np(X[b]), "bf16")
        assert_close(to_np(Ob[b, :, :D]), want, "bf16", "combine, strided rows")
        Rr, Sr, _ = ref_full_step_residual_ema(to_np(F[b]), to_np(V[b]), to_np(S[0][b]), to_np(Rp[b]), 0.3, 0.4,
                                               False, "bf16")
        assert_close(to_np(Rs[b, :, :D]), Rr, "bf16", "residual smoothing, strided rows", floor_of=to_np(F[b]))
        assert_close(to_np(S1[b]), Sr, "f32", "S")
    assert not Ob[:, :, D:].any() and not Rs[:, :, D:].any()


def test_whole_step_sequence_under_hip_graph_capture():
    """Callers that capture their step loop into a HIP graph: the allocation-free fit, the packing and both step
    kernels are recorded into one graph (no memset nodes: the library clears with kernels) and replayed several
    times with eager work and synchronisations in between; every replay must reproduce the eager results."""
    B, N, D, k = 2, 700, 512, 32
    wl = WORKLOADS["flux1"].with_(N=N, D=D, k=k, signal_rank=96)
    F0 = torch.stack([FeatureStream(wl, b).at(0) for b in range(B)]).to(DEV)
    F1 = torch.stack([FeatureStream(wl, b).at(5) for b in range(B)]).to(DEV)
    shape = pkg.make_shape(F0, k)
    V = torch.empty(B, D, k, device=DEV)
    sigma, fro2 = torch.empty(B, k, device=DEV), torch.empty(B, device=DEV)
    status = torch.empty(B, dtype=torch.int32, device=DEV)
    packed = torch.empty(pkg.svdcache_packed_basis_bytes(shape), dtype=torch.uint8, device=DEV)
    Sp = pkg.alloc_packed_state(shape, DEV)
    R, Fh = torch.empty_like(F0), torch.empty_like(F0)
    S = torch.empty(B, N, k, device=DEV)
    Fin = F0.clone()

    def sequence():
        pkg.svdcache_fit_basis_static(shape, Fin, V, sigma, fro2, status, q=6, seed=3)
        pkg.svdcache_pack_basis(shape, V, packed)
        pkg.svdcache_full_step_packed(shape, Fin, V, packed, R, S, None, Sp, 0.5, True)
        pkg.svdcache_full_step_packed(shape, F1, V, packed, R, S, None, Sp, 0.5, False)
        pkg.svdcache_forecast_packed(shape, Sp, packed, R, Fh)

    sequence()                                     # eager: also resolves the static workspace before any capture
    torch.cuda.synchronize()
    want = [t.clone() for t in (sigma, S, R, Fh)]
    want_V = V.clone()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            sequence()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in (V, sigma, S, R, Fh):
            t.fill_(float("nan"))                  # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (sigma, S, R, Fh)
        # the small launches of the fit sum with float atomics: same values up to the last bits, same subspace
        # (values deep in the flat part of the spectrum move most)
        rel = (sigma / want[0] - 1).abs()
        assert rel[:, :k // 2].max() <= 1e-4 and rel.max() <= 5e-3, f"replay {rep}: sigma differs by {rel.max():.2e}"
        for b in range(B):
            sines = principal_sines(to_np(V[b][:, :k // 2]), to_np(want_V[b][:, :k // 2]))
            assert sines.max() <= 1e-3, f"replay {rep}: basis"
        assert torch.isfinite(Fh.float()).all() and torch.isfinite(S).all()
        # the steps themselves are deterministic given V: recompute them eagerly on the replay's V and compare bits
        V_rep, S_rep, R_rep, Fh_rep = V.clone(), S.clone(), R.clone(), Fh.clone()
        pkg.svdcache_pack_basis(shape, V_rep, packed)
        pkg.svdcache_full_step_packed(shape, Fin, V_rep, packed, R, S, None, Sp, 0.5, True)
        pkg.svdcache_full_step_packed(shape, F1, V_rep, packed, R, S, None, Sp, 0.5, False)
        pkg.svdcache_forecast_packed(shape, Sp, packed, R, Fh)
        torch.cuda.synchronize()
        assert torch.equal(S, S_rep) and torch.equal(R, R_rep) and torch.equal(Fh, Fh_rep), f"replay {rep}: steps"
