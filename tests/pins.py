"""Checks that pin the oracle to things other than itself.

Each check takes the implementation under test as an argument, so the same
checks run (a) against the real oracle and (b) against deliberately broken
copies of it (tests/test_oracle_mutants.py) to show that a plausible mistake
fails at least one of them.

Everything here is float64 and CPU-only.
"""
from __future__ import annotations

import numpy as np

from oracle import jacobi_svd


def rng(seed):
    return np.random.default_rng(seed)


def random_orthonormal(r, n, m):
    q, _ = np.linalg.qr(r.standard_normal((n, m)))
    return q


def principal_sines(Va, Vb):
    """sines of the principal angles between span(Va) and span(Vb)
    (both with orthonormal columns)."""
    s = np.linalg.svd(Va.T @ Vb, compute_uv=False)
    return np.sqrt(np.maximum(0.0, 1.0 - np.minimum(s, 1.0) ** 2))


# ---------------------------------------------------------------------------
# the brute-force SVD itself, against the definition (Eq. 4)
# ---------------------------------------------------------------------------

def check_jacobi_definition(svd=jacobi_svd):
    r = rng(11)
    for (n, d) in [(32, 16), (16, 16), (7, 5), (5, 9), (1, 4), (6, 1)]:
        F = r.standard_normal((n, d))
        U, s, V = svd(F)
        m = min(n, d)
        assert U.shape == (n, m) and V.shape == (d, m) and s.shape == (m,)
        assert np.abs(F - (U * s) @ V.T).max() <= 1e-12 * max(1.0, np.abs(F).max())
        assert np.abs(U.T @ U - np.eye(m)).max() <= 1e-12
        assert np.abs(V.T @ V - np.eye(m)).max() <= 1e-12
        assert np.all(np.diff(s) <= 0) and np.all(s >= 0)


# ---------------------------------------------------------------------------
# basis fit (Eq. 4-5): fit(F, k) -> (V [D,k], sigma [k], fro2)
# ---------------------------------------------------------------------------

def check_fit_vs_bruteforce(fit):
    """LAPACK/Gram route against the loop-level Jacobi SVD on tiny inputs."""
    r = rng(5)
    for (n, d, k) in [(32, 16, 4), (24, 12, 12), (10, 16, 3)]:
        F = r.standard_normal((n, d)) * (np.arange(1, d + 1) ** -0.7)
        V, sig, fro2 = fit(F, k)
        _, s_ref, V_ref = jacobi_svd(F)
        assert V.shape == (d, k) and sig.shape == (k,)
        assert np.allclose(sig, s_ref[:k], rtol=1e-10, atol=0)
        # distinct singular values => vectors agree up to sign
        dots = np.abs(np.sum(V * V_ref[:, :k], axis=0))
        assert np.all(np.abs(dots - 1.0) <= 1e-9)
        assert abs(fro2 - np.sum(F * F)) <= 1e-12 * fro2


def check_fit_constructed_spectrum(fit):
    """F = U diag(s) V^T with known factors: sigma = s and span(V_k) is the
    span of the first k columns of V."""
    r = rng(6)
    n, d, k = 40, 24, 6
    U = random_orthonormal(r, n, d)
    V0 = random_orthonormal(r, d, d)
    s = 10.0 * np.arange(1, d + 1) ** -1.5
    F = (U * s) @ V0.T
    V, sig, fro2 = fit(F, k)
    assert np.allclose(sig, s[:k], rtol=1e-10)
    assert principal_sines(V, V0[:, :k]).max() <= 1e-7
    assert abs(fro2 - np.sum(s ** 2)) <= 1e-10 * fro2
    assert np.abs(V.T @ V - np.eye(k)).max() <= 1e-12


def check_fit_invariances(fit):
    """sigma is invariant under a permutation of the tokens (rows) and under
    right-multiplication by an orthogonal matrix; V rotates with the latter."""
    r = rng(7)
    n, d, k = 30, 12, 5
    F = r.standard_normal((n, d)) * (np.arange(1, d + 1) ** -1.0)
    V, sig, _ = fit(F, k)
    perm = r.permutation(n)
    Vp, sigp, _ = fit(F[perm], k)
    assert np.allclose(sigp, sig, rtol=1e-12)
    assert principal_sines(Vp, V).max() <= 1e-7
    Q = random_orthonormal(r, d, d)
    Vq, sigq, _ = fit(F @ Q, k)
    assert np.allclose(sigq, sig, rtol=1e-11)
    assert principal_sines(Vq, Q.T @ V).max() <= 1e-7


def check_fit_eckart_young_and_energy(fit):
    """||F - F V_k V_k^T||_F^2 = sum_{i>k} sigma_i^2, and at k = min(N, D) the
    squared singular values add up to ||F||_F^2."""
    r = rng(8)
    n, d = 28, 10
    F = r.standard_normal((n, d))
    s_all = jacobi_svd(F)[1]
    for k in (1, 4, 9):
        V, sig, _ = fit(F, k)
        tail = np.sum((F - (F @ V) @ V.T) ** 2)
        assert abs(tail - np.sum(s_all[k:] ** 2)) <= 1e-10 * np.sum(s_all ** 2)
    V, sig, fro2 = fit(F, d)
    assert abs(np.sum(sig ** 2) - fro2) <= 1e-11 * fro2


def check_fit_closed_forms(fit):
    """rank-1 outer product and a 2 x 2 matrix with a hand-computed SVD."""
    u = np.array([3.0, 0.0, 4.0])
    v = np.array([1.0, 2.0, 2.0, 0.0])
    V, sig, _ = fit(np.outer(u, v), 1)
    assert abs(sig[0] - 5.0 * 3.0) <= 1e-12          # ||u|| * ||v||
    assert np.allclose(np.abs(V[:, 0]), v / 3.0, atol=1e-12)
    # F = [[3, 0], [4, 5]]: F^T F = [[25, 20], [20, 25]] has eigenvalues 45, 5
    # with eigenvectors (1, 1)/sqrt2 and (1, -1)/sqrt2.
    V, sig, _ = fit(np.array([[3.0, 0.0], [4.0, 5.0]]), 2)
    assert np.allclose(sig, [np.sqrt(45.0), np.sqrt(5.0)], rtol=1e-13)
    assert np.allclose(np.abs(V), np.full((2, 2), np.sqrt(0.5)), atol=1e-13)
    assert V[0, 1] * V[1, 1] < 0 < V[0, 0] * V[1, 0]


def check_fit_methods_agree(fit):
    r = rng(9)
    F = r.standard_normal((50, 20)) * (np.arange(1, 21) ** -1.2)
    Va, sa, _ = fit(F, 6, method="svd")
    Vb, sb, _ = fit(F, 6, method="gram")
    assert np.allclose(sa, sb, rtol=1e-10)
    assert principal_sines(Va, Vb).max() <= 1e-7


# ---------------------------------------------------------------------------
# full step (Eq. 8-11): full(F, V, S_prev, alpha, init, store) -> (R, S, C)
# ---------------------------------------------------------------------------

def _problem(seed=21, n=24, d=16, k=5):
    r = rng(seed)
    F = r.standard_normal((n, d))
    V = random_orthonormal(r, d, k)
    S0 = r.standard_normal((n, k))
    return r, F, V, S0


def check_full_identities(full):
    r, F, V, S0 = _problem()
    R, S, C = full(F, V, None, 0.5, True, "f64")
    k = V.shape[1]
    # exact recombination, orthogonality of the residual, Pythagoras
    assert np.abs(C @ V.T + R - F).max() <= 1e-13
    assert np.abs(R @ V).max() <= 1e-13
    assert abs(np.sum(F ** 2) - np.sum(C ** 2) - np.sum(R ** 2)) <= 1e-12 * np.sum(F ** 2)
    assert np.array_equal(S, C)
    # C is the coefficient of each token in the basis: column j = F v_j
    for j in range(k):
        assert np.abs(C[:, j] - F @ V[:, j]).max() <= 1e-13
    # recombination also holds for a V that is NOT orthonormal (used as given)
    W = r.standard_normal(V.shape)
    R2, _, C2 = full(F, W, None, 0.5, True, "f64")
    assert np.abs(C2 @ W.T + R2 - F).max() <= 1e-12
    assert np.abs(C2 - F @ W).max() <= 1e-13


def check_full_special_bases(full):
    r, F, _, _ = _problem(22)
    n, d = F.shape
    # k = D with V = I: everything is principal
    R, S, C = full(F, np.eye(d), None, 0.3, True, "f64")
    assert np.array_equal(C, F) and np.abs(R).max() == 0.0
    # one-hot columns: C gathers columns of F, R zeroes exactly those columns
    cols = [3, 0, 7]
    V = np.zeros((d, len(cols)))
    V[cols, np.arange(len(cols))] = 1.0
    R, S, C = full(F, V, None, 0.3, True, "f64")
    assert np.array_equal(C, F[:, cols])
    expect = F.copy()
    expect[:, cols] = 0.0
    assert np.array_equal(R, expect)


def check_ema_closed_forms(full):
    """Eq. 11 with state kept in coefficient space; alpha = 1 - beta."""
    r, F0, V, _ = _problem(23, n=12, d=10, k=4)
    d, k = V.shape
    Vc = np.concatenate([V, random_orthonormal(r, d, d)[:, : d - k]], axis=1)
    Vc, _ = np.linalg.qr(Vc)           # orthonormal completion; first k cols span V
    V = Vc[:, :k]
    a = 0.3
    # constant coefficients -> state equals them for ever
    S = None
    for n_ in range(6):
        _, S, C = full(F0, V, S, a, n_ == 0, "f64")
        assert np.abs(S - C).max() <= 1e-14
    # linear trajectory C_n = c0 + n d  ->  S_n = C_n - d (1-a)(1-(1-a)^n)/a
    c0 = r.standard_normal((12, k))
    dl = r.standard_normal((12, k))
    rest = r.standard_normal((12, d - k)) @ Vc[:, k:].T     # lives outside span(V)
    S = None
    hist = []
    for n_ in range(8):
        Cn = c0 + n_ * dl
        F = Cn @ V.T + rest
        _, S, C = full(F, V, S, a, n_ == 0, "f64")
        assert np.abs(C - Cn).max() <= 1e-12
        hist.append(Cn)
        lag = dl * (1 - a) * (1 - (1 - a) ** n_) / a
        assert np.abs(S - (Cn - lag)).max() <= 1e-12
        # unrolled form: S_n = (1-a)^n C_0 + a sum_j (1-a)^(n-j) C_j
        unrolled = (1 - a) ** n_ * hist[0] + a * sum((1 - a) ** (n_ - j) * hist[j] for j in range(1, n_ + 1))
        assert np.abs(S - unrolled).max() <= 1e-12
    # alpha = 1: the state is the newest observation (plain reuse)
    S_prev = r.standard_normal((12, k))
    _, S, C = full(F, V, S_prev, 1.0, False, "f64")
    assert np.abs(S - C).max() <= 1e-15
    # beta = 0.9 (the paper's setting) is alpha = 0.1: new state = 0.9 old + 0.1 new
    _, S, C = full(F, V, S_prev, 0.1, False, "f64")
    assert np.abs(S - (0.9 * S_prev + 0.1 * C)).max() <= 1e-14
    # init ignores S_prev
    _, S, C = full(F, V, S_prev, 0.1, True, "f64")
    assert np.array_equal(S, C)


def check_full_storage_rounding(full):
    """bf16 storage: R is within half a bf16 ulp (at most 2^-8 relative) of the exact
    residual, C and S are float32 values; inputs already bf16 stay exact."""
    from oracle import round_bf16
    r, F, V, S0 = _problem(24)
    F = round_bf16(F)
    R64, S64, C64 = full(F, V, S0, 0.5, False, "f64")
    R, S, C = full(F, V, S0, 0.5, False, "bf16")
    assert np.array_equal(R, round_bf16(R)) and np.array_equal(C, C.astype(np.float32).astype(np.float64))
    assert np.all(np.abs(R - R64) <= 2.0 ** -8 * np.abs(R64) + 1e-300)
    assert np.all(np.abs(C - C64) <= 2.0 ** -24 * np.abs(C64) + 1e-300)
    assert np.all(np.abs(S - S64) <= 2.0 ** -24 * np.abs(S64) + 1e-300)
    assert np.abs(C @ V.T + R - F).max() <= 2.0 ** -8 * np.abs(F).max()
    # hand-picked halfway cases of bf16 rounding (ties to even)
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8), 1.0 + 2.0 ** -8 + 2.0 ** -30])
    assert np.array_equal(round_bf16(x), [1.0, 1.0 + 2.0 ** -6, -1.0, 1.0 + 2.0 ** -7])


# ---------------------------------------------------------------------------
# cached step (Sec. 3.5): forecast(S, V, R, store) -> Fhat
# ---------------------------------------------------------------------------

def check_forecast(full, forecast):
    r, F, V, S0 = _problem(25)
    # right after an initial full step the forecast reproduces F exactly
    R, S, C = full(F, V, None, 0.5, True, "f64")
    assert np.abs(forecast(S, V, R, "f64") - F).max() <= 1e-13
    # in general Fhat = F_t + (S - C_t) V^T
    R, S, C = full(F, V, S0, 0.5, False, "f64")
    Fh = forecast(S, V, R, "f64")
    assert np.abs(Fh - (F + (S - C) @ V.T)).max() <= 1e-13
    # element-wise definition, written out
    n, d = F.shape
    for (i, j) in [(0, 0), (5, 3), (n - 1, d - 1)]:
        assert abs(Fh[i, j] - (sum(S[i, m] * V[j, m] for m in range(V.shape[1])) + R[i, j])) <= 1e-13
    # V = 0 (nothing is principal): plain reuse of the cached feature (Eq. 3)
    Z = np.zeros_like(V)
    R0, S_, _ = full(F, Z, None, 0.5, True, "f64")
    assert np.array_equal(forecast(S_, Z, R0, "f64"), F)
    # the forecast does not depend on anything but (S, V, R): no hidden state
    assert np.array_equal(forecast(S, V, R, "f64"), Fh)


# ---------------------------------------------------------------------------
# rank selection by retained energy (Eq. 6)
# ---------------------------------------------------------------------------

def check_select_rank(select, rank_all):
    """select(sigma_lead, fro2, tau) -> (k_star, reached);  rank_all(sigma_all, tau) -> k_star."""
    # equal singular values: k of n hold the fraction k/n, so k* = ceil(tau n)
    n = 20
    sig = np.full(n, 3.0, dtype=np.float32)
    for tau, want in [(0.04, 1), (0.26, 6), (0.5, 10), (0.51, 11), (1.0, 20)]:   # no ties except exact binary fractions
        assert select(sig, float(9.0 * n), tau) == (want, True)
    # geometric energies sigma_i^2 = 2^-i (i >= 1, infinitely many: total energy 1):
    # the k leading ones hold 1 - 2^-k, so k* = ceil(-log2(1 - tau))
    sig = np.sqrt(2.0 ** -np.arange(1, 25)).astype(np.float32)
    for tau, want in [(0.4, 1), (0.55, 2), (0.7, 2), (0.85, 3), (0.9, 4), (0.99, 7)]:
        assert select(sig, 1.0, tau) == (want, True), tau
    # only 3 values kept: they hold 87.5 % -- enough for 0.85, not for 0.9
    assert select(sig[:3], 1.0, 0.85) == (3, True)
    assert select(sig[:3], 1.0, 0.9) == (3, False)
    assert select(sig[:2], 1.0, 0.85) == (2, False)
    # with the whole spectrum known it is the textbook cumulative-energy rule
    r = rng(41)
    for trial in range(20):
        s_all = np.sort(np.abs(r.standard_normal(30)) + 0.01)[::-1].astype(np.float32)
        fro2 = float(np.sum(s_all.astype(np.float64) ** 2))
        tau = float(r.uniform(0.05, 0.97))
        frac = np.cumsum(s_all.astype(np.float64) ** 2) / fro2
        if np.min(np.abs(frac - tau)) < 1e-6:      # a tie in the last bits: either answer is right
            continue
        assert select(s_all, fro2, tau) == (rank_all(s_all, tau), True)
    # monotone in tau
    ks = [select(s_all, fro2, t)[0] for t in np.linspace(0.01, 0.99, 50)]
    assert all(a <= b for a, b in zip(ks, ks[1:]))


def check_truncate_basis(truncate, full):
    """A step with the truncated basis is the rank-k* step."""
    r, F, V, S0 = _problem(33, n=30, d=18, k=6)
    for ks in (1, 4, 6):
        Vt, st = truncate(V, np.arange(6, 0, -1.0), ks)
        assert np.array_equal(Vt[:, :ks], V[:, :ks]) and not Vt[:, ks:].any()
        assert np.array_equal(st[:ks], np.arange(6, 6 - ks, -1.0)) and not st[ks:].any()
        R, S, C = full(F, Vt, None, 0.5, True, "f64")
        R_k, S_k, C_k = full(F, V[:, :ks], None, 0.5, True, "f64")
        assert np.abs(R - R_k).max() <= 1e-13
        assert np.abs(C[:, :ks] - C_k).max() <= 1e-13 and not C[:, ks:].any() and not S[:, ks:].any()
    assert V[:, 5].any()          # the input was not modified


# ---------------------------------------------------------------------------
# forecasters that are linear in stored coefficient states (Sec. 5.3, Fig. 5(b))
# ---------------------------------------------------------------------------

def check_extrapolation_weights(weights):
    # order 0: reuse; order 1: the straight line through the last two states
    assert np.allclose(weights(0, 3, 6), [1.0], atol=0, rtol=0)
    for j, d in [(1, 6), (5, 6), (2, 3)]:
        assert np.allclose(weights(1, j, d), [1 + j / d, -j / d], rtol=1e-15)
    # a polynomial of degree <= order is extrapolated exactly
    r = rng(5)
    for order in (1, 2, 3):
        coef = r.standard_normal(order + 1)
        poly = lambda t: sum(c * t ** i for i, c in enumerate(coef))
        for j, d in [(1.0, 6.0), (4.0, 5.0), (7.0, 2.0)]:
            w = weights(order, j, d)
            t0 = 11.0
            got = sum(w[m] * poly(t0 - m * d) for m in range(order + 1))
            assert abs(got - poly(t0 + j)) <= 1e-9 * max(1.0, abs(poly(t0 + j))), (order, j, d)
            assert abs(sum(w) - 1.0) <= 1e-12
    # offset 0 returns the latest state itself
    assert np.allclose(weights(3, 0, 6), [1, 0, 0, 0], atol=1e-15)
    # offset -interval returns the state before it
    assert np.allclose(weights(2, -6, 6), [0, 1, 0], atol=1e-15)


def check_forecast_combine(combine, forecast, full, weights):
    r, F, V, S0 = _problem(27)
    R, S, C = full(F, V, None, 0.5, True, "f64")
    # one state, weight 1: the paper's cached step
    assert np.array_equal(combine([S], [1.0], V, R, None, "f64"), forecast(S, V, R, "f64"))
    # linear in the states
    S2 = r.standard_normal(S.shape)
    w = [0.75, -1.5]
    got = combine([S, S2], w, V, R, None, "f64")
    want = R + w[0] * (S @ V.T) + w[1] * (S2 @ V.T)
    assert np.abs(got - want).max() <= 1e-12
    # order matters with unequal weights (a swapped pair is caught)
    assert np.abs(got - combine([S2, S], w, V, R, None, "f64")).max() > 1e-3
    # element-wise definition written out
    n, d = F.shape
    for (i, j) in [(0, 0), (7, 2), (n - 1, d - 1)]:
        e = sum((w[0] * S[i, m] + w[1] * S2[i, m]) * V[j, m] for m in range(V.shape[1])) + R[i, j]
        assert abs(got[i, j] - e) <= 1e-12
    # added tensor
    X = r.standard_normal(F.shape)
    assert np.abs(combine([S, S2], w, V, R, X, "f64") - (want + X)).max() <= 1e-12
    # a feature whose principal coefficients move on a straight line and whose residual is constant is
    # forecast exactly by the order-1 weights on the last two observed coefficient sets
    Cs = [C + t * S2 for t in (0.0, 6.0)]                  # observed at t = 0 and t = 6
    j = 3.0          # weights 1.5 and -0.5 are exact in float32
    F_future = (C + (6.0 + j) * S2) @ V.T + R
    got = combine([Cs[1], Cs[0]], weights(1, j, 6.0), V, R, None, "f64")
    assert np.abs(got - F_future).max() <= 1e-10
    # storage rounding happens once, at the end
    out = combine([S, S2], w, V, R, X, "bf16")
    exact = want + X
    assert np.all(np.abs(out - exact) <= np.abs(exact) * 2.0 ** -8 + 1e-30)


def check_residual_ema(full_ema, full):
    r, F, V, S0 = _problem(29)
    R_prev = r.standard_normal(F.shape)
    # alpha_r = 1 and init: the paper's full step
    for init in (True, False):
        a = full_ema(F, V, S0, R_prev, 0.3, 1.0, init, "f64")
        b = full(F, V, S0, 0.3, init, "f64")
        assert all(np.array_equal(x, y) for x, y in zip(a, b))
    R_new, S, C = full(F, V, S0, 0.3, False, "f64")
    Rs, S2, C2 = full_ema(F, V, S0, R_prev, 0.3, 0.25, False, "f64")
    assert np.abs(Rs - (0.75 * R_prev + 0.25 * R_new)).max() <= 1e-13
    assert np.array_equal(S2, S) and np.array_equal(C2, C)
    # init ignores the previous residual
    Ri, _, _ = full_ema(F, V, None, R_prev, 0.3, 0.25, True, "f64")
    assert np.array_equal(Ri, full(F, V, None, 0.3, True, "f64")[0])
    # a constant feature gives a constant residual state, whatever alpha_r
    Rc = R_new
    for _ in range(4):
        Rc, _, _ = full_ema(F, V, S0, Rc, 0.3, 0.4, False, "f64")
    assert np.abs(Rc - R_new).max() <= 1e-13


# ---------------------------------------------------------------------------
# basis reuse and re-basing (Sec. 3.3, Fig. 1(b))
# ---------------------------------------------------------------------------

def check_rebase(overlap, rebase, forecast):
    r = rng(61)
    n, d, k = 40, 24, 6
    V = random_orthonormal(r, d, k)
    S = r.standard_normal((n, k))
    R = r.standard_normal((n, d))
    # same basis: M = I, state unchanged
    M = overlap(V, V)
    assert np.abs(M - np.eye(k)).max() <= 1e-14
    assert np.abs(rebase(S, M) - S).max() <= 1e-13
    # a rotation inside the same subspace changes the coefficients but not the feature they stand for
    Q = random_orthonormal(r, k, k)
    V2 = V @ Q
    M = overlap(V, V2)
    assert np.abs(M - Q).max() <= 1e-13
    S2 = rebase(S, M)
    assert np.abs(S2 - S).max() > 0.1
    assert np.abs(forecast(S2, V2, R, "f64") - forecast(S, V, R, "f64")).max() <= 1e-12
    # entry (i, j) is the inner product of old direction i with new direction j (not the transpose)
    W = random_orthonormal(r, d, k)
    M = overlap(V, W)
    assert abs(M[1, 4] - float(V[:, 1] @ W[:, 4])) <= 1e-14 and abs(M[1, 4] - M[4, 1]) > 1e-3
    # general new basis: the new coefficients are those of the orthogonal projection of S V^T onto span(W)
    P_old = S @ V.T
    best = np.linalg.lstsq(W, P_old.T, rcond=None)[0].T          # argmin_X |X W^T - P_old|
    assert np.abs(rebase(S, M) - best).max() <= 1e-12
    # a basis orthogonal to the old one carries nothing over
    full = random_orthonormal(r, d, 2 * k)
    assert np.abs(rebase(S, overlap(full[:, :k], full[:, k:]))).max() <= 1e-13


def check_basis_similarity(similarity):
    r = rng(62)
    d, k = 30, 5
    V = random_orthonormal(r, d, k)
    s = np.array([9.0, 5.0, 3.0, 2.0, 1.0])
    sd, ss = similarity(V, s, V, s)
    assert np.abs(sd - 1).max() <= 1e-14 and abs(ss - 1) <= 1e-14
    # a sign flip of a singular vector changes nothing; scaling the spectrum by c costs min(c, 1/c)
    V2 = V.copy()
    V2[:, 2] *= -1
    sd, ss = similarity(V, s, V2, 0.5 * s)
    assert np.abs(sd - 1).max() <= 1e-14 and abs(ss - 0.5) <= 1e-14
    sd, ss = similarity(V, s, V2, 4.0 * s)
    assert abs(ss - 0.25) <= 1e-14
    # a direction rotated by the angle phi inside a plane has similarity cos(phi)
    phi = 0.3
    V3 = V.copy()
    V3[:, 0] = np.cos(phi) * V[:, 0] + np.sin(phi) * V[:, 1]
    sd, _ = similarity(V, s, V3, s)
    assert abs(sd[0] - np.cos(phi)) <= 1e-14 and np.abs(sd[1:] - 1).max() <= 1e-14
    # orthogonal directions: zero; a non-unit vector pays its norm ratio
    full = random_orthonormal(r, d, 2 * k)
    sd, _ = similarity(full[:, :k], s, full[:, k:], s)
    assert np.abs(sd).max() <= 1e-14
    V4 = V.copy()
    V4[:, 1] *= 0.8
    sd, _ = similarity(V, s, V4, s)
    assert abs(sd[1] - 0.8) <= 1e-14
    # different spectra: the textbook cosine times the norm ratio
    t = np.array([8.0, 6.0, 1.0, 1.0, 0.5])
    _, ss = similarity(V, s, V, t)
    cos = float(s @ t) / (np.linalg.norm(s) * np.linalg.norm(t))
    assert abs(ss - cos * min(np.linalg.norm(s), np.linalg.norm(t)) / max(np.linalg.norm(s), np.linalg.norm(t))) <= 1e-14
    assert ss < 1
