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
