"""CPU oracle for the SVD-Cache step.  TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may
import this module; the GPU library never does, and this module imports
nothing from the GPU package.  It is deliberately plain: numpy, float64,
one statement per equation of the paper, no blocking, no fusion.

Conventions
-----------
* All inputs are numpy arrays; every input is promoted to float64.  A "bf16"
  or "f32" tensor is passed as the float64 array holding exactly its values
  (the caller converts losslessly), so input rounding never counts as error.
* ``store`` names the storage type of F / R / Fhat ("f64", "f32", "bf16").
  Results are computed in float64 and rounded ONCE to that type (R, Fhat) or
  to float32 (C, S) at the very end, then returned as float64 arrays holding
  the rounded values.  ``store="f64"`` disables all rounding (used by the
  algebraic pins).
* alpha is the weight on the NEW observation, alpha = 1 - beta in the symbols
  of Eq. 11 (the paper's beta = 0.9 is alpha = 0.1).

Pins: tests/test_oracle_*.py (brute-force Jacobi SVD, constructed spectra,
Eckart-Young, permutation invariance, closed-form EMA, exact identities).
"""
from __future__ import annotations

import numpy as np

# ----------------------------------------------------------------------------
# rounding to the storage types
# ----------------------------------------------------------------------------


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round float64 values to the nearest bfloat16 (8 significant bits,
    ties to even), returned as float64.  Done directly from float64 so there
    is no double rounding through float32."""
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)                      # x = m * 2^e, 0.5 <= |m| < 1
    e = np.maximum(e, -125)                 # bf16 subnormals share the quantum 2^-133
    quantum = np.ldexp(1.0, e - 8)
    y = np.rint(x / quantum) * quantum      # np.rint rounds half to even
    bf16_max = (2.0 - 2.0 ** -7) * 2.0 ** 127
    y = np.where(np.abs(y) > bf16_max, np.sign(x) * np.inf, y)
    return np.where(np.isfinite(x), y, x)


def round_store(x: np.ndarray, store: str) -> np.ndarray:
    if store == "f64":
        return np.asarray(x, dtype=np.float64)
    if store == "f32":
        return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)
    if store == "bf16":
        return round_bf16(x)
    raise ValueError(f"unknown storage type {store!r}")


def _round_f32(x: np.ndarray, store: str) -> np.ndarray:
    """C and S are kept in float32 whatever the feature storage type is."""
    return x if store == "f64" else round_store(x, "f32")


# ----------------------------------------------------------------------------
# basis fit: exact truncated SVD (Sec. 3.2, Eq. 4-5)
# ----------------------------------------------------------------------------


def canonical_sign(V: np.ndarray) -> np.ndarray:
    """Flip each column so its largest-magnitude entry is positive.  Cosmetic:
    singular vectors are defined up to sign and nothing relies on this."""
    idx = np.argmax(np.abs(V), axis=0)
    sgn = np.sign(V[idx, np.arange(V.shape[1])])
    sgn[sgn == 0] = 1.0
    return V * sgn


def ref_fit_basis(F: np.ndarray, k: int, method: str = "auto"):
    """Top-k right singular vectors and singular values of F (Eq. 4-5).

    Returns (V_k [D,k], sigma_k [k] descending, fro2 = ||F||_F^2).

    method "svd":  LAPACK SVD of F itself (the definition).
    method "gram": eigen-decomposition of the D x D Gram matrix F^T F, whose
                   eigenvectors are F's right singular vectors and whose
                   eigenvalues are sigma^2.  Same result, affordable at
                   FLUX size.  Checked against "svd" in the oracle's tests.
    """
    F = np.asarray(F, dtype=np.float64)
    N, D = F.shape
    if not (1 <= k <= min(N, D)):
        raise ValueError("need 1 <= k <= min(N, D)")
    if method == "auto":
        method = "svd" if N * D * min(N, D) <= 2e9 else "gram"
    fro2 = float(np.sum(F * F))
    if method == "svd":
        _, s, Vt = np.linalg.svd(F, full_matrices=False)
        V = Vt.T[:, :k]
        sigma = s[:k]
    elif method == "gram":
        G = F.T @ F
        lam, W = np.linalg.eigh(G)          # ascending
        order = np.argsort(lam)[::-1][:k]
        V = W[:, order]
        sigma = np.sqrt(np.maximum(lam[order], 0.0))
    else:
        raise ValueError(method)
    return canonical_sign(V), sigma, fro2


def ref_rank_for_energy(sigma_all: np.ndarray, tau: float) -> int:
    """Smallest k whose leading singular values hold a fraction tau of the
    energy sum(sigma^2) (rank-selection rule, Eq. 6)."""
    e = np.asarray(sigma_all, dtype=np.float64) ** 2
    frac = np.cumsum(e) / np.sum(e)
    return int(np.searchsorted(frac, tau, side="left") + 1) if tau > 0 else 1


def ref_select_rank(sigma_lead, fro2: float, tau: float):
    """Energy rule of Eq. 6 when only the k leading singular values and the
    total energy ||F||_F^2 = sum over ALL sigma_i^2 are known (what a truncated
    fit returns): the smallest k* <= k with sum_{i<=k*} sigma_i^2 >= tau * fro2.

    Returns (k_star, reached).  If even all k values hold less than tau of the
    energy, k_star = k and reached = False (the fitted rank is too small).

    The decision is taken in float64 on the float32 inputs, the partial sums
    formed left to right, the threshold formed as float64(tau32) * float64(fro2),
    so that an implementation doing the same arithmetic gets the same integer."""
    sig = np.asarray(sigma_lead, dtype=np.float32).astype(np.float64)
    thr = float(np.float32(tau)) * float(np.float32(fro2))
    acc = 0.0
    for i, s_i in enumerate(sig):
        acc = acc + s_i * s_i
        if acc >= thr:
            return i + 1, True
    return len(sig), False


def ref_truncate_basis(V, sigma, k_star: int):
    """Rank-k* basis stored in the frame of a rank-k one: columns (and singular
    values) from k* on are set to zero.  A step taken with this basis is the
    rank-k* step: the extra coefficients are identically zero."""
    V = np.array(V, dtype=np.float64, copy=True)
    V[:, k_star:] = 0.0
    if sigma is None:
        return V, None
    sigma = np.array(sigma, dtype=np.float64, copy=True)
    sigma[k_star:] = 0.0
    return V, sigma


# ----------------------------------------------------------------------------
# full-compute step (Eq. 8-11)
# ----------------------------------------------------------------------------


def ref_full_step(F, V, S_prev, alpha: float, init: bool, store: str = "f64"):
    """One full-compute step for one block.

    C = F V_k                    coefficients in the cached basis.  Eq. 8 forms
                                 U = F V diag(sigma)^-1 and Eq. 9 multiplies by
                                 diag(sigma_k) again, so sigma cancels and the
                                 rank-k part is F_k = (F V_k) V_k^T.
    R = F - C V_k^T              residual, Eq. 10.
    S = C                        if init (first full step: state starts at the
                                 observation), else
    S = (1-alpha) S_prev + alpha C     EMA of Eq. 11 with beta = 1-alpha, kept in
                                 coefficient space (V_k is fixed, so averaging
                                 C and then multiplying by V_k^T equals
                                 averaging F_k).

    V is used as given (not re-orthonormalised).  Returns (R, S, C).
    """
    F = np.asarray(F, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    if not (0.0 < alpha <= 1.0):
        raise ValueError("alpha must lie in (0, 1]")
    C = F @ V
    R = F - C @ V.T
    if init:
        S = C.copy()
    else:
        S = (1.0 - alpha) * np.asarray(S_prev, dtype=np.float64) + alpha * C
    return round_store(R, store), _round_f32(S, store), _round_f32(C, store)


# ----------------------------------------------------------------------------
# cached step (Sec. 3.5)
# ----------------------------------------------------------------------------


def ref_forecast(S, V, R, store: str = "f64"):
    """Cached step: the EMA state is the forecast of the principal
    coefficients, the residual is reused unchanged, and the feature is their
    sum:  Fhat = S V_k^T + R  (Sec. 3.4 last paragraph, Sec. 3.5)."""
    S = np.asarray(S, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    R = np.asarray(R, dtype=np.float64)
    return round_store(S @ V.T + R, store)


def ref_extrapolation_weights(order: int, offset: float, interval: float):
    """Weights w_0..w_order on the states observed at times t, t - interval, ...,
    t - order*interval such that sum_m w_m x(t - m*interval) is the value at
    t + offset of the polynomial of degree `order` through those states
    (Lagrange form; order 0 is plain reuse of the latest state).  This is how a
    finite-difference / Taylor-type forecaster in the principal subspace
    (Sec. 5.3, Fig. 5(b)) is expressed as a
    linear combination of stored coefficient states."""
    from fractions import Fraction
    x = Fraction(offset).limit_denominator(1 << 20) / Fraction(interval).limit_denominator(1 << 20)
    nodes = [Fraction(-m) for m in range(order + 1)]
    w = []
    for m, xm in enumerate(nodes):
        num, den = Fraction(1), Fraction(1)
        for i, xi in enumerate(nodes):
            if i != m:
                num *= (x - xi)
                den *= (xm - xi)
        w.append(float(num / den))
    return np.array(w, dtype=np.float64)


def ref_forecast_combine(S_list, weights, V, R, X=None, store: str = "f64"):
    """Cached step with a forecaster that is linear in stored coefficient states
    (Sec. 5.3, Fig. 5(b): other predictors applied to the low-rank part):
        C_hat = sum_m w_m S_m,   Fhat = C_hat V_k^T + R   [+ X]
    With one state and weight 1 this is the paper's cached step.  X, if given,
    is a tensor the forecast is added to (the hidden state of a residual
    connection), so that Fhat itself need not be written."""
    V = np.asarray(V, dtype=np.float64)
    R = np.asarray(R, dtype=np.float64)
    w = np.asarray(weights, dtype=np.float32).astype(np.float64)
    if len(S_list) != len(w) or len(w) < 1:
        raise ValueError("one weight per state")
    C_hat = np.zeros_like(np.asarray(S_list[0], dtype=np.float64))
    for w_m, S_m in zip(w, S_list):
        C_hat = C_hat + w_m * np.asarray(S_m, dtype=np.float64)
    out = C_hat @ V.T + R
    if X is not None:
        out = out + np.asarray(X, dtype=np.float64)
    return round_store(out, store)


def ref_full_step_residual_ema(F, V, S_prev, R_prev, alpha: float, alpha_r: float, init: bool, store: str = "f64"):
    """Ablation "EMA on both parts" (Sec. 4.5, Fig. 5(c)): as ref_full_step, and the
    residual state is smoothed too,
        R_state = R_new                                   if init
        R_state = (1 - alpha_r) R_prev + alpha_r R_new     otherwise,
    with R_new = F - C V_k^T.  alpha_r = 1 is the paper's method (plain reuse of
    the latest residual)."""
    if not (0.0 < alpha_r <= 1.0):
        raise ValueError("alpha_r must lie in (0, 1]")
    R_new, S, C = ref_full_step(F, V, S_prev, alpha, init, store="f64")
    if init:
        R_state = R_new
    else:
        R_state = (1.0 - alpha_r) * np.asarray(R_prev, dtype=np.float64) + alpha_r * R_new
    return round_store(R_state, store), _round_f32(S, store), _round_f32(C, store)


# ----------------------------------------------------------------------------
# basis reuse across prompts and re-basing (Sec. 3.3, Fig. 1(b))
# ----------------------------------------------------------------------------


def ref_basis_overlap(V_old, V_new):
    """M = V_old^T V_new  (k_old x k_new): entry (i, j) is the cosine between the
    i-th old and the j-th new basis direction (both sets orthonormal)."""
    return np.asarray(V_old, dtype=np.float64).T @ np.asarray(V_new, dtype=np.float64)


def ref_rebase_state(S, M, store: str = "f64"):
    """Coefficient state carried over to a refitted basis.  The principal part the
    state stands for is S V_old^T; its coefficients in the new basis are
    (S V_old^T) V_new = S (V_old^T V_new) = S M.  If both bases span the same
    subspace nothing is lost: S_new V_new^T = S V_old^T."""
    out = np.asarray(S, dtype=np.float64) @ np.asarray(M, dtype=np.float64)
    return _round_f32(out, store)


def ref_basis_similarity(V_a, sigma_a, V_b, sigma_b):
    """Similarity of two fitted bases as in Fig. 1(b): cosine similarity times
    magnitude similarity, for each pair of right singular vectors and for the two
    singular-value vectors.  Reading taken here (the caption gives no formula):
    cosine = |<a, b>| / (|a| |b|) (singular vectors are defined up to sign, so the
    absolute value), magnitude similarity = min(|a|, |b|) / max(|a|, |b|).
    Returns (sim_dir [k], sim_sigma)."""
    Va, Vb = np.asarray(V_a, dtype=np.float64), np.asarray(V_b, dtype=np.float64)
    sa, sb = np.asarray(sigma_a, dtype=np.float64), np.asarray(sigma_b, dtype=np.float64)

    def sim(a, b, signed):
        na, nb = np.sqrt(np.sum(a * a)), np.sqrt(np.sum(b * b))
        if na == 0.0 or nb == 0.0:
            return 0.0
        dot = np.sum(a * b)
        cos = (dot if signed else abs(dot)) / (na * nb)
        return cos * min(na, nb) / max(na, nb)

    sim_dir = np.array([sim(Va[:, j], Vb[:, j], False) for j in range(Va.shape[1])])
    return sim_dir, sim(sa, sb, True)


# ----------------------------------------------------------------------------
# a whole sampling trajectory for one block
# ----------------------------------------------------------------------------


def ref_trajectory(features, k: int, interval: int, alpha: float, store: str = "f64", V=None):
    """Run the schedule "full step iff t mod interval == 0" over a list of
    feature matrices F_0 .. F_{T-1}.

    The basis is fitted once, on F_0 (one-time SVD, Sec. 3.3), unless V is
    given.  On a full step the block output is F_t itself and (R, S) are
    refreshed; on a cached step the output is the forecast and the state is
    left untouched.  Returns a dict with V, sigma and per-step lists.
    """
    sigma = None
    if V is None:
        V, sigma, _ = ref_fit_basis(features[0], k)
        V = round_store(V, "f32") if store != "f64" else V
    out, Rs, Ss, kinds = [], [], [], []
    R = S = None
    for t, F in enumerate(features):
        if t % interval == 0:
            R, S, _ = ref_full_step(F, V, S, alpha, init=(S is None), store=store)
            out.append(np.asarray(F, dtype=np.float64))
            kinds.append("full")
        else:
            out.append(ref_forecast(S, V, R, store=store))
            kinds.append("cached")
        Rs.append(R)
        Ss.append(S)
    return {"V": V, "sigma": sigma, "out": out, "R": Rs, "S": Ss, "kind": kinds}
