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
