"""Brute-force one-sided (Hestenes) Jacobi SVD.  TEST INFRASTRUCTURE.

Used only on tiny matrices, as an independent check of the LAPACK-based
``ref_fit_basis`` (which is the definition of Eq. 4 evaluated by a library
routine).  Plain Python loops over column pairs; float64.

Method: repeatedly pick a pair of columns (p, q) of the working matrix A and
apply the plane rotation (on the right) that makes them orthogonal,
accumulating the same rotations into V.  When every pair is orthogonal,
A = U diag(sigma) with sigma_j = ||A[:, j]||, and F = U diag(sigma) V^T.
"""
from __future__ import annotations

import numpy as np


def jacobi_svd(F: np.ndarray, tol: float = 1e-15, max_sweeps: int = 60):
    """Thin SVD F = U diag(s) V^T with s descending.

    Returns (U [N,r], s [r], V [D,r]) with r = min(N, D).  If N < D the
    decomposition of F^T is computed and the factors swapped."""
    F = np.asarray(F, dtype=np.float64)
    N, D = F.shape
    if N < D:
        V, s, U = jacobi_svd(F.T, tol, max_sweeps)
        return U, s, V
    A = F.copy()
    V = np.eye(D)
    for _ in range(max_sweeps):
        rotated = False
        for p in range(D - 1):
            for q in range(p + 1, D):
                app = float(A[:, p] @ A[:, p])
                aqq = float(A[:, q] @ A[:, q])
                apq = float(A[:, p] @ A[:, q])
                if abs(apq) <= tol * np.sqrt(app * aqq) or apq == 0.0:
                    continue
                rotated = True
                # rotation angle that zeroes the (p, q) inner product
                zeta = (aqq - app) / (2.0 * apq)
                t = (1.0 if zeta >= 0 else -1.0) / (abs(zeta) + np.sqrt(1.0 + zeta * zeta))
                c = 1.0 / np.sqrt(1.0 + t * t)
                s = c * t
                ap = A[:, p].copy()
                A[:, p] = c * ap - s * A[:, q]
                A[:, q] = s * ap + c * A[:, q]
                vp = V[:, p].copy()
                V[:, p] = c * vp - s * V[:, q]
                V[:, q] = s * vp + c * V[:, q]
        if not rotated:
            break
    else:
        raise RuntimeError("Jacobi SVD did not converge")
    sig = np.sqrt(np.sum(A * A, axis=0))
    order = np.argsort(-sig, kind="stable")
    sig = sig[order]
    A = A[:, order]
    V = V[:, order]
    U = np.zeros_like(A)
    nz = sig > 0
    U[:, nz] = A[:, nz] / sig[nz]
    return U, sig, V
