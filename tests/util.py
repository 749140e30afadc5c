"""Helpers shared by the GPU parity tests (metrics only; no method arithmetic)."""
from __future__ import annotations

import numpy as np
import torch

# Tolerances from the benchmark spec: norm-wise relative error per block,
# 1e-4 for float32 storage, 2e-2 for bf16 storage with fp32 accumulation.
TOL = {"f32": 1e-4, "bf16": 2e-2}


def to_np(t: torch.Tensor) -> np.ndarray:
    """Exact float64 copy of a float32 / bfloat16 tensor."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def rel_err(got, ref) -> float:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    num = np.linalg.norm(got - ref)
    return float(num / den) if den > 0 else float(num)


def row_err(got, ref) -> float:
    """Largest per-row error scaled by the RMS row norm of the reference: catches single bad rows
    that a whole-matrix norm would hide."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rows = np.linalg.norm(got - ref, axis=-1)
    scale = np.sqrt(np.mean(np.linalg.norm(ref, axis=-1) ** 2))
    return float(rows.max() / scale) if scale > 0 else float(rows.max())


def principal_sines(Va, Vb) -> np.ndarray:
    s = np.linalg.svd(np.asarray(Va).T @ np.asarray(Vb), compute_uv=False)
    return np.sqrt(np.maximum(0.0, 1.0 - np.minimum(s, 1.0) ** 2))


def assert_close(got, ref, store: str, what: str, factor: float = 1.0, floor_of=None):
    """Norm-wise relative error <= TOL[store] (and no single row worse than 4x that).

    ``floor_of``: for a result that is a small difference of large terms (R = F - C V^T, which
    vanishes when V spans everything) the fp32 accumulation error is proportional to the large
    terms, not to the result; pass F there and 1e-6 * ||F|| is added to the allowance."""
    tol = TOL[store] * factor
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    floor = 0.0 if floor_of is None else 1e-6 * np.linalg.norm(floor_of)
    err = np.linalg.norm(got - ref)
    allow = tol * np.linalg.norm(ref) + floor
    assert err <= allow, f"{what}: error {err:.3e} > allowed {allow:.3e} (rel {rel_err(got, ref):.3e})"
    rows = np.linalg.norm(got - ref, axis=-1)
    scale = np.sqrt(np.mean(np.linalg.norm(ref, axis=-1) ** 2))
    row_floor = floor / np.sqrt(max(1, ref.shape[0])) * 4
    assert rows.max() <= 4 * tol * scale + row_floor, \
        f"{what}: worst-row error {rows.max():.3e} > {4 * tol * scale + row_floor:.3e}"
