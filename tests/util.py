"""Helpers shared by the GPU parity tests (metrics only; no method arithmetic)."""
from __future__ import annotations

import os

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


# Element-wise allowance, on top of the norm-wise bars above:  |got - ref| <= REL[store] * |ref| + c * rms_i,
# rms_i = root mean square of row i of the large terms the result is formed from (the features for R and Fhat;
# the reference itself where no such tensor is passed).  REL: one bf16 unit in the last place for values stored
# as bf16 (the oracle rounds a float64 result, the device a float32 one: next to a rounding boundary the two may
# land on neighbouring bf16 values), nothing for float32.  c: accumulated arithmetic error relative to the size
# of the terms summed, by arithmetic mode (see ELEM_C).
ELEM_REL = {"f32": 0.0, "bf16": 2.0 ** -7}
ELEM_C = {
    # float32 results.  On the matrix cores both factors enter as bf16 high + low parts (16 significant bits) and the
    # low x low product is dropped: 2^-16 per term, relative to the largest term of the sum, which for R and Fhat is
    # |C_i1 V_d1| <= ||F_i|| max|V| ~ 4 rms_i.  Measured worst over all cases: 7e-5.
    "f32": 2e-4,
    # bf16 storage, split operands (SVDC_PRECISE): the same arithmetic; measured worst 4.4e-5
    "bf16": 1e-4,
    # single bf16 operands (SVDC_FAST): 2^-9 per factor; sum_j |C_ij| |V_dj| <= ||C_i|| ||V_d,:|| ~ sqrt(D) rms_i x
    # 2 sqrt(k / D), i.e. 2^-8 sqrt(k) rms_i: 0.044 at k = 128.  Measured worst 2.4e-2.
    "bf16-fast": 5e-2,
}
_ELEM_LOG = []           # (what, store key, worst normalised excess) of every call, for calibration runs


def elem_excess(got, ref, store: str, scale_of=None, ulp_of=None) -> float:
    """max over elements of (|got - ref| - REL (|ref| + |ulp_of|)) / rms_i, to be compared with ELEM_C[...]."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    base = ref if scale_of is None else np.asarray(scale_of, dtype=np.float64)
    rms = np.sqrt(np.mean(base.reshape(ref.shape[0], -1) ** 2, axis=1)) if ref.ndim >= 2 else np.sqrt(np.mean(base ** 2))
    rms = np.maximum(rms, np.finfo(np.float64).tiny)
    exc = np.abs(got - ref) - ELEM_REL[store] * np.abs(ref)
    if ulp_of is not None:
        exc = exc - ELEM_REL[store] * np.abs(np.asarray(ulp_of, dtype=np.float64))
    if ref.ndim >= 2:
        exc = exc.reshape(ref.shape[0], -1) / rms[:, None]
    else:
        exc = exc / rms
    return float(exc.max()) if exc.size else 0.0


def assert_close(got, ref, store: str, what: str, factor: float = 1.0, floor_of=None, fast: bool = False,
                 scale_of=None, ulp_of=None):
    """Norm-wise relative error <= TOL[store], no single row worse than 4x that, and every ELEMENT within
    ELEM_REL[store] * |ref| + ELEM_C[mode] * rms(row of the large terms).

    ``floor_of``: for a result that is a small difference of large terms (R = F - C V^T, which
    vanishes when V spans everything) the fp32 accumulation error is proportional to the large
    terms, not to the result; pass F there and 1e-6 * ||F|| is added to the norm allowance, and the
    element-wise allowance is scaled by the rows of F.  ``scale_of``: the same for the element-wise
    allowance only.  ``fast``: the result was computed with single bf16 operands (SVDC_FAST).
    ``ulp_of``: a stored INPUT of the result that the two sides hold separately (the cached step reads each
    side's own residual, and two correctly rounded residuals may differ in their last place): one unit in the
    last place of it is allowed on top, element by element."""
    tol = TOL[store] * factor
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, f"{what}: shape {got.shape} != {ref.shape}"
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
    key = "bf16-fast" if (fast and store == "bf16") else store
    base = scale_of if scale_of is not None else floor_of
    exc = elem_excess(got, ref, store, base, ulp_of)
    _ELEM_LOG.append((what + " | " + os.environ.get("PYTEST_CURRENT_TEST", ""), key, exc))
    if os.environ.get("SVDC_ELEM_LOG"):      # calibration run: record every call, judge nothing element-wise
        return
    assert exc <= ELEM_C[key] * factor, \
        f"{what}: an element is off by {exc:.3e} x rms(row) beyond {ELEM_REL[store]:.1e} |ref| (allowed {ELEM_C[key] * factor:.1e})"
