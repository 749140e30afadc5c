"""CPU oracle for the SVD-Cache hot path: test infrastructure only.

Nothing in the GPU package imports this; only tests, the smoke check and the
benchmark's cpu_baseline leg do.
"""
from .svdcache_ref import (round_bf16, round_store, canonical_sign, ref_fit_basis,
                           ref_rank_for_energy, ref_select_rank, ref_truncate_basis, ref_full_step,
                           ref_forecast, ref_extrapolation_weights, ref_forecast_combine,
                           ref_full_step_residual_ema, ref_basis_overlap, ref_rebase_state,
                           ref_basis_similarity, ref_trajectory)
from .jacobi_svd import jacobi_svd

__all__ = ["round_bf16", "round_store", "canonical_sign", "ref_fit_basis", "ref_rank_for_energy",
           "ref_select_rank", "ref_truncate_basis", "ref_full_step", "ref_forecast", "ref_extrapolation_weights",
           "ref_forecast_combine", "ref_full_step_residual_ema", "ref_basis_overlap", "ref_rebase_state",
           "ref_basis_similarity", "ref_trajectory", "jacobi_svd"]
