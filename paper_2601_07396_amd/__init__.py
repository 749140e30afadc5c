"""MI355X-native SVD-Cache hot path: thin Python binding over libsvdcache.so.

Every arithmetic step runs in the HIP kernels behind the C ABI declared in
include/svdcache.h; this package only marshals torch tensors (device memory
and the current stream) into that ABI.  There is no CPU fallback: calling any
function without the compiled library, or with tensors that are not on the
GPU, raises.
"""
from .binding import (
    SvdcError, Shape, SVDC_PRECISE, SVDC_FAST, lib_path, load_library, exported_symbols,
    svdcache_version, svdcache_strerror, svdcache_fit_workspace_bytes, svdcache_workspace_bytes,
    svdcache_fit_status_offset, SVDC_FIT_JACOBI_CAPPED, SVDC_FIT_RANK_DEFICIENT, svdcache_packed_basis_bytes,
    svdcache_has_mfma_path, svdcache_fit_basis, svdcache_fit_basis_static, SVDC_STATIC_SCRATCH_BYTES,
    svdcache_pack_basis, svdcache_full_step, svdcache_forecast,
    svdcache_full_step_residual_ema,
    svdcache_packed_state_bytes, svdcache_pack_state, svdcache_full_step_packed, svdcache_forecast_packed,
    alloc_packed_state,
    svdcache_select_rank, svdcache_truncate_basis, svdcache_extrapolation_weights, svdcache_forecast_combine,
    svdcache_basis_overlap, svdcache_rebase_state, svdcache_basis_similarity,
    make_shape, fit_basis, fit_basis_for_energy, pack_basis, save_basis, load_basis,
)

__all__ = [
    "SvdcError", "Shape", "SVDC_PRECISE", "SVDC_FAST", "lib_path", "load_library", "exported_symbols",
    "svdcache_version", "svdcache_strerror", "svdcache_fit_workspace_bytes", "svdcache_workspace_bytes",
    "svdcache_fit_status_offset", "SVDC_FIT_JACOBI_CAPPED", "SVDC_FIT_RANK_DEFICIENT", "svdcache_packed_basis_bytes",
    "svdcache_has_mfma_path", "svdcache_fit_basis", "svdcache_fit_basis_static", "SVDC_STATIC_SCRATCH_BYTES",
    "svdcache_pack_basis", "svdcache_full_step",
    "svdcache_forecast", "svdcache_full_step_residual_ema", "svdcache_packed_state_bytes", "svdcache_pack_state",
    "svdcache_full_step_packed", "svdcache_forecast_packed", "alloc_packed_state", "svdcache_select_rank", "svdcache_truncate_basis", "svdcache_extrapolation_weights",
    "svdcache_forecast_combine", "svdcache_basis_overlap", "svdcache_rebase_state", "svdcache_basis_similarity",
    "make_shape", "fit_basis", "fit_basis_for_energy", "pack_basis", "save_basis", "load_basis",
]
