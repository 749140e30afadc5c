"""The oracle against what the paper and the mathematics fix (CPU only)."""
import numpy as np
import pytest

import pins
from oracle import ref_fit_basis, ref_full_step, ref_forecast, ref_rank_for_energy, jacobi_svd


def test_jacobi_svd_satisfies_definition():
    pins.check_jacobi_definition(jacobi_svd)


@pytest.mark.parametrize("check", [
    pins.check_fit_vs_bruteforce, pins.check_fit_constructed_spectrum, pins.check_fit_invariances,
    pins.check_fit_eckart_young_and_energy, pins.check_fit_closed_forms, pins.check_fit_methods_agree,
], ids=lambda f: f.__name__)
def test_fit_basis(check):
    check(ref_fit_basis)


@pytest.mark.parametrize("method", ["svd", "gram"])
def test_fit_basis_each_method_against_bruteforce(method):
    fit = lambda F, k: ref_fit_basis(F, k, method=method)
    pins.check_fit_vs_bruteforce(fit)
    pins.check_fit_closed_forms(fit)
    pins.check_fit_constructed_spectrum(fit)


@pytest.mark.parametrize("check", [
    pins.check_full_identities, pins.check_full_special_bases, pins.check_ema_closed_forms,
    pins.check_full_storage_rounding,
], ids=lambda f: f.__name__)
def test_full_step(check):
    check(ref_full_step)


def test_forecast():
    pins.check_forecast(ref_full_step, ref_forecast)


def test_rank_selection_rule():
    # energies 16, 4, 1, 1 -> cumulative fractions 16/22, 20/22, 21/22, 1
    s = np.array([4.0, 2.0, 1.0, 1.0])
    assert ref_rank_for_energy(s, 0.5) == 1
    assert ref_rank_for_energy(s, 16 / 22) == 1
    assert ref_rank_for_energy(s, 0.85) == 2      # the paper's preferred threshold
    assert ref_rank_for_energy(s, 0.92) == 3
    assert ref_rank_for_energy(s, 1.0) == 4


def test_argument_errors():
    F = np.zeros((4, 3))
    with pytest.raises(ValueError):
        ref_fit_basis(F, 4)
    with pytest.raises(ValueError):
        ref_full_step(F, np.zeros((3, 1)), None, 0.0, True)
    with pytest.raises(ValueError):
        ref_full_step(F, np.zeros((3, 1)), None, 1.5, True)


def test_select_rank():
    from oracle import ref_select_rank
    pins.check_select_rank(ref_select_rank, ref_rank_for_energy)


def test_truncate_basis():
    from oracle import ref_truncate_basis
    pins.check_truncate_basis(ref_truncate_basis, ref_full_step)


def test_extrapolation_weights():
    from oracle import ref_extrapolation_weights
    pins.check_extrapolation_weights(ref_extrapolation_weights)


def test_forecast_combine():
    from oracle import ref_forecast_combine, ref_extrapolation_weights
    pins.check_forecast_combine(ref_forecast_combine, ref_forecast, ref_full_step, ref_extrapolation_weights)


def test_residual_ema():
    from oracle import ref_full_step_residual_ema
    pins.check_residual_ema(ref_full_step_residual_ema, ref_full_step)


def test_rebase_state():
    from oracle import ref_basis_overlap, ref_rebase_state
    pins.check_rebase(ref_basis_overlap, ref_rebase_state, ref_forecast)


def test_basis_similarity():
    from oracle import ref_basis_similarity
    pins.check_basis_similarity(ref_basis_similarity)
