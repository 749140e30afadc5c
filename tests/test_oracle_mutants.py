"""Plant plausible mistakes in copies of the oracle (on the CPU) and show that
the pins catch each one: a dropped term, a wrong sign, a transposed operand,
a swapped EMA weight, a wrong ordering."""
import numpy as np
import pytest

import pins
from oracle import ref_fit_basis, ref_full_step, ref_forecast


def _full(mut):
    def f(F, V, S_prev, alpha, init, store="f64"):
        F = np.asarray(F, float); V = np.asarray(V, float)
        C = F @ V
        if mut == "residual_sign":
            R = F + C @ V.T
        elif mut == "no_residual":
            R = F.copy()
        elif mut == "gram_instead_of_projector":          # C (V^T V)^-1-like slip: uses V V^T V
            R = F - (C @ (V.T @ V)) @ V.T
        else:
            R = F - C @ V.T
        if init:
            S = C.copy() if mut != "zero_init" else alpha * C
        elif mut == "ema_weights_swapped":
            S = alpha * np.asarray(S_prev, float) + (1 - alpha) * C
        elif mut == "ema_no_decay":
            S = np.asarray(S_prev, float) + alpha * C
        else:
            S = (1 - alpha) * np.asarray(S_prev, float) + alpha * C
        return R, S, C
    return f


FULL_CHECKS = [pins.check_full_identities, pins.check_full_special_bases, pins.check_ema_closed_forms]


@pytest.mark.parametrize("mut", ["residual_sign", "no_residual", "gram_instead_of_projector",
                                 "zero_init", "ema_weights_swapped", "ema_no_decay"])
def test_full_step_mutants_are_caught(mut):
    caught = 0
    for chk in FULL_CHECKS:
        try:
            chk(_full(mut))
        except AssertionError:
            caught += 1
    assert caught >= 1, mut


def test_unmutated_copy_passes():
    for chk in FULL_CHECKS:
        chk(_full(None))


@pytest.mark.parametrize("mut", ["drop_residual", "drop_principal", "untransposed_sign", "uses_C_not_S"])
def test_forecast_mutants_are_caught(mut):
    state = {}

    def full(F, V, S_prev, alpha, init, store="f64"):
        R, S, C = ref_full_step(F, V, S_prev, alpha, init, store)
        state["C"] = C
        return R, S, C

    def fc(S, V, R, store="f64"):
        if mut == "drop_residual":
            return S @ V.T
        if mut == "drop_principal":
            return R.copy()
        if mut == "untransposed_sign":
            return R - S @ V.T
        return state["C"] @ V.T + R
    with pytest.raises(AssertionError):
        pins.check_forecast(full, fc)


@pytest.mark.parametrize("mut", ["left_vectors", "ascending", "sigma_squared", "fro_norm_not_squared"])
def test_fit_mutants_are_caught(mut):
    def fit(F, k, method="auto"):
        F = np.asarray(F, float)
        U, s, Vt = np.linalg.svd(F, full_matrices=False)
        V = Vt.T
        if mut == "left_vectors":
            V = U[: F.shape[1], :] if U.shape[0] >= F.shape[1] else np.pad(U, ((0, F.shape[1] - U.shape[0]), (0, 0)))
        if mut == "ascending":
            V, s = V[:, ::-1], s[::-1]
        if mut == "sigma_squared":
            s = s ** 2
        fro2 = np.sum(F * F) if mut != "fro_norm_not_squared" else np.sqrt(np.sum(F * F))
        return V[:, :k], s[:k], fro2
    caught = 0
    for chk in [pins.check_fit_vs_bruteforce, pins.check_fit_constructed_spectrum,
                pins.check_fit_eckart_young_and_energy, pins.check_fit_closed_forms]:
        try:
            chk(fit)
        except AssertionError:
            caught += 1
    assert caught >= 1, mut
