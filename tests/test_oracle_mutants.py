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


@pytest.mark.parametrize("mut", ["sigma_not_squared", "strict_inequality_off_by_one", "index_not_count",
                                 "normalised_by_kept_energy", "never_reports_unreached"])
def test_select_rank_mutants_are_caught(mut):
    from oracle import ref_rank_for_energy

    def select(sigma_lead, fro2, tau):
        sig = np.asarray(sigma_lead, np.float64)
        e = sig if mut == "sigma_not_squared" else sig * sig
        total = np.sum(e) if mut == "normalised_by_kept_energy" else float(fro2)
        thr = float(np.float32(tau)) * total
        acc = 0.0
        for i, x in enumerate(e):
            acc += x
            if acc >= thr:
                k = i + 1
                if mut == "strict_inequality_off_by_one":
                    k = min(len(e), k + 1)
                if mut == "index_not_count":
                    k = max(1, i)
                return k, True
        return len(e), (mut == "never_reports_unreached")
    with pytest.raises(AssertionError):
        pins.check_select_rank(select, ref_rank_for_energy)


@pytest.mark.parametrize("mut", ["nodes_forward", "offset_sign", "not_normalised"])
def test_extrapolation_weight_mutants_are_caught(mut):
    def weights(order, offset, interval):
        x = offset / interval
        if mut == "offset_sign":
            x = -x
        nodes = [float(m) if mut == "nodes_forward" else -float(m) for m in range(order + 1)]
        w = []
        for m, xm in enumerate(nodes):
            num = den = 1.0
            for i, xi in enumerate(nodes):
                if i != m:
                    num *= (x - xi)
                    den *= (xm - xi) if mut != "not_normalised" else 1.0
            w.append(num / den)
        return np.array(w)
    with pytest.raises(AssertionError):
        pins.check_extrapolation_weights(weights)


@pytest.mark.parametrize("mut", ["weights_ignored", "weights_swapped", "residual_weighted", "added_tensor_dropped",
                                 "first_state_only"])
def test_forecast_combine_mutants_are_caught(mut):
    from oracle import ref_extrapolation_weights

    def combine(S_list, w, V, R, X, store="f64"):
        from oracle import round_store
        w = list(w)
        if mut == "weights_ignored":
            w = [1.0 / len(w)] * len(w)
        if mut == "weights_swapped":
            w = w[::-1]
        if mut == "first_state_only":
            S_list, w = S_list[:1], w[:1]
        Ch = sum(wm * np.asarray(Sm, float) for wm, Sm in zip(w, S_list))
        out = Ch @ V.T + (R * sum(w) if mut == "residual_weighted" else R)
        if X is not None and mut != "added_tensor_dropped":
            out = out + X
        return round_store(out, store)
    with pytest.raises(AssertionError):
        pins.check_forecast_combine(combine, ref_forecast, ref_full_step, ref_extrapolation_weights)


@pytest.mark.parametrize("mut", ["weights_swapped", "init_blends", "principal_state_smoothed_with_alpha_r"])
def test_residual_ema_mutants_are_caught(mut):
    def full_ema(F, V, S_prev, R_prev, alpha, alpha_r, init, store="f64"):
        a = alpha_r if mut == "principal_state_smoothed_with_alpha_r" else alpha
        R_new, S, C = ref_full_step(F, V, S_prev, a, init, "f64")
        if init and mut != "init_blends":
            return R_new, S, C
        if mut == "weights_swapped":
            return alpha_r * R_prev + (1 - alpha_r) * R_new, S, C
        return (1 - alpha_r) * R_prev + alpha_r * R_new, S, C
    with pytest.raises(AssertionError):
        pins.check_residual_ema(full_ema, ref_full_step)


@pytest.mark.parametrize("mut", ["overlap_transposed", "rebase_transposed", "rebase_left_multiply_pinv"])
def test_rebase_mutants_are_caught(mut):
    def overlap(Va, Vb):
        return (Vb.T @ Va) if mut == "overlap_transposed" else (Va.T @ Vb)

    def rebase(S, M, store="f64"):
        if mut == "rebase_transposed":
            return S @ M.T
        if mut == "rebase_left_multiply_pinv":
            return S @ np.linalg.pinv(M)
        return S @ M
    with pytest.raises(AssertionError):
        pins.check_rebase(overlap, rebase, ref_forecast)


@pytest.mark.parametrize("mut", ["signed_cosine", "no_magnitude_term", "magnitude_ratio_inverted", "rows_not_columns"])
def test_basis_similarity_mutants_are_caught(mut):
    def similarity(Va, sa, Vb, sb):
        def sim(a, b, signed):
            na, nb = np.linalg.norm(a), np.linalg.norm(b)
            if na == 0 or nb == 0:
                return 0.0
            dot = float(a @ b)
            cos = (dot if (signed or mut == "signed_cosine") else abs(dot)) / (na * nb)
            mag = min(na, nb) / max(na, nb)
            if mut == "no_magnitude_term":
                mag = 1.0
            if mut == "magnitude_ratio_inverted":
                mag = max(na, nb) / min(na, nb)
            return cos * mag
        if mut == "rows_not_columns":
            return np.array([sim(Va[j], Vb[j], False) for j in range(Va.shape[1])]), sim(sa, sb, True)
        return np.array([sim(Va[:, j], Vb[:, j], False) for j in range(Va.shape[1])]), sim(sa, sb, True)
    with pytest.raises(AssertionError):
        pins.check_basis_similarity(similarity)
