"""Trajectory-level pins of the oracle and of the shared schedule rule (CPU)."""
import os

import numpy as np
import torch

from oracle import ref_fit_basis, ref_full_step, ref_forecast, ref_trajectory
from synth import WORKLOADS, FeatureStream, is_full_step

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_flops_ratios.txt")


def test_schedule_matches_paper_flops_ratios():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for model, n, steps, base, ours, printed, *_ in rows:
        n, steps = int(n), int(steps)
        full = sum(is_full_step(t, n) for t in range(steps))
        assert abs(steps / full - float(printed)) <= 0.01           # printed to 2 decimals
        assert abs(float(base) / float(ours) - steps / full) <= 0.01


def _tiny_features(block=0, noise=True, T=None):
    wl = WORKLOADS["tiny"]
    fs = FeatureStream(wl, block)
    T = wl.T if T is None else T
    return wl, fs, [fs.at(t, noise=noise).double().numpy() for t in range(T)]


def test_trajectory_runner_equals_manual_loop_and_split_resume():
    wl, fs, feats = _tiny_features()
    tr = ref_trajectory(feats, wl.k, wl.interval, wl.alpha, store="f32")
    V = tr["V"]
    # manual loop, interrupted after 5 steps and resumed from the saved (R, S)
    R = S = None
    outs = []
    for t in range(5):
        if is_full_step(t, wl.interval):
            R, S, _ = ref_full_step(feats[t], V, S, wl.alpha, S is None, "f32")
            outs.append(feats[t])
        else:
            outs.append(ref_forecast(S, V, R, "f32"))
    saved = (R.copy(), S.copy())
    R, S = saved
    for t in range(5, wl.T):
        if is_full_step(t, wl.interval):
            R, S, _ = ref_full_step(feats[t], V, S, wl.alpha, False, "f32")
            outs.append(feats[t])
        else:
            outs.append(ref_forecast(S, V, R, "f32"))
    for a, b in zip(outs, tr["out"]):
        assert np.array_equal(a, b)
    assert [k for k in tr["kind"]] == ["full" if t % 3 == 0 else "cached" for t in range(10)]
    # every cached step of one interval returns the same forecast
    assert np.array_equal(tr["out"][1], tr["out"][2])
    # right after the first (initialising) full step the forecast is F_0 up to fp32 rounding
    assert np.abs(tr["out"][1] - feats[0]).max() <= 1e-5 * np.abs(feats[0]).max()


def test_noise_free_generator_gives_closed_form_state():
    """Without residual noise and with the generator's own V as basis, the
    coefficients are C_t = U diag(s a(t)) exactly, so the EMA state has the
    unrolled closed form column by column."""
    wl, fs, feats = _tiny_features(noise=False)
    # tiny is stored as fp32; rebuild the noise-free features in float64
    feats = [fs.signal(t).numpy() for t in range(wl.T)]
    k = wl.k
    V = fs.V[:, :k].numpy()
    U = fs.U[:, :k].numpy()
    a = wl.alpha
    full_ts = [t for t in range(wl.T) if is_full_step(t, wl.interval)]
    tr = ref_trajectory(feats, k, wl.interval, a, store="f64", V=V)
    Cs = [U * (fs.s[:k] * fs.coeff_scale(t)[:k]).numpy() for t in full_ts]
    for n, t in enumerate(full_ts):
        expect = (1 - a) ** n * Cs[0] + a * sum((1 - a) ** (n - j) * Cs[j] for j in range(1, n + 1))
        assert np.abs(tr["S"][t] - expect).max() <= 1e-11 * np.abs(expect).max()
    # and the fitted basis of the noise-free F_0 spans the generator's leading directions
    Vfit, sig, _ = ref_fit_basis(feats[0], k)
    order = np.argsort(-(fs.s * fs.coeff_scale(0)).numpy())[:k]
    overlap = np.linalg.svd(Vfit.T @ fs.V[:, order].numpy(), compute_uv=False)
    assert overlap.min() >= 1 - 1e-9
    assert np.allclose(sig, np.sort((fs.s * fs.coeff_scale(0)).numpy())[::-1][:k], rtol=1e-9)


def test_alpha_one_reduces_to_plain_reuse():
    """With alpha = 1 the state is the newest coefficients, so every cached step
    returns the last fully computed feature: the plain-reuse cache of Eq. 3."""
    wl = WORKLOADS["flux1"].with_(N=192, D=96, k=8, signal_rank=32, T=12, interval=3)
    fs = FeatureStream(wl, 0)
    feats = [fs.at(t).double().numpy() for t in range(wl.T)]
    tr = ref_trajectory(feats, wl.k, wl.interval, 1.0, store="f64")
    last_full = None
    for t in range(wl.T):
        if is_full_step(t, wl.interval):
            last_full = feats[t]
        else:
            assert np.abs(tr["out"][t] - last_full).max() <= 1e-12 * np.abs(last_full).max()
