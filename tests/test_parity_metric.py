"""The parity metric itself (tests/util.assert_close), on the CPU: a result that differs from the oracle only by
its storage rounding passes, and a LOCAL mistake of the size a kernel indexing bug would make -- one lane's
8-channel piece of one row written to the wrong place -- fails, although the block norm and the worst-row norm at
their loose bars would let it through."""
import numpy as np
import pytest

from oracle import ref_full_step, ref_forecast, round_bf16
from util import assert_close, TOL


def _problem(seed=0, N=96, D=3072, k=32):
    g = np.random.default_rng(seed)
    V = np.linalg.qr(g.standard_normal((D, k)))[0]
    C = g.standard_normal((N, k)) * np.arange(1, k + 1) ** -0.6 * np.sqrt(D)
    F = round_bf16(C @ V.T + 0.22 * g.standard_normal((N, D)))
    return F, V.astype(np.float32).astype(np.float64)


def test_rounding_differences_pass_and_a_misplaced_lane_piece_fails():
    F, V = _problem()
    R, S, C = ref_full_step(F, V, None, 0.5, True, "bf16")
    # a device-like result: float32 arithmetic error of a few 1e-6 of the row scale, then its own bf16 rounding
    g = np.random.default_rng(1)
    got = round_bf16((F - (F @ V) @ V.T) + 3e-6 * g.standard_normal(F.shape))
    assert_close(got, R, "bf16", "R", floor_of=F)
    # one 16-byte piece (8 channels of one token) lands one row further down: 8 wrong elements out of 295 thousand
    scale = np.sqrt(np.mean(np.linalg.norm(R, axis=-1) ** 2))
    for c0 in range(512, 1024, 8):          # the first piece whose misplacement the row bar lets through (most do)
        bad = got.copy()
        bad[41, c0:c0 + 8] = got[40, c0:c0 + 8]
        rows = np.linalg.norm(bad - R, axis=-1)
        if rows.max() <= 4 * TOL["bf16"] * scale:
            break
    assert np.linalg.norm(bad - R) <= TOL["bf16"] * np.linalg.norm(R)         # the block norm does not see it
    assert rows.max() <= 4 * TOL["bf16"] * scale                              # nor does the worst-row norm
    with pytest.raises(AssertionError, match="an element is off"):
        assert_close(bad, R, "bf16", "R with a misplaced piece", floor_of=F)
    # the same for the cached step and for a float32 coefficient
    Fh = ref_forecast(S, V, R, "bf16")
    assert_close(round_bf16(S @ V.T + got), Fh, "bf16", "Fhat", scale_of=F, ulp_of=R)
    badh = Fh.copy()
    badh[7, 64:72] = Fh[8, 64:72]
    with pytest.raises(AssertionError):
        assert_close(badh, Fh, "bf16", "Fhat with a misplaced piece", scale_of=F, ulp_of=R)
    badc = C.copy()
    badc[3, 5] = C[3, 6]
    with pytest.raises(AssertionError):
        assert_close(badc, C, "f32", "C with a swapped coefficient")
