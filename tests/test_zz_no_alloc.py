"""The allocation-free basis fit (svdcache_fit_basis_static) against svdcache_fit_basis, through the C ABI: two
calls in a row on the library's static device workspace, the second on a smaller problem (so it runs over the
first call's leftovers), each compared with the existing entry point on the same features and seed."""
import numpy as np
import pytest
import torch

import paper_2601_07396_amd as pkg
from oracle import ref_fit_basis
from synth import WORKLOADS, FeatureStream
from util import TOL, to_np, principal_sines

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(B, N, D, k, dtype, seed):
    store = "f32" if dtype == torch.float32 else "bf16"
    wl = WORKLOADS["flux1"].with_(N=N, D=D, k=k, dtype=store, signal_rank=min(96, D, N))
    F = torch.stack([FeatureStream(wl, b).at(0) for b in range(B)]).contiguous()
    Fd = F.to(DEV)
    shape = pkg.make_shape(Fd, k)
    V0, s0, f0, st0 = pkg.fit_basis(Fd, k, q=8, seed=seed, return_status=True)
    V1 = torch.full_like(V0, float("nan"))
    s1 = torch.full_like(s0, float("nan"))
    f1 = torch.full_like(f0, float("nan"))
    st1 = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    before = torch.cuda.memory_stats(DEV)["allocation.all.allocated"]
    pkg.svdcache_fit_basis_static(shape, Fd, V1, s1, f1, st1, q=8, seed=seed)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats(DEV)["allocation.all.allocated"] == before      # torch's allocator was not asked
    assert torch.equal(st0, st1)
    for b in range(B):
        # same algorithm, same seed, same Gaussian sketch: the two differ only through the summation order of
        # float atomics in small launches, amplified by at most the inverse spectral gaps
        assert np.abs(to_np(s1[b]) / to_np(s0[b]) - 1).max() <= 1e-5
        assert abs(float(f1[b]) / float(f0[b]) - 1) <= 1e-6
        # (the trailing directions sit in the flat part of the spectrum, where a change in the last bits of the
        # sketch rotates them most: the leading half is held tighter than the whole)
        lead = max(1, k // 2)
        assert principal_sines(to_np(V0[b][:, :lead]), to_np(V1[b][:, :lead])).max() <= 1e-3
        assert principal_sines(to_np(V0[b]), to_np(V1[b])).max() <= TOL["bf16"]
        # and against the oracle, at the bar of the other fit tests
        Fb = to_np(F[b])
        _, sr, fr = ref_fit_basis(Fb, k)
        Vg, sg = to_np(V1[b]), to_np(s1[b])
        assert np.abs(Vg.T @ Vg - np.eye(k)).max() <= 1e-5
        assert np.abs(sg / sr - 1).max() <= TOL[store]
        assert 1 - np.sum((Fb @ Vg) ** 2) / np.sum(sr ** 2) <= TOL[store]
        assert abs(float(f1[b]) / fr - 1) <= 1e-5


def test_static_workspace_fit_matches_the_workspace_fit_twice_in_a_row():
    _case(3, 1000, 512, 32, torch.bfloat16, seed=5)      # matrix-core products, 3 blocks
    _case(1, 300, 256, 8, torch.bfloat16, seed=6)        # smaller: runs over what the first call left behind
    _case(2, 260, 96, 12, torch.float32, seed=7)         # general products


def test_static_workspace_fit_refuses_what_does_not_fit():
    F = torch.zeros(16, 4608, 3072, dtype=torch.bfloat16, device=DEV)
    shape = pkg.make_shape(F, 32)
    assert pkg.svdcache_workspace_bytes(shape) > pkg.SVDC_STATIC_SCRATCH_BYTES
    V = torch.zeros(16, 3072, 32, device=DEV)
    sigma, fro2 = torch.zeros(16, 32, device=DEV), torch.zeros(16, device=DEV)
    with pytest.raises(pkg.SvdcError) as e:
        pkg.svdcache_fit_basis_static(shape, F, V, sigma, fro2)
    assert e.value.code == -6
    torch.cuda.synchronize()
    assert not V.any()                                    # nothing was launched
