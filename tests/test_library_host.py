"""CPU-only checks of the HIP library: it loads, exports what the header declares, and its
host-side construction code agrees with the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2110_14871_amd as gd
from workloads import rng

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "gdws.h")).read()
    body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b((?:gdws|conv_dense)_\w+)\s*\(", body))
    assert declared == set(gd.EXPORTS)
    L = ctypes.CDLL(gd.LIB_PATH)
    for name in declared:
        assert getattr(L, name) is not None
    assert gd.lib().gdws_strerror(0) == b"ok" and gd.lib().gdws_strerror(-4) != gd.lib().gdws_strerror(-5)


@pytest.mark.parametrize("M,C,K,seed", [(16, 5, 3, 400), (4, 3, 2, 401), (8, 4, 1, 402), (32, 6, 5, 403), (3, 4, 3, 404)])
def test_singular_values_match_oracle(M, C, K, seed):
    W = rng.normal(seed, (M, C, K, K), std=0.1)
    if seed == 400:
        W[:, 2] = 0.0                                       # an all-zero slice has rank 0
        W[:, 3] = np.outer(np.arange(1, M + 1), np.arange(1, K * K + 1)).reshape(M, K, K) * 0.01   # rank 1
    s, r = gd.gdws_singular_values(W)
    _, S, _ = oracle.svd_slices(W)
    assert s.shape == S.shape and np.abs(s - S).max() < 1e-12
    want = [oracle.numerical_rank(S[c], max(M, K * K)) for c in range(C)]
    assert r.tolist() == want


@pytest.mark.parametrize("seed", [410, 411, 412])
def test_greedy_allocations_match_oracle_bit_for_bit(seed):
    C, M = 24, 32
    W = rng.normal(seed, (M, C, 3, 3), std=0.05)
    alpha = np.abs(rng.normal(seed + 1, (C,))).astype(np.float64) + 0.1
    s, r = gd.gdws_singular_values(W)
    _, S, _ = oracle.svd_slices(W)
    for gamma in (0, 1, C, 57, 9 * C, 9 * C + 5):
        assert (gd.gdws_mego(s, r, gamma) == oracle.mego(S, gamma, dim=M)).all()
        assert (gd.gdws_mego(s, r, gamma, alpha) == oracle.mego(S, gamma, alpha, dim=M)).all()
    g1 = gd.gdws_mego(s, r, 60, g_init=np.ones(C, np.int32), cap=9)
    assert (g1 == oracle.mego(S, 60, g_init=np.ones(C, np.int32), cap=9, dim=M)).all() and g1.sum() == 60
    g2 = gd.gdws_mego(s, r, 1000, cap=4)
    assert (g2 == 4).all()
    emax = oracle.error_from_sigmas(S, np.zeros(C, int))
    for beta in (0.0, 0.1 * emax, 0.5 * emax, 0.99 * emax, 1.01 * emax):
        assert (gd.gdws_lego(s, r, beta) == oracle.lego(S, beta, dim=M)).all()
        assert (gd.gdws_lego(s, r, beta, alpha, g_min=1) == oracle.lego(S, beta, alpha, g_min=1, dim=M)).all()
        # the algorithm-box reading of the bound (no printed value pins either side: the two are only compared)
        assert (gd.gdws_lego(s, r, beta, compare=gd.LEGO_LISTING) == oracle.lego(S, beta, compare="beta", dim=M)).all()


def test_budget_gamma_matches_oracle():
    for rho, C, K, M in [(0.25, 128, 3, 128), (0.4, 64, 3, 64), (0.4, 3, 3, 64), (0.4, 512, 3, 512), (1.0, 4, 3, 16),
                         (5.0, 4, 3, 16), (0.0, 7, 5, 3), (0.4, 256, 3, 512), (0.1, 16, 1, 8)]:
        assert gd.gdws_budget_gamma(rho, C, K, M) == oracle.gamma_from_budget(rho, C, K, M)
    assert gd.gdws_budget_gamma(0.25, 128, 3, 128) == 269
    assert gd.lib().gdws_budget_gamma(-1.0, 4, 3, 4) == -1 and gd.lib().gdws_budget_gamma(0.5, 0, 3, 4) == -1


@pytest.mark.parametrize("seed,M,C,K,keep", [(420, 16, 12, 3, 0.05), (421, 64, 24, 3, 0.02), (422, 4, 3, 2, 0.1)])
def test_sparse_aware_reduction_matches_oracle(seed, M, C, K, keep):
    """gdws_compact_factors against the oracle's reduction, bit for bit, on the oracle's factors of a pruned W."""
    import workloads
    W = workloads.pruned_weight(seed, M, C, K, keep)
    g_full = np.full(C, min(M, K * K), np.int32)
    D, Pw = oracle.truncated_factors(W, g_full)
    D, Pw = D.astype(np.float32), Pw.astype(np.float32)
    g2, D2, Pw2, keep2 = oracle.compact_factors(g_full, D, Pw)
    g3, D3, Pw3, keep3 = gd.gdws_compact_factors(g_full, D, Pw)
    assert (g3 == g2).all() and (keep3 == keep2).all()
    assert (D3 == D2.astype(np.float32)).all() and (Pw3 == Pw2.astype(np.float32)).all()
    s, r = gd.gdws_singular_values(W)
    assert (r == oracle.sparse_g(W)).all() and (g3 == r).all()


def test_argument_errors_are_reported_not_thrown():
    L = gd.lib()
    assert L.gdws_singular_values(None, 4, 4, 3, None, None) == -2
    s = np.zeros((2, 4))
    r = np.zeros(2, np.int32)
    g = np.zeros(2, np.int32)
    vp = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    assert L.gdws_mego(vp(s), vp(r), 0, 4, None, 3, 0, vp(g)) == -1
    assert L.gdws_mego(vp(s), vp(r), 2, 4, None, -1, 0, vp(g)) == -1
    assert L.gdws_lego(vp(s), vp(r), 2, 4, None, -0.5, 0, 0, vp(g)) == -1
    assert L.gdws_lego(vp(s), vp(r), 2, 4, None, 0.5, 0, 2, vp(g)) == -1       # unknown reading of the bound
    d = gd.make_desc(4, 4, 3, 1, 1)
    h = ctypes.c_void_p()
    assert L.gdws_plan(None, vp(g), None, None, None, None, ctypes.byref(h)) == -2
    bad = gd.make_desc(0, 4, 3, 1, 1)
    w = np.zeros((4, 4, 3, 3), np.float32)
    g4 = np.ones(4, np.int32)
    assert L.gdws_plan(ctypes.byref(bad), vp(g4), vp(w), None, None, None, ctypes.byref(h)) == -1
    assert L.gdws_plan(ctypes.byref(d), vp(g4), None, None, None, None, ctypes.byref(h)) == -1      # no weights
    assert L.gdws_plan(ctypes.byref(d), vp(g4), vp(w), vp(w), vp(w), None, ctypes.byref(h)) == -1   # both
    g_neg = np.array([1, -1, 1, 1], np.int32)
    assert L.gdws_plan(ctypes.byref(d), vp(g_neg), vp(w), None, None, None, ctypes.byref(h)) == -1
    g_big = np.array([1, 10, 1, 1], np.int32)                                                         # > K^2 with W given
    assert L.gdws_plan(ctypes.byref(d), vp(g_big), vp(w), None, None, None, ctypes.byref(h)) == -1
    g_zero = np.zeros(4, np.int32)
    assert L.gdws_plan(ctypes.byref(d), vp(g_zero), vp(w), None, None, None, ctypes.byref(h)) == -1
    db = gd.make_desc(4, 4, 3, 1, 1, has_bias=True)
    assert L.gdws_plan(ctypes.byref(db), vp(g4), vp(w), None, None, None, ctypes.byref(h)) == -2     # bias missing
    assert h.value is None
    assert L.gdws_forward(None, None, None, None, 1, 4, 4, None, 0, 0, None) == -2
    assert L.gdws_network_forward(None, None, None, 1, 4, 4, None, 0, None) == -2
    assert L.gdws_net_create(None, 0, ctypes.byref(h)) == -2
    assert L.gdws_workspace_bytes(None, 1, 4, 4, 0) == 0
