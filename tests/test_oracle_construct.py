"""Pins for the oracle's construction side: tables, SVD factors, error closed form, greedy optimality."""
import itertools
import os

import numpy as np
import pytest

import oracle
import workloads
from workloads import rng

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "toy_example.txt")


def _read_toy():
    d = {"pw": [], "gdw": []}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        if k in ("pw", "gdw"):
            d[k].append([float(t) for t in v])
        else:
            d[k] = [float(t) for t in v]
    return d


def test_offset_tables():
    """Property 2: channel c owns rows h_c .. h_c + g_c - 1; chan_of inverts the prefix sum."""
    g = np.array([3, 0, 1, 4, 0, 2], np.int32)
    h = oracle.offsets(g)
    co = oracle.chan_of(g)
    assert h.dtype == np.int32 and co.dtype == np.int32
    assert h[0] == 0 and h[-1] == g.sum() and (np.diff(h) == g).all()
    assert (h == np.concatenate([[0], np.cumsum(g)])).all()
    assert (co == np.repeat(np.arange(6), g)).all()
    assert (np.diff(co) >= 0).all()
    for j in range(int(g.sum())):
        assert h[co[j]] <= j < h[co[j] + 1]
    with pytest.raises(ValueError):
        oracle.offsets([1, -1])


def test_svd_slices_are_valid_svds():
    W = rng.normal(300, (12, 5, 3, 3), std=0.2).astype(np.float64)
    U, S, Vt = oracle.svd_slices(W)
    Wc = oracle.slices(W)
    assert Wc.shape == (5, 12, 9) and (Wc[2] == W[:, 2].reshape(12, 9)).all()
    for c in range(5):
        assert np.abs(U[c].T @ U[c] - np.eye(9)).max() < 1e-12
        assert np.abs(Vt[c] @ Vt[c].T - np.eye(9)).max() < 1e-12
        assert (np.diff(S[c]) <= 0).all() and (S[c] >= 0).all()
        assert np.abs((U[c] * S[c]) @ Vt[c] - Wc[c]).max() < 1e-12
        for i in range(9):                                  # sign convention
            assert Vt[c, i, np.argmax(np.abs(Vt[c, i]))] > 0
    # singular values are the square roots of the eigenvalues of the Gram matrix
    ev = np.sort(np.linalg.eigvalsh(Wc[0].T @ Wc[0]))[::-1]
    assert np.abs(np.sqrt(np.maximum(ev, 0)) - S[0]).max() < 1e-10


@pytest.mark.parametrize("seed", [310, 311, 312])
def test_truncation_error_is_the_discarded_singular_values(seed):
    """Lemma 3 with the Eckart-Young closed form: ||W - W_hat||_F^2 = sum_c sum_{i > g_c} sigma_{i,c}^2."""
    C, M = 6, 16
    W = rng.normal(seed, (M, C, 3, 3), std=0.1).astype(np.float64)
    g = rng.uniform_int(seed + 50, (C,), 0, 9)
    alpha = np.abs(rng.normal(seed + 60, (C,))).astype(np.float64) + 0.1
    D, Pw = oracle.truncated_factors(W, g)
    assert D.shape == (g.sum(), 3, 3) and Pw.shape == (M, g.sum())
    Wh = oracle.expand_weight(D, Pw, g)
    _, S, _ = oracle.svd_slices(W)
    assert abs(oracle.weight_error(W, Wh) - oracle.error_from_sigmas(S, g)) < 1e-12
    assert abs(oracle.weight_error(W, Wh, alpha) - oracle.error_from_sigmas(S, g, alpha)) < 1e-12
    assert abs(oracle.weight_error(W, Wh) ** 2 - np.sum((W - Wh) ** 2)) < 1e-12       # alpha = 1 is Frobenius
    # depthwise rows are unit vectors, singular values sit in the pointwise columns
    h = oracle.offsets(g)
    for c in range(C):
        for i in range(g[c]):
            assert abs(np.linalg.norm(D[h[c] + i]) - 1) < 1e-12
            assert abs(np.linalg.norm(Pw[:, h[c] + i]) - S[c, i]) < 1e-12
    # rank-g_c optimality spot check: no random rank-g_c matrix does better on any slice
    Wc, Whc = oracle.slices(W), oracle.slices(Wh)
    for c in range(C):
        best = np.sum((Wc[c] - Whc[c]) ** 2)
        for t in range(5 if g[c] > 0 else 0):
            A = rng.normal(seed + 100 + t, (M, g[c])).astype(np.float64)
            B = np.linalg.lstsq(A, Wc[c], rcond=None)[0]
            assert np.sum((Wc[c] - A @ B) ** 2) >= best - 1e-12


def test_rank_deficient_slices_get_zero_filters():
    W = np.zeros((8, 3, 2, 2))
    W[:, 0] = np.outer(np.arange(1, 9), [1, 2, 3, 4]).reshape(8, 2, 2)          # rank 1
    W[:, 2] = rng.normal(320, (8, 2, 2))                                          # rank 4; channel 1 is all zero
    g = np.array([3, 2, 4], np.int32)
    D, Pw = oracle.truncated_factors(W, g)
    assert np.abs(D[1:3]).max() == 0 and np.abs(Pw[:, 1:5]).max() == 0
    assert oracle.weight_error(W, oracle.expand_weight(D, Pw, g)) < 1e-12
    _, S, _ = oracle.svd_slices(W)
    assert [oracle.numerical_rank(S[c], 8) for c in range(3)] == [1, 0, 4]


def test_worked_example_from_the_paper():
    """Appendix B toy (3,2,4) convolution: g = [2,1,1], zero error, printed factors, 48 -> 32 MACs."""
    t = _read_toy()
    w1, w2, w3, w4 = t["w"]
    Wm = np.zeros((4, 12))
    Wm[0, 0], Wm[1, 4], Wm[2, 8], Wm[3, 2] = w1, w2, w3, w4
    W = Wm.reshape(4, 3, 2, 2)
    _, S, _ = oracle.svd_slices(W)
    g = oracle.lego(S, 0.0)                         # least-complex exact representation = the slice ranks
    assert g.tolist() == [int(v) for v in t["g"]]
    assert oracle.mego(S, 4).tolist() == g.tolist() and oracle.mego(S, 100).tolist() == g.tolist()
    D, Pw = oracle.truncated_factors(W, g)
    assert oracle.weight_error(W, oracle.expand_weight(D, Pw, g)) < 1e-14
    assert np.abs(Pw - np.array(t["pw"])).max() < 1e-14
    WD = np.zeros((4, 12))
    h = oracle.offsets(g)
    for c in range(3):
        for j in range(h[c], h[c + 1]):
            WD[j, 4 * c:4 * c + 4] = D[j].reshape(-1)
    assert np.abs(WD - np.array(t["gdw"])).max() < 1e-14
    assert oracle.macs_dense(3, 2, 4, 1, 1) == t["macs_dense"][0]
    assert oracle.macs_gdws(g, 2, 4, 1, 1) == t["macs_gdws"][0]
    assert np.count_nonzero(np.abs(Pw) > 1e-14) + np.count_nonzero(np.abs(WD) > 1e-14) == t["nonzeros"][0]
    x = rng.normal(330, (1, 3, 4, 4)).astype(np.float64)
    y, macs = oracle.gdws_forward(x, g, D, Pw, return_macs=True)
    assert np.abs(y - oracle.conv_dense(x, W)).max() < 1e-14
    assert macs == 9 * 32


def test_worked_example_through_the_sparse_aware_reduction():
    """Appendix B from the other side: start from the exact g_c = K^2 = 4 of Lemma 1 on the pruned toy weight and
    let the reduction drop the dead channels: what is left is the printed g = [2,1,1] with the printed factors."""
    t = _read_toy()
    w1, w2, w3, w4 = t["w"]
    Wm = np.zeros((4, 12))
    Wm[0, 0], Wm[1, 4], Wm[2, 8], Wm[3, 2] = w1, w2, w3, w4
    W = Wm.reshape(4, 3, 2, 2)
    assert oracle.sparse_g(W).tolist() == [int(v) for v in t["g"]]
    g_full = np.full(3, 4, np.int32)
    D, Pw = oracle.truncated_factors(W, g_full)
    assert oracle.macs_gdws(g_full, 2, 4, 1, 1) == 4 * 12 + 12 * 4            # exact but dearer than the dense 48
    g2, D2, Pw2, keep = oracle.compact_factors(g_full, D, Pw)
    assert g2.tolist() == [int(v) for v in t["g"]] and keep.tolist() == [0, 1, 4, 8]
    assert np.abs(Pw2 - np.array(t["pw"])).max() < 1e-14
    assert np.abs(D2.reshape(4, 4) - np.array(t["gdw"]).reshape(4, 3, 4)[np.arange(4), [0, 0, 1, 2]]).max() < 1e-14
    assert oracle.weight_error(W, oracle.expand_weight(D2, Pw2, g2)) < 1e-14
    assert oracle.macs_gdws(g2, 2, 4, 1, 1) == t["macs_gdws"][0]
    assert np.count_nonzero(Pw2) + np.count_nonzero(D2) == t["nonzeros"][0]


@pytest.mark.parametrize("seed,M,C,K,keep", [(370, 16, 12, 3, 0.05), (371, 64, 24, 3, 0.02), (372, 8, 6, 2, 0.15)])
def test_sparse_aware_reduction_on_pruned_weights(seed, M, C, K, keep):
    """Pruned W: g_c = rank(W_c) is exact (Lemma 1); dropping dead channels changes neither the product W_P W_D nor
    the output, only the MAC count; rank(W_c) is bounded by the slice's non-zero rows and columns."""
    W = workloads.pruned_weight(seed, M, C, K, keep).astype(np.float64)
    Wc = oracle.slices(W)
    r = oracle.sparse_g(W)
    for c in range(C):
        assert r[c] == np.linalg.matrix_rank(Wc[c])
        assert r[c] <= min(np.count_nonzero(np.abs(Wc[c]).sum(0)), np.count_nonzero(np.abs(Wc[c]).sum(1)))
    assert r.sum() < C * min(M, K * K)                       # the pruning did lower some ranks
    _, S, _ = oracle.svd_slices(W)
    assert (oracle.lego(S, 0.0, dim=max(M, K * K)) == r).all()
    g_full = np.full(C, min(M, K * K), np.int32)
    D, Pw = oracle.truncated_factors(W, g_full)
    g2, D2, Pw2, keep_idx = oracle.compact_factors(g_full, D, Pw)
    assert (g2 == r).all() and len(keep_idx) == r.sum()
    h = oracle.offsets(g_full)
    for q, j in enumerate(keep_idx):                         # kept channels are the leading ones of each slice
        c = oracle.chan_of(g_full)[j]
        assert j - h[c] < r[c]
    assert oracle.weight_error(W, oracle.expand_weight(D2, Pw2, g2)) < 1e-12
    x = rng.normal(seed + 5, (2, C, 6, 5)).astype(np.float64)
    y_full, m_full = oracle.gdws_forward(x, g_full, D, Pw, stride=1, pad=1, return_macs=True)
    y_red, m_red = oracle.gdws_forward(x, g2, D2, Pw2, stride=1, pad=1, return_macs=True)
    assert np.abs(y_full - y_red).max() < 1e-13 and m_red < m_full
    assert m_red == oracle.macs_gdws(g2, K, M, 6 + 2 - K + 1, 5 + 2 - K + 1) * 2
    assert np.abs(y_red - oracle.conv_dense(x, W, stride=1, pad=1)).max() < 1e-12
    # a zero pointwise column is dead as well, and zeros elsewhere are not
    Pw3 = Pw2.copy()
    Pw3[:, 0] = 0.0
    g3, _, _, k3 = oracle.compact_factors(g2, D2, Pw3)
    assert g3.sum() == g2.sum() - 1 and 0 not in k3


def _all_g(ranks):
    return itertools.product(*[range(r + 1) for r in ranks])


@pytest.mark.parametrize("seed", [340, 341, 342, 343])
def test_mego_is_optimal_by_brute_force(seed):
    """Theorem 1: Algorithm 1 minimises e subject to sum(g) <= gamma, for any positive alpha."""
    W = rng.normal(seed, (5, 3, 2, 2)).astype(np.float64)
    alpha = np.abs(rng.normal(seed + 1, (3,))).astype(np.float64) + 0.05
    _, S, _ = oracle.svd_slices(W)
    prev = None
    for gamma in range(0, 14):
        g = oracle.mego(S, gamma, alpha)
        assert g.sum() == min(gamma, 12)
        e = oracle.error_from_sigmas(S, g, alpha)
        best = min(oracle.error_from_sigmas(S, q, alpha) for q in _all_g([4, 4, 4]) if sum(q) <= gamma)
        assert abs(e - best) < 1e-12
        if prev is not None:                        # proof of Theorem 1: one more unit changes one entry
            assert np.abs(g - prev).sum() <= 1 and e <= prev_e + 1e-15
        prev, prev_e = g, e


@pytest.mark.parametrize("seed", [350, 351, 352])
def test_lego_is_optimal_by_brute_force(seed):
    """Theorem 2: Algorithm 2 minimises sum(g) subject to e <= beta."""
    W = rng.normal(seed, (5, 3, 2, 2)).astype(np.float64)
    alpha = np.abs(rng.normal(seed + 1, (3,))).astype(np.float64) + 0.05
    _, S, _ = oracle.svd_slices(W)
    emax = oracle.error_from_sigmas(S, [0, 0, 0], alpha)
    for beta in np.linspace(0, emax * 1.1, 23):
        g = oracle.lego(S, beta, alpha)
        assert oracle.error_from_sigmas(S, g, alpha) <= beta + 1e-12
        best = min(sum(q) for q in _all_g([4, 4, 4]) if oracle.error_from_sigmas(S, q, alpha) <= beta + 1e-12)
        assert g.sum() == best
    assert oracle.lego(S, 0.0, alpha).tolist() == [4, 4, 4]
    assert oracle.lego(S, emax * 1.0001, alpha).tolist() == [0, 0, 0]
    assert oracle.lego(S, emax * 1.0001, alpha, g_min=1).tolist() == [1, 1, 1]


def test_mego_with_floor_and_cap_and_budget():
    """The benchmark recipe: start every channel at 1, cap at K^2, fill up to the MAC budget."""
    W = rng.normal(360, (32, 8, 3, 3), std=0.05).astype(np.float64)
    _, S, _ = oracle.svd_slices(W)
    gam = oracle.gamma_from_budget(0.25, 8, 3, 32)
    assert gam * (9 + 32) <= 0.25 * 8 * 9 * 32 < (gam + 1) * (9 + 32)
    g = oracle.mego(S, gam, g_init=np.ones(8, np.int32), cap=9)
    assert g.sum() == gam and g.min() >= 1 and g.max() <= 9
    # with a floor the greedy still picks, at every step, the largest remaining sigma^2
    taken = sorted((S[c, i] ** 2 for c in range(8) for i in range(1, g[c])), reverse=True)
    left = max(S[c, g[c]] ** 2 for c in range(8) if g[c] < 9)
    assert not taken or taken[-1] >= left
    # eq. 3 against eq. 2 by brute force: the largest G whose MACs fit, then the clamp to [C, min(K^2, M) C]
    for rho, C, K, M in [(0.25, 128, 3, 128), (0.4, 64, 3, 64), (0.4, 3, 3, 64), (0.4, 512, 3, 512), (1.0, 4, 3, 16)]:
        fits = max(G for G in range(0, 9 * C + 2) if G * (K * K + M) <= rho * C * K * K * M)
        assert oracle.gamma_from_budget(rho, C, K, M) == max(C, min(min(K * K, M) * C, fits))
    assert oracle.gamma_from_budget(0.25, 128, 3, 128) == 269
    assert oracle.gamma_from_budget(1.0, 4, 3, 16) == 23 and oracle.gamma_from_budget(5.0, 4, 3, 16) == 36
