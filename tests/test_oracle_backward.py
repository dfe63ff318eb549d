"""Pins of the oracle's backward pass (CPU only).

The gradients are the adjoints of the two linear operators of Section 3.1, so they are pinned by
(1) a library routine: torch.autograd through the layer written as channel duplication + grouped
convolution + 1 x 1 convolution (the mapping of Appendix A) in float64; (2) the adjoint identity
<dy, F(x)> = <F*(dy), x>; (3) exact finite differences (the loss is linear in each argument);
(4) hand cases.  A dropped term, a transposed weight, a wrong stride or padding offset fails one of them.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from workloads import rng

CASES = [
    # N, C, H, W, M, K, stride, pad, g
    (2, 3, 6, 7, 4, 3, 1, 1, [2, 1, 3]),
    (1, 4, 9, 8, 5, 3, 2, 1, [1, 0, 2, 4]),       # stride 2, a channel without filters
    (2, 2, 7, 7, 3, 5, 1, 2, [3, 2]),             # K = 5
    (1, 3, 8, 9, 2, 3, 2, 0, [1, 1, 1]),          # no padding, stride 2 (last rows/columns unused)
    (2, 5, 4, 4, 6, 1, 1, 0, [1, 2, 1, 1, 2]),    # K = 1
]


def _tensors(case, seed):
    N, C, H, W, M, K, s, p, g = case
    g = np.array(g, np.int32)
    G = int(g.sum())
    Ho, Wo = (H + 2 * p - K) // s + 1, (W + 2 * p - K) // s + 1
    x = rng.normal(seed, (N, C, H, W)).astype(np.float64)
    D = rng.normal(seed + 1, (G, K, K), std=0.5).astype(np.float64)
    Pw = rng.normal(seed + 2, (M, G), std=0.5).astype(np.float64)
    dy = rng.normal(seed + 3, (N, M, Ho, Wo)).astype(np.float64)
    return x, g, D, Pw, dy


@pytest.mark.parametrize("case", range(len(CASES)))
def test_against_autograd(case):
    N, C, H, W, M, K, s, p, _ = CASES[case]
    x, g, D, Pw, dy = _tensors(CASES[case], 7000 + 10 * case)
    G = int(g.sum())
    xt = torch.tensor(x, requires_grad=True)
    Dt = torch.tensor(D, requires_grad=True)
    Pt = torch.tensor(Pw, requires_grad=True)
    bt = torch.zeros(M, dtype=torch.float64, requires_grad=True)
    idx = torch.tensor(np.repeat(np.arange(C), g))
    t = F.conv2d(xt.index_select(1, idx), Dt.reshape(G, 1, K, K), stride=s, padding=p, groups=G)
    y = F.conv2d(t, Pt.reshape(M, G, 1, 1), bias=bt)
    (y * torch.tensor(dy)).sum().backward()
    dx, dD, dPw, db = oracle.gdws_backward(x, g, D, Pw, dy, s, p)
    for ours, ref in ((dx, xt.grad), (dD, Dt.grad), (dPw, Pt.grad), (db, bt.grad)):
        ref = ref.numpy()
        assert ours.shape == ref.shape
        assert np.max(np.abs(ours - ref)) <= 1e-11 * max(1.0, np.max(np.abs(ref)))


@pytest.mark.parametrize("case", range(len(CASES)))
def test_adjoint_identity_and_finite_differences(case):
    N, C, H, W, M, K, s, p, _ = CASES[case]
    x, g, D, Pw, dy = _tensors(CASES[case], 7100 + 10 * case)
    dx, dD, dPw, db = oracle.gdws_backward(x, g, D, Pw, dy, s, p)
    L = lambda x_, D_, P_, b_=None: float((oracle.gdws_forward(x_, g, D_, P_, b_, stride=s, pad=p) * dy).sum())
    L0 = L(x, D, Pw)
    assert abs(L0 - float((dx * x).sum())) <= 1e-10 * max(1.0, abs(L0))      # <dy, F(x)> = <F*(dy), x>
    # L is linear in x, in D and in Pw separately, so a finite difference of any size is exact up to rounding
    for k in range(4):
        i = tuple(int(rng.uniform_int(7200 + 10 * case + k, (1,), 0, n - 1)[0]) for n in D.shape)
        D2 = D.copy(); D2[i] += 0.75
        assert abs((L(x, D2, Pw) - L0) / 0.75 - dD[i]) <= 1e-9 * max(1.0, abs(dD[i]))
        i = tuple(int(rng.uniform_int(7300 + 10 * case + k, (1,), 0, n - 1)[0]) for n in Pw.shape)
        P2 = Pw.copy(); P2[i] -= 1.5
        assert abs((L(x, D, P2) - L0) / -1.5 - dPw[i]) <= 1e-9 * max(1.0, abs(dPw[i]))
        i = tuple(int(rng.uniform_int(7400 + 10 * case + k, (1,), 0, n - 1)[0]) for n in x.shape)
        x2 = x.copy(); x2[i] += 2.0
        assert abs((L(x2, D, Pw) - L0) / 2.0 - dx[i]) <= 1e-9 * max(1.0, abs(dx[i]))
    b = np.zeros(M); b[M - 1] = 1.0
    assert abs(L(x, D, Pw, b) - L0 - db[M - 1]) <= 1e-9 * max(1.0, abs(db[M - 1]))


def test_hand_case_single_tap():
    """One channel, one 3 x 3 filter with a single non-zero tap at (0, 2), pad 1: T[y, x] = 2 X[y - 1, x + 1];
    dx is dT shifted back, dD picks the matching correlation."""
    x = np.arange(16, dtype=np.float64).reshape(1, 1, 4, 4)
    D = np.zeros((1, 3, 3)); D[0, 0, 2] = 2.0
    Pw = np.array([[3.0]])
    dy = np.zeros((1, 1, 4, 4)); dy[0, 0, 2, 1] = 1.0
    dx, dD, dPw, db = oracle.gdws_backward(x, np.array([1], np.int32), D, Pw, dy, 1, 1)
    ref_dx = np.zeros((1, 1, 4, 4)); ref_dx[0, 0, 1, 2] = 6.0           # Y[2,1] = 3 * 2 * X[1,2]
    assert (dx == ref_dx).all()
    assert dPw[0, 0] == 2.0 * x[0, 0, 1, 2] and db[0] == 1.0
    ref_dD = np.zeros((3, 3))
    for u in range(3):
        for v in range(3):
            yy, xx = 2 + u - 1, 1 + v - 1
            ref_dD[u, v] = 3.0 * x[0, 0, yy, xx] if 0 <= yy < 4 and 0 <= xx < 4 else 0.0
    assert (dD[0] == ref_dD).all()


def test_zero_multiplier_channel_gets_no_gradient():
    x, g, D, Pw, dy = _tensors(CASES[1], 7500)
    dx = oracle.gdws_backward(x, g, D, Pw, dy, 2, 1)[0]
    assert (dx[:, 1] == 0).all() and np.abs(dx[:, 0]).max() > 0
