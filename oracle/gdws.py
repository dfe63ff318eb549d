"""CPU oracle: GDWS construction (numpy, float64) and forward pass (plain C loops, float64).

TEST INFRASTRUCTURE ONLY -- never imported by the product package.

Every function names the passage of the paper it follows.  Where the paper is
silent the reading taken is stated in the docstring.  Tensors use the paper's
C x H x W order with a leading batch axis; weights are [M, C, K, K]; the K^2
entries of one channel of one filter are vectorised row-major (u*K + v).

Parity status: every function here is pinned by tests/test_oracle_*.py against
closed forms, identities, brute force, a library routine or the paper's worked example, except the
choice between the two readings of the error-constrained greedy's stopping rule
(`lego(..., compare=...)`): the default follows the theorem and its proof and is
pinned by brute force; the literal algorithm-box variant is "parity unpinned".
"""
import ctypes
import os
import subprocess

import numpy as np

from workloads.storage import from_storage, to_storage

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gdws_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force=False):
    """Compile the C loops with gcc (-O2, OpenMP for the optional multi-thread timing)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


def _c():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        dp, ip, i, i64 = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        L.oracle_conv_dense.restype = i64
        L.oracle_conv_dense.argtypes = [dp, dp, dp, dp, i, i, i, i, i, i, i, i, i]
        L.oracle_gdw.restype = i64
        L.oracle_gdw.argtypes = [dp, ip, dp, dp, i, i, i, i, i, i, i, i]
        L.oracle_pw.restype = i64
        L.oracle_pw.argtypes = [dp, dp, dp, dp, i, i, i, i, i]
        L.oracle_duplicate_channels.restype = None
        L.oracle_duplicate_channels.argtypes = [dp, ip, dp, i, i, i]
        L.oracle_add_relu.restype = None
        L.oracle_add_relu.argtypes = [dp, dp, ctypes.c_size_t, i]
        L.oracle_maxpool.restype = None
        L.oracle_maxpool.argtypes = [dp, dp, i, i, i, i, i, i, i]
        L.oracle_max_threads.restype = i
        _lib = L
    return _lib


def max_threads():
    return int(_c().oracle_max_threads())


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


# ----------------------------------------------------------------------------
# index tables  (Property 2; proof of Lemma 1, definition of h_c)
# ----------------------------------------------------------------------------

def offsets(g):
    """h[c] = g[0] + ... + g[c-1] for c = 0..C (zero-based form of the paper's h_c); h[C] = G."""
    g = np.asarray(g)
    h = np.zeros(len(g) + 1, dtype=np.int32)
    for c in range(len(g)):
        if g[c] < 0:
            raise ValueError("g must be non-negative")
        h[c + 1] = h[c] + int(g[c])
    return h


def chan_of(g):
    """For each intermediate channel j, the input channel it is computed from.

    This is the index vector that duplicates channel c g[c] times (Appendix A,
    "Mapping GDWS Convolutions").
    """
    out = []
    for c, gc in enumerate(np.asarray(g)):
        out.extend([c] * int(gc))
    return np.asarray(out, dtype=np.int32)


# ----------------------------------------------------------------------------
# construction  (Section 3.2 Lemma 1; Section 3.3 Algorithms 1 and 2; Appendix C Lemma 3)
# ----------------------------------------------------------------------------

def slices(W):
    """[C, M, K^2]: the sub-matrices W_c of W = [W_1 | ... | W_C] (Section 3 "2D Convolution as Matrix Multiplication")."""
    W = _f64(W)
    M, C, K, _ = W.shape
    return np.ascontiguousarray(W.reshape(M, C, K * K).transpose(1, 0, 2))


def numerical_rank(s, dim=None):
    """Number of singular values above dim * eps * s[0]; dim = max(M, K^2), or len(s) if not given.

    The paper only says "rank r_c"; this is the usual floating-point reading.
    """
    s = np.asarray(s, dtype=np.float64)
    if s.size == 0 or s[0] == 0.0:
        return 0
    dim = len(s) if dim is None else dim
    return int(np.sum(s > s[0] * np.finfo(np.float64).eps * dim))


def svd_slices(W):
    """Per-channel SVD W_c = sum_i sigma_i u_i v_i^T, sigma descending (Algorithm 1, first step).

    Returns U [C, M, R], S [C, R], Vt [C, R, K^2] with R = min(M, K^2).  Each
    (u_i, v_i) pair has its sign fixed so that the largest-magnitude entry of
    v_i (lowest index on ties) is positive -- the paper does not discuss the
    sign freedom; the product is unaffected.
    """
    Wc = slices(W)
    U, S, Vt = np.linalg.svd(Wc, full_matrices=False)
    for c in range(Wc.shape[0]):
        for i in range(S.shape[1]):
            k = int(np.argmax(np.abs(Vt[c, i])))
            if Vt[c, i, k] < 0:
                Vt[c, i] = -Vt[c, i]
                U[c, :, i] = -U[c, :, i]
    return U, S, Vt


def truncated_factors(W, g):
    """Depthwise filters D [G, K, K] and pointwise matrix Pw [M, G] of the rank-g_c truncated SVDs.

    Lemma 3 (optimal fixed-g approximation) with the split of Property 1 and the
    row placement of Property 2: for i < g_c, row h_c + i of W_D holds v_i^T and
    column h_c + i of W_P holds sigma_i u_i (the singular value goes to the
    pointwise side, as in the worked example of Appendix B where the unit
    vectors sit in the depthwise matrix).  Filters beyond the numerical rank of
    W_c are zero (proof of Lemma 3, the g_c > r_c remark).
    """
    W = _f64(W)
    M, C, K, _ = W.shape
    h = offsets(g)
    G = int(h[-1])
    U, S, Vt = svd_slices(W)
    D = np.zeros((G, K, K))
    Pw = np.zeros((M, G))
    for c in range(C):
        r = numerical_rank(S[c], max(M, K * K))
        for i in range(int(g[c])):
            if i < r:
                D[h[c] + i] = Vt[c, i].reshape(K, K)
                Pw[:, h[c] + i] = S[c, i] * U[c, :, i]
    return D, Pw


def expand_weight(D, Pw, g):
    """The equivalent standard weight W = W_P W_D as [M, C, K, K] (Property 1 with the block structure of Property 2)."""
    D, Pw = _f64(D), _f64(Pw)
    G, K, _ = D.shape
    C = len(g)
    h = offsets(g)
    WD = np.zeros((G, C * K * K))
    for c in range(C):
        for j in range(h[c], h[c + 1]):
            WD[j, c * K * K:(c + 1) * K * K] = D[j].reshape(-1)
    return (Pw @ WD).reshape(Pw.shape[0], C, K, K)


def weight_error(W, Q, alpha=None):
    """e(W, Q, alpha) = sqrt(sum_c alpha_c ||W_c - Q_c||_F^2)  (eq. 4)."""
    Wc, Qc = slices(W), slices(Q)
    C = Wc.shape[0]
    a = np.ones(C) if alpha is None else _f64(alpha)
    return float(np.sqrt(sum(a[c] * np.sum((Wc[c] - Qc[c]) ** 2) for c in range(C))))


def error_from_sigmas(S, g, alpha=None):
    """e(g) = sqrt(sum_c alpha_c sum_{i > g_c} sigma_{i,c}^2)  (closed form in the proofs of Lemma 3 / Theorem 2)."""
    S = _f64(S)
    a = np.ones(S.shape[0]) if alpha is None else _f64(alpha)
    return float(np.sqrt(sum(a[c] * np.sum(S[c, int(g[c]):] ** 2) for c in range(S.shape[0]))))


def mego(S, gamma, alpha=None, g_init=None, cap=None, dim=None):
    """Algorithm 1 (MEGO): greedy g minimising the weighted error subject to sum(g) <= gamma.

    S [C, R] singular values per channel (descending).  Starting from g_init
    (all zeros in the paper), repeatedly give one more filter to the channel
    with the largest alpha_c * sigma_{g_c+1,c}^2 among channels that are not
    saturated (g_c < r_c, and g_c < cap if a cap is given).  Ties go to the lowest
    channel index; the loop stops early once every channel is saturated (proof
    of Theorem 1, last remark of the induction step).
    """
    S = _f64(S)
    C, R = S.shape
    a = np.ones(C) if alpha is None else _f64(alpha)
    r = np.array([numerical_rank(S[c], dim) for c in range(C)])
    lim = r if cap is None else np.minimum(r, cap)
    g = np.zeros(C, dtype=np.int32) if g_init is None else np.array(g_init, dtype=np.int32)
    while int(g.sum()) < gamma:
        best, best_gain = -1, -1.0
        for c in range(C):
            if g[c] < lim[c]:
                gain = a[c] * S[c, g[c]] ** 2
                if gain > best_gain:
                    best, best_gain = c, gain
        if best < 0:
            break
        g[best] += 1
    return g


def lego(S, beta, alpha=None, compare="beta_squared", g_min=0, dim=None):
    """Algorithm 2 (LEGO): least-complex g with e(g) <= beta.

    Start from g = r and keep dropping the filter with the smallest
    alpha_c * sigma_{g_c,c}^2 while the accumulated squared error stays within
    the bound.  compare="beta_squared" (default) is the reading of Theorem 2
    and its proof: stop when adding the next term would make the sum exceed
    beta^2.  compare="beta" is the algorithm box taken literally (accumulated
    squared terms compared with beta itself, strict inequality).  Ties go to the
    lowest channel index.  Channels are never reduced below g_min.
    """
    S = _f64(S)
    C, R = S.shape
    a = np.ones(C) if alpha is None else _f64(alpha)
    g = np.array([numerical_rank(S[c], dim) for c in range(C)], dtype=np.int32)
    b = 0.0
    while True:
        best, h = -1, np.inf
        for c in range(C):
            if g[c] > g_min:
                term = a[c] * S[c, g[c] - 1] ** 2
                if term < h:
                    best, h = c, term
        if best < 0:
            break
        ok = (b + h <= beta * beta) if compare == "beta_squared" else (b + h < beta)
        if not ok:
            break
        b += h
        g[best] -= 1
    return g


def sparse_g(W):
    """g_c = rank(W_c): the smallest g whose GDWS convolution reproduces a (pruned) W with no error.

    Appendix B: very sparse weight matrices have low-rank sub-matrices W_c, and by Lemma 1 a
    GDWS convolution with g_c = rank(W_c) is exact.
    """
    _, S, _ = svd_slices(W)
    M, _, K, _ = np.shape(W)
    return np.array([numerical_rank(S[c], max(M, K * K)) for c in range(S.shape[0])], dtype=np.int32)


def compact_factors(g, D, Pw):
    """Drop the intermediate channels that cannot contribute (Appendix B: the factors of a pruned W are sparse too).

    Channel j is dead if its depthwise filter D[j] is all zero (its map is zero) or its pointwise
    column Pw[:, j] is all zero (its map is never read).  Returns (g', D', Pw', keep) with keep[q] the
    index in the original of kept channel q; g'_c counts the kept channels of input channel c.
    """
    D, Pw = _f64(D), _f64(Pw)
    h = offsets(g)
    keep, g2 = [], np.zeros(len(g), dtype=np.int32)
    for c in range(len(g)):
        for j in range(h[c], h[c + 1]):
            if np.any(D[j] != 0.0) and np.any(Pw[:, j] != 0.0):
                keep.append(j)
                g2[c] += 1
    keep = np.asarray(keep, dtype=np.int32)
    return g2, D[keep], Pw[:, keep], keep


def gamma_from_budget(rho, C, K, M):
    """Largest G with G (K^2 + M) <= rho * C K^2 M (eq. 3 against eq. 2), kept within [C, min(K^2, M) C]."""
    gam = int(np.floor(rho * C * K * K * M / (K * K + M) + 1e-9))
    return max(C, min(min(K * K, M) * C, gam))


def macs_dense(C, K, M, Ho, Wo):
    """eq. 2."""
    return Ho * Wo * M * C * K * K


def macs_gdws(g, K, M, Ho, Wo):
    """eq. 3."""
    return Ho * Wo * int(np.sum(g)) * (K * K + M)


# ----------------------------------------------------------------------------
# forward pass (C loops)
# ----------------------------------------------------------------------------

def _osz(n, K, s, p):
    return (n + 2 * p - K) // s + 1


def conv_dense(x, W, bias=None, stride=1, pad=0, threads=1, return_macs=False):
    """Standard (C,K,M) convolution, eq. 1.  x [N,C,H,W], W [M,C,K,K] -> [N,M,H',W']."""
    x, W = _f64(x), _f64(W)
    N, C, H, Wd = x.shape
    M, C2, K, _ = W.shape
    assert C == C2
    b = None if bias is None else _f64(bias)
    y = np.empty((N, M, _osz(H, K, stride, pad), _osz(Wd, K, stride, pad)))
    macs = _c().oracle_conv_dense(_ptr(x), _ptr(W), _ptr(b), _ptr(y), N, C, H, Wd, M, K, stride, pad, max(1, threads))
    return (y, macs) if return_macs else y


def gdw(x, g, D, stride=1, pad=0, threads=1, return_macs=False):
    """Generalized depthwise convolution (Section 3.1 Definition).  x [N,C,H,W], D [G,K,K] -> [N,G,H',W']."""
    x, D = _f64(x), _f64(D)
    g = np.ascontiguousarray(g, dtype=np.int32)
    N, C, H, Wd = x.shape
    G, K, _ = D.shape
    assert len(g) == C and int(g.sum()) == G and (g >= 0).all()
    t = np.empty((N, G, _osz(H, K, stride, pad), _osz(Wd, K, stride, pad)))
    macs = _c().oracle_gdw(_ptr(x), _ptr(g), _ptr(D), _ptr(t), N, C, H, Wd, K, stride, pad, max(1, threads))
    return (t, macs) if return_macs else t


def pw(t, Pw, bias=None, threads=1, return_macs=False):
    """Pointwise (G,1,M) convolution (Section 3.1 Definition).  t [N,G,H,W], Pw [M,G] -> [N,M,H,W]."""
    t, Pw = _f64(t), _f64(Pw)
    N, G, H, Wd = t.shape
    M, G2 = Pw.shape
    assert G == G2
    b = None if bias is None else _f64(bias)
    y = np.empty((N, M, H, Wd))
    macs = _c().oracle_pw(_ptr(t), _ptr(Pw), _ptr(b), _ptr(y), N, G, H * Wd, M, max(1, threads))
    return (y, macs) if return_macs else y


def duplicate_channels(x, g):
    """X' of Appendix A: channel c repeated g[c] times."""
    x = _f64(x)
    g = np.ascontiguousarray(g, dtype=np.int32)
    N, C, H, Wd = x.shape
    xd = np.empty((N, int(g.sum()), H, Wd))
    _c().oracle_duplicate_channels(_ptr(x), _ptr(g), _ptr(xd), N, C, H * Wd)
    return xd


def add_relu(y, residual=None, relu=True):
    y = _f64(y).copy()
    r = None if residual is None else _f64(residual)
    _c().oracle_add_relu(_ptr(y), _ptr(r), y.size, int(bool(relu)))
    return y


def maxpool(x, k=2, s=2, pad=0):
    x = _f64(x)
    N, C, H, Wd = x.shape
    y = np.empty((N, C, _osz(H, k, s, pad), _osz(Wd, k, s, pad)))
    _c().oracle_maxpool(_ptr(x), _ptr(y), N, C, H, Wd, k, s, pad)
    return y


def round_to(x, dtype):
    """Values of x after a round trip through the storage type (f32 / f16 / bf16, round to nearest even)."""
    x = np.asarray(x)
    return from_storage(to_storage(x.astype(np.float32), dtype), dtype).reshape(x.shape)


def gdws_forward(x, g, D, Pw, bias=None, residual=None, relu=False, stride=1, pad=0,
                 round_intermediate=None, threads=1, return_macs=False):
    """(C,K,g,M) GDWS convolution: GDW then PW, then the optional bias / residual add / ReLU.

    round_intermediate: None keeps the G-channel intermediate in double; "f16" /
    "bf16" rounds it to that storage type first (what a 16-bit matrix-core path
    does), to separate rounding from logic errors.
    """
    t, m1 = gdw(x, g, D, stride, pad, threads, True)
    if round_intermediate:
        t = round_to(t, round_intermediate)
    y, m2 = pw(t, Pw, bias, threads, True)
    if residual is not None or relu:
        y = add_relu(y, residual, relu)
    return (y, m1 + m2) if return_macs else y


def gdws_backward(x, g, D, Pw, dy, stride=1, pad=0, threads=1):
    """Gradients of L through the linear map Y = PW(GDW(X)) + bias, given dy = dL/dY (what fine-tuning a GDWS
    network needs, Section 4's fine-tuning ablation; the paper prints no formulas: these are the adjoints of the
    two operators of Section 3.1, written out).

    x [N,C,H,W], D [G,K,K], Pw [M,G], dy [N,M,H',W'].  Returns (dx [N,C,H,W], dD [G,K,K], dPw [M,G], dbias [M]):
      T          = GDW(x)                                        (recomputed)
      dbias[m]   = sum_{n,p} dy[n,m,p]
      dPw[m,j]   = sum_{n,p} dy[n,m,p] T[n,j,p]
      dT[n,j,p]  = sum_m Pw[m,j] dy[n,m,p]
      dD[j,u,v]  = sum_{n,y,x} dT[n,j,y,x] X[n,chan_of[j], y s + u - pad, x s + v - pad]     (zero outside)
      dx[n,c,.]  = sum_{j in channel c} sum_{u,v} D[j,u,v] dT[n,j,y,x] scattered to (y s + u - pad, x s + v - pad)
    A ReLU or a residual add after the layer is the caller's: dy is the gradient at the layer's linear output.
    """
    x, D, Pw, dy = _f64(x), _f64(D), _f64(Pw), _f64(dy)
    g = np.ascontiguousarray(g, dtype=np.int32)
    N, C, H, Wd = x.shape
    G, K, _ = D.shape
    M = Pw.shape[0]
    Ho, Wo = _osz(H, K, stride, pad), _osz(Wd, K, stride, pad)
    assert dy.shape == (N, M, Ho, Wo) and Pw.shape == (M, G)
    T = gdw(x, g, D, stride, pad, threads)
    dbias = dy.sum(axis=(0, 2, 3))
    dPw = np.zeros((M, G))
    for m in range(M):
        dPw[m] = (dy[:, m][:, None] * T).sum(axis=(0, 2, 3))
    dT = np.zeros((N, G, Ho, Wo))
    for j in range(G):
        for m in range(M):
            dT[:, j] += Pw[m, j] * dy[:, m]
    xp = np.zeros((N, C, H + 2 * pad, Wd + 2 * pad))
    xp[:, :, pad:pad + H, pad:pad + Wd] = x
    dxp = np.zeros_like(xp)
    ch = chan_of(g)
    dD = np.zeros((G, K, K))
    for j in range(G):
        c = int(ch[j])
        for u in range(K):
            for v in range(K):
                # input positions (y s + u, x s + v) of the padded image, for all output positions (y, x)
                window = (slice(None), c, slice(u, u + (Ho - 1) * stride + 1, stride), slice(v, v + (Wo - 1) * stride + 1, stride))
                dD[j, u, v] = (dT[:, j] * xp[window]).sum()
                dxp[window] += D[j, u, v] * dT[:, j]
    return dxp[:, :, pad:pad + H, pad:pad + Wd].copy(), dD, dPw, dbias


def network_forward(layers, params, x, store=None, round_intermediate=None, threads=1, keep=False):
    """Run a feed-forward graph of `workloads.LayerShape` nodes.

    params[i] is a dict for layer i: {"g","D","Pw","bias"} for "gdws",
    {"W","bias"} for "dense", nothing for "maxpool".  `store` (None / "f16" /
    "bf16") rounds every layer output to the storage type, as a network whose
    activations live in 16-bit memory does.  Returns the last output (or all).
    """
    outs = []
    for i, l in enumerate(layers):
        src = _f64(x) if l.src < 0 else outs[l.src]
        res = None if l.residual is None else outs[l.residual]
        p = params[i]
        if l.kind == "gdws":
            y = gdws_forward(src, p["g"], p["D"], p["Pw"], p.get("bias"), res, l.relu, l.stride, l.pad,
                             round_intermediate, threads)
        elif l.kind == "dense":
            y = conv_dense(src, p["W"], p.get("bias"), l.stride, l.pad, threads)
            if res is not None or l.relu:
                y = add_relu(y, res, l.relu)
        elif l.kind == "maxpool":
            y = maxpool(src, l.K, l.stride, l.pad)
        else:
            raise ValueError(l.kind)
        if store:
            y = round_to(y, store)
        outs.append(y)
    return outs if keep else outs[-1]
