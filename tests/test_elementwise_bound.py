"""The element-wise parity bound of the GPU tests, exercised on the CPU: a float32 emulation of the kernels'
arithmetic (fp32 sums, intermediate and output rounded to the storage type) must lie inside it, and a single wrong
input pixel, tap or weight must fall outside it somewhere."""
import numpy as np
import pytest

import oracle
import workloads
from workloads import rng

from gpu_util import assert_elementwise, elementwise_bound, elementwise_bound_f32, quantise


def _emulate(x, g, dw, pw, bias, residual, relu, pad, dtype, order):
    """fp32 arithmetic in a given summation order; 16-bit: T and y rounded to the storage type."""
    N, C, H, W = x.shape
    co = oracle.chan_of(g)
    G, M = len(co), pw.shape[0]
    xp = np.zeros((N, C, H + 2 * pad, W + 2 * pad), np.float32)
    xp[:, :, pad:pad + H, pad:pad + W] = x
    Ho, Wo = H + 2 * pad - 2, W + 2 * pad - 2
    t = np.zeros((N, G, Ho, Wo), np.float32)
    taps = [(u, v) for u in range(3) for v in range(3)]
    for u, v in (taps if order == 0 else taps[::-1]):
        t += dw[:, u, v].astype(np.float32)[None, :, None, None] * xp[:, co, u:u + Ho, v:v + Wo]
    if dtype != "f32":
        t = oracle.round_to(t, dtype).astype(np.float32)
    y = np.zeros((N, M, Ho, Wo), np.float32)
    js = range(G) if order == 0 else range(G - 1, -1, -1)
    for j in js:
        y += pw[:, j].astype(np.float32)[None, :, None, None] * t[:, j][:, None]
    if bias is not None:
        y += bias.astype(np.float32)[None, :, None, None]
    if residual is not None:
        y += residual.astype(np.float32)
    if relu:
        y = np.maximum(y, 0)
    return oracle.round_to(y, dtype) if dtype != "f32" else y.astype(np.float64)


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("seed,C,M,relu,res", [(950, 24, 40, True, False), (951, 64, 16, False, True)])
def test_bound_holds_for_fp32_arithmetic_and_catches_single_errors(dtype, seed, C, M, relu, res):
    N, H, W = 2, 9, 7
    g = rng.uniform_int(seed, (C,), 0, 5)
    G = int(g.sum())
    q = (lambda a: quantise(a, dtype)) if dtype != "f32" else (lambda a: np.asarray(a, np.float32))
    x, dw, pw = q(rng.normal(seed + 1, (N, C, H, W))), q(rng.normal(seed + 2, (G, 3, 3), std=0.3)), \
        q(rng.normal(seed + 3, (M, G), std=0.2))
    b = rng.normal(seed + 4, (M,), std=0.1)
    r = q(rng.normal(seed + 5, (N, M, H, W))) if res else None

    def check(y):
        if dtype == "f32":
            ref = oracle.gdws_forward(x, g, dw, pw, b, r, relu, 1, 1)
            assert_elementwise(y, ref, elementwise_bound_f32(x, g, dw, pw, b, r, 1, 1) + 2.0 ** -23 * np.abs(ref))
        else:
            ref, bound = elementwise_bound(y, x, g, dw, pw, b, r, relu, 1, 1, dtype)
            assert_elementwise(y, ref, bound)

    for order in (0, 1):
        check(_emulate(x, g, dw, pw, b, r, relu, 1, dtype, order))
    # one wrong input pixel (what a bad halo index produces), one wrong tap, one wrong pointwise weight
    x2 = x.copy(); x2[1, 3, 4, 0] = x[1, 3, 4, 1]
    dw2 = dw.copy(); dw2[G // 2, 2, 0] = dw[G // 2, 0, 2]
    pw2 = pw.copy(); pw2[M // 3, G // 3] = pw[M // 3, G // 3 + 1]
    for bad in (_emulate(x2, g, dw, pw, b, r, relu, 1, dtype, 0), _emulate(x, g, dw2, pw, b, r, relu, 1, dtype, 0),
                _emulate(x, g, dw, pw2, b, r, relu, 1, dtype, 0)):
        with pytest.raises(AssertionError):
            check(bad)
