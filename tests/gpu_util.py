"""Helpers for the GPU parity tests: host<->device conversion by storage type and layout."""
import numpy as np
import torch

import workloads

TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
TOL = {"f32": 1e-5, "f16": 2e-2, "bf16": 2e-2}          # rel-L2 bars: fp32, 16-bit storage


def to_device(x_nchw, dtype, layout):
    """fp32 NCHW numpy -> (torch tensor on cuda:0 in storage dtype and layout, float64 NCHW values it holds)."""
    x_nchw = np.ascontiguousarray(x_nchw, dtype=np.float32)
    s = workloads.to_storage(x_nchw, dtype)
    exact = workloads.from_storage(s, dtype).reshape(x_nchw.shape)
    if layout == "nhwc":
        s = np.ascontiguousarray(s.transpose(0, 2, 3, 1))
    if dtype == "bf16":
        t = torch.from_numpy(s.view(np.int16)).view(torch.bfloat16)
    else:
        t = torch.from_numpy(s)
    return t.cuda(), exact


def from_device(t, dtype, layout):
    """torch device tensor (N,C,H,W or N,H,W,C) -> float64 NCHW numpy."""
    a = t.detach().cpu()
    a = a.view(torch.int16).numpy().view(np.uint16) if dtype == "bf16" else a.numpy()
    v = workloads.from_storage(a, dtype).reshape(a.shape)
    if layout == "nhwc":
        v = v.transpose(0, 3, 1, 2)
    return np.ascontiguousarray(v)


def empty_act(N, C, H, W, dtype, layout, fill=None):
    shape = (N, H, W, C) if layout == "nhwc" else (N, C, H, W)
    t = torch.empty(shape, dtype=TORCH_DTYPE[dtype], device="cuda")
    if fill is not None:
        t.fill_(fill)
    return t


def rel_l2(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    den = np.sqrt(np.sum(b * b))
    return float(np.sqrt(np.sum((a - b) ** 2)) / (den if den > 0 else 1.0))


def quantise(w, dtype):
    """fp32 weights -> the fp32 values they take after rounding to the storage dtype."""
    return workloads.from_storage(workloads.to_storage(w, dtype), dtype).astype(np.float32).reshape(np.shape(w))


# ------------------------------------------------------------------------------------------
# element-wise bound
# ------------------------------------------------------------------------------------------

_MANT = {"bf16": 7, "f16": 10}
_MIN_EXP = {"bf16": -126, "f16": -14}          # exponent of the smallest normal number


def spacing(v, dtype):
    """Distance from |v| to the next representable value of larger magnitude in the storage type."""
    a = np.abs(np.asarray(v, np.float64))
    e = np.floor(np.log2(np.maximum(a, 2.0 ** _MIN_EXP[dtype])))
    return 2.0 ** (np.maximum(e, _MIN_EXP[dtype]) - _MANT[dtype])


def elementwise_bound(y, x, g, dw, pw, bias, residual, relu, stride, pad, dtype):
    """(ref, bound): the oracle's output with the intermediate rounded as the kernels round it, and for every
    output element the largest |y - ref| that the kernels' arithmetic can produce.

    16-bit storage.  The kernels differ from that oracle in three places only:
      * the depthwise sums are accumulated in fp32, so an intermediate value T can land on the other side of a
        rounding boundary of the storage type when it lies within eps_T = 16 * 2^-24 * sum|taps * inputs| of one;
        such a T is off by one spacing, which reaches output m as |Pw[m,j]| * spacing(T);
      * the pointwise sums are accumulated in fp32: (G + 16) * 2^-24 * sum_j |Pw[m,j] T[j]|;
      * the result is rounded once to the storage type: half a spacing of the output.
    Bias, residual add and ReLU are fp32 operations on exact inputs (2^-23 relative), and ReLU and rounding are
    monotone and 1-Lipschitz, so the bound passes through them.
    """
    import oracle
    G = int(np.sum(g))
    t = oracle.gdw(x, g, dw, stride, pad, threads=8)
    a = oracle.gdw(np.abs(x), g, np.abs(dw), stride, pad, threads=8)
    tr = oracle.round_to(t, dtype)
    sp = spacing(tr, dtype)
    eps_t = 16.0 * 2.0 ** -24 * a
    # distance from T to the nearer rounding boundary: half a spacing from the rounded value, a quarter where the
    # rounded value is a power of two and T lies below it (the spacing halves there)
    at = np.abs(tr)
    pow2 = (at > 2.0 ** _MIN_EXP[dtype]) & (at == 2.0 ** np.floor(np.log2(np.maximum(at, 1e-300))))
    half = np.where(pow2 & (np.abs(t) < at), 0.25, 0.5) * sp
    near = (half - np.abs(t - tr)) <= eps_t
    flip = oracle.pw(np.where(near, sp, 0.0), np.abs(pw), threads=8)
    s_abs = oracle.pw(np.abs(tr) + np.where(near, sp, 0.0), np.abs(pw), threads=8)
    ref = oracle.pw(tr, pw, bias, threads=8)
    pre = np.abs(ref) + (0.0 if residual is None else np.abs(residual))
    if residual is not None or relu:
        ref = oracle.add_relu(ref, residual, relu)
    delta = flip + (G + 16) * 2.0 ** -24 * s_abs + 2.0 ** -22 * pre
    bound = 0.5 * spacing(np.maximum(np.abs(ref), np.abs(y)), dtype) * (1 + 2.0 ** -10) + delta
    return ref, bound


def elementwise_bound_f32(x, g, dw, pw, bias, residual, stride, pad):
    """fp32 storage: nothing is rounded but the fp32 sums themselves: |y - ref| <= (G + K^2 + 8) * 2^-24 * S with S
    the sum of the magnitudes of every product that enters the element (plus bias and residual)."""
    import oracle
    G, KK = int(np.sum(g)), dw.shape[1] * dw.shape[2]
    a = oracle.gdw(np.abs(x), g, np.abs(dw), stride, pad, threads=8)
    s_abs = oracle.pw(a, np.abs(pw), None if bias is None else np.abs(bias), threads=8)
    if residual is not None:
        s_abs = s_abs + np.abs(residual)
    return (G + KK + 8) * 2.0 ** -24 * s_abs


def assert_elementwise(y, ref, bound, what=""):
    """Every element within its bound; the message names the worst element."""
    excess = np.abs(y - ref) - bound
    k = int(np.argmax(excess))
    idx = np.unravel_index(k, y.shape)
    assert excess.flat[k] <= 0, (f"{what}: element {idx}: got {y.flat[k]!r}, want {ref.flat[k]!r}, "
                                 f"bound {bound.flat[k]:.3e}, {int((excess > 0).sum())} of {y.size} outside")
