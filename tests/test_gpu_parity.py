"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Bars: rel-L2 <= 1e-5 for fp32 storage, <= 2e-2 for fp16 / bf16 storage (both sides use the same
rounded inputs and weights; the oracle keeps the G-channel intermediate in double, the GPU rounds it
to the storage type), index tables bit-exact.  On top of the norm, every output element of a single
layer must lie within the bound that the kernels' arithmetic allows around the oracle's value
(gpu_util.elementwise_bound: fp32 accumulation, the rounding of the intermediate, one rounding of the
output), so that a single wrong pixel, tap or weight fails the test however large the tensor is.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2110_14871_amd as gd
import workloads
from workloads import rng

from gpu_util import (TOL, assert_elementwise, elementwise_bound, elementwise_bound_f32, empty_act, from_device,
                      quantise, rel_l2, to_device)

pytestmark = pytest.mark.gpu

MODES = [gd.MODE_UNFUSED, gd.MODE_FUSED]


def _osz(n, K, s, p):
    return (n + 2 * p - K) // s + 1


def run_layer(x_nchw, g, dw, pw, *, K, stride, pad, dtype, layout, mode, bias=None, residual=None, relu=False):
    """One GDWS layer on the GPU from explicit factors.  Returns (y float64 NCHW, exact inputs dict) or None
    if `mode` is not available for this shape."""
    N, C, H, W = x_nchw.shape
    M = pw.shape[0]
    desc = gd.make_desc(C, M, K, stride, pad, dtype, layout, relu, bias is not None, residual is not None)
    plan = gd.gdws_plan(desc, g, dw=dw, pw=pw, bias=bias)
    Ho, Wo = _osz(H, K, stride, pad), _osz(W, K, stride, pad)
    xd, x_exact = to_device(x_nchw, dtype, layout)
    rd, r_exact = (None, None) if residual is None else to_device(residual, dtype, layout)
    y = empty_act(N, M, Ho, Wo, dtype, layout, fill=float("nan"))
    nbytes = gd.gdws_workspace_bytes(plan, N, H, W, mode)
    ws = torch.empty(max(nbytes, 1), dtype=torch.uint8, device="cuda")
    try:
        gd.gdws_forward(plan, xd, y, N, H, W, residual=rd, workspace=ws, mode=mode)
    except gd.GdwsError as e:
        if e.code == -3 and mode == gd.MODE_FUSED:
            return None
        raise
    torch.cuda.synchronize()
    dwq, pwq = gd.gdws_plan_factors(plan)
    return from_device(y, dtype, layout), dict(x=x_exact, residual=r_exact, dw=dwq, pw=pwq)


def check_layer(seed, N, C, H, W, M, K, stride, pad, g, dtype, layout, mode, bias=False, residual=False, relu=False,
                std_w=0.2):
    G = int(np.sum(g))
    x = rng.normal(seed, (N, C, H, W))
    dw = rng.normal(seed + 1, (G, K, K), std=std_w)
    pw = rng.normal(seed + 2, (M, G), std=std_w)
    b = rng.normal(seed + 3, (M,), std=0.1) if bias else None
    Ho, Wo = _osz(H, K, stride, pad), _osz(W, K, stride, pad)
    r = rng.normal(seed + 4, (N, M, Ho, Wo)) if residual else None
    out = run_layer(x, g, dw, pw, K=K, stride=stride, pad=pad, dtype=dtype, layout=layout, mode=mode, bias=b,
                    residual=r, relu=relu)
    if out is None:
        pytest.skip("no fused kernel for this shape")
    y, ex = out
    assert (ex["dw"] == quantise(dw, dtype)).all() and (ex["pw"] == quantise(pw, dtype)).all()
    ref = oracle.gdws_forward(ex["x"], g, ex["dw"], ex["pw"], b, ex["residual"], relu, stride, pad)
    assert y.shape == ref.shape
    assert np.isfinite(y).all()
    err = rel_l2(y, ref)
    assert err <= TOL[dtype], f"rel-L2 {err:.3e}"
    check_elements(y, ref, ex, g, b, relu, stride, pad, dtype)
    return err


def check_elements(y, ref, ex, g, b, relu, stride, pad, dtype):
    """Every element of y against the oracle, within the bound of the kernels' arithmetic (see gpu_util)."""
    if dtype == "f32":
        bound = elementwise_bound_f32(ex["x"], g, ex["dw"], ex["pw"], b, ex["residual"], stride, pad)
        assert_elementwise(y, ref, bound + 2.0 ** -23 * np.abs(ref), "fp32")
        return
    # with the intermediate rounded like the GPU does, only output rounding is left
    ref2, bound = elementwise_bound(y, ex["x"], g, ex["dw"], ex["pw"], b, ex["residual"], relu, stride, pad, dtype)
    assert rel_l2(y, ref2) <= (1.5e-3 if dtype == "f16" else 6e-3)
    assert_elementwise(y, ref2, bound, dtype)


# ------------------------------------------------------------------------------------------
# configuration 1: small fp32 layer, factors made by the library from W
# ------------------------------------------------------------------------------------------

@pytest.mark.parametrize("layout", ["nchw", "nhwc"])
@pytest.mark.parametrize("mode", MODES)
def test_config1_from_weights(layout, mode):
    c = workloads.config1()
    desc = gd.make_desc(c["C"], c["M"], c["K"], c["stride"], c["pad"], "f32", layout)
    plan = gd.gdws_plan(desc, c["g"], W=c["Wt"])
    info = gd.gdws_plan_info(plan)
    # tables: bit-exact
    assert info["G"] == int(c["g"].sum())
    assert info["offsets"].dtype == np.int32 and (info["offsets"] == oracle.offsets(c["g"])).all()
    assert (info["chan_of"] == oracle.chan_of(c["g"])).all()
    assert info["macs_per_pixel"] * 32 * 32 == oracle.macs_gdws(c["g"], 3, 32, 32, 32)
    # factors: compared through the product they form and the singular values they carry
    dw, pw = gd.gdws_plan_factors(plan)
    D0, P0 = oracle.truncated_factors(c["Wt"], c["g"])
    assert rel_l2(oracle.expand_weight(dw, pw, c["g"]), oracle.expand_weight(D0, P0, c["g"])) < 1e-6
    assert np.abs(np.linalg.norm(pw, axis=0) - np.linalg.norm(P0, axis=0)).max() < 1e-6
    xd, x_exact = to_device(c["X"], "f32", layout)
    y = empty_act(1, 32, 32, 32, "f32", layout, fill=float("nan"))
    ws = torch.empty(max(1, gd.gdws_workspace_bytes(plan, 1, 32, 32, mode)), dtype=torch.uint8, device="cuda")
    try:
        gd.gdws_forward(plan, xd, y, 1, 32, 32, workspace=ws, mode=mode)
    except gd.GdwsError as e:
        if e.code == -3 and mode == gd.MODE_FUSED:
            pytest.skip("no fused kernel for this shape")
        raise
    torch.cuda.synchronize()
    yh = from_device(y, "f32", layout)
    ref = oracle.gdws_forward(x_exact, c["g"], dw, pw, stride=1, pad=1)
    assert rel_l2(yh, ref) <= 1e-5
    check_elements(yh, ref, dict(x=x_exact, dw=dw, pw=pw, residual=None), c["g"], None, False, 1, 1, "f32")
    # against the oracle's own factors the difference is that of the two SVDs
    assert rel_l2(yh, oracle.gdws_forward(x_exact, c["g"], D0, P0, stride=1, pad=1)) <= 1e-5


@pytest.mark.parametrize("layout", ["nchw", "nhwc"])
def test_stages_separately(layout):
    g = np.array([2, 0, 3, 1, 1, 4, 9, 1], np.int32)
    G, C, M, N, H, W = int(g.sum()), 8, 24, 2, 13, 11
    for dtype in ("f32", "f16", "bf16"):
        x = rng.normal(500, (N, C, H, W))
        dw = rng.normal(501, (G, 3, 3), std=0.3)
        pw = rng.normal(502, (M, G), std=0.3)
        b = rng.normal(503, (M,), std=0.1)
        desc = gd.make_desc(C, M, 3, 1, 1, dtype, layout, relu=True, has_bias=True)
        plan = gd.gdws_plan(desc, g, dw=dw, pw=pw, bias=b)
        dwq, pwq = gd.gdws_plan_factors(plan)
        xd, x_exact = to_device(x, dtype, layout)
        Gt = gd.gdws_intermediate_channels(plan)          # G, or G padded with zero channels (NHWC, 16-bit)
        assert Gt == (G if (layout == "nchw" or dtype == "f32") else -(-G // 16) * 16)
        t = empty_act(N, Gt, H, W, dtype, layout, fill=float("nan"))
        gd.gdws_gdw_forward(plan, xd, t, N, H, W)
        torch.cuda.synchronize()
        th = from_device(t, dtype, layout)
        assert np.all(th[:, G:] == 0)
        th = np.ascontiguousarray(th[:, :G])
        assert rel_l2(th, oracle.gdw(x_exact, g, dwq, 1, 1)) <= (1e-6 if dtype == "f32" else 4e-3)
        y = empty_act(N, M, H, W, dtype, layout, fill=float("nan"))
        gd.gdws_pw_forward(plan, t, y, N, H, W)
        torch.cuda.synchronize()
        ref = oracle.add_relu(oracle.pw(th, pwq, b), None, True)          # from the GPU's own intermediate
        assert rel_l2(from_device(y, dtype, layout), ref) <= (1e-6 if dtype == "f32" else 4e-3)


@pytest.mark.parametrize("case", [
    # C, N, H, W, rule: layers of several input stages (C > 128), whose depthwise stage alone runs on the matrix cores
    # with stages that overlap by 8 channels
    (256, 3, 8, 8, "u14"),
    (136, 2, 10, 12, "u13"),        # a last stage of 24 channels, C no multiple of 16
    (320, 2, 5, 7, "u09"),          # channels without filters: groups of 8 intermediate channels that reach further
    (192, 1, 16, 16, "all9"),
    (512, 2, 4, 4, "all1"),
])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_depthwise_stage_alone_many_channels(case, dtype):
    C, N, H, W, rule = case
    g = _g(rule, C, 640 + C)
    G, M = int(g.sum()), 16
    x = rng.normal(510 + C, (N, C, H, W))
    dw = rng.normal(511 + C, (G, 3, 3), std=0.3)
    pw = rng.normal(512 + C, (M, G), std=0.1)
    plan = gd.gdws_plan(gd.make_desc(C, M, 3, 1, 1, dtype, "nhwc"), g, dw=dw, pw=pw)
    dwq, _ = gd.gdws_plan_factors(plan)
    xd, x_exact = to_device(x, dtype, "nhwc")
    Gt = gd.gdws_intermediate_channels(plan)
    t = empty_act(N, Gt, H, W, dtype, "nhwc", fill=float("nan"))
    gd.gdws_gdw_forward(plan, xd, t, N, H, W)
    torch.cuda.synchronize()
    th = from_device(t, dtype, "nhwc")
    assert np.all(th[:, G:] == 0)
    ref = oracle.gdw(x_exact, g, dwq, 1, 1)
    th = th[:, :G]
    assert rel_l2(th, ref) <= 4e-3
    # every element: the fp32 sum of nine products, rounded once to the storage type
    ulp = np.abs(ref) * 2.0 ** (-8 if dtype == "bf16" else -11)
    slack = 9 * 2.0 ** -24 * oracle.gdw(np.abs(x_exact), g, np.abs(dwq), 1, 1) + (2.0 ** -133 if dtype == "bf16" else 2.0 ** -24)
    assert np.all(np.abs(th - ref) <= ulp * (1 + 2.0 ** -6) + slack)


@pytest.mark.parametrize("case", [
    # C, N, H, W, rule: ragged images (tiles that hang over the edge), row blocks that own one to four groups of 8
    # intermediate channels, images narrower than a tile row
    (32, 3, 13, 11, "u13"),
    (64, 2, 17, 5, "all1"),
    (128, 2, 9, 19, "u09"),
    (48, 5, 3, 3, "u14"),
    (160, 2, 7, 9, "u13"),          # several input stages
])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_depthwise_stage_alone_writes_only_its_output(case, dtype):
    """The depthwise stage alone stores T through a bounds-checked descriptor, masked lanes carrying an offset outside
    it: T is right on ragged shapes and the memory on either side of T keeps its contents."""
    C, N, H, W, rule = case
    g = _g(rule, C, 700 + C)
    G, M = int(g.sum()), 16
    x = rng.normal(520 + C, (N, C, H, W))
    dw = rng.normal(521 + C, (G, 3, 3), std=0.3)
    pw = rng.normal(522 + C, (M, G), std=0.1)
    plan = gd.gdws_plan(gd.make_desc(C, M, 3, 1, 1, dtype, "nhwc"), g, dw=dw, pw=pw)
    dwq, _ = gd.gdws_plan_factors(plan)
    xd, x_exact = to_device(x, dtype, "nhwc")
    Gt = gd.gdws_intermediate_channels(plan)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float16
    n, guard = N * H * W * Gt, 4096
    buf = torch.full((n + 2 * guard,), 7.0, dtype=tdt, device="cuda")
    t = buf[guard:guard + n].view(N, H, W, Gt)
    t.fill_(float("nan"))
    gd.gdws_gdw_forward(plan, xd, t, N, H, W)
    torch.cuda.synchronize()
    assert bool((buf[:guard] == 7.0).all()) and bool((buf[guard + n:] == 7.0).all())
    th = from_device(t, dtype, "nhwc")
    assert np.all(th[:, G:] == 0)
    assert rel_l2(th[:, :G], oracle.gdw(x_exact, g, dwq, 1, 1)) <= 4e-3


# ------------------------------------------------------------------------------------------
# shape sweep: several tiles, ragged tails, strides, kernel sizes, degenerate multipliers
# ------------------------------------------------------------------------------------------

SWEEP = [
    # N, C, H, W, M, K, stride, pad, g-rule
    (2, 16, 32, 32, 32, 3, 1, 1, "u13"),
    (3, 24, 17, 19, 40, 3, 1, 1, "u09"),     # odd sizes, zero-multiplier channels, ragged everything
    (2, 32, 16, 16, 64, 3, 2, 1, "u14"),     # stride 2
    (2, 8, 15, 15, 16, 3, 2, 1, "u13"),      # stride 2, odd
    (1, 6, 9, 9, 12, 5, 1, 2, "u13"),        # K = 5
    (2, 4, 19, 18, 24, 7, 2, 3, "u14"),      # K = 7, stride 2, pad 3 (an ImageNet stem's geometry)
    (2, 10, 8, 8, 7, 1, 1, 0, "u13"),        # K = 1
    (2, 12, 12, 12, 20, 3, 1, 0, "u13"),     # no padding
    (5, 64, 4, 4, 128, 3, 1, 1, "u14"),      # tiny images, many channels
    (4, 48, 2, 2, 96, 3, 1, 1, "u14"),       # 2 x 2 images
    (1, 3, 33, 33, 64, 3, 1, 1, "u14"),      # network stem shape
    (2, 20, 7, 7, 36, 3, 1, 1, "all9"),      # exact-representation multiplier
    (2, 20, 14, 14, 36, 3, 1, 1, "all1"),    # plain depthwise-separable
    (1, 5, 6, 6, 4, 3, 1, 1, "big"),         # g_c > K^2 allowed when factors are given
    (2, 256, 8, 8, 256, 3, 1, 1, "u14"),     # several input stages (double-buffered) and two blocks of outputs
    (1, 136, 10, 12, 130, 3, 1, 1, "u13"),   # channel counts that are no multiples of 16 / 8
    (2, 64, 12, 12, 96, 3, 2, 1, "u14"),     # stride 2 with several input stages
]


def _g(rule, C, seed):
    if rule == "all9":
        return np.full(C, 9, np.int32)
    if rule == "all1":
        return np.ones(C, np.int32)
    if rule == "big":
        return np.array([12, 1, 0, 11, 2], np.int32)
    lo, hi = int(rule[1]), int(rule[2])
    g = rng.uniform_int(seed, (C,), lo, hi)
    if g.sum() == 0:
        g[0] = 1
    return g


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("layout", ["nhwc", "nchw"])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("case", range(len(SWEEP)))
def test_shape_sweep(case, dtype, layout, mode):
    N, C, H, W, M, K, stride, pad, rule = SWEEP[case]
    g = _g(rule, C, 600 + case)
    check_layer(700 + 10 * case, N, C, H, W, M, K, stride, pad, g, dtype, layout, mode,
                bias=case % 2 == 0, residual=case % 3 == 0, relu=case % 2 == 1)


# ------------------------------------------------------------------------------------------
# configuration 2 (bf16, C = M = 128, 16 x 16): reduced batch element by element, full batch on a sample
# ------------------------------------------------------------------------------------------

def _config2_g(kind, c2):
    if kind == "budget":
        s, r = gd.gdws_singular_values(c2["Wt"])
        gamma = gd.gdws_budget_gamma(c2["rho"], 128, 3, 128)
        assert gamma == oracle.gamma_from_budget(c2["rho"], 128, 3, 128)
        g = gd.gdws_mego(s, r, gamma, g_init=np.ones(128, np.int32), cap=9)
        _, S, _ = oracle.svd_slices(c2["Wt"])
        assert (g == oracle.mego(S, gamma, g_init=np.ones(128, np.int32), cap=9, dim=128)).all()
        assert g.sum() == 269
        return g
    return np.full(128, 9 if kind == "all9" else 1, np.int32)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("layout", ["nhwc", "nchw"])
@pytest.mark.parametrize("kind", ["budget", "all9", "all1"])
def test_config2_reduced_batch(kind, layout, mode):
    c2 = workloads.config2(N=6)
    g = _config2_g(kind, c2)
    desc = gd.make_desc(128, 128, 3, 1, 1, "bf16", layout)
    plan = gd.gdws_plan(desc, g, W=c2["Wt"])
    dw, pw = gd.gdws_plan_factors(plan)
    if kind == "all9":       # Lemma 1: the full multiplier reproduces W itself (up to bf16 rounding of the factors)
        assert rel_l2(oracle.expand_weight(dw, pw, g), c2["Wt"]) < 1e-2
    xd, x_exact = to_device(c2["X"], "bf16", layout)
    y = empty_act(6, 128, 16, 16, "bf16", layout, fill=float("nan"))
    ws = torch.empty(max(1, gd.gdws_workspace_bytes(plan, 6, 16, 16, mode)), dtype=torch.uint8, device="cuda")
    try:
        gd.gdws_forward(plan, xd, y, 6, 16, 16, workspace=ws, mode=mode)
    except gd.GdwsError as e:
        if e.code == -3 and mode == gd.MODE_FUSED:
            pytest.skip("no fused kernel for this shape")
        raise
    torch.cuda.synchronize()
    ref = oracle.gdws_forward(x_exact, g, dw, pw, stride=1, pad=1, threads=8)
    yh = from_device(y, "bf16", layout)
    assert rel_l2(yh, ref) <= 2e-2
    check_elements(yh, ref, dict(x=x_exact, dw=dw, pw=pw, residual=None), g, None, False, 1, 1, "bf16")


@pytest.mark.parametrize("mode", [gd.MODE_AUTO, gd.MODE_UNFUSED])
@pytest.mark.parametrize("layout", ["nhwc", "nchw"])
def test_config2_full_batch_sampled(layout, mode):
    """Batch 256 in the launch configuration the bench times; the oracle checks images 0, 1, 127, 254, 255."""
    c2 = workloads.config2(N=256)
    g = _config2_g("budget", c2)
    desc = gd.make_desc(128, 128, 3, 1, 1, "bf16", layout)
    plan = gd.gdws_plan(desc, g, W=c2["Wt"])
    dw, pw = gd.gdws_plan_factors(plan)
    xd, x_exact = to_device(c2["X"], "bf16", layout)
    y = empty_act(256, 128, 16, 16, "bf16", layout, fill=float("nan"))
    ws = torch.empty(max(1, gd.gdws_workspace_bytes(plan, 256, 16, 16, mode)), dtype=torch.uint8, device="cuda")
    gd.gdws_forward(plan, xd, y, 256, 16, 16, workspace=ws, mode=mode)
    torch.cuda.synchronize()
    yh = from_device(y, "bf16", layout)
    assert np.isfinite(yh).all()
    pick = [0, 1, 127, 254, 255]
    ref = oracle.gdws_forward(x_exact[pick], g, dw, pw, stride=1, pad=1, threads=8)
    assert rel_l2(yh[pick], ref) <= 2e-2
    check_elements(yh[pick], ref, dict(x=x_exact[pick], dw=dw, pw=pw, residual=None), g, None, False, 1, 1, "bf16")
    # images are independent: permuting the batch permutes the output
    perm = np.arange(255, -1, -1)
    xd2, _ = to_device(c2["X"][perm], "bf16", layout)
    y2 = empty_act(256, 128, 16, 16, "bf16", layout, fill=float("nan"))
    gd.gdws_forward(plan, xd2, y2, 256, 16, 16, workspace=ws, mode=mode)
    torch.cuda.synchronize()
    assert (from_device(y2, "bf16", layout)[perm] == yh).all()


# ------------------------------------------------------------------------------------------
# seeded random shapes: channel counts around the stage and slice boundaries, images smaller than a tile, batches that
# give one or many tiles per CU (the launch picks 256- or 128-pixel tiles and 128- or 64-channel slices from these)
# ------------------------------------------------------------------------------------------

def _random_case(R, big):
    C = int(R.choice([16, 64, 128, 136, 256] if big else [8, 16, 24, 40, 64, 72, 128, 136, 200, 256]))
    M = int(R.choice([32, 64, 128, 256] if big else [8, 24, 32, 64, 72, 128, 136, 256, 320]))
    stride = int(R.choice([1, 1, 1, 2]))
    H = int(R.choice([2, 3, 4, 5, 7, 8, 9, 12, 16, 17, 24, 33]))
    W = int(R.choice([2, 3, 4, 6, 8, 11, 16, 20, 31, 32]))
    budget = int(R.choice([20000, 50000])) if big else 6000
    N = max(1, min(int(R.choice([1, 2, 3, 5, 9, 17, 40])) if not big else 10 ** 9, budget // (H * W)))
    kind = R.randint(3)
    g = (np.ones(C) if kind == 0 else R.randint(1, 10, C) if kind == 1 else np.minimum(R.geometric(0.5, C), 9))
    return dict(N=N, C=C, H=H, W=W, M=M, stride=stride, g=g.astype(np.int32), dtype=str(R.choice(["bf16", "f16"])),
                layout=str(R.choice(["nhwc", "nhwc", "nchw"])), mode=int(R.choice(MODES)), bias=bool(R.randint(2)),
                residual=bool(R.randint(2)), relu=bool(R.randint(2)))


@pytest.mark.parametrize("block", range(8))
def test_random_shapes(block):
    R = np.random.RandomState(4200 + block)
    for i in range(6 if block >= 6 else 40):
        c = _random_case(R, big=block >= 6)
        check_layer(4300 + 100 * block + i, c["N"], c["C"], c["H"], c["W"], c["M"], 3, c["stride"], 1, c["g"], c["dtype"],
                    c["layout"], c["mode"], bias=c["bias"], residual=c["residual"], relu=c["relu"])


# ------------------------------------------------------------------------------------------
# reference point, pooling, networks, error paths
# ------------------------------------------------------------------------------------------

DENSE = [(2, 16, 12, 12, 24, 3, 1, 1), (2, 3, 20, 20, 16, 7, 2, 3), (3, 32, 8, 8, 48, 1, 2, 0), (1, 8, 9, 7, 8, 3, 2, 1),
         # 3 x 3, stride 1, C a multiple of 16: the implicit GEMM on the matrix cores (16-bit NHWC); several tiles per
         # image, a last chunk of 16 channels, two slices of output channels with a ragged end, images narrower than a tile
         (3, 128, 16, 16, 128, 3, 1, 1), (2, 80, 19, 37, 72, 3, 1, 1), (1, 32, 5, 7, 200, 3, 1, 1), (2, 144, 33, 8, 36, 3, 1, 1)]


@pytest.mark.parametrize("layout", ["nhwc", "nchw"])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("case", range(len(DENSE)))
def test_conv_dense_reference_point(case, dtype, layout):
    N, C, H, W, M, K, stride, pad = DENSE[case]
    x = rng.normal(800 + case, (N, C, H, W))
    w = rng.normal(810 + case, (M, C, K, K), std=0.2)
    b = rng.normal(820 + case, (M,), std=0.1)
    Ho, Wo = _osz(H, K, stride, pad), _osz(W, K, stride, pad)
    r = rng.normal(830 + case, (N, M, Ho, Wo))
    desc = gd.make_desc(C, M, K, stride, pad, dtype, layout, relu=True, has_bias=True, has_residual=True)
    xd, x_exact = to_device(x, dtype, layout)
    rd, r_exact = to_device(r, dtype, layout)
    wd, w_exact = to_device(w, dtype, "nchw")
    bd = torch.from_numpy(b).cuda()
    y = empty_act(N, M, Ho, Wo, dtype, layout, fill=float("nan"))
    ws = torch.empty(max(1, gd.conv_dense_workspace_bytes(desc)), dtype=torch.uint8, device="cuda")
    gd.conv_dense_forward(desc, wd, xd, y, N, H, W, bias=bd, residual=rd, workspace=ws)
    torch.cuda.synchronize()
    ref = oracle.add_relu(oracle.conv_dense(x_exact, w_exact, b, stride, pad), r_exact, True)
    assert rel_l2(from_device(y, dtype, layout), ref) <= TOL[dtype]


from net_util import build_network as _build_network  # noqa: E402


def _run_network(net, shapes, x, dtype, layout):
    N, C, H, W = x.shape
    last = shapes[-1]
    xd, x_exact = to_device(x, dtype, layout)
    y = empty_act(N, last.M, last.Ho, last.Wo, dtype, layout, fill=float("nan"))
    nbytes = gd.gdws_net_workspace_bytes(net, N, H, W)
    ws = torch.empty(max(1, nbytes), dtype=torch.uint8, device="cuda")
    gd.gdws_network_forward(net, xd, y, N, H, W, workspace=ws)
    torch.cuda.synchronize()
    return from_device(y, dtype, layout), x_exact


NETS = {"vgg16": workloads.vgg16_shape, "resnet18": workloads.resnet18_shape, "resnet50": workloads.resnet50_shape,
        "wrn28_4": workloads.wrn28_4_shape}


@pytest.mark.parametrize("layout", ["nhwc", "nchw"])
@pytest.mark.parametrize("name,dtype,N,size", [("vgg16", "f16", 2, 32), ("resnet18", "bf16", 2, 32),
                                                ("resnet50", "bf16", 1, 64), ("vgg16", "f32", 1, 32),
                                                ("wrn28_4", "bf16", 2, 32)])
def test_network_shapes(name, dtype, N, size, layout):
    shapes = NETS[name](size, size)
    net, params = _build_network(shapes, dtype, layout)
    x = rng.normal(900, (N, 3, size, size))
    yh, x_exact = _run_network(net, shapes, x, dtype, layout)
    store = None if dtype == "f32" else dtype
    ref = oracle.network_forward(shapes, params, x_exact, store=store, round_intermediate=store, threads=8)
    check_network_output(yh, ref, dtype)
    if store:    # and against the oracle that keeps every layer's intermediate in double
        assert rel_l2(yh, oracle.network_forward(shapes, params, x_exact, store=store, threads=8)) <= TOL[dtype]


def check_network_output(yh, ref, dtype):
    """Whole tensor and every image within the rel-L2 bar; no single element further off than the rounding of a
    deep stack of layers can put it (a wrong element is off by about the tensor's rms)."""
    assert yh.shape == ref.shape and np.isfinite(yh).all()
    assert rel_l2(yh, ref) <= TOL[dtype]
    rtol = {"f32": 1e-4, "f16": 2e-2, "bf16": 1e-1}[dtype]
    for n in range(ref.shape[0]):
        assert rel_l2(yh[n], ref[n]) <= TOL[dtype], f"image {n}"
        rms = float(np.sqrt(np.mean(ref[n] ** 2)))
        assert_elementwise(yh[n], ref[n], rtol * (np.abs(ref[n]) + rms), f"image {n}")


# the three network workloads at their full batch (the launch configurations the benchmark times: tile sizes, channel
# slices and buffer reuse depend on the batch); images are independent, so the oracle runs a sample of them alone
FULL = [("vgg16", "f16", 256, 32, [0, 1, 130, 255]), ("resnet18", "bf16", 512, 32, [0, 255, 256, 511]),
        ("resnet50", "bf16", 128, 224, [0, 127]), ("wrn28_4", "bf16", 256, 32, [0, 128, 255])]


@pytest.mark.parametrize("name,dtype,N,size,pick", FULL)
def test_network_full_batch_sampled(name, dtype, N, size, pick):
    shapes = NETS[name](size, size)
    net, params = _build_network(shapes, dtype, "nhwc")
    x = rng.normal(901, (N, 3, size, size))
    yh, x_exact = _run_network(net, shapes, x, dtype, "nhwc")
    assert np.isfinite(yh).all()
    ref = oracle.network_forward(shapes, params, x_exact[pick], store=dtype, round_intermediate=dtype, threads=16)
    check_network_output(yh[pick], ref, dtype)
    # a second forward through the same workspace gives the same bits (no layer reads what another one is writing)
    yh2, _ = _run_network(net, shapes, x, dtype, "nhwc")
    assert (yh2 == yh).all()


# first layers of a network (3 input channels): the implicit-GEMM kernel, at sizes with ragged tiles, images
# smaller than the filter's reach, and an output channel count that is not a multiple of 8
STEM = [(3, 37, 29, 64, 7, 2, 3), (2, 9, 11, 40, 7, 2, 3), (5, 16, 16, 96, 3, 1, 1), (1, 3, 5, 12, 3, 1, 1)]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("case", range(len(STEM)))
def test_network_first_layer(case, dtype):
    from workloads.configs import LayerShape
    N, H, W, M, K, stride, pad = STEM[case]
    shapes = [LayerShape(kind="dense", C=3, M=M, K=K, stride=stride, pad=pad, relu=(case % 2 == 0), bias=True, src=-1,
                         residual=None, seed=850 + case, H=H, W=W)]
    net, params = _build_network(shapes, dtype, "nhwc")
    x = rng.normal(860 + case, (N, 3, H, W))
    yh, x_exact = _run_network(net, shapes, x, dtype, "nhwc")
    ref = oracle.network_forward(shapes, params, x_exact, store=dtype, threads=8)
    assert yh.shape == ref.shape and np.isfinite(yh).all()
    assert rel_l2(yh, ref) <= TOL[dtype]


@pytest.mark.parametrize("residual", [False, True])
def test_pointwise_gemm_many_tiles(residual):
    """A 1 x 1 convolution with more pixel tiles than resident workgroups: every workgroup of the pointwise GEMM
    walks over several work items (ragged last tile, output channels not a multiple of 8 in the second slice)."""
    from workloads.configs import LayerShape
    N, C, H, W, M = 3, 16, 250, 211, (40 if residual else 136)   # (sizes the oracle finishes in seconds)
    shapes = [LayerShape(kind="dense", C=C, M=M, K=1, stride=1, pad=0, relu=True, bias=True, src=-1, residual=None,
                         seed=870, H=H, W=W)]
    if residual:
        shapes.append(LayerShape(kind="dense", C=M, M=M, K=1, stride=1, pad=0, relu=True, bias=True, src=0, residual=0,
                                 seed=871, H=H, W=W))
    net, params = _build_network(shapes, "bf16", "nhwc")
    x = rng.normal(872, (N, C, H, W))
    yh, x_exact = _run_network(net, shapes, x, "bf16", "nhwc")
    ref = oracle.network_forward(shapes, params, x_exact, store="bf16", threads=8)
    assert yh.shape == ref.shape and np.isfinite(yh).all()
    assert rel_l2(yh, ref) <= TOL["bf16"]


# images at most four pixels wide (the deep layers of the CIFAR networks): tiles with four-pixel rows, several images
# per tile, one and several input stages, 128- and 64-channel workgroups, stride 2 down to four pixels
# (the library takes four-pixel rows only when the grid still fills the chip: the cases with many images)
NARROW = [(9, 32, 4, 4, 128, 1), (5, 16, 2, 2, 64, 1), (3, 144, 3, 4, 160, 1), (6, 24, 8, 8, 96, 2),
          (33, 16, 1, 3, 32, 1), (70, 64, 4, 4, 256, 1), (2, 16, 7, 3, 40, 1), (20, 32, 7, 6, 64, 2),
          (2100, 16, 4, 4, 32, 1), (1030, 16, 4, 4, 128, 1), (600, 8, 8, 8, 256, 2), (4200, 16, 2, 2, 32, 1),
          (1500, 72, 3, 4, 72, 1)]


@pytest.mark.parametrize("residual", [False, True])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("case", range(len(NARROW)))
def test_narrow_images(case, dtype, residual):
    N, C, H, W, M, stride = NARROW[case]
    g = _g("u14", C, 4700 + case)
    check_layer(4710 + 10 * case, N, C, H, W, M, 3, stride, 1, g, dtype, "nhwc", gd.MODE_FUSED, bias=True,
                residual=residual, relu=(case % 2 == 1))


# few pixels, many channels (the deep layers of the networks): the kernel whose four waves share a 32-pixel block and
# split the output channels.  Channel counts that are no multiples of 16 / 256, both LDS pixel sizes (C up to 256, up
# to 512), four- and eight-pixel tile rows, 2 x 2 images (half the lanes idle), odd image sizes, a partial last slice
# of output channels; batch sizes chosen so that the library's grid rule takes that kernel.
DEEP = [(64, 264, 4, 4, 264), (128, 256, 2, 2, 512), (32, 512, 7, 7, 256), (40, 160, 8, 8, 512), (130, 136, 3, 4, 384),
        (33, 200, 5, 6, 320), (70, 512, 4, 4, 512)]


# the same kernel on a batch of one or two images: the launch is split over runs of row blocks, partial sums through the
# workspace (gdws_workspace_bytes is then non-zero for the fused path), a second kernel adds them up
DEEP += [(1, 512, 4, 4, 512), (2, 256, 2, 2, 512), (1, 264, 8, 8, 264), (3, 384, 7, 7, 256), (1, 136, 1, 5, 256)]


@pytest.mark.parametrize("residual", [False, True])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("case", range(len(DEEP)))
def test_deep_layers(case, dtype, residual):
    N, C, H, W, M = DEEP[case]
    g = _g("u14" if case % 2 == 0 else "u09", C, 4900 + case)
    check_layer(4910 + 10 * case, N, C, H, W, M, 3, 1, 1, g, dtype, "nhwc", gd.MODE_FUSED, bias=True,
                residual=residual, relu=(case % 2 == 1))


# the layer with the 2 x 2 max-pool in its epilogue: one and several images per tile, odd sizes (the last row and
# column drop out of the pool), stride 2, both stage-size classes, 64- and 128-channel workgroups, 128-pixel tiles
POOLED = [(3, 32, 16, 16, 128, 1), (2, 16, 13, 11, 64, 1), (5, 64, 8, 8, 256, 1), (2, 24, 18, 34, 40, 2),
          (1, 128, 32, 32, 128, 1), (7, 16, 4, 4, 64, 1), (4, 16, 2, 2, 32, 1), (2, 144, 9, 40, 96, 1), (3, 16, 3, 19, 64, 1),
          (2100, 16, 4, 4, 32, 1), (4200, 16, 2, 2, 64, 1),   # (four-pixel tile rows)
          (64, 264, 4, 4, 264, 1), (128, 256, 2, 2, 512, 1), (40, 160, 8, 8, 512, 1), (36, 384, 6, 6, 256, 1)]  # (deep layers)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("case", range(len(POOLED)))
def test_forward_with_pool_epilogue(case, dtype):
    N, C, H, W, M, stride = POOLED[case]
    seed = 4600 + 10 * case
    g = _g("u14", C, seed)
    G = int(g.sum())
    x = rng.normal(seed, (N, C, H, W))
    dw = rng.normal(seed + 1, (G, 3, 3), std=0.2)
    pw = rng.normal(seed + 2, (M, G), std=0.2)
    b = rng.normal(seed + 3, (M,), std=0.1)
    relu = case % 2 == 0
    desc = gd.make_desc(C, M, 3, stride, 1, dtype, "nhwc", relu, True, False)
    plan = gd.gdws_plan(desc, g, dw=dw, pw=pw, bias=b)
    Ho, Wo = _osz(H, 3, stride, 1), _osz(W, 3, stride, 1)
    xd, x_exact = to_device(x, dtype, "nhwc")
    y = empty_act(N, M, Ho // 2, Wo // 2, dtype, "nhwc", fill=float("nan"))
    gd.gdws_forward_maxpool2(plan, xd, y, N, H, W)
    torch.cuda.synchronize()
    dwq, pwq = gd.gdws_plan_factors(plan)
    full = oracle.gdws_forward(x_exact, g, dwq, pwq, b, None, relu, stride, 1)
    ref = oracle.maxpool(oracle.round_to(full, dtype), 2, 2, 0)
    yh = from_device(y, dtype, "nhwc")
    assert yh.shape == ref.shape and np.isfinite(yh).all()
    assert rel_l2(yh, ref) <= TOL[dtype]
    # the same layer through the plain entry point, pooled by the oracle: the epilogue pools what that one stores
    y2 = empty_act(N, M, Ho, Wo, dtype, "nhwc", fill=float("nan"))
    gd.gdws_forward(plan, xd, y2, N, H, W, mode=gd.MODE_FUSED)
    torch.cuda.synchronize()
    assert (yh == oracle.maxpool(from_device(y2, dtype, "nhwc"), 2, 2, 0)).all()


def test_pool_epilogue_unsupported_shapes():
    g = np.ones(16, np.int32)
    dw, pw = np.ones((16, 3, 3), np.float32), np.ones((36, 16), np.float32)
    x = torch.zeros(1, 16, 8, 8, device="cuda", dtype=torch.bfloat16)
    y = torch.zeros(1, 36, 4, 4, device="cuda", dtype=torch.bfloat16)
    for layout, M in (("nchw", 32), ("nhwc", 36)):       # not NHWC; output channels not a multiple of 8
        plan = gd.gdws_plan(gd.make_desc(16, M, 3, 1, 1, "bf16", layout), g, dw=dw, pw=pw[:M])
        with pytest.raises(gd.GdwsError) as e:
            gd.gdws_forward_maxpool2(plan, x, y, 1, 8, 8)
        assert e.value.code == -3
    plan = gd.gdws_plan(gd.make_desc(16, 32, 3, 1, 1, "bf16", "nhwc"), g, dw=dw, pw=pw[:32])
    with pytest.raises(gd.GdwsError) as e:
        gd.gdws_forward_maxpool2(plan, x, y, 1, 1, 8)    # nothing to pool
    assert e.value.code == -1
    torch.cuda.synchronize()


@pytest.mark.parametrize("residual", [False, True])
@pytest.mark.parametrize("M", [40, 136])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_pointwise_gemm_deep_contraction(dtype, M, residual):
    """A 1 x 1 convolution over many channels and few pixels (33 steps of 16 channels, which no unrolling of the
    contraction loop divides); ragged last tile, two slices of output channels for M = 136, residuals."""
    from workloads.configs import LayerShape
    N, C, H, W = 3, 528, 7, 9
    shapes = [LayerShape(kind="dense", C=C, M=M, K=1, stride=1, pad=0, relu=True, bias=True, src=-1, residual=None,
                         seed=880, H=H, W=W)]
    if residual:
        shapes.append(LayerShape(kind="dense", C=M, M=M, K=1, stride=1, pad=0, relu=False, bias=True, src=0, residual=0,
                                 seed=881, H=H, W=W))
        shapes.append(LayerShape(kind="dense", C=M, M=C, K=1, stride=1, pad=0, relu=True, bias=False, src=1,
                                 residual=None, seed=882, H=H, W=W))
        shapes.append(LayerShape(kind="dense", C=C, M=M, K=1, stride=1, pad=0, relu=True, bias=True, src=2, residual=1,
                                 seed=883, H=H, W=W))
    net, params = _build_network(shapes, dtype, "nhwc")
    x = rng.normal(884, (N, C, H, W))
    yh, x_exact = _run_network(net, shapes, x, dtype, "nhwc")
    ref = oracle.network_forward(shapes, params, x_exact, store=dtype, threads=8)
    assert yh.shape == ref.shape and np.isfinite(yh).all()
    assert rel_l2(yh, ref) <= TOL[dtype]


def test_error_paths_on_device():
    g = np.array([1, 2, 1, 1], np.int32)
    desc = gd.make_desc(4, 8, 3, 1, 1, "f32", "nchw", has_residual=True)
    plan = gd.gdws_plan(desc, g, dw=np.ones((5, 3, 3), np.float32), pw=np.ones((8, 5), np.float32))
    x = torch.zeros(1, 4, 6, 6, device="cuda")
    y = torch.zeros(1, 8, 6, 6, device="cuda")
    ws = torch.empty(gd.gdws_workspace_bytes(plan, 1, 6, 6, gd.MODE_UNFUSED), dtype=torch.uint8, device="cuda")
    assert ws.numel() == 5 * 36 * 4
    with pytest.raises(gd.GdwsError) as e:
        gd.gdws_forward(plan, x, y, 1, 6, 6, workspace=ws, mode=gd.MODE_UNFUSED)      # residual missing
    assert e.value.code == -2
    with pytest.raises(gd.GdwsError) as e:
        gd.gdws_forward(plan, x, y, 1, 6, 6, residual=y, workspace=ws[:16], mode=gd.MODE_UNFUSED)
    assert e.value.code == -4
    with pytest.raises(gd.GdwsError) as e:
        gd.gdws_forward(plan, x, y, 0, 6, 6, residual=y, workspace=ws, mode=gd.MODE_UNFUSED)
    assert e.value.code == -1
    with pytest.raises(gd.GdwsError) as e:
        gd.gdws_forward(plan, x, y, 1, 6, 6, residual=y, workspace=ws, mode=7)
    assert e.value.code == -1
    gd.gdws_forward(plan, x, y, 1, 6, 6, residual=y, workspace=ws, mode=gd.MODE_UNFUSED)
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------------------
# batch-1 protocol (Appendix A): the forward recorded once and replayed as a launch graph
# ------------------------------------------------------------------------------------------

@pytest.mark.parametrize("name,dtype,size", [("vgg16", "f16", 32), ("resnet18", "bf16", 32), ("resnet50", "bf16", 64)])
def test_launch_graph_replays_equal_eager(name, dtype, size):
    shapes = NETS[name](size, size)
    net, params = _build_network(shapes, dtype, "nhwc")
    last = shapes[-1]
    x = rng.normal(905, (1, 3, size, size))
    xd, x_exact = to_device(x, dtype, "nhwc")
    y_eager = empty_act(1, last.M, last.Ho, last.Wo, dtype, "nhwc", fill=float("nan"))
    y_graph = empty_act(1, last.M, last.Ho, last.Wo, dtype, "nhwc", fill=float("nan"))
    ws = torch.empty(max(1, gd.gdws_net_workspace_bytes(net, 1, size, size)), dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        gd.gdws_network_forward(net, xd, y_eager, 1, size, size, workspace=ws, stream=side)
        gd.gdws_network_forward(net, xd, y_graph, 1, size, size, workspace=ws, stream=side)
        side.synchronize()
        gd.gdws_capture_begin(side)
        gd.gdws_network_forward(net, xd, y_graph, 1, size, size, workspace=ws, stream=side)
        graph = gd.gdws_capture_end(side)
        want = from_device(y_eager, dtype, "nhwc")
        for rep in range(4):
            # between replays: the program's own eager work on the same buffers, and a synchronisation
            y_graph.fill_(float("nan"))
            ws.fill_(0xFF if rep % 2 else 0)
            gd.gdws_network_forward(net, xd, y_eager, 1, size, size, workspace=ws, stream=side)
            ws.fill_(0x7F)
            side.synchronize()
            gd.gdws_graph_launch(graph, side)
            side.synchronize()
            assert (from_device(y_graph, dtype, "nhwc") == want).all(), f"replay {rep}"
            assert (from_device(y_eager, dtype, "nhwc") == want).all()
    ref = oracle.network_forward(shapes, params, x_exact, store=dtype, round_intermediate=dtype, threads=8)
    check_network_output(want, ref, dtype)
    with pytest.raises(gd.GdwsError) as e:
        gd.gdws_capture_begin(0)          # the default stream cannot be captured
    assert e.value.code == -1


# ------------------------------------------------------------------------------------------
# sparse-aware plan (Appendix B): a pruned weight, dead intermediate channels dropped at plan time
# ------------------------------------------------------------------------------------------

@pytest.mark.parametrize("mode", [gd.MODE_AUTO, gd.MODE_UNFUSED])
@pytest.mark.parametrize("dtype,layout", [("bf16", "nhwc"), ("f16", "nhwc"), ("f32", "nchw")])
@pytest.mark.parametrize("M,C,keep", [(64, 64, 0.02), (128, 32, 0.01), (16, 24, 0.05)])
def test_sparse_aware_plan(M, C, keep, dtype, layout, mode):
    N, H, W = 3, 12, 10
    Wt = workloads.pruned_weight(960 + M, M, C, 3, keep)
    Wq = quantise(Wt, dtype) if dtype != "f32" else Wt
    r = oracle.sparse_g(Wq)
    if r.sum() == 0:
        pytest.skip("nothing survived the pruning")
    g_full = np.full(C, min(M, 9), np.int32)
    desc = gd.make_desc(C, M, 3, 1, 1, dtype, layout)
    full = gd.gdws_plan(desc, g_full, W=Wq)
    sparse = gd.gdws_plan(desc, g_full, W=Wq, sparse=True)
    fi, si = gd.gdws_plan_info(full), gd.gdws_plan_info(sparse)
    assert fi["G"] == int(g_full.sum())
    # the reduced tables are those of g' = rank(W_c) (rounding the factors can only zero more of them)
    g2 = np.diff(si["offsets"])
    assert (g2 <= r).all() and si["G"] == int(g2.sum()) and si["G"] < fi["G"]
    assert (si["offsets"] == oracle.offsets(g2)).all() and (si["chan_of"] == oracle.chan_of(g2)).all()
    assert si["macs_per_pixel"] == si["G"] * (9 + M)
    dwf, pwf = gd.gdws_plan_factors(full)
    dws, pws = gd.gdws_plan_factors(sparse)
    og, od, op, _ = oracle.compact_factors(g_full, dwf, pwf)
    assert (og == g2).all() and (od == dws).all() and (op == pws).all()
    x = rng.normal(970, (N, C, H, W))
    xd, x_exact = to_device(x, dtype, layout)
    outs = []
    for plan, g in ((full, g_full), (sparse, g2)):
        y = empty_act(N, M, H, W, dtype, layout, fill=float("nan"))
        ws = torch.empty(max(1, gd.gdws_workspace_bytes(plan, N, H, W, mode)), dtype=torch.uint8, device="cuda")
        gd.gdws_forward(plan, xd, y, N, H, W, workspace=ws, mode=mode)
        torch.cuda.synchronize()
        outs.append(from_device(y, dtype, layout))
    ref = oracle.gdws_forward(x_exact, g2, dws, pws, stride=1, pad=1)
    for yh in outs:
        assert rel_l2(yh, ref) <= TOL[dtype]
    check_elements(outs[1], ref, dict(x=x_exact, dw=dws, pw=pws, residual=None), g2, None, False, 1, 1, dtype)
    check_elements(outs[0], ref, dict(x=x_exact, dw=dwf, pw=pwf, residual=None), g_full, None, False, 1, 1, dtype)
    # the layer is the pruned standard convolution itself, up to the rounding of the factors (Lemma 1)
    dense = oracle.conv_dense(x_exact, Wq, stride=1, pad=1)
    assert rel_l2(outs[1], dense) <= (1e-5 if dtype == "f32" else 2e-2)


# ------------------------------------------------------------------------------------------
# batched singular values on the device (the ranking step of Algorithms 1 and 2)
# ------------------------------------------------------------------------------------------

SVD_CASES = [
    # M, C, K, std, note
    (128, 128, 3),     # config 2's weight
    (12, 6, 5),        # K = 5
    (4, 10, 3),        # fewer rows than taps: R = M
    (64, 3, 7),        # a 7 x 7 stem: K^2 = 49 < M
    (1, 5, 1),         # 1 x 1, one output channel
]


@pytest.mark.gpu
@pytest.mark.parametrize("case", range(len(SVD_CASES)))
def test_singular_values_device(case):
    """sigma, rank and V from the device routine against the oracle's SVD (numpy) of the same slices."""
    M, C, K = SVD_CASES[case]
    KK, R = K * K, min(M, K * K)
    W = rng.normal(9100 + case, (M, C, K, K), std=0.05)
    if C > 2:
        W[:, 2] = 0.0                                    # a zero slice: rank 0
    if C > 3 and M > 2 and KK > 2:
        W[:, 3] = np.outer(W[:, 3, 0, 0], W[0, 3].reshape(-1)).reshape(M, K, K)   # a rank-1 slice
    w = torch.from_numpy(W).cuda()
    sigma = torch.full((C, R), float("nan"), dtype=torch.float64, device="cuda")
    rank = torch.full((C,), -1, dtype=torch.int32, device="cuda")
    v = torch.full((C, R, KK), float("nan"), dtype=torch.float64, device="cuda")
    gd.gdws_singular_values_device(w, sigma, rank, v)
    torch.cuda.synchronize()
    sigma, rank, v = sigma.cpu().numpy(), rank.cpu().numpy(), v.cpu().numpy()
    U, S, Vt = oracle.svd_slices(W.astype(np.float64))
    s1 = max(S.max(), 1e-300)
    # the Gram matrix resolves sigma to eps * sigma_1^2 / sigma; relative to sigma_1 the error is below sqrt(eps)
    assert np.max(np.abs(sigma - S)) <= 2e-8 * s1
    big = S > 1e-3 * s1
    assert np.max(np.abs(sigma - S)[big]) <= 1e-11 * s1
    # (the device routine's rank rule, on squares: see the header) applied to the oracle's singular values
    ref_rank = (S ** 2 > 64 * max(M, KK) * np.finfo(np.float64).eps * S[:, :1] ** 2).sum(axis=1)
    assert np.array_equal(rank, ref_rank), (rank, ref_rank)
    Wc = oracle.slices(W.astype(np.float64))                          # [C, M, KK]
    for c in range(C):
        r = int(ref_rank[c])
        Vc = v[c]                                                      # rows: v_i
        assert np.allclose(Vc @ Vc.T, np.eye(R), atol=1e-12)          # orthonormal (also inside a null space)
        G = Wc[c].T @ Wc[c]
        assert np.allclose(Vc @ G @ Vc.T, np.diag(sigma[c] ** 2), atol=1e-12 * max(s1 * s1, 1e-300))
        for i in range(r):                                             # sign convention, and the oracle's vectors
            k = int(np.argmax(np.abs(Vc[i])))
            assert Vc[i, k] > 0
            gap = min([abs(S[c, i] - S[c, j]) for j in range(R) if j != i] + [S[c, i]])
            if gap > 1e-6 * s1:
                assert np.allclose(Vc[i], Vt[c, i], atol=1e-7 * s1 / gap)


# ------------------------------------------------------------------------------------------
# backward pass through the layer's linear part (fine-tuning)
# ------------------------------------------------------------------------------------------

BACKWARD = [
    # N, C, H, W, M, K, stride, pad, g-rule
    (2, 16, 12, 12, 24, 3, 1, 1, "u13"),
    (3, 10, 9, 11, 7, 3, 2, 1, "u09"),       # stride 2, odd sizes, channels without filters
    (1, 6, 9, 9, 12, 5, 1, 2, "u13"),        # K = 5
    (2, 8, 8, 8, 20, 3, 2, 0, "u13"),        # no padding: the last row and column of x get no gradient
    (2, 12, 5, 5, 9, 1, 1, 0, "u13"),        # K = 1
    (4, 40, 16, 16, 48, 3, 1, 1, "u14"),     # several tiles of every kernel
]


@pytest.mark.gpu
@pytest.mark.parametrize("layout", ["nhwc", "nchw"])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("case", range(len(BACKWARD)))
def test_backward(case, dtype, layout):
    N, C, H, W, M, K, stride, pad, rule = BACKWARD[case]
    seed = 5200 + 10 * case
    g = _g(rule, C, seed)
    G = int(g.sum())
    Ho, Wo = _osz(H, K, stride, pad), _osz(W, K, stride, pad)
    x = rng.normal(seed, (N, C, H, W))
    dw = rng.normal(seed + 1, (G, K, K), std=0.3)
    pw = rng.normal(seed + 2, (M, G), std=0.3)
    dy = rng.normal(seed + 3, (N, M, Ho, Wo))
    desc = gd.make_desc(C, M, K, stride, pad, dtype, layout)
    plan = gd.gdws_plan(desc, g, dw=dw, pw=pw)
    dwq, pwq = gd.gdws_plan_factors(plan)
    xd, x_exact = to_device(x, dtype, layout)
    dyd, dy_exact = to_device(dy, dtype, layout)
    dx = empty_act(N, C, H, W, dtype, layout, fill=float("nan"))
    d_dw = torch.full((G, K, K), float("nan"), dtype=torch.float32, device="cuda")
    d_pw = torch.full((M, G), float("nan"), dtype=torch.float32, device="cuda")
    d_b = torch.full((M,), float("nan"), dtype=torch.float32, device="cuda")
    nbytes = gd.gdws_backward_workspace_bytes(plan, N, H, W)
    assert nbytes >= 2 * N * G * Ho * Wo * 4
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    with pytest.raises(gd.GdwsError):
        gd.gdws_backward(plan, xd, dyd, N, H, W, dx=dx, workspace=ws[:nbytes - 4])
    gd.gdws_backward(plan, xd, dyd, N, H, W, dx=dx, d_dw=d_dw, d_pw=d_pw, d_bias=d_b, workspace=ws)
    torch.cuda.synchronize()
    rdx, rdD, rdP, rdb = oracle.gdws_backward(x_exact, g, dwq, pwq, dy_exact, stride, pad)
    # weight gradients: fp32 sums of exact products of the (rounded) inputs; dx is rounded to the storage type
    for got, ref in ((d_dw, rdD), (d_pw, rdP), (d_b, rdb)):
        got = got.cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all()
        assert rel_l2(got, ref) <= 1e-5
    dxh = from_device(dx, dtype, layout)
    assert np.isfinite(dxh).all()
    assert rel_l2(dxh, rdx) <= TOL[dtype]
    # element by element: fp32 accumulation of the sums' absolute terms, plus the storage rounding of dx
    a_dx, a_dD, a_dP, a_db = oracle.gdws_backward(np.abs(x_exact), g, np.abs(dwq), np.abs(pwq), np.abs(dy_exact), stride, pad)
    terms = N * Ho * Wo + G * K * K + M
    ulp = {"f32": 2.0 ** -24, "f16": 2.0 ** -11, "bf16": 2.0 ** -8}[dtype]
    assert (np.abs(d_dw.cpu().numpy() - rdD) <= terms * 2.0 ** -23 * a_dD + 1e-30).all()
    assert (np.abs(d_pw.cpu().numpy() - rdP) <= terms * 2.0 ** -23 * a_dP + 1e-30).all()
    assert (np.abs(dxh - rdx) <= terms * 2.0 ** -23 * a_dx + ulp * 1.01 * np.abs(rdx) + 1e-30).all()
    # a second call that asks for dx only leaves the other buffers alone
    d_pw.fill_(7.0)
    gd.gdws_backward(plan, xd, dyd, N, H, W, dx=dx, workspace=ws)
    torch.cuda.synchronize()
    assert (d_pw == 7.0).all() and (from_device(dx, dtype, layout) == dxh).all()


@pytest.mark.gpu
def test_split_launch_needs_its_workspace_and_matches_the_unsplit_one():
    """A batch-1 deep layer: with the workspace the fused path asks for, the launch is split over row blocks; without
    it the same call still works (unsplit).  Both agree with the oracle; the split one is repeatable bit for bit."""
    N, C, H, W, M = 1, 512, 4, 4, 512
    g = _g("u14", C, 6100)
    G = int(g.sum())
    x = rng.normal(6101, (N, C, H, W))
    dw = rng.normal(6102, (G, 3, 3), std=0.2)
    pw = rng.normal(6103, (M, G), std=0.2)
    b = rng.normal(6104, (M,), std=0.1)
    plan = gd.gdws_plan(gd.make_desc(C, M, 3, 1, 1, "bf16", "nhwc", True, True, False), g, dw=dw, pw=pw, bias=b)
    nbytes = gd.gdws_workspace_bytes(plan, N, H, W, gd.MODE_FUSED)
    assert nbytes > 0 and nbytes == gd.gdws_workspace_bytes(plan, N, H, W, gd.MODE_AUTO)
    assert gd.gdws_workspace_bytes(plan, 256, H, W, gd.MODE_FUSED) == 0          # a full batch is not split
    xd, x_exact = to_device(x, "bf16", "nhwc")
    dwq, pwq = gd.gdws_plan_factors(plan)
    ref = oracle.gdws_forward(x_exact, g, dwq, pwq, b, None, True, 1, 1)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    outs = []
    for workspace in (ws, ws, None, ws[: nbytes - 16]):
        y = empty_act(N, M, H, W, "bf16", "nhwc", fill=float("nan"))
        gd.gdws_forward(plan, xd, y, N, H, W, workspace=workspace, mode=gd.MODE_FUSED)
        torch.cuda.synchronize()
        outs.append(from_device(y, "bf16", "nhwc"))
        assert np.isfinite(outs[-1]).all() and rel_l2(outs[-1], ref) <= TOL["bf16"]
    assert (outs[0] == outs[1]).all()
    assert (outs[2] == outs[3]).all()                                            # both unsplit
    assert rel_l2(outs[0], outs[2]) <= 4e-3                                       # same sums in another order


@pytest.mark.gpu
def test_error_codes_of_the_later_entry_points():
    """gdws_singular_values_device and gdws_backward refuse what they cannot do, with the documented codes."""
    w = torch.zeros(4, 2, 9, 9, dtype=torch.float32, device="cuda")
    sigma = torch.zeros(2, 4, dtype=torch.float64, device="cuda")
    with pytest.raises(gd.GdwsError) as e:
        gd.gdws_singular_values_device(w, sigma)                    # K = 9: beyond the kernel's 7 x 7
    assert e.value.code == -3
    with pytest.raises(gd.GdwsError) as e:
        gd.gdws_singular_values_device(w[:, :, :3, :3].contiguous(), None)
    assert e.value.code == -2
    g = np.ones(8, np.int32)
    plan = gd.gdws_plan(gd.make_desc(8, 16, 3, 1, 1, "f16", "nhwc"), g, dw=np.ones((8, 3, 3), np.float32),
                        pw=np.ones((16, 8), np.float32))
    x = torch.zeros(1, 6, 6, 8, device="cuda", dtype=torch.float16)
    dy = torch.zeros(1, 6, 6, 16, device="cuda", dtype=torch.float16)
    ws = torch.empty(gd.gdws_backward_workspace_bytes(plan, 1, 6, 6), dtype=torch.uint8, device="cuda")
    with pytest.raises(gd.GdwsError) as e:
        gd.gdws_backward(plan, x, None, 1, 6, 6, dx=torch.empty_like(x), workspace=ws)
    assert e.value.code == -2
    with pytest.raises(gd.GdwsError) as e:
        gd.gdws_backward(plan, x, dy, 1, 6, 6, dx=torch.empty_like(x), workspace=None)
    assert e.value.code == -4
    with pytest.raises(gd.GdwsError) as e:
        gd.gdws_backward(plan, x, dy, 0, 6, 6, dx=torch.empty_like(x), workspace=ws)
    assert e.value.code == -1
    assert gd.gdws_backward_workspace_bytes(plan, 0, 6, 6) == 0
    gd.gdws_backward(plan, x, dy, 1, 6, 6, workspace=ws)              # nothing asked for: still a valid call
    torch.cuda.synchronize()


# layers with three to nine filters per channel: the plan takes the depthwise stage with two taps per MFMA (8-channel
# windows).  256- and 128-pixel tiles, 64- and 128-channel workgroups, with and without loader waves, one and several
# input stages, stride 2, four-pixel tile rows, ragged sizes, channels with no filter in between.
TWO_TAP = [(3, 128, 16, 16, 128, 1, "u39"), (2, 64, 32, 32, 64, 1, "u35"), (2, 32, 17, 19, 40, 1, "u39"),
           (2, 256, 8, 8, 256, 1, "u36"), (2, 64, 12, 12, 96, 2, "u39"), (70, 64, 4, 4, 256, 1, "u39"),
           (2100, 16, 4, 4, 32, 1, "u39"), (1, 136, 10, 12, 136, 1, "u09"), (5, 24, 9, 9, 72, 2, "u39"),
           (300, 64, 8, 8, 64, 1, "all9")]


@pytest.mark.gpu
@pytest.mark.parametrize("residual", [False, True])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("case", range(len(TWO_TAP)))
def test_two_tap_layers(case, dtype, residual):
    N, C, H, W, M, stride, rule = TWO_TAP[case]
    g = _g(rule, C, 5300 + case)
    check_layer(5310 + 10 * case, N, C, H, W, M, 3, stride, 1, g, dtype, "nhwc", gd.MODE_FUSED, bias=True,
                residual=residual, relu=(case % 2 == 0))


@pytest.mark.gpu
def test_one_plan_on_two_streams_at_once():
    """A plan is immutable: forwards on different streams with their own buffers may overlap.  Same results, bit for
    bit, as one after the other (general kernel, deep-layer kernel and its split launch with separate workspaces)."""
    for (N, C, H, W, M) in ((64, 128, 16, 16, 128), (48, 512, 4, 4, 512), (1, 512, 4, 4, 512)):
        g = _g("u14", C, 6200)
        G = int(g.sum())
        dw = rng.normal(6201, (G, 3, 3), std=0.2)
        pw = rng.normal(6202, (M, G), std=0.2)
        plan = gd.gdws_plan(gd.make_desc(C, M, 3, 1, 1, "bf16", "nhwc", True), g, dw=dw, pw=pw)
        nbytes = max(1, gd.gdws_workspace_bytes(plan, N, H, W, gd.MODE_FUSED))
        xs = [to_device(rng.normal(6210 + k, (N, C, H, W)), "bf16", "nhwc")[0] for k in range(2)]
        wss = [torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(2)]
        seq = []
        for k in range(2):
            y = empty_act(N, M, H, W, "bf16", "nhwc", fill=float("nan"))
            gd.gdws_forward(plan, xs[k], y, N, H, W, workspace=wss[k], mode=gd.MODE_FUSED)
            torch.cuda.synchronize()
            seq.append(y.clone())
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        ys = [empty_act(N, M, H, W, "bf16", "nhwc", fill=float("nan")) for _ in range(2)]
        torch.cuda.synchronize()
        for rep in range(20):                      # interleaved launches: the two streams' kernels overlap on the chip
            for k in range(2):
                gd.gdws_forward(plan, xs[k], ys[k], N, H, W, workspace=wss[k], mode=gd.MODE_FUSED, stream=streams[k])
        for st in streams:
            st.synchronize()
        for k in range(2):
            assert torch.equal(ys[k].view(torch.int16), seq[k].view(torch.int16))
