"""The entry point that allocates nothing (the intermediate in the library's static device array) against
gdws_forward in its unfused mode: same kernels, same bits.  Two calls in a row share the array, the second with a
smaller input; a layer whose intermediate exceeds the array is refused."""
import numpy as np
import pytest
import torch

import oracle
import paper_2110_14871_amd as gd
from workloads import rng

from gpu_util import TOL, empty_act, from_device, rel_l2, to_device

pytestmark = pytest.mark.gpu


def _layer(seed, N, C, H, W, M, g, dtype, layout, residual):
    G = int(g.sum())
    x = rng.normal(seed, (N, C, H, W))
    dw = rng.normal(seed + 1, (G, 3, 3), std=0.2)
    pw = rng.normal(seed + 2, (M, G), std=0.2)
    b = rng.normal(seed + 3, (M,), std=0.1)
    r = rng.normal(seed + 4, (N, M, H, W)) if residual else None
    desc = gd.make_desc(C, M, 3, 1, 1, dtype, layout, True, True, residual)
    plan = gd.gdws_plan(desc, g, dw=dw, pw=pw, bias=b)
    xd, x_exact = to_device(x, dtype, layout)
    rd, r_exact = (None, None) if r is None else to_device(r, dtype, layout)
    return plan, xd, rd, dict(x=x_exact, r=r_exact, b=b, g=g)


@pytest.mark.parametrize("dtype,layout", [("bf16", "nhwc"), ("f16", "nchw"), ("f32", "nchw")])
def test_static_scratch_forward_two_calls(dtype, layout):
    out = []
    # a layer with several tiles, then a smaller one: the second call finds the first call's intermediate in the array
    for seed, N, C, H, W, M, residual in ((3000, 5, 64, 16, 16, 128, True), (3010, 2, 24, 9, 7, 40, False)):
        g = rng.uniform_int(seed + 9, (C,), 1, 4)
        plan, xd, rd, ex = _layer(seed, N, C, H, W, M, g, dtype, layout, residual)
        y0 = empty_act(N, M, H, W, dtype, layout, fill=float("nan"))
        y1 = empty_act(N, M, H, W, dtype, layout, fill=float("nan"))
        ws = torch.empty(gd.gdws_workspace_bytes(plan, N, H, W, gd.MODE_UNFUSED), dtype=torch.uint8, device="cuda")
        assert 0 < ws.numel() <= gd.STATIC_SCRATCH_BYTES
        out.append((plan, xd, rd, ex, y0, y1, ws, (N, H, W)))
    for plan, xd, rd, ex, y0, y1, ws, (N, H, W) in out:
        gd.gdws_forward(plan, xd, y0, N, H, W, residual=rd, workspace=ws, mode=gd.MODE_UNFUSED)
    torch.cuda.synchronize()
    for plan, xd, rd, ex, y0, y1, ws, (N, H, W) in out:          # the two calls in a row, on one stream
        gd.gdws_forward_static(plan, xd, y1, N, H, W, residual=rd)
    torch.cuda.synchronize()
    for plan, xd, rd, ex, y0, y1, ws, (N, H, W) in out:
        a, b = from_device(y0, dtype, layout), from_device(y1, dtype, layout)
        assert np.isfinite(b).all() and (a == b).all()
        dw, pw = gd.gdws_plan_factors(plan)
        ref = oracle.gdws_forward(ex["x"], ex["g"], dw, pw, ex["b"], ex["r"], True, 1, 1, threads=8)
        assert rel_l2(b, ref) <= TOL[dtype]


def test_static_scratch_forward_refuses_what_does_not_fit():
    g = np.full(64, 9, np.int32)
    plan = gd.gdws_plan(gd.make_desc(64, 32, 3, 1, 1, "bf16", "nhwc"), g, dw=np.ones((576, 3, 3), np.float32),
                        pw=np.ones((32, 576), np.float32))
    N, H, W = 64, 32, 32                                   # 64 x 576 x 1024 x 2 bytes = 72 MiB > 64 MiB
    assert gd.gdws_workspace_bytes(plan, N, H, W, gd.MODE_UNFUSED) > gd.STATIC_SCRATCH_BYTES
    x = torch.zeros(N, H, W, 64, device="cuda", dtype=torch.bfloat16)
    y = torch.zeros(N, H, W, 32, device="cuda", dtype=torch.bfloat16)
    with pytest.raises(gd.GdwsError) as e:
        gd.gdws_forward_static(plan, x, y, N, H, W)
    assert e.value.code == -4
    with pytest.raises(gd.GdwsError) as e:
        gd.gdws_forward_static(plan, x, y, 0, H, W)
    assert e.value.code == -1
    gd.gdws_forward_static(plan, x, y, 8, H, W)            # a batch that fits runs
    torch.cuda.synchronize()
    assert float(y[:8].float().abs().sum()) == 0.0
