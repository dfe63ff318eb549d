"""Shape descriptors and tensor recipes for the five benchmark workloads.

These stand in for the image-classification workloads the paper measures
(32x32 and 224x224 inputs through VGG-16 / ResNet-18 / ResNet-50 shaped
stacks): only the shapes, value distributions and per-channel multiplier
distributions are reproduced; every tensor is drawn from `workloads.rng`.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from . import rng


@dataclass
class LayerShape:
    """One node of a feed-forward network graph (NCHW semantics).

    kind      "gdws" (KxK conv given as depthwise+pointwise factors),
              "dense" (ordinary conv) or "maxpool".
    src       index of the layer whose output feeds this one, -1 = network input.
    residual  index of a layer whose output is added before the ReLU, or None.
    """
    kind: str
    C: int
    M: int
    K: int
    stride: int = 1
    pad: int = 0
    relu: bool = True
    bias: bool = True
    src: int = -1
    residual: Optional[int] = None
    seed: int = 0
    g_rule: str = ""          # how g is drawn for "gdws" layers (see draw_g)
    H: int = 0                # input spatial size (filled by the builders)
    W: int = 0

    @property
    def Ho(self):
        return (self.H + 2 * self.pad - self.K) // self.stride + 1

    @property
    def Wo(self):
        return (self.W + 2 * self.pad - self.K) // self.stride + 1


def he_weight(seed, M, C, K):
    """[M, C, K, K] fp32, N(0, 2 / (C K^2)) -- He initialisation."""
    return rng.normal(seed, (M, C, K, K), std=float(np.sqrt(2.0 / (C * K * K))))


def small_bias(seed, M):
    """[M] fp32, N(0, 0.05^2): stands in for a folded batch-norm shift."""
    return rng.normal(seed, (M,), std=0.05)


def pruned_weight(seed, M, C, K, keep=0.02):
    """[M, C, K, K] fp32: a He-initialised weight with all but a fraction `keep` of its entries set to zero.

    Stands in for an unstructured-pruned layer (the paper prunes to 90 - 99 % sparsity): the surviving
    entries are scattered, so no filter is all zero, yet every M x K^2 slice has few non-zero columns.
    """
    W = he_weight(seed, M, C, K)
    u = rng.bits64(seed + 1, 0, W.size).astype(np.float64) / 2.0 ** 64
    return (W * (u.reshape(W.shape) < keep)).astype(np.float32)


def skewed_g(seed, C, gamma, cap=9, p=0.5):
    """int32[C] with sum exactly gamma: geometric(p) draws clipped to [1, cap], then adjusted.

    Adjustment walks a seeded random channel order, adding (or removing) one
    filter at a time from channels that still have room, until the sum matches.
    """
    g = np.minimum(rng.geometric(seed, (C,), p), cap).astype(np.int64)
    order = np.argsort(rng.bits64(seed + 7919, 0, C), kind="stable")
    i = 0
    guard = 0
    while g.sum() != gamma:
        c = order[i % C]
        if g.sum() < gamma and g[c] < cap:
            g[c] += 1
        elif g.sum() > gamma and g[c] > 1:
            g[c] -= 1
        i += 1
        guard += 1
        if guard > 64 * C * cap:
            raise ValueError("gamma unreachable with 1 <= g_c <= cap")
    return g.astype(np.int32)


def draw_g(layer: LayerShape, budget_gamma=None):
    """Per-channel multipliers for a "gdws" layer according to its g_rule.

    The "skewed:rho" rule needs the total multiplier that a fraction rho of the dense layer's
    MACs allows; that figure is the method's arithmetic, so the caller supplies it as
    budget_gamma(rho, C, K, M) (the library's planner on the GPU side, the oracle on the CPU side).
    """
    cap = min(layer.K * layer.K, layer.M)
    rule = layer.g_rule
    if rule.startswith("uniform"):           # "uniform:lo:hi"
        _, lo, hi = rule.split(":")
        return np.minimum(rng.uniform_int(layer.seed + 2, (layer.C,), int(lo), int(hi)), cap).astype(np.int32)
    if rule.startswith("skewed"):            # "skewed:rho"
        rho = float(rule.split(":")[1])
        if budget_gamma is None:
            raise ValueError("the skewed rule needs the caller's budget_gamma(rho, C, K, M)")
        return skewed_g(layer.seed + 2, layer.C, int(budget_gamma(rho, layer.C, layer.K, layer.M)), cap=cap)
    raise ValueError(rule)


def layer_tensors(layer: LayerShape):
    """(W fp32 [M,C,K,K], bias fp32 [M] or None) for a conv layer."""
    W = he_weight(layer.seed, layer.M, layer.C, layer.K)
    b = small_bias(layer.seed + 1, layer.M) if layer.bias else None
    return W, b


# --------------------------------------------------------------------------
# single-layer workloads
# --------------------------------------------------------------------------

def config1():
    """Small fp32 layer: X [1,16,32,32] ~ N(0,1), W [32,16,3,3] ~ N(0, 0.1^2), g_c ~ U{1,2,3}."""
    X = rng.normal(1, (1, 16, 32, 32))
    W = rng.normal(2, (32, 16, 3, 3), std=0.1)
    g = rng.uniform_int(3, (16,), 1, 3)
    return dict(N=1, C=16, H=32, W=32, M=32, K=3, stride=1, pad=1, dtype="f32", X=X, Wt=W, g=g)


def config2(N=256):
    """bf16 layer: X [N,128,16,16] ~ N(0,1), W [128,128,3,3] ~ N(0, 0.05^2); g is chosen by the caller.

    The caller derives g from the singular values of W for a 25 % MAC budget
    (`rho`; the total multiplier that budget allows is 269), or uses the
    all-9 / all-1 edge cases.
    """
    X = rng.normal(11, (N, 128, 16, 16))
    W = rng.normal(12, (128, 128, 3, 3), std=0.05)
    return dict(N=N, C=128, H=16, W=16, M=128, K=3, stride=1, pad=1, dtype="bf16", X=X, Wt=W,
                rho=0.25)


# --------------------------------------------------------------------------
# network-shaped workloads
# --------------------------------------------------------------------------

def _finish(layers: List[LayerShape], H, W):
    """Fill each layer's input spatial size by walking the graph."""
    sizes = []
    for l in layers:
        h, w = (H, W) if l.src < 0 else sizes[l.src]
        l.H, l.W = h, w
        sizes.append((l.Ho, l.Wo))
    return layers


def vgg16_shape(H=32, W=32, seed0=21):
    """13 3x3 convs (all GDWS, g_c ~ U{1..4}) with ReLU, 2x2/2 max-pool after convs 2, 4, 7, 10, 13."""
    chans = [64, 64, "P", 128, 128, "P", 256, 256, 256, "P", 512, 512, 512, "P", 512, 512, 512, "P"]
    layers, c, idx = [], 3, 0
    for v in chans:
        src = len(layers) - 1
        if v == "P":
            layers.append(LayerShape("maxpool", c, c, 2, 2, 0, relu=False, bias=False, src=src))
        else:
            layers.append(LayerShape("gdws", c, v, 3, 1, 1, relu=True, bias=True, src=src,
                                     seed=1000 * (seed0 + idx), g_rule="uniform:1:4"))
            c = v
            idx += 1
    return _finish(layers, H, W)


def resnet18_shape(H=32, W=32, seed0=31, rho=0.4):
    """3x3 stem + 4 stages x 2 basic blocks (64/128/256/512); every 3x3 is GDWS on a rho MAC budget.

    Post-activation form with folded batch norm: out = relu(conv2(relu(conv1(x))) + shortcut(x)),
    shortcut = identity, or a dense 1x1 stride-2 projection where the shape changes.
    """
    layers, idx = [], 0

    def gd(C, M, s, src, relu, residual=None):
        nonlocal idx
        layers.append(LayerShape("gdws", C, M, 3, s, 1, relu=relu, bias=True, src=src, residual=residual,
                                 seed=1000 * (seed0 + idx), g_rule=f"skewed:{rho}"))
        idx += 1
        return len(layers) - 1

    cur = gd(3, 64, 1, -1, True)
    c = 64
    for width, stride in [(64, 1), (128, 2), (256, 2), (512, 2)]:
        for b in range(2):
            s = stride if b == 0 else 1
            if s != 1 or c != width:
                layers.append(LayerShape("dense", c, width, 1, s, 0, relu=False, bias=True, src=cur,
                                         seed=1000 * (seed0 + idx) + 500))
                short = len(layers) - 1
            else:
                short = cur
            a = gd(c, width, s, cur, True)
            cur = gd(width, width, 1, a, True, residual=short)
            c = width
    return _finish(layers, H, W)


def wrn28_4_shape(H=32, W=32, seed0=61, rho=0.4):
    """WideResNet-28-4: 3x3 stem (3 -> 16), three groups of four basic blocks of widths 64 / 128 / 256 (stride 2
    entering groups 2 and 3), dense 1x1 projection shortcuts where the shape changes: 25 3x3 convolutions, all
    GDWS on a rho MAC budget with the skewed per-channel draw, plus three 1x1 convolutions.  Same post-activation
    form with folded batch norm as the ResNet-18 shape."""
    layers, idx = [], 0

    def gd(C, M, s, src, relu, residual=None):
        nonlocal idx
        layers.append(LayerShape("gdws", C, M, 3, s, 1, relu=relu, bias=True, src=src, residual=residual,
                                 seed=1000 * (seed0 + idx), g_rule=f"skewed:{rho}"))
        idx += 1
        return len(layers) - 1

    cur = gd(3, 16, 1, -1, True)
    c = 16
    for width, stride in [(64, 1), (128, 2), (256, 2)]:
        for b in range(4):
            s = stride if b == 0 else 1
            if s != 1 or c != width:
                layers.append(LayerShape("dense", c, width, 1, s, 0, relu=False, bias=True, src=cur,
                                         seed=1000 * (seed0 + idx) + 500))
                short = len(layers) - 1
            else:
                short = cur
            a = gd(c, width, s, cur, True)
            cur = gd(width, width, 1, a, True, residual=short)
            c = width
    return _finish(layers, H, W)


def resnet50_shape(H=224, W=224, seed0=41):
    """7x7/2 dense stem, 3x3/2 max-pool, bottlenecks [3,4,6,3]; 1x1 convs dense, 3x3 convs GDWS with g_c ~ U{1..9}."""
    layers, idx = [], 0

    def conv(kind, C, M, K, s, p, src, relu, residual=None):
        nonlocal idx
        layers.append(LayerShape(kind, C, M, K, s, p, relu=relu, bias=True, src=src, residual=residual,
                                 seed=1000 * (seed0 + idx), g_rule="uniform:1:9" if kind == "gdws" else ""))
        idx += 1
        return len(layers) - 1

    cur = conv("dense", 3, 64, 7, 2, 3, -1, True)
    layers.append(LayerShape("maxpool", 64, 64, 3, 2, 1, relu=False, bias=False, src=cur))
    cur = len(layers) - 1
    c = 64
    for width, blocks, stride in [(64, 3, 1), (128, 4, 2), (256, 6, 2), (512, 3, 2)]:
        for b in range(blocks):
            s = stride if b == 0 else 1
            if b == 0:
                short = conv("dense", c, 4 * width, 1, s, 0, cur, False)
            else:
                short = cur
            a = conv("dense", c, width, 1, 1, 0, cur, True)
            a = conv("gdws", width, width, 3, s, 1, a, True)
            cur = conv("dense", width, 4 * width, 1, 1, 0, a, True, residual=short)
            c = 4 * width
    return _finish(layers, H, W)
