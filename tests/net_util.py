"""Builds a gdws network object (and the matching oracle parameters) from a list of workloads.LayerShape nodes."""
import workloads
import paper_2110_14871_amd as gd
from gpu_util import quantise


def build_network(shapes, dtype, layout):
    layers, params = [], []
    for l in shapes:
        if l.kind == "gdws":
            W, b = workloads.configs.layer_tensors(l)
            g = workloads.configs.draw_g(l, gd.gdws_budget_gamma)
            desc = gd.make_desc(l.C, l.M, l.K, l.stride, l.pad, dtype, layout, l.relu, l.bias, l.residual is not None)
            plan = gd.gdws_plan(desc, g, W=W, bias=b)
            dw, pw = gd.gdws_plan_factors(plan)
            layers.append(dict(kind=gd.LAYER_GDWS, src=l.src, residual=l.residual, plan=plan))
            params.append(dict(g=g, D=dw, Pw=pw, bias=b))
        elif l.kind == "dense":
            W, b = workloads.configs.layer_tensors(l)
            desc = gd.make_desc(l.C, l.M, l.K, l.stride, l.pad, dtype, layout, l.relu, l.bias, l.residual is not None)
            layers.append(dict(kind=gd.LAYER_DENSE, src=l.src, residual=l.residual, desc=desc, w=W, bias=b))
            params.append(dict(W=quantise(W, dtype), bias=b))
        else:
            desc = gd.make_desc(l.C, l.C, l.K, l.stride, l.pad, dtype, layout)
            layers.append(dict(kind=gd.LAYER_MAXPOOL, src=l.src, residual=None, desc=desc))
            params.append({})
    return gd.gdws_net_create(layers), params
