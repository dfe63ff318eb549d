"""ctypes binding of libgdws: the same entry points as include/gdws.h, argument marshalling only.

Device tensors are torch tensors (used for their memory and streams only); host
arrays are numpy.  Every function raises GdwsError on a non-zero status.  There
is no CPU fallback: if the shared library is missing the import fails.
"""
import ctypes
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libgdws.so")

F32, F16, BF16 = 0, 1, 2
NCHW, NHWC = 0, 1
MODE_AUTO, MODE_FUSED, MODE_UNFUSED = 0, 1, 2
LAYER_GDWS, LAYER_DENSE, LAYER_MAXPOOL = 0, 1, 2
DTYPES = {"f32": F32, "f16": F16, "bf16": BF16}
LAYOUTS = {"nchw": NCHW, "nhwc": NHWC}


class GdwsError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {lib().gdws_strerror(code).decode()} ({code})")


class LayerDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("C", "M", "K", "stride", "pad", "dtype", "layout", "relu", "has_bias", "has_residual")]


class NetLayer(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("src", ctypes.c_int32), ("residual", ctypes.c_int32),
                ("plan", ctypes.c_void_p), ("desc", LayerDesc), ("w", ctypes.c_void_p), ("bias", ctypes.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2110_14871_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t, ctypes.c_double
        pdesc = ctypes.POINTER(LayerDesc)
        sig = {
            "gdws_strerror": (ctypes.c_char_p, [ctypes.c_int]),
            "gdws_singular_values": (ctypes.c_int, [vp, i32, i32, i32, vp, vp]),
            "gdws_singular_values_device": (ctypes.c_int, [vp, i32, i32, i32, vp, vp, vp, vp]),
            "gdws_mego": (ctypes.c_int, [vp, vp, i32, i32, vp, i64, i32, vp]),
            "gdws_lego": (ctypes.c_int, [vp, vp, i32, i32, vp, dbl, i32, i32, vp]),
            "gdws_budget_gamma": (i64, [dbl, i32, i32, i32]),
            "gdws_compact_factors": (ctypes.c_int, [i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]),
            "gdws_plan_sparse": (ctypes.c_int, [pdesc, vp, vp, vp, vp, vp, ctypes.POINTER(vp)]),
            "gdws_plan": (ctypes.c_int, [pdesc, vp, vp, vp, vp, vp, ctypes.POINTER(vp)]),
            "gdws_plan_destroy": (ctypes.c_int, [vp]),
            "gdws_plan_info": (ctypes.c_int, [vp, ctypes.POINTER(i32), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                              ctypes.POINTER(i64)]),
            "gdws_plan_factors": (ctypes.c_int, [vp, vp, vp]),
            "gdws_intermediate_channels": (i32, [vp]),
            "gdws_workspace_bytes": (sz, [vp, i32, i32, i32, ctypes.c_int]),
            "gdws_forward": (ctypes.c_int, [vp, vp, vp, vp, i32, i32, i32, vp, sz, ctypes.c_int, vp]),
            "gdws_forward_maxpool2": (ctypes.c_int, [vp, vp, vp, i32, i32, i32, vp]),
            "gdws_forward_static": (ctypes.c_int, [vp, vp, vp, vp, i32, i32, i32, vp]),
            "gdws_gdw_forward": (ctypes.c_int, [vp, vp, vp, i32, i32, i32, vp]),
            "gdws_pw_forward": (ctypes.c_int, [vp, vp, vp, vp, i32, i32, i32, vp]),
            "gdws_backward_workspace_bytes": (sz, [vp, i32, i32, i32]),
            "gdws_backward": (ctypes.c_int, [vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, vp, sz, vp]),
            "conv_dense_workspace_bytes": (sz, [pdesc]),
            "conv_dense_forward": (ctypes.c_int, [pdesc, vp, vp, vp, vp, vp, i32, i32, i32, vp, sz, vp]),
            "gdws_net_create": (ctypes.c_int, [ctypes.POINTER(NetLayer), i32, ctypes.POINTER(vp)]),
            "gdws_net_destroy": (ctypes.c_int, [vp]),
            "gdws_net_workspace_bytes": (sz, [vp, i32, i32, i32]),
            "gdws_network_forward": (ctypes.c_int, [vp, vp, vp, i32, i32, i32, vp, sz, vp]),
            "gdws_capture_begin": (ctypes.c_int, [vp]),
            "gdws_capture_end": (ctypes.c_int, [vp, ctypes.POINTER(vp)]),
            "gdws_graph_launch": (ctypes.c_int, [vp, vp]),
            "gdws_graph_destroy": (ctypes.c_int, [vp]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


EXPORTS = ("gdws_strerror", "gdws_singular_values", "gdws_singular_values_device", "gdws_mego", "gdws_lego", "gdws_budget_gamma",
           "gdws_compact_factors", "gdws_plan_sparse", "gdws_plan", "gdws_plan_destroy",
           "gdws_plan_info", "gdws_plan_factors", "gdws_intermediate_channels", "gdws_workspace_bytes", "gdws_forward",
           "gdws_forward_maxpool2", "gdws_forward_static", "gdws_gdw_forward",
           "gdws_pw_forward", "gdws_backward_workspace_bytes", "gdws_backward", "conv_dense_workspace_bytes", "conv_dense_forward", "gdws_net_create",
           "gdws_net_destroy", "gdws_net_workspace_bytes", "gdws_network_forward", "gdws_capture_begin",
           "gdws_capture_end", "gdws_graph_launch", "gdws_graph_destroy")


def _check(code, where):
    if code != 0:
        raise GdwsError(code, where)


def _host(a, dtype):
    """(array kept alive, pointer) for an optional host array."""
    if a is None:
        return None, None
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _dev(t):
    """Device pointer of an optional torch tensor (must be contiguous and on the GPU)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("device tensors must be contiguous GPU tensors")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    return ctypes.c_void_p(stream if isinstance(stream, int) else stream.cuda_stream)


def make_desc(C, M, K, stride=1, pad=0, dtype="f32", layout="nchw", relu=False, has_bias=False, has_residual=False):
    return LayerDesc(C, M, K, stride, pad, DTYPES[dtype] if isinstance(dtype, str) else dtype,
                     LAYOUTS[layout] if isinstance(layout, str) else layout, int(relu), int(has_bias),
                     int(has_residual))


# ---- construction -----------------------------------------------------------------

def gdws_singular_values(W):
    """(sigma float64 [C, R], rank int32 [C]) of the per-channel slices of W [M, C, K, K]."""
    Wk, wp = _host(W, np.float32)
    M, C, K, _ = Wk.shape
    R = min(M, K * K)
    sigma = np.zeros((C, R), dtype=np.float64)
    rank = np.zeros(C, dtype=np.int32)
    _check(lib().gdws_singular_values(wp, M, C, K, sigma.ctypes.data_as(ctypes.c_void_p),
                                      rank.ctypes.data_as(ctypes.c_void_p)), "gdws_singular_values")
    return sigma, rank


def gdws_singular_values_device(w, sigma, rank=None, v=None, stream=None):
    """Device version: w float32 [M, C, K, K], sigma float64 [C, R], rank int32 [C], v float64 [C, R, K*K], all GPU tensors."""
    M, C, K, _ = w.shape
    _check(lib().gdws_singular_values_device(_dev(w), M, C, K, _dev(sigma), _dev(rank), _dev(v), _stream(stream)),
           "gdws_singular_values_device")


def gdws_mego(sigma, rank, gamma, alpha=None, g_init=None, cap=0):
    sk, sp = _host(sigma, np.float64)
    rk, rp = _host(rank, np.int32)
    ak, ap = _host(alpha, np.float64)
    C, R = sk.shape
    g = np.zeros(C, dtype=np.int32) if g_init is None else np.array(g_init, dtype=np.int32)
    _check(lib().gdws_mego(sp, rp, C, R, ap, int(gamma), int(cap), g.ctypes.data_as(ctypes.c_void_p)), "gdws_mego")
    return g


LEGO_THEOREM, LEGO_LISTING = 0, 1


def gdws_lego(sigma, rank, beta, alpha=None, g_min=0, compare=LEGO_THEOREM):
    sk, sp = _host(sigma, np.float64)
    rk, rp = _host(rank, np.int32)
    ak, ap = _host(alpha, np.float64)
    C, R = sk.shape
    g = np.zeros(C, dtype=np.int32)
    _check(lib().gdws_lego(sp, rp, C, R, ap, float(beta), int(g_min), int(compare),
                           g.ctypes.data_as(ctypes.c_void_p)), "gdws_lego")
    return g


def gdws_budget_gamma(rho, C, K, M):
    v = int(lib().gdws_budget_gamma(float(rho), C, K, M))
    _check(min(v, 0), "gdws_budget_gamma")
    return v


def gdws_compact_factors(g, dw, pw):
    """(g' int32 [C], dw' [G', K, K], pw' [M, G'], keep int32 [G']): the factors without their dead channels."""
    gk, gp = _host(g, np.int32)
    dk, dp = _host(dw, np.float32)
    pk, pp = _host(pw, np.float32)
    G, K = dk.shape[0], dk.shape[1]
    M = pk.shape[0]
    if pk.shape[1] != G or int(gk.sum()) != G:
        raise ValueError("g, dw [G, K, K] and pw [M, G] do not agree")
    g_out = np.zeros(len(gk), np.int32)
    dw_out, pw_out, keep = np.zeros((G, K, K), np.float32), np.zeros(M * G, np.float32), np.zeros(G, np.int32)
    vp = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    n = lib().gdws_compact_factors(len(gk), M, K, gp, dp, pp, vp(g_out), vp(dw_out), vp(pw_out), vp(keep))
    _check(min(n, 0), "gdws_compact_factors")
    return g_out, dw_out[:n].copy(), pw_out[:M * n].reshape(M, n).copy(), keep[:n].copy()


class Plan:
    """Owner of a gdws_plan_t handle."""

    def __init__(self, handle, desc):
        self.handle, self.desc = handle, desc

    def destroy(self):
        if self.handle:
            lib().gdws_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def gdws_plan(desc, g, W=None, dw=None, pw=None, bias=None, sparse=False):
    """sparse=True: gdws_plan_sparse (dead intermediate channels are dropped at plan time)."""
    gk, gp = _host(g, np.int32)
    if len(gk) != desc.C:
        raise ValueError("g must have C entries")
    Wk, wp = _host(W, np.float32)
    dk, dp = _host(dw, np.float32)
    pk, pp = _host(pw, np.float32)
    bk, bp = _host(bias, np.float32)
    G, KK = int(gk.sum()), desc.K * desc.K
    if Wk is not None and Wk.size != desc.M * desc.C * KK:
        raise ValueError("W must be [M, C, K, K]")
    if dk is not None and dk.size != G * KK:
        raise ValueError("dw must be [G, K, K]")
    if pk is not None and pk.size != desc.M * G:
        raise ValueError("pw must be [M, G]")
    if bk is not None and bk.size != desc.M:
        raise ValueError("bias must be [M]")
    h = ctypes.c_void_p()
    fn = lib().gdws_plan_sparse if sparse else lib().gdws_plan
    _check(fn(ctypes.byref(desc), gp, wp, dp, pp, bp, ctypes.byref(h)), "gdws_plan_sparse" if sparse else "gdws_plan")
    return Plan(h, desc)


def gdws_plan_destroy(plan):
    plan.destroy()


def gdws_plan_info(plan):
    """dict(G, offsets int32[C+1], chan_of int32[G], macs_per_pixel)."""
    G, off, co, macs = ctypes.c_int32(), ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_int64()
    _check(lib().gdws_plan_info(plan.handle, ctypes.byref(G), ctypes.byref(off), ctypes.byref(co),
                                ctypes.byref(macs)), "gdws_plan_info")
    offsets = np.ctypeslib.as_array(ctypes.cast(off, ctypes.POINTER(ctypes.c_int32)), (plan.desc.C + 1,)).copy()
    chan_of = np.ctypeslib.as_array(ctypes.cast(co, ctypes.POINTER(ctypes.c_int32)), (G.value,)).copy()
    return dict(G=G.value, offsets=offsets, chan_of=chan_of, macs_per_pixel=macs.value)


def gdws_plan_factors(plan):
    """(dw float32 [G, K, K], pw float32 [M, G]) as the kernels see them (rounded to the plan's dtype)."""
    G = gdws_plan_info(plan)["G"]
    d = plan.desc
    dw = np.zeros((G, d.K, d.K), dtype=np.float32)
    pw = np.zeros((d.M, G), dtype=np.float32)
    _check(lib().gdws_plan_factors(plan.handle, dw.ctypes.data_as(ctypes.c_void_p),
                                   pw.ctypes.data_as(ctypes.c_void_p)), "gdws_plan_factors")
    return dw, pw


# ---- forward ----------------------------------------------------------------------

def gdws_intermediate_channels(plan):
    return int(lib().gdws_intermediate_channels(plan.handle))


def gdws_workspace_bytes(plan, N, H, W, mode=MODE_AUTO):
    return int(lib().gdws_workspace_bytes(plan.handle, N, H, W, mode))


def gdws_forward(plan, x, y, N, H, W, residual=None, workspace=None, mode=MODE_AUTO, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().gdws_forward(plan.handle, _dev(x), _dev(residual), _dev(y), N, H, W, _dev(workspace), ws_bytes,
                              mode, _stream(stream)), "gdws_forward")


def gdws_forward_maxpool2(plan, x, y, N, H, W, stream=None):
    _check(lib().gdws_forward_maxpool2(plan.handle, _dev(x), _dev(y), N, H, W, _stream(stream)),
           "gdws_forward_maxpool2")


STATIC_SCRATCH_BYTES = 64 << 20


def gdws_forward_static(plan, x, y, N, H, W, residual=None, stream=None):
    _check(lib().gdws_forward_static(plan.handle, _dev(x), _dev(residual), _dev(y), N, H, W, _stream(stream)),
           "gdws_forward_static")


def gdws_gdw_forward(plan, x, t, N, H, W, stream=None):
    _check(lib().gdws_gdw_forward(plan.handle, _dev(x), _dev(t), N, H, W, _stream(stream)), "gdws_gdw_forward")


def gdws_pw_forward(plan, t, y, N, Ho, Wo, residual=None, stream=None):
    _check(lib().gdws_pw_forward(plan.handle, _dev(t), _dev(residual), _dev(y), N, Ho, Wo, _stream(stream)),
           "gdws_pw_forward")


def gdws_backward_workspace_bytes(plan, N, H, W):
    return lib().gdws_backward_workspace_bytes(plan.handle, N, H, W)


def gdws_backward(plan, x, dy, N, H, W, dx=None, d_dw=None, d_pw=None, d_bias=None, workspace=None, stream=None):
    """Gradients through the layer's linear part; the outputs given (GPU tensors) are filled, the others skipped."""
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().gdws_backward(plan.handle, _dev(x), _dev(dy), _dev(dx), _dev(d_dw), _dev(d_pw), _dev(d_bias), N, H, W,
                               _dev(workspace), nbytes, _stream(stream)), "gdws_backward")


def conv_dense_workspace_bytes(desc):
    return int(lib().conv_dense_workspace_bytes(ctypes.byref(desc)))


def conv_dense_forward(desc, w, x, y, N, H, W, bias=None, residual=None, workspace=None, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().conv_dense_forward(ctypes.byref(desc), _dev(w), _dev(bias), _dev(x), _dev(residual), _dev(y), N, H, W,
                                    _dev(workspace), ws_bytes, _stream(stream)), "conv_dense_forward")


# ---- networks ---------------------------------------------------------------------

class Net:
    """Owner of a gdws_net_t handle; keeps the plans it borrows alive."""

    def __init__(self, handle, plans):
        self.handle, self.plans = handle, plans

    def destroy(self):
        if self.handle:
            lib().gdws_net_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def gdws_net_create(layers):
    """layers: list of dicts {kind, src, residual (None = no residual), plan | (desc, w, bias) | desc}."""
    arr = (NetLayer * len(layers))()
    keep, plans = [], []
    for i, l in enumerate(layers):
        arr[i].kind = l["kind"]
        arr[i].src = l.get("src", i - 1)
        arr[i].residual = -2 if l.get("residual") is None else l["residual"]
        if l["kind"] == LAYER_GDWS:
            arr[i].plan = l["plan"].handle
            plans.append(l["plan"])
        else:
            arr[i].desc = l["desc"]
            wk, wp = _host(l.get("w"), np.float32)
            bk, bp = _host(l.get("bias"), np.float32)
            keep += [wk, bk]
            arr[i].w, arr[i].bias = wp, bp
    h = ctypes.c_void_p()
    _check(lib().gdws_net_create(arr, len(layers), ctypes.byref(h)), "gdws_net_create")
    return Net(h, plans)


def gdws_net_destroy(net):
    net.destroy()


def gdws_net_workspace_bytes(net, N, H, W):
    return int(lib().gdws_net_workspace_bytes(net.handle, N, H, W))


def gdws_network_forward(net, x, y, N, H, W, workspace=None, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().gdws_network_forward(net.handle, _dev(x), _dev(y), N, H, W, _dev(workspace), ws_bytes,
                                      _stream(stream)), "gdws_network_forward")


# ---- launch graphs ------------------------------------------------------------------

class Graph:
    """Owner of a gdws_graph_t handle."""

    def __init__(self, handle):
        self.handle = handle

    def destroy(self):
        if self.handle:
            lib().gdws_graph_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def gdws_capture_begin(stream):
    _check(lib().gdws_capture_begin(_stream(stream)), "gdws_capture_begin")


def gdws_capture_end(stream):
    h = ctypes.c_void_p()
    _check(lib().gdws_capture_end(_stream(stream), ctypes.byref(h)), "gdws_capture_end")
    return Graph(h)


def gdws_graph_launch(graph, stream=None):
    _check(lib().gdws_graph_launch(graph.handle, _stream(stream)), "gdws_graph_launch")


def gdws_graph_destroy(graph):
    graph.destroy()
