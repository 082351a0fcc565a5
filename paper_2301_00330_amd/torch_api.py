"""Tensor-level convenience layer over ``binding``: allocates outputs and the
workspace with torch on the tensor's device and enqueues on torch's current
stream.  Plumbing only -- every arithmetic step runs inside libgf.so."""
from __future__ import annotations

import torch

from . import binding as B
from .workloads import Layer


def desc_for(layer: Layer, N: int, r: int, dtype: str) -> B.ConvDesc:
    return B.ConvDesc(N=N, C_in=layer.C_in, C_out=layer.C_out, H_in=layer.H, W_in=layer.W,
                      K_h=layer.K, K_w=layer.K, stride=layer.stride, pad=layer.pad,
                      dilation=layer.dilation, groups=layer.groups, r=r,
                      dtype=B.GF_BF16 if dtype == "bf16" else B.GF_F32)


def _tdtype(d: B.ConvDesc):
    return torch.bfloat16 if d.dtype == B.GF_BF16 else torch.float32


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def _check(t: torch.Tensor, d: B.ConvDesc, shape, what: str, dtype=None):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{what} must be a contiguous device tensor")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{what}: expected shape {tuple(shape)}, got {tuple(t.shape)}")
    if t.dtype != (dtype or _tdtype(d)):
        raise ValueError(f"{what}: expected dtype {dtype or _tdtype(d)}, got {t.dtype}")


def shapes(d: B.ConvDesc) -> dict:
    Hy, Wy, Hp, Wp = B.gf_out_shape(d)
    cg = d.C_in // d.groups
    return {
        "x": (d.N, d.C_in, d.H_in, d.W_in), "g_y": (d.N, d.C_out, Hy, Wy),
        "w": (d.C_out, cg, d.K_h, d.K_w),
        "x_u": (d.N, d.C_in, d.H_in, d.W_in) if d.r == 1 else (d.N, d.C_in, Hp, Wp),
        "gy_u": (d.N, d.C_out, Hp, Wp),
        "g_x_u": (d.N, d.C_in, d.H_in, d.W_in) if d.r == 1 else (d.N, d.C_in, Hp, Wp),
    }


class Workspace:
    """A reusable device scratch buffer (grown on demand, never inside a call to libgf).  One
    Workspace serves ONE stream at a time: two calls that may run concurrently need two."""

    def __init__(self, device="cuda"):
        self.device = device
        self.buf = None

    def get(self, nbytes: int):
        if nbytes == 0:
            return 0, 0
        if self.buf is None or self.buf.numel() < nbytes:
            if self.buf is not None:
                # the old buffer goes back to the caching allocator: tell it that work already
                # enqueued on the current stream may still be using it
                self.buf.record_stream(torch.cuda.current_stream(self.buf.device))
            self.buf = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.device)
        return int(self.buf.data_ptr()), int(self.buf.numel())


_default_ws = {}


def _ws(t: torch.Tensor, ws: Workspace | None) -> Workspace:
    """The caller's workspace, else a default one per (device, current stream): calls on different
    streams may overlap in time and must not share scratch memory."""
    if ws is not None:
        return ws
    key = (str(t.device), int(torch.cuda.current_stream(t.device).cuda_stream))
    if key not in _default_ws:
        _default_ws[key] = Workspace(t.device)
    return _default_ws[key]


def pool_activation(d: B.ConvDesc, x: torch.Tensor, out: torch.Tensor | None = None):
    s = shapes(d)
    _check(x, d, s["x"], "x")
    out = torch.empty(s["x_u"], dtype=x.dtype, device=x.device) if out is None else out
    B.gf_pool_activation(d, B.ptr(x), B.ptr(out), _stream())
    return out


def pool_activation_batch(descs, xs):
    """x_u of several layers from one launch (gf_pool_activation_batch)."""
    outs = []
    for d, x in zip(descs, xs):
        s = shapes(d)
        _check(x, d, s["x"], "x")
        outs.append(torch.empty(s["x_u"], dtype=x.dtype, device=x.device))
    B.gf_pool_activation_batch(B.PoolBatch(descs, [B.ptr(x) for x in xs], [B.ptr(o) for o in outs]), _stream())
    return outs


def pool_activation_batch_q8(descs, xs, inv_deltas):
    """x_q of several layers from one launch (gf_pool_activation_batch_q8)."""
    outs = []
    for d, x in zip(descs, xs):
        s = shapes(d)
        _check(x, d, s["x"], "x")
        outs.append(torch.empty(s["x_u"], dtype=torch.int8, device=x.device))
    B.gf_pool_activation_batch_q8(B.PoolBatchQ8(descs, [B.ptr(x) for x in xs], list(inv_deltas), [B.ptr(o) for o in outs]),
                                  _stream())
    return outs


def pool_activation_mask(d: B.ConvDesc, x: torch.Tensor, hi: float = float("inf")):
    """(x_u, m_u): patch sums of x and the share of each patch with 0 < x < hi (the gradient mask of the
    ReLU / clipped ReLU that produced x, averaged over the patch)."""
    s = shapes(d)
    _check(x, d, s["x"], "x")
    x_u = torch.empty(s["x_u"], dtype=x.dtype, device=x.device)
    m_u = torch.empty(s["x_u"], dtype=x.dtype, device=x.device)
    B.gf_pool_activation_mask(d, B.ptr(x), hi, B.ptr(x_u), B.ptr(m_u), _stream())
    return x_u, m_u


def filter_grad(d: B.ConvDesc, g_y: torch.Tensor, out: torch.Tensor | None = None):
    s = shapes(d)
    _check(g_y, d, s["g_y"], "g_y")
    out = torch.empty(s["gy_u"], dtype=g_y.dtype, device=g_y.device) if out is None else out
    B.gf_filter_grad(d, B.ptr(g_y), B.ptr(out), _stream())
    return out


def conv_bwd_weight(d: B.ConvDesc, x_u: torch.Tensor, gy_u: torch.Tensor,
                    out: torch.Tensor | None = None, ws: Workspace | None = None):
    s = shapes(d)
    _check(x_u, d, s["x_u"], "x_u")
    _check(gy_u, d, s["gy_u"], "gy_u")
    out = torch.empty(s["w"], dtype=torch.float32, device=x_u.device) if out is None else out
    p, n = _ws(x_u, ws).get(B.gf_workspace_bytes(d, B.GF_OP_BWD_WEIGHT))
    B.gf_conv_bwd_weight(d, B.ptr(x_u), B.ptr(gy_u), B.ptr(out), p, n, _stream())
    return out


def conv_bwd_input(d: B.ConvDesc, gy_u: torch.Tensor, w: torch.Tensor, reduced_out: bool = False,
                   out: torch.Tensor | None = None, ws: Workspace | None = None):
    s = shapes(d)
    _check(gy_u, d, s["gy_u"], "gy_u")
    _check(w, d, s["w"], "w")
    shape = s["g_x_u"] if reduced_out else s["x"]
    out = torch.empty(shape, dtype=gy_u.dtype, device=gy_u.device) if out is None else out
    p, n = _ws(gy_u, ws).get(B.gf_workspace_bytes(d, B.GF_OP_BWD_INPUT))
    B.gf_conv_bwd_input(d, B.ptr(gy_u), B.ptr(w), B.ptr(out), reduced_out, p, n, _stream())
    return out


def conv_bwd_filtered(d: B.ConvDesc, g_y: torch.Tensor, x_u: torch.Tensor, w: torch.Tensor,
                      want_gyu: bool = True, ws: Workspace | None = None):
    """(g_w, g_x, gy_u or None) from one call of gf_conv_bwd_filtered."""
    s = shapes(d)
    _check(g_y, d, s["g_y"], "g_y")
    _check(x_u, d, s["x_u"], "x_u")
    _check(w, d, s["w"], "w")
    g_w = torch.empty(s["w"], dtype=torch.float32, device=g_y.device)
    g_x = torch.empty(s["x"], dtype=g_y.dtype, device=g_y.device)
    gy_u = torch.empty(s["gy_u"], dtype=g_y.dtype, device=g_y.device) if want_gyu else None
    p, n = _ws(g_y, ws).get(B.gf_workspace_bytes(d, B.GF_OP_BWD_FILTERED))
    B.gf_conv_bwd_filtered(d, B.ptr(g_y), B.ptr(x_u), B.ptr(w), B.ptr(gy_u), B.ptr(g_w), B.ptr(g_x),
                           p, n, _stream())
    return g_w, g_x, gy_u


def filter_grad_snr(d: B.ConvDesc, g_y: torch.Tensor, ws: Workspace | None = None):
    """(gy_u, stats) with stats = [sum g_y^2, sum (g_y - patch mean)^2] as a float64 device tensor."""
    s = shapes(d)
    _check(g_y, d, s["g_y"], "g_y")
    gy_u = torch.empty(s["gy_u"], dtype=g_y.dtype, device=g_y.device)
    stats = torch.empty(2, dtype=torch.float64, device=g_y.device)
    p, n = _ws(g_y, ws).get(B.gf_workspace_bytes(d, B.GF_OP_FILTER_SNR))
    B.gf_filter_grad_snr(d, B.ptr(g_y), B.ptr(gy_u), B.ptr(stats), p, n, _stream())
    return gy_u, stats


def conv_bwd_chained(d: B.ConvDesc, gy_u: torch.Tensor, x_u: torch.Tensor, w: torch.Tensor,
                     reduced_out: bool = True, mask_u: torch.Tensor | None = None, ws: Workspace | None = None):
    """(g_w, g_x) from one call of gf_conv_bwd_chained; g_x is the reduced map unless reduced_out is False.
    mask_u (from pool_activation_mask of this layer's input) is multiplied into the reduced g_x."""
    s = shapes(d)
    _check(gy_u, d, s["gy_u"], "gy_u")
    _check(x_u, d, s["x_u"], "x_u")
    _check(w, d, s["w"], "w")
    g_w = torch.empty(s["w"], dtype=torch.float32, device=gy_u.device)
    g_x = torch.empty(s["g_x_u"] if reduced_out else s["x"], dtype=gy_u.dtype, device=gy_u.device)
    if mask_u is not None:
        _check(mask_u, d, tuple(g_x.shape), "mask_u")
    p, n = _ws(gy_u, ws).get(B.gf_workspace_bytes(d, B.GF_OP_BWD_CHAINED))
    B.gf_conv_bwd_chained(d, B.ptr(gy_u), B.ptr(x_u), B.ptr(w), B.ptr(g_w), B.ptr(g_x), reduced_out,
                          0 if mask_u is None else B.ptr(mask_u), p, n, _stream())
    return g_w, g_x


def conv_bwd_exact(d: B.ConvDesc, x, w, g_y, want_gw: bool = True, want_gx: bool = True,
                   ws: Workspace | None = None):
    s = shapes(d.with_(r=1))
    _check(g_y, d, s["g_y"], "g_y")
    g_w = g_x = None
    if want_gw:
        _check(x, d, s["x"], "x")
        g_w = torch.empty(s["w"], dtype=torch.float32, device=g_y.device)
    if want_gx:
        _check(w, d, s["w"], "w")
        g_x = torch.empty(s["x"], dtype=g_y.dtype, device=g_y.device)
    p, n = _ws(g_y, ws).get(B.gf_workspace_bytes(d, B.GF_OP_BWD_EXACT))
    B.gf_conv_bwd_exact(d, B.ptr(x) if want_gw else 0, B.ptr(w) if want_gx else 0, B.ptr(g_y),
                        B.ptr(g_w), B.ptr(g_x), p, n, _stream())
    return g_w, g_x


# ---- gradient filtering on signed 8-bit codes (one step size per tensor, chosen by the caller) ----

def filter_grad_q8(d: B.ConvDesc, g_y: torch.Tensor, inv_delta: float) -> torch.Tensor:
    s = shapes(d)
    _check(g_y, d, s["g_y"], "g_y")
    out = torch.empty(s["gy_u"], dtype=torch.int8, device=g_y.device)
    B.gf_filter_grad_q8(d, B.ptr(g_y), inv_delta, B.ptr(out), _stream())
    return out


def pool_activation_q8(d: B.ConvDesc, x: torch.Tensor, inv_delta: float) -> torch.Tensor:
    s = shapes(d)
    _check(x, d, s["x"], "x")
    out = torch.empty(s["x_u"], dtype=torch.int8, device=x.device)
    B.gf_pool_activation_q8(d, B.ptr(x), inv_delta, B.ptr(out), _stream())
    return out


def kernel_sum_q8(d: B.ConvDesc, w: torch.Tensor, inv_delta: float) -> torch.Tensor:
    s = shapes(d)
    _check(w, d, s["w"], "w")
    out = torch.empty(s["w"][:2], dtype=torch.int8, device=w.device)
    B.gf_kernel_sum_q8(d, B.ptr(w), inv_delta, B.ptr(out), _stream())
    return out


def conv_bwd_unique(d: B.ConvDesc, gy_u: torch.Tensor, x_u: torch.Tensor, w: torch.Tensor, reduced_out: bool = False,
                    ws: Workspace | None = None):
    """(g_w, g_x) of gf_conv_bwd_unique: vanilla BP of the layer's kernel on the patch grid."""
    s = shapes(d)
    _check(gy_u, d, s["gy_u"], "gy_u")
    _check(x_u, d, s["x_u"], "x_u")
    _check(w, d, s["w"], "w")
    g_w = torch.empty(s["w"], dtype=torch.float32, device=gy_u.device)
    g_x = torch.empty(s["g_x_u"] if (reduced_out and d.r > 1) else s["x"], dtype=_tdtype(d), device=gy_u.device)
    p, n = _ws(gy_u, ws).get(B.gf_workspace_bytes(d, B.GF_OP_BWD_UNIQUE))
    B.gf_conv_bwd_unique(d, B.ptr(gy_u), B.ptr(x_u), B.ptr(w), B.ptr(g_w), B.ptr(g_x), reduced_out, p, n, _stream())
    return g_w, g_x


def conv_bwd_weight_q8(d: B.ConvDesc, x_q: torch.Tensor, gy_q: torch.Tensor, scale: float,
                       ws: Workspace | None = None) -> torch.Tensor:
    s = shapes(d)
    _check(x_q, d, s["x_u"], "x_q", torch.int8)
    _check(gy_q, d, s["gy_u"], "gy_q", torch.int8)
    g_w = torch.empty(s["w"], dtype=torch.float32, device=x_q.device)
    p, n = _ws(x_q, ws).get(B.gf_workspace_bytes(d, B.GF_OP_BWD_WEIGHT_Q8))
    B.gf_conv_bwd_weight_q8(d, B.ptr(x_q), B.ptr(gy_q), scale, B.ptr(g_w), p, n, _stream())
    return g_w


def conv_bwd_filtered_q8(d: B.ConvDesc, g_y: torch.Tensor, inv_delta_gy: float, x_q: torch.Tensor, w: torch.Tensor,
                         inv_delta_w: float, scale_w: float, scale_x: float, want_gyq: bool = False,
                         ws: Workspace | None = None):
    """Filter with code output + kernel-sum codes + Eq. 5 and Eq. 3 on codes in one call: (g_w, g_x[, gy_q])."""
    s = shapes(d)
    _check(g_y, d, s["g_y"], "g_y")
    _check(x_q, d, s["x_u"], "x_q", torch.int8)
    _check(w, d, s["w"], "w")
    g_w = torch.empty(s["w"], dtype=torch.float32, device=g_y.device)
    g_x = torch.empty(s["x"], dtype=_tdtype(d), device=g_y.device)
    gy_q = torch.empty(s["gy_u"], dtype=torch.int8, device=g_y.device) if want_gyq else None
    p, n = _ws(g_y, ws).get(B.gf_workspace_bytes(d, B.GF_OP_BWD_FILTERED_Q8))
    B.gf_conv_bwd_filtered_q8(d, B.ptr(g_y), inv_delta_gy, B.ptr(x_q), B.ptr(w), inv_delta_w, scale_w, scale_x,
                              B.ptr(gy_q) if want_gyq else 0, B.ptr(g_w), B.ptr(g_x), p, n, _stream())
    return (g_w, g_x, gy_q) if want_gyq else (g_w, g_x)


def conv_bwd_input_q8(d: B.ConvDesc, gy_q: torch.Tensor, w_q: torch.Tensor, scale: float,
                      reduced_out: bool = False, ws: Workspace | None = None) -> torch.Tensor:
    s = shapes(d)
    _check(gy_q, d, s["gy_u"], "gy_q", torch.int8)
    _check(w_q, d, s["w"][:2], "w_q", torch.int8)
    g_x = torch.empty(s["g_x_u"] if reduced_out else s["x"], dtype=_tdtype(d), device=gy_q.device)
    p, n = _ws(gy_q, ws).get(B.gf_workspace_bytes(d, B.GF_OP_BWD_INPUT_Q8))
    B.gf_conv_bwd_input_q8(d, B.ptr(gy_q), B.ptr(w_q), scale, B.ptr(g_x), reduced_out, p, n, _stream())
    return g_x
