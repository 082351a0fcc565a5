"""CPU oracle for gradient-filtered convolution backward -- TEST INFRASTRUCTURE ONLY.

A thin numpy/ctypes front for ``gf_ref.c``: every function takes and returns
contiguous float64 NCHW arrays.  Only ``tests/``, the smoke check and the
benchmark's ``cpu_baseline`` leg may import this package; the GPU library and
its Python binding never do, and nothing here imports them.

The arithmetic lives in ``gf_ref.c`` (plain loops, fp64 accumulation), each
function citing the passage of the paper it follows in ``gf_ref.h``.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libgf_ref.so")
_SRC = [os.path.join(_HERE, "gf_ref.c"), os.path.join(_HERE, "gf_ref.h")]
_lib = None


def build(force: bool = False) -> str:
    """Compile gf_ref.c into libgf_ref.so with gcc (OpenMP over outer loops)."""
    stale = force or not os.path.exists(_SO) or any(
        os.path.getmtime(s) > os.path.getmtime(_SO) for s in _SRC)
    if stale:
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _SO, _SRC[0]]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _SO


class _Desc(C.Structure):
    _fields_ = [(k, C.c_int) for k in ("N", "C_in", "C_out", "H_in", "W_in", "K_h", "K_w",
                                        "stride", "pad", "dilation", "groups", "r")]


class _Cost(C.Structure):
    _fields_ = [(k, C.c_double) for k in ("flops_exact_gx", "flops_gf_gx", "flops_gf_min",
                                           "overhead_fwd", "overhead_bwd", "act_elems_exact",
                                           "act_elems_gf")]


@dataclass(frozen=True)
class Desc:
    """Layer description in the paper's symbols (x is [N, C_in, H_in, W_in])."""
    N: int
    C_in: int
    C_out: int
    H_in: int
    W_in: int
    K_h: int = 1
    K_w: int = 1
    stride: int = 1
    pad: int = 0
    dilation: int = 1
    groups: int = 1
    r: int = 2

    def _c(self) -> _Desc:
        return _Desc(self.N, self.C_in, self.C_out, self.H_in, self.W_in, self.K_h, self.K_w,
                     self.stride, self.pad, self.dilation, self.groups, self.r)


class OracleError(ValueError):
    pass


def _L():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_SO)
    return _lib


def _chk(rc: int, what: str):
    if rc != 0:
        raise OracleError(f"{what}: oracle rejected the call (code {rc})")


def _in(a, shape) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float64)
    if tuple(a.shape) != tuple(shape):
        raise OracleError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_double))


def num_threads() -> int:
    return int(_L().gf_ref_num_threads())


def out_shape(d: Desc):
    """(H_y, W_y, H_p, W_p): output map and patch grid (Sec. 3.3)."""
    v = [C.c_int() for _ in range(4)]
    cd = d._c()
    _chk(_L().gf_ref_out_shape(C.byref(cd), *[C.byref(t) for t in v]), "out_shape")
    return tuple(int(t.value) for t in v)


def xu_shape(d: Desc):
    Hy, Wy, Hp, Wp = out_shape(d)
    return (d.N, d.C_in, d.H_in, d.W_in) if d.r == 1 else (d.N, d.C_in, Hp, Wp)


def w_shape(d: Desc):
    return (d.C_out, d.C_in // d.groups, d.K_h, d.K_w)


def filter_grad(d: Desc, g_y) -> np.ndarray:
    Hy, Wy, Hp, Wp = out_shape(d)
    g_y = _in(g_y, (d.N, d.C_out, Hy, Wy))
    out = np.empty((d.N, d.C_out, Hp, Wp), np.float64)
    cd = d._c()
    _chk(_L().gf_ref_filter_grad(C.byref(cd), _p(g_y), _p(out)), "filter_grad")
    return out


def filter_snr(d: Desc, g_y):
    """(energy, noise) of the filter (first line of Eq. 8 in the pixel domain); SNR = energy / noise."""
    Hy, Wy, Hp, Wp = out_shape(d)
    g_y = _in(g_y, (d.N, d.C_out, Hy, Wy))
    e, v = C.c_double(0.0), C.c_double(0.0)
    cd = d._c()
    _chk(_L().gf_ref_filter_snr(C.byref(cd), _p(g_y), C.byref(e), C.byref(v)), "filter_snr")
    return e.value, v.value


def pool_activation(d: Desc, x) -> np.ndarray:
    x = _in(x, (d.N, d.C_in, d.H_in, d.W_in))
    out = np.empty(xu_shape(d), np.float64)
    cd = d._c()
    _chk(_L().gf_ref_pool_activation(C.byref(cd), _p(x), _p(out)), "pool_activation")
    return out


def pool_activation_mask(d: Desc, x, hi: float = float("inf")):
    """(x_u, m_u): the patch sums of x and the fraction of each patch through which a ReLU
    (clipped at `hi`) that produced x passes a gradient."""
    x = _in(x, (d.N, d.C_in, d.H_in, d.W_in))
    x_u = np.empty(xu_shape(d), np.float64)
    m_u = np.empty(xu_shape(d), np.float64)
    cd = d._c()
    _chk(_L().gf_ref_pool_activation_mask(C.byref(cd), _p(x), C.c_double(hi), _p(x_u), _p(m_u)), "pool_activation_mask")
    return x_u, m_u


def kernel_sum(d: Desc, w) -> np.ndarray:
    w = _in(w, w_shape(d))
    out = np.empty((d.C_out, d.C_in // d.groups), np.float64)
    cd = d._c()
    _chk(_L().gf_ref_kernel_sum(C.byref(cd), _p(w), _p(out)), "kernel_sum")
    return out


def bwd_weight(d: Desc, x_u, gy_u) -> np.ndarray:
    Hy, Wy, Hp, Wp = out_shape(d)
    x_u = _in(x_u, xu_shape(d))
    gy_u = _in(gy_u, (d.N, d.C_out, Hp, Wp))
    out = np.empty(w_shape(d), np.float64)
    cd = d._c()
    _chk(_L().gf_ref_bwd_weight(C.byref(cd), _p(x_u), _p(gy_u), _p(out)), "bwd_weight")
    return out


def bwd_input(d: Desc, gy_u, w, reduced_out: bool = False) -> np.ndarray:
    Hy, Wy, Hp, Wp = out_shape(d)
    gy_u = _in(gy_u, (d.N, d.C_out, Hp, Wp))
    w = _in(w, w_shape(d))
    full = (d.N, d.C_in, d.H_in, d.W_in)
    shape = (d.N, d.C_in, Hp, Wp) if (reduced_out and d.r > 1) else full
    out = np.empty(shape, np.float64)
    cd = d._c()
    _chk(_L().gf_ref_bwd_input(C.byref(cd), _p(gy_u), _p(w), _p(out), int(bool(reduced_out))),
         "bwd_input")
    return out


def bwd_exact(d: Desc, x, w, g_y, want_gw: bool = True, want_gx: bool = True):
    e = Desc(**{**d.__dict__, "r": 1})
    Hy, Wy, _, _ = out_shape(e)
    g_y = _in(g_y, (d.N, d.C_out, Hy, Wy))
    x = _in(x, (d.N, d.C_in, d.H_in, d.W_in)) if want_gw else None
    w = _in(w, w_shape(d)) if want_gx else None
    g_w = np.empty(w_shape(d), np.float64) if want_gw else None
    g_x = np.empty((d.N, d.C_in, d.H_in, d.W_in), np.float64) if want_gx else None
    cd = d._c()
    _chk(_L().gf_ref_bwd_exact(C.byref(cd), _p(x) if want_gw else None,
                               _p(w) if want_gx else None, _p(g_y),
                               _p(g_w) if want_gw else None, _p(g_x) if want_gx else None),
         "bwd_exact")
    return g_w, g_x


def bwd_unique(d: Desc, x_u, gy_u, w, reduced_out: bool = False):
    """'Fewer unique elements' alone (Sec. 4.2, the middle cost line of Fig. 3): the gradient map is
    replaced by its one value per patch, but the K x K kernel is kept.  The backward then runs on the
    r^2 times smaller maps as it stands:
        g_w[co, ci, u, v] = sum_{n, hp, wp} x_u[n, ci, hp + u d - p, wp + v d - p] gy_u[n, co, hp, wp]
        g_xu[n, ci, hp, wp] = sum_{co, u, v} w[co, ci, u, v] gy_u[n, co, hp - u d + p, wp - v d + p]
    i.e. vanilla BP (Sec. 3.1) of the same kernel on the patch grid, x_u being the patch sums and
    gy_u the patch means; every pixel of an input patch then receives its patch's g_xu (or, with
    reduced_out, g_xu itself is returned).  Stride-1 layers whose padding keeps the map size only;
    r = 1 is vanilla BP.  Returns (g_w, g_x)."""
    if d.r == 1:
        return bwd_exact(d, x_u, w, gy_u)
    if d.stride != 1:
        raise OracleError("bwd_unique: stride-1 layers only")
    Hy, Wy, Hp, Wp = out_shape(d)
    ds = Desc(N=d.N, C_in=d.C_in, C_out=d.C_out, H_in=Hp, W_in=Wp, K_h=d.K_h, K_w=d.K_w, stride=1,
              pad=d.pad, dilation=d.dilation, groups=d.groups, r=1)
    if out_shape(ds)[:2] != (Hp, Wp):
        raise OracleError("bwd_unique: the padding must keep the map size")
    g_w, g_xu = bwd_exact(ds, x_u, w, gy_u)
    if reduced_out:
        return g_w, g_xu
    g_x = np.repeat(np.repeat(g_xu, d.r, axis=2), d.r, axis=3)[:, :, :d.H_in, :d.W_in]
    return g_w, np.ascontiguousarray(g_x)


def conv_fwd(d: Desc, x, w) -> np.ndarray:
    e = Desc(**{**d.__dict__, "r": 1})
    Hy, Wy, _, _ = out_shape(e)
    x = _in(x, (d.N, d.C_in, d.H_in, d.W_in))
    w = _in(w, w_shape(d))
    y = np.empty((d.N, d.C_out, Hy, Wy), np.float64)
    cd = d._c()
    _chk(_L().gf_ref_conv_fwd(C.byref(cd), _p(x), _p(w), _p(y)), "conv_fwd")
    return y


# ---- gradient filtering on 8-bit codes (reading of Supp. H, see gf_ref.h) ----

def _q(a, shape) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.int8)
    if tuple(a.shape) != tuple(shape):
        raise OracleError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _pq(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_byte))


def quantize_q8(v, inv_delta: float) -> np.ndarray:
    """codes = clip(round_half_even(float32(v) * inv_delta), -127, 127), int8, same shape."""
    v = np.ascontiguousarray(v, dtype=np.float64)
    q = np.empty(v.shape, np.int8)
    _chk(_L().gf_ref_quantize_q8(_p(v), C.c_long(v.size), C.c_float(inv_delta), _pq(q)), "quantize_q8")
    return q


def filter_grad_q8(d: Desc, g_y, inv_delta: float) -> np.ndarray:
    return quantize_q8(filter_grad(d, g_y), inv_delta)


def pool_activation_q8(d: Desc, x, inv_delta: float) -> np.ndarray:
    return quantize_q8(pool_activation(d, x), inv_delta)


def kernel_sum_q8(d: Desc, w, inv_delta: float) -> np.ndarray:
    return quantize_q8(kernel_sum(d, w), inv_delta)


def _scale32(d: Desc, scale: float) -> np.float32:
    """step-size product times 1/s^2, formed in binary32 as the library's host code forms it"""
    return np.float32(scale) / (np.float32(d.stride) * np.float32(d.stride))


def bwd_weight_q8(d: Desc, x_q, gy_q, scale: float) -> np.ndarray:
    """Eq. 5 on codes, float32 [C_out, C_in/groups, K_h, K_w]: float32(integer sum) * scale / s^2 on every tap."""
    Hy, Wy, Hp, Wp = out_shape(d)
    x_q = _q(x_q, (d.N, d.C_in, Hp, Wp))
    gy_q = _q(gy_q, (d.N, d.C_out, Hp, Wp))
    acc = np.empty((d.C_out, d.C_in // d.groups), np.int64)
    cd = d._c()
    _chk(_L().gf_ref_bwd_weight_q8(C.byref(cd), _pq(x_q), _pq(gy_q), acc.ctypes.data_as(C.POINTER(C.c_longlong))),
         "bwd_weight_q8")
    val = acc.astype(np.float32) * _scale32(d, scale)
    return np.broadcast_to(val[:, :, None, None], w_shape(d)).copy()


def bwd_input_q8(d: Desc, gy_q, w_q, scale: float, reduced_out: bool = False) -> np.ndarray:
    """Eq. 3 on codes, float32: float32(integer sum) * scale / s^2, one value per patch
    ([N, C_in, H_p, W_p]) or replicated over the input-side patches ([N, C_in, H_in, W_in])."""
    Hy, Wy, Hp, Wp = out_shape(d)
    gy_q = _q(gy_q, (d.N, d.C_out, Hp, Wp))
    w_q = _q(w_q, (d.C_out, d.C_in // d.groups))
    acc = np.empty((d.N, d.C_in, Hp, Wp), np.int64)
    cd = d._c()
    _chk(_L().gf_ref_bwd_input_q8(C.byref(cd), _pq(gy_q), _pq(w_q), acc.ctypes.data_as(C.POINTER(C.c_longlong))),
         "bwd_input_q8")
    val = acc.astype(np.float32) * _scale32(d, scale)
    if reduced_out:
        return val
    rx = d.r * d.stride
    full = np.repeat(np.repeat(val, rx, axis=2), rx, axis=3)
    return np.ascontiguousarray(full[:, :, :d.H_in, :d.W_in])


def cost_model(d: Desc) -> dict:
    c = _Cost()
    cd = d._c()
    _chk(_L().gf_ref_cost_model(C.byref(cd), C.byref(c)), "cost_model")
    return {k: float(getattr(c, k)) for k, _ in _Cost._fields_}


def gf_backward(d: Desc, x, w, g_y, reduced_out: bool = False):
    """The whole filtered backward in the paper's order (lower half of Fig. 2(a)):
    x_u (forward time), gy_u, then g_theta and g_x from the reduced maps."""
    x_u = pool_activation(d, x)
    gy_u = filter_grad(d, g_y)
    return bwd_weight(d, x_u, gy_u), bwd_input(d, gy_u, w, reduced_out), x_u, gy_u
