"""ctypes binding of libgf's C ABI (include/gf.h): argument marshalling only.

Every function takes raw device pointers (ints) -- use ``ptr(tensor)`` for a
torch tensor -- plus a ``ConvDesc``.  Nothing is computed here, and there is no
fallback: if libgf.so is missing the import of the library fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, replace

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libgf.so")

GF_OK = 0
GF_ERR_NULL, GF_ERR_BAD_DESC, GF_ERR_SHAPE, GF_ERR_UNSUPPORTED, GF_ERR_WORKSPACE, GF_ERR_DEVICE = range(1, 7)
GF_F32, GF_BF16 = 0, 1
GF_OP_BWD_WEIGHT, GF_OP_BWD_INPUT, GF_OP_BWD_EXACT, GF_OP_BWD_FILTERED, GF_OP_BWD_CHAINED = 0, 1, 2, 3, 4
GF_OP_FILTER_SNR = 5
GF_OP_BWD_WEIGHT_Q8, GF_OP_BWD_INPUT_Q8, GF_OP_BWD_FILTERED_Q8 = 6, 7, 8
GF_OP_BWD_UNIQUE = 9

EXPORTS = ("gf_out_shape", "gf_workspace_bytes", "gf_pool_activation", "gf_pool_activation_batch",
           "gf_pool_activation_mask", "gf_filter_grad",
           "gf_filter_grad_snr",
           "gf_conv_bwd_weight", "gf_conv_bwd_input", "gf_conv_bwd_filtered", "gf_conv_bwd_filtered_static",
           "gf_conv_bwd_chained",
           "gf_conv_bwd_exact",
           "gf_filter_grad_q8", "gf_pool_activation_q8", "gf_kernel_sum_q8", "gf_conv_bwd_weight_q8",
           "gf_conv_bwd_input_q8", "gf_conv_bwd_filtered_q8", "gf_pool_activation_batch_q8", "gf_conv_bwd_unique",
           "gf_cost_model",
           "gf_status_string", "gf_version", "gf_set_launch_observer")


class _Desc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32)] + [(k, C.c_int32) for k in (
        "N", "C_in", "C_out", "H_in", "W_in", "K_h", "K_w", "stride", "pad", "dilation", "groups",
        "r", "dtype")]


class _Cost(C.Structure):
    _fields_ = [(k, C.c_double) for k in (
        "flops_exact_gx", "flops_gf_gx", "flops_gf_min", "overhead_fwd", "overhead_bwd",
        "act_elems_exact", "act_elems_gf", "bytes_pool", "bytes_filter", "bytes_bwd_weight",
        "bytes_bwd_input", "bytes_exact", "flops_bwd_weight", "flops_bwd_input", "flops_exact")]


@dataclass(frozen=True)
class ConvDesc:
    """gf_conv_desc: the layer in the paper's symbols; x is [N, C_in, H_in, W_in]."""
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
    dtype: int = GF_F32

    def c(self) -> _Desc:
        return _Desc(C.sizeof(_Desc), self.N, self.C_in, self.C_out, self.H_in, self.W_in,
                     self.K_h, self.K_w, self.stride, self.pad, self.dilation, self.groups, self.r,
                     self.dtype)

    def with_(self, **kw) -> "ConvDesc":
        return replace(self, **kw)


class GfError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


_lib = None


def lib() -> C.CDLL:
    """Load libgf.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with "
                              "`python -m paper_2301_00330_amd.build` (needs hipcc)")
        L = C.CDLL(LIB_PATH)
        vp, dp = C.c_void_p, C.POINTER(_Desc)
        i32p = C.POINTER(C.c_int32)
        L.gf_out_shape.argtypes = [dp, i32p, i32p, i32p, i32p]
        L.gf_workspace_bytes.argtypes = [dp, C.c_int, C.POINTER(C.c_size_t)]
        L.gf_pool_activation.argtypes = [dp, vp, vp, vp]
        L.gf_pool_activation_batch.argtypes = [C.c_int32, dp, C.POINTER(vp), C.POINTER(vp), vp]
        L.gf_pool_activation_batch_q8.argtypes = [C.c_int32, dp, C.POINTER(vp), C.POINTER(C.c_float), C.POINTER(vp), vp]
        L.gf_filter_grad.argtypes = [dp, vp, vp, vp]
        L.gf_filter_grad_snr.argtypes = [dp, vp, vp, vp, vp, C.c_size_t, vp]
        L.gf_conv_bwd_weight.argtypes = [dp, vp, vp, vp, vp, C.c_size_t, vp]
        L.gf_conv_bwd_input.argtypes = [dp, vp, vp, vp, C.c_int, vp, C.c_size_t, vp]
        L.gf_conv_bwd_exact.argtypes = [dp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.gf_conv_bwd_filtered.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.gf_conv_bwd_filtered_static.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp]
        L.gf_conv_bwd_chained.argtypes = [dp, vp, vp, vp, vp, vp, C.c_int, vp, vp, C.c_size_t, vp]
        L.gf_pool_activation_mask.argtypes = [dp, vp, C.c_float, vp, vp, vp]
        L.gf_filter_grad_q8.argtypes = [dp, vp, C.c_float, vp, vp]
        L.gf_pool_activation_q8.argtypes = [dp, vp, C.c_float, vp, vp]
        L.gf_kernel_sum_q8.argtypes = [dp, vp, C.c_float, vp, vp]
        L.gf_conv_bwd_weight_q8.argtypes = [dp, vp, vp, C.c_float, vp, vp, C.c_size_t, vp]
        L.gf_conv_bwd_input_q8.argtypes = [dp, vp, vp, C.c_float, vp, C.c_int, vp, C.c_size_t, vp]
        L.gf_conv_bwd_unique.argtypes = [dp, vp, vp, vp, vp, vp, C.c_int, vp, C.c_size_t, vp]
        L.gf_conv_bwd_filtered_q8.argtypes = [dp, vp, C.c_float, vp, vp, C.c_float, C.c_float, C.c_float, vp, vp, vp,
                                              vp, C.c_size_t, vp]
        L.gf_cost_model.argtypes = [dp, C.POINTER(_Cost)]
        L.gf_status_string.argtypes = [C.c_int]
        L.gf_status_string.restype = C.c_char_p
        L.gf_version.restype = C.c_int
        L.gf_set_launch_observer.argtypes = [LAUNCH_OBSERVER, vp]
        L.gf_set_launch_observer.restype = None
        for name in EXPORTS:
            getattr(L, name)
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().gf_status_string(int(status)).decode()


def _chk(status: int, where: str):
    if status != GF_OK:
        raise GfError(status, where)


def ptr(t) -> int:
    """Device address of a torch tensor (None -> NULL)."""
    return 0 if t is None else int(t.data_ptr())


LAUNCH_OBSERVER = C.CFUNCTYPE(None, C.c_void_p, C.c_char_p, C.c_int, C.c_void_p)
_observer_keepalive = None


def gf_set_launch_observer(fn=None):
    """fn(kernel_name: str, phase: int, stream: int) is called before (0) / after (1) every kernel launch
    of the library; None removes the observer."""
    global _observer_keepalive
    if fn is None:
        lib().gf_set_launch_observer(LAUNCH_OBSERVER(0), None)
        _observer_keepalive = None
        return
    cb = LAUNCH_OBSERVER(lambda user, name, phase, stream: fn(name.decode(), int(phase), int(stream or 0)))
    lib().gf_set_launch_observer(cb, None)
    _observer_keepalive = cb


def gf_version() -> int:
    return int(lib().gf_version())


def gf_out_shape(d: ConvDesc):
    v = [C.c_int32() for _ in range(4)]
    cd = d.c()
    _chk(lib().gf_out_shape(C.byref(cd), *[C.byref(t) for t in v]), "gf_out_shape")
    return tuple(int(t.value) for t in v)


def gf_workspace_bytes(d: ConvDesc, op: int) -> int:
    n = C.c_size_t()
    cd = d.c()
    _chk(lib().gf_workspace_bytes(C.byref(cd), int(op), C.byref(n)), "gf_workspace_bytes")
    return int(n.value)


def gf_pool_activation(d: ConvDesc, x: int, x_u: int, stream: int = 0):
    cd = d.c()
    _chk(lib().gf_pool_activation(C.byref(cd), x, x_u, stream), "gf_pool_activation")


class PoolBatch:
    """Marshalled arguments of gf_pool_activation_batch (build once, call many times)."""

    def __init__(self, descs, xs, x_us):
        n = len(descs)
        assert n == len(xs) == len(x_us)
        self.n = n
        self.descs = (_Desc * max(n, 1))(*[d.c() for d in descs])
        self.xs = (C.c_void_p * max(n, 1))(*xs)
        self.x_us = (C.c_void_p * max(n, 1))(*x_us)


def gf_pool_activation_batch(batch: PoolBatch, stream: int = 0):
    _chk(lib().gf_pool_activation_batch(batch.n, batch.descs, batch.xs, batch.x_us, stream), "gf_pool_activation_batch")


class PoolBatchQ8(PoolBatch):
    """Marshalled arguments of gf_pool_activation_batch_q8: PoolBatch plus one step-size reciprocal per layer
    (x_us then holds the int8 code tensors)."""

    def __init__(self, descs, xs, inv_deltas, x_qs):
        super().__init__(descs, xs, x_qs)
        assert len(inv_deltas) == self.n
        self.inv = (C.c_float * max(self.n, 1))(*inv_deltas)


def gf_pool_activation_batch_q8(batch: PoolBatchQ8, stream: int = 0):
    _chk(lib().gf_pool_activation_batch_q8(batch.n, batch.descs, batch.xs, batch.inv, batch.x_us, stream),
         "gf_pool_activation_batch_q8")


def gf_filter_grad(d: ConvDesc, g_y: int, gy_u: int, stream: int = 0):
    cd = d.c()
    _chk(lib().gf_filter_grad(C.byref(cd), g_y, gy_u, stream), "gf_filter_grad")


def gf_conv_bwd_weight(d: ConvDesc, x_u: int, gy_u: int, g_w: int, ws: int, ws_bytes: int,
                       stream: int = 0):
    cd = d.c()
    _chk(lib().gf_conv_bwd_weight(C.byref(cd), x_u, gy_u, g_w, ws, ws_bytes, stream),
         "gf_conv_bwd_weight")


def gf_conv_bwd_input(d: ConvDesc, gy_u: int, w: int, g_x: int, reduced_out: bool, ws: int,
                      ws_bytes: int, stream: int = 0):
    cd = d.c()
    _chk(lib().gf_conv_bwd_input(C.byref(cd), gy_u, w, g_x, int(bool(reduced_out)), ws, ws_bytes,
                                 stream), "gf_conv_bwd_input")


def gf_conv_bwd_filtered(d: ConvDesc, g_y: int, x_u: int, w: int, gy_u: int, g_w: int, g_x: int,
                         ws: int, ws_bytes: int, stream: int = 0):
    cd = d.c()
    _chk(lib().gf_conv_bwd_filtered(C.byref(cd), g_y, x_u, w, gy_u, g_w, g_x, ws, ws_bytes, stream),
         "gf_conv_bwd_filtered")


GF_STATIC_SCRATCH_BYTES = 64 << 20


def gf_conv_bwd_filtered_static(d: ConvDesc, g_y: int, x_u: int, w: int, gy_u: int, g_w: int, g_x: int,
                                stream: int = 0):
    cd = d.c()
    _chk(lib().gf_conv_bwd_filtered_static(C.byref(cd), g_y, x_u, w, gy_u, g_w, g_x, stream),
         "gf_conv_bwd_filtered_static")


def gf_filter_grad_snr(d: ConvDesc, g_y: int, gy_u: int, stats: int, ws: int, ws_bytes: int, stream: int = 0):
    cd = d.c()
    _chk(lib().gf_filter_grad_snr(C.byref(cd), g_y, gy_u, stats, ws, ws_bytes, stream), "gf_filter_grad_snr")


def gf_conv_bwd_chained(d: ConvDesc, gy_u: int, x_u: int, w: int, g_w: int, g_x: int,
                        reduced_out: bool, mask_u: int, ws: int, ws_bytes: int, stream: int = 0):
    cd = d.c()
    _chk(lib().gf_conv_bwd_chained(C.byref(cd), gy_u, x_u, w, g_w, g_x, int(bool(reduced_out)), mask_u, ws,
                                   ws_bytes, stream), "gf_conv_bwd_chained")


def gf_pool_activation_mask(d: ConvDesc, x: int, hi: float, x_u: int, m_u: int, stream: int = 0):
    cd = d.c()
    _chk(lib().gf_pool_activation_mask(C.byref(cd), x, C.c_float(hi), x_u, m_u, stream), "gf_pool_activation_mask")


def gf_conv_bwd_exact(d: ConvDesc, x: int, w: int, g_y: int, g_w: int, g_x: int, ws: int,
                      ws_bytes: int, stream: int = 0):
    cd = d.c()
    _chk(lib().gf_conv_bwd_exact(C.byref(cd), x, w, g_y, g_w, g_x, ws, ws_bytes, stream),
         "gf_conv_bwd_exact")


def gf_filter_grad_q8(d: ConvDesc, g_y: int, inv_delta: float, gy_q: int, stream: int = 0):
    cd = d.c()
    _chk(lib().gf_filter_grad_q8(C.byref(cd), g_y, inv_delta, gy_q, stream), "gf_filter_grad_q8")


def gf_pool_activation_q8(d: ConvDesc, x: int, inv_delta: float, x_q: int, stream: int = 0):
    cd = d.c()
    _chk(lib().gf_pool_activation_q8(C.byref(cd), x, inv_delta, x_q, stream), "gf_pool_activation_q8")


def gf_kernel_sum_q8(d: ConvDesc, w: int, inv_delta: float, w_q: int, stream: int = 0):
    cd = d.c()
    _chk(lib().gf_kernel_sum_q8(C.byref(cd), w, inv_delta, w_q, stream), "gf_kernel_sum_q8")


def gf_conv_bwd_weight_q8(d: ConvDesc, x_q: int, gy_q: int, scale: float, g_w: int, ws: int, ws_bytes: int,
                          stream: int = 0):
    cd = d.c()
    _chk(lib().gf_conv_bwd_weight_q8(C.byref(cd), x_q, gy_q, scale, g_w, ws, ws_bytes, stream),
         "gf_conv_bwd_weight_q8")


def gf_conv_bwd_unique(d: ConvDesc, gy_u: int, x_u: int, w: int, g_w: int, g_x: int, reduced_out: bool, ws: int,
                       ws_bytes: int, stream: int = 0):
    cd = d.c()
    _chk(lib().gf_conv_bwd_unique(C.byref(cd), gy_u, x_u, w, g_w, g_x, int(bool(reduced_out)), ws, ws_bytes, stream),
         "gf_conv_bwd_unique")


def gf_conv_bwd_filtered_q8(d: ConvDesc, g_y: int, inv_delta_gy: float, x_q: int, w: int, inv_delta_w: float,
                            scale_w: float, scale_x: float, gy_q: int, g_w: int, g_x: int, ws: int, ws_bytes: int,
                            stream: int = 0):
    cd = d.c()
    _chk(lib().gf_conv_bwd_filtered_q8(C.byref(cd), g_y, inv_delta_gy, x_q, w, inv_delta_w, scale_w, scale_x, gy_q,
                                       g_w, g_x, ws, ws_bytes, stream), "gf_conv_bwd_filtered_q8")


def gf_conv_bwd_input_q8(d: ConvDesc, gy_q: int, w_q: int, scale: float, g_x: int, reduced_out: bool, ws: int,
                         ws_bytes: int, stream: int = 0):
    cd = d.c()
    _chk(lib().gf_conv_bwd_input_q8(C.byref(cd), gy_q, w_q, scale, g_x, int(bool(reduced_out)), ws, ws_bytes,
                                    stream), "gf_conv_bwd_input_q8")


def gf_cost_model(d: ConvDesc) -> dict:
    c = _Cost()
    cd = d.c()
    _chk(lib().gf_cost_model(C.byref(cd), C.byref(c)), "gf_cost_model")
    return {k: float(getattr(c, k)) for k, _ in _Cost._fields_}
