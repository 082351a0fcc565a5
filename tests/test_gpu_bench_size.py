"""GPU parity at the sizes bench.py times: every layer of every configuration at its full
batch, through the one-call entry (gf_conv_bwd_filtered) the timed step issues, against the
oracle run end to end in fp64 from the same rounded inputs; and vanilla BP (Sec. 3.1) at the
same full shapes on sampled outputs the oracle evaluates one by one.

Beside the per-tensor figure max|gpu - ref| / max|ref| the comparisons here are also
normalised per channel: over each c_o row of g_w and over each (n, c_i) plane of g_x, so a
single wrong row or plane cannot hide below the tensor's largest value.
"""
import numpy as np
import pytest
import torch

import paper_2301_00330_amd.binding as B
import paper_2301_00330_amd.torch_api as T
from paper_2301_00330_amd import workloads as WL

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    B.lib()


def to64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def odesc(oracle, d: B.ConvDesc, **kw):
    f = dict(N=d.N, C_in=d.C_in, C_out=d.C_out, H_in=d.H_in, W_in=d.W_in, K_h=d.K_h, K_w=d.K_w,
             stride=d.stride, pad=d.pad, dilation=d.dilation, groups=d.groups, r=d.r)
    f.update(kw)
    return oracle.Desc(**f)


def rel_err(g: np.ndarray, ref: np.ndarray) -> float:
    assert g.shape == ref.shape, (g.shape, ref.shape)
    den = np.abs(ref).max()
    return float(np.abs(g - ref).max() / (den if den > 0 else 1.0))


def rel_err_rows(g: np.ndarray, ref: np.ndarray, keep: int, scale: np.ndarray = None) -> float:
    """Largest per-row figure, a row being everything behind the first `keep` axes: one c_o of
    g_w (keep = 1), one (n, c_i) plane of g_x (keep = 2).  A row's error is measured against the
    row's largest reference value, or against the row's largest value of `scale` when given."""
    assert g.shape == ref.shape, (g.shape, ref.shape)
    rows = int(np.prod(ref.shape[:keep]))
    a = np.abs(g - ref).reshape(rows, -1).max(axis=1)
    den = np.abs(ref if scale is None else scale).reshape(rows, -1).max(axis=1)
    assert den.min() > 0.0, "a reference row is identically zero"
    return float((a / den).max())


# Per-row tolerances.  The end-to-end fp64 oracle rounds nothing on the way, the library rounds the
# reduced maps and the kernel sum once to the storage type; on a row whose terms cancel (a c_o
# whose patch means sum to almost nothing against nearly constant post-ReLU patch sums) those
# 2^-9 roundings are a few per cent of the row's own largest value although they are 1e-3 of the
# tensor's.  The per-row reference therefore rounds at the library's rounding points too
# (oracle-made reduced maps and kernel sum, each rounded once to the storage type); what is
# left is the fp32 summation order, the output rounding (bf16 g_x: 2^-9 of the value) and the
# rare patch whose fp32 sum lands on the other side of a rounding boundary.
# Depthwise layers: a "row" of g_w is ONE dot product over (n, patch) and a plane of g_x is the
# patch means times ONE sum of K_h K_w taps; both may cancel to almost nothing, so their error is
# measured against the same contraction of the absolute values (the forward error bound of a
# sum), and the kernel sum stays in fp32 as the depthwise kernels keep it.
TOL_ROW = {"f32": {"g_w": 1e-5, "g_x": 1e-5}, "bf16": {"g_w": 2e-3, "g_x": 8e-3}}


def rounded64(a: np.ndarray, dtype: str) -> np.ndarray:
    """fp64 -> the storage type (one round-to-nearest-even) -> fp64"""
    return torch.from_numpy(np.ascontiguousarray(a)).to(WL.torch_dtype(dtype)).to(torch.float64).numpy()


def check_one_call(oracle, cfg, layer, dtype, r):
    """gf_pool_activation + gf_conv_bwd_filtered at the configuration's own batch size: the
    launches bench.py times.  The oracle runs the whole path in fp64 from the same inputs."""
    d = T.desc_for(layer, cfg.N, r, dtype)
    od = odesc(oracle, d)
    x, w, gy = WL.make_inputs(cfg, layer, dtype)
    x_u = T.pool_activation(d, x.cuda())
    g_w, g_x, gy_u = T.conv_bwd_filtered(d, gy.cuda(), x_u, w.cuda(), want_gyu=True)
    g_w2, g_x2, none = T.conv_bwd_filtered(d, gy.cuda(), x_u, w.cuda(), want_gyu=False)
    torch.cuda.synchronize()
    assert none is None and torch.equal(g_x, g_x2) and torch.equal(g_w, g_w2)   # also run to run
    ref_gw, ref_gx, ref_xu, ref_gyu = oracle.gf_backward(od, to64(x), to64(w), to64(gy))
    tol = TOL[dtype]
    gw, gx = to64(g_w), to64(g_x)
    errs = {"x_u": rel_err(to64(x_u), ref_xu), "gy_u": rel_err(to64(gy_u), ref_gyu),
            "g_w": rel_err(gw, ref_gw), "g_x": rel_err(gx, ref_gx),
            "x_u/plane": rel_err_rows(to64(x_u), ref_xu, 2), "gy_u/plane": rel_err_rows(to64(gy_u), ref_gyu, 2)}
    # per row, against the oracle continued from its own reduced maps rounded where the library rounds
    xu_r, gyu_r = rounded64(ref_xu, dtype), rounded64(ref_gyu, dtype)
    row_gw = oracle.bwd_weight(od, xu_r, gyu_r)
    depthwise = layer.groups == layer.C_in == layer.C_out and layer.groups > 1
    ksum = oracle.kernel_sum(od, to64(w))
    if not depthwise:
        ksum = rounded64(ksum, dtype)
    od1 = odesc(oracle, d, K_h=1, K_w=1, pad=0, dilation=1)        # the collapsed kernel as a 1x1 layer
    assert oracle.out_shape(od1) == oracle.out_shape(od)
    row_gx = oracle.bwd_input(od1, gyu_r, ksum[:, :, None, None])
    abs_gw = abs_gx = None
    if depthwise:
        abs_gw = oracle.bwd_weight(od, np.abs(xu_r), np.abs(gyu_r))
        abs_gx = oracle.bwd_input(od1, np.abs(gyu_r), oracle.kernel_sum(od, np.abs(to64(w)))[:, :, None, None])
    errs["g_w/c_o"] = rel_err_rows(gw, row_gw, 1, abs_gw)
    errs["g_x/plane"] = rel_err_rows(gx, row_gx, 2, abs_gx)
    print(f"\n{cfg.cfg_id}/{layer.name}/{dtype}/r{r}: " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    for k in ("x_u", "gy_u", "g_w", "g_x", "x_u/plane", "gy_u/plane"):
        assert errs[k] <= tol, k
    assert errs["g_w/c_o"] <= TOL_ROW[dtype]["g_w"], "g_w per c_o"
    assert errs["g_x/plane"] <= TOL_ROW[dtype]["g_x"], "g_x per (n, c_i) plane"
    # structure with one right answer
    assert torch.equal(g_w, g_w[:, :, :1, :1].expand_as(g_w))
    rx = r * layer.stride
    rep = g_x[:, :, ::rx, ::rx].repeat_interleave(rx, 2).repeat_interleave(rx, 3)[:, :, :layer.H, :layer.W]
    assert torch.equal(rep, g_x)


@pytest.mark.parametrize("r", [2, 4])
@pytest.mark.parametrize("li", [0, 1, 2])
def test_config3_full_size_one_call(oracle, li, r):
    cfg = WL.CONFIGS[3]
    check_one_call(oracle, cfg, cfg.layers[li], "bf16", r)


@pytest.mark.parametrize("r", [2, 4, 8])
@pytest.mark.parametrize("li", [0, 1, 2, 3])
def test_config4_full_size_one_call(oracle, li, r):
    cfg = WL.CONFIGS[4]
    check_one_call(oracle, cfg, cfg.layers[li], "bf16", r)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("li", list(range(10)))
def test_config5_full_size_one_call(oracle, li, dtype):
    cfg = WL.CONFIGS[5]
    check_one_call(oracle, cfg, cfg.layers[li], dtype, 2)


@pytest.mark.parametrize("r", [2, 4])
@pytest.mark.parametrize("li", [2, 3, 4, 5, 6])
def test_paper_cases_full_size_one_call(oracle, li, r):
    """Table 7's shapes with the smaller maps (Supp. E) at the paper's batch of 32, fp32."""
    cfg = WL.CONFIGS[7]
    check_one_call(oracle, cfg, cfg.layers[li], "f32", r)


# ---------------------------------------------------------------------------
# vanilla BP (Sec. 3.1) at full size, sampled
# ---------------------------------------------------------------------------
def check_exact_sampled(oracle, cfg, layer, dtype, seed, rows=2, planes=2):
    """gf_conv_bwd_exact at the configuration's batch size.  The oracle evaluates sampled outputs
    one by one: the c_o row of g_w (all c_i, all taps) is the weight gradient of the layer
    restricted to that output channel; an (n, c_i) plane of g_x is the input gradient of the
    layer restricted to that image and that input channel.  Every sample is compared against
    its own largest reference value (per-row normalisation)."""
    N = cfg.N
    d = T.desc_for(layer, N, 1, dtype)
    x, w, gy = WL.make_inputs(cfg, layer, dtype)
    g_w, g_x = T.conv_bwd_exact(d, x.cuda(), w.cuda(), gy.cuda())
    g_w2, g_x2 = T.conv_bwd_exact(d, x.cuda(), w.cuda(), gy.cuda())
    torch.cuda.synchronize()
    assert torch.equal(g_w, g_w2) and torch.equal(g_x, g_x2)
    gw_c, gx_c = g_w.cpu(), g_x.cpu()
    tol = TOL[dtype]
    rs = np.random.default_rng(seed)
    dw = layer.groups > 1
    assert (not dw) or layer.groups == layer.C_in == layer.C_out, "sampling covers dense and depthwise layers"
    x64 = None if dw else to64(x)
    worst_w = worst_x = 0.0
    # first and last channels are always among the samples (tile edges)
    for co in [0, layer.C_out - 1] + [int(v) for v in rs.integers(0, layer.C_out, rows)]:
        if dw:
            sd = odesc(oracle, d, C_in=1, C_out=1, groups=1)
            ref, _ = oracle.bwd_exact(sd, to64(x[:, co:co + 1]), None, to64(gy[:, co:co + 1]), want_gx=False)
        else:
            sd = odesc(oracle, d, C_out=1)
            ref, _ = oracle.bwd_exact(sd, x64, None, to64(gy[:, co:co + 1]), want_gx=False)
        e = rel_err(to64(gw_c[co:co + 1]), ref)
        worst_w = max(worst_w, e)
        assert e <= tol, f"g_w[{co}]"
    ns = [0, N - 1] + [int(v) for v in rs.integers(0, N, planes)]
    cs = [layer.C_in - 1, 0] + [int(v) for v in rs.integers(0, layer.C_in, planes)]
    for n, ci in zip(ns, cs):
        if dw:
            sd = odesc(oracle, d, N=1, C_in=1, C_out=1, groups=1)
            _, ref = oracle.bwd_exact(sd, None, to64(w[ci:ci + 1]), to64(gy[n:n + 1, ci:ci + 1]), want_gw=False)
        else:
            sd = odesc(oracle, d, N=1, C_in=1)
            _, ref = oracle.bwd_exact(sd, None, to64(w[:, ci:ci + 1]), to64(gy[n:n + 1]), want_gw=False)
        e = rel_err(to64(gx_c[n:n + 1, ci:ci + 1]), ref)
        worst_x = max(worst_x, e)
        assert e <= tol, f"g_x[{n},{ci}]"
    print(f"\nexact {cfg.cfg_id}/{layer.name}/{dtype}: g_w/c_o={worst_w:.2e} g_x/plane={worst_x:.2e}", flush=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("li", [0, 1, 2])
def test_config2_exact_full_size_sampled(oracle, li, dtype):
    cfg = WL.CONFIGS[2]
    check_exact_sampled(oracle, cfg, cfg.layers[li], dtype, 20 + li)


@pytest.mark.parametrize("li", [0, 1, 2])
def test_config3_exact_full_size_sampled(oracle, li):
    cfg = WL.CONFIGS[3]
    check_exact_sampled(oracle, cfg, cfg.layers[li], "bf16", 30 + li)


@pytest.mark.parametrize("li", [0, 1, 2, 3])
def test_config4_exact_full_size_sampled(oracle, li):
    cfg = WL.CONFIGS[4]
    check_exact_sampled(oracle, cfg, cfg.layers[li], "bf16", 40 + li)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("li", list(range(10)))
def test_config5_exact_full_size_sampled(oracle, li, dtype):
    cfg = WL.CONFIGS[5]
    check_exact_sampled(oracle, cfg, cfg.layers[li], dtype, 50 + li)


@pytest.mark.parametrize("li", [2, 3, 4, 5, 6])
def test_paper_cases_exact_full_size_sampled(oracle, li):
    cfg = WL.CONFIGS[7]
    check_exact_sampled(oracle, cfg, cfg.layers[li], "f32", 70 + li)
