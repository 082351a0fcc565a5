"""gf_conv_bwd_filtered_static (the entry point for callers that cannot allocate: its scratch is a
static device array inside the library) against gf_conv_bwd_filtered with a caller's workspace:
same kernels, so every output must match bit for bit -- on two calls in a row, the second on a
smaller layer (the shared scratch then still holds the first call's contents), and for the
different scratch users (partial weight-gradient slabs, kernel sums, an own gy_u)."""
import pytest
import torch

import paper_2301_00330_amd.binding as B
import paper_2301_00330_amd.torch_api as T
from paper_2301_00330_amd import workloads as WL

pytestmark = pytest.mark.gpu


def _inputs(d, seed, dtype):
    s = T.shapes(d)
    g = torch.Generator(device="cpu").manual_seed(seed)
    td = WL.torch_dtype(dtype)
    x_u = torch.randn(s["x_u"], generator=g).abs().to(td).cuda()
    w = (torch.randn(s["w"], generator=g) * 0.1).to(td).cuda()
    gy = (torch.randn(s["g_y"], generator=g) * 1e-2).to(td).cuda()
    return x_u, w, gy


def _static(d, gy, x_u, w, want_gyu):
    s = T.shapes(d)
    g_w = torch.full(s["w"], float("nan"), dtype=torch.float32, device="cuda")
    g_x = torch.full(s["x"], float("nan"), dtype=gy.dtype, device="cuda")
    gy_u = torch.full(s["gy_u"], float("nan"), dtype=gy.dtype, device="cuda") if want_gyu else None
    B.gf_conv_bwd_filtered_static(d, B.ptr(gy), B.ptr(x_u), B.ptr(w), B.ptr(gy_u), B.ptr(g_w), B.ptr(g_x),
                                  int(torch.cuda.current_stream().cuda_stream))
    return g_w, g_x, gy_u


def mk(N, Ci, Co, H, W, K=1, s=1, p=0, g=1, r=2, dtype="f32"):
    return B.ConvDesc(N=N, C_in=Ci, C_out=Co, H_in=H, W_in=W, K_h=K, K_w=K, stride=s, pad=p, dilation=1,
                      groups=g, r=r, dtype=B.GF_BF16 if dtype == "bf16" else B.GF_F32)


PAIRS = [
    # a large layer, then a smaller one of the same kind (dense 3x3: slabs + kernel sums + own gy_u)
    (mk(16, 128, 160, 14, 14, 3, 1, 1), mk(3, 40, 24, 7, 7, 3, 1, 1)),
    # pointwise with few input channels (one-pass kernel: per-tile slabs), then a depthwise layer
    (mk(8, 24, 144, 56, 56), mk(4, 48, 48, 28, 28, 3, 1, 1, 48)),
    # strided dense, then vanilla BP (r = 1) through the same entry
    (mk(8, 64, 128, 14, 14, 3, 2, 1, r=2), mk(2, 16, 24, 9, 9, 3, 1, 1, r=1)),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("want_gyu", [True, False])
@pytest.mark.parametrize("pair", PAIRS)
def test_static_scratch_entry_matches_workspace_entry(pair, want_gyu, dtype):
    assert torch.cuda.is_available(), "these tests need the MI355X"
    code = B.GF_BF16 if dtype == "bf16" else B.GF_F32
    for k, d0 in enumerate(pair):                 # two calls in a row, the second on the smaller layer
        d = d0.with_(dtype=code)
        x_u, w, gy = _inputs(d, 77 + k, dtype)
        assert B.gf_workspace_bytes(d, B.GF_OP_BWD_FILTERED) <= B.GF_STATIC_SCRATCH_BYTES
        ref_gw, ref_gx, ref_gyu = T.conv_bwd_filtered(d, gy, x_u, w, want_gyu=want_gyu)
        g_w, g_x, gy_u = _static(d, gy, x_u, w, want_gyu)
        torch.cuda.synchronize()
        assert torch.equal(g_w, ref_gw), f"g_w, call {k}"
        assert torch.equal(g_x, ref_gx), f"g_x, call {k}"
        if want_gyu:
            assert torch.equal(gy_u, ref_gyu), f"gy_u, call {k}"


def test_static_scratch_entry_rejects_layers_beyond_its_size():
    """Config 4's 2048 -> 256 layer at r = 2 needs 73 MB of scratch: refused on the host, nothing runs."""
    cfg = WL.CONFIGS[4]
    d = T.desc_for(cfg.layers[0], cfg.N, 2, "bf16")
    assert B.gf_workspace_bytes(d, B.GF_OP_BWD_FILTERED) > B.GF_STATIC_SCRATCH_BYTES
    t = torch.zeros(64, dtype=torch.bfloat16, device="cuda")   # never touched: the size check comes first
    with pytest.raises(B.GfError) as e:
        B.gf_conv_bwd_filtered_static(d, B.ptr(t), B.ptr(t), B.ptr(t), 0, B.ptr(t), B.ptr(t), 0)
    assert e.value.status == B.GF_ERR_WORKSPACE
