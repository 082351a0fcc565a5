"""GPU parity: every entry point of libgf, called through the C ABI, against the
CPU oracle on the same seeded inputs.

Tolerances (per output tensor, max|gpu - ref| / max|ref|): 1e-5 for fp32 and
2e-2 for bf16 storage with fp32 accumulation; the oracle accumulates in fp64 and
consumes the same (already rounded) inputs.  Layout / index tests use
integer-coded inputs whose sums are exact, and must agree bit for bit.
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
    B.lib()  # fail loudly if libgf.so was not built


def to64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def rel_err(gpu: torch.Tensor, ref: np.ndarray) -> float:
    g = to64(gpu)
    assert g.shape == ref.shape, (g.shape, ref.shape)
    den = np.abs(ref).max()
    return float(np.abs(g - ref).max() / (den if den > 0 else 1.0))


def rounded(a: np.ndarray, dtype: str) -> torch.Tensor:
    """oracle result -> the storage dtype (one round-to-nearest-even), as a CPU tensor"""
    return torch.from_numpy(np.ascontiguousarray(a)).to(WL.torch_dtype(dtype))


def odesc(oracle, d: B.ConvDesc):
    return oracle.Desc(N=d.N, C_in=d.C_in, C_out=d.C_out, H_in=d.H_in, W_in=d.W_in, K_h=d.K_h,
                       K_w=d.K_w, stride=d.stride, pad=d.pad, dilation=d.dilation, groups=d.groups, r=d.r)


def mk(N, Ci, Co, H, W, K=1, s=1, p=0, dl=1, g=1, r=2, dtype="f32"):
    return B.ConvDesc(N=N, C_in=Ci, C_out=Co, H_in=H, W_in=W, K_h=K, K_w=K, stride=s, pad=p,
                      dilation=dl, groups=g, r=r, dtype=B.GF_BF16 if dtype == "bf16" else B.GF_F32)


def randn(shape, seed, dtype, scale=1.0, relu=False):
    g = torch.Generator(device="cpu").manual_seed(seed)
    t = torch.randn(shape, generator=g, dtype=torch.float32) * scale
    if relu:
        t = t.abs()
    return t.to(WL.torch_dtype(dtype))


# ---------------------------------------------------------------------------
# S0 / S1: patch sum and patch mean
# ---------------------------------------------------------------------------
REDUCE_CASES = [
    # N  C   H   W   r  s
    (2, 3, 8, 8, 2, 1), (3, 5, 7, 7, 2, 1), (3, 5, 7, 7, 4, 1), (2, 4, 14, 14, 2, 2), (2, 4, 14, 14, 4, 2),
    (1, 2, 56, 56, 2, 1), (2, 3, 64, 64, 8, 1), (1, 3, 9, 5, 3, 1), (2, 2, 7, 7, 7, 1), (1, 2, 5, 6, 8, 1),
    (4, 37, 7, 7, 2, 1), (1, 1, 1, 1, 2, 1), (2, 3, 30, 40, 4, 1), (1, 2, 160, 120, 2, 1), (1, 1, 33, 4100, 4, 1),
    (1, 1, 12, 9000, 8, 1),     # one strip larger than the LDS staging budget
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", REDUCE_CASES)
def test_pool_and_filter(oracle, case, dtype):
    N, C, H, W, r, s = case
    # a "same"-padded 3x3 layer with that stride: H_y = ceil(H / s)
    d = mk(N, C, C, H, W, K=3, s=s, p=1, r=r, dtype=dtype)
    Hy, Wy, Hp, Wp = B.gf_out_shape(d)
    x = randn((N, C, H, W), 11, dtype)
    gy = randn((N, C, Hy, Wy), 12, dtype)
    od = odesc(oracle, d)
    x_u = T.pool_activation(d, x.cuda())
    gy_u = T.filter_grad(d, gy.cuda())
    torch.cuda.synchronize()
    assert tuple(x_u.shape) == (N, C, Hp, Wp) and tuple(gy_u.shape) == (N, C, Hp, Wp)
    assert rel_err(x_u, oracle.pool_activation(od, to64(x))) <= TOL[dtype]
    assert rel_err(gy_u, oracle.filter_grad(od, to64(gy))) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("H,W,r,s", [(8, 8, 2, 1), (16, 16, 4, 1), (56, 56, 2, 1), (64, 64, 8, 1), (16, 16, 2, 2),
                                     (7, 7, 2, 1), (14, 14, 4, 1)])
def test_patch_layout_bit_exact(oracle, H, W, r, s, dtype):
    """Integer-coded maps: all sums are exact, so patch positions, the ragged-edge
    rule and the row-major [N, C, H_p, W_p] layout must match bit for bit.  (Ragged
    patches here hold 1, 2, 4, 8 or 16 pixels and g_y is a multiple of r*r, so the
    means are exact too.)"""
    N, C = 3, 5
    d = mk(N, C, C, H, W, K=3, s=s, p=1, r=r, dtype=dtype)
    Hy, Wy, Hp, Wp = B.gf_out_shape(d)
    x = WL.integer_coded((N, C, H, W), 5, dtype=dtype)
    gy = WL.integer_coded((N, C, Hy, Wy), 6, dtype=dtype) * (r * r)
    od = odesc(oracle, d)
    x_u = T.pool_activation(d, x.cuda())
    gy_u = T.filter_grad(d, gy.cuda())
    ref_x = oracle.pool_activation(od, to64(x))
    ref_g = oracle.filter_grad(od, to64(gy))
    assert np.array_equal(to64(x_u), ref_x)
    assert np.array_equal(to64(gy_u), ref_g)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", REDUCE_CASES + [(2, 3, 9, 9, 1, 1), (8, 64, 56, 56, 2, 1), (8, 96, 28, 28, 4, 1)])
def test_filter_with_noise_figures(oracle, case, dtype):
    """The filter's by-product (Sec. 3.4, first line of Eq. 8): energy of g_y and of what the
    filter removes, against the fp64 oracle on the same (rounded) input; the filtered map itself
    is the one gf_filter_grad writes, bit for bit."""
    N, C, H, W, r, s = case
    d = mk(N, C, C, H, W, K=3, s=s, p=1, r=r, dtype=dtype)
    Hy, Wy, Hp, Wp = B.gf_out_shape(d)
    gy = randn((N, C, Hy, Wy), 13, dtype) + 0.25
    gyg = gy.cuda()
    gy_u, stats = T.filter_grad_snr(d, gyg)
    plain = T.filter_grad(d, gyg)
    torch.cuda.synchronize()
    assert torch.equal(gy_u, plain)
    e, v = oracle.filter_snr(odesc(oracle, d), to64(gy))
    got = stats.cpu().numpy()
    assert abs(got[0] - e) <= 1e-5 * e
    if r == 1 or (Hy <= 1 and Wy <= 1):
        assert got[1] == 0.0 and v == 0.0
    else:
        assert abs(got[1] - v) <= 1e-5 * v


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("H,W,r", [(8, 8, 2), (16, 16, 4), (16, 16, 8), (14, 14, 2), (32, 32, 2)])
def test_noise_figures_bit_exact_on_integers(oracle, H, W, r, dtype):
    """Small integers times r*r: means and squares are integers and every partial sum stays
    below 2^24 (at most 6144 terms of at most 96^2), so both sums equal the oracle's whatever
    the order; a patch-constant map has no noise at all."""
    N, C = 2, 3
    d = mk(N, C, C, H, W, K=3, p=1, r=r, dtype=dtype)
    gy = WL.integer_coded((N, C, H, W), 8, lo=-3, hi=3, dtype=dtype) * (r * r)
    _, stats = T.filter_grad_snr(d, gy.cuda())
    e, v = oracle.filter_snr(odesc(oracle, d), to64(gy))
    assert stats.cpu().tolist() == [e, v]
    const = WL.integer_coded((N, C, H // r, W // r), 9, dtype=dtype)
    const = const.repeat_interleave(r, 2).repeat_interleave(r, 3).contiguous()
    gy_u, stats = T.filter_grad_snr(d, const.cuda())
    assert stats[1].item() == 0.0 and stats[0].item() == float((to64(const) ** 2).sum())
    assert torch.equal(gy_u.cpu(), const[:, :, ::r, ::r])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("hi", [float("inf"), 6.0])
@pytest.mark.parametrize("case", REDUCE_CASES + [(2, 3, 9, 9, 1, 1), (4, 24, 56, 56, 2, 1)])
def test_pool_with_mask_fraction(oracle, case, dtype, hi):
    """gf_pool_activation_mask: x_u bit-identical to gf_pool_activation, m_u = the share of each patch
    through which a (clipped) ReLU passes a gradient, against the oracle on the same rounded x."""
    N, C, H, W, r, s = case
    d = mk(N, C, C, H, W, K=3, s=s, p=1, r=r, dtype=dtype)
    x = (randn((N, C, H, W), 21, dtype) * 4.0 + 2.0).clamp(min=0.0)     # a ReLU output with values beyond 6
    xg = x.cuda()
    x_u, m_u = T.pool_activation_mask(d, xg, hi)
    plain = T.pool_activation(d, xg)
    torch.cuda.synchronize()
    assert torch.equal(x_u, plain)
    _, ref_m = oracle.pool_activation_mask(odesc(oracle, d), to64(x), hi)
    assert tuple(m_u.shape) == ref_m.shape
    # counts over at most 64 pixels divided by the in-bounds count: one rounding of an exact quotient
    assert np.abs(to64(m_u) - ref_m).max() <= (4e-3 if dtype == "bf16" else 1e-6)
    pow2 = (r * s) in (1, 2, 4, 8) and H % (r * s) == 0 and W % (r * s) == 0
    if pow2:
        assert np.array_equal(to64(m_u), ref_m)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", [(3, 24, 40, 12, 12, 1, 1, 0, 1, 1, 2), (4, 48, 48, 12, 12, 3, 1, 1, 1, 48, 2),
                                  (2, 32, 48, 14, 14, 3, 2, 1, 1, 1, 2), (2, 16, 16, 24, 24, 3, 1, 6, 6, 1, 4),
                                  (3, 12, 18, 10, 10, 3, 1, 1, 1, 3, 2), (3, 24, 144, 56, 56, 1, 1, 0, 1, 1, 2)])
def test_chained_entry_with_mask(oracle, case, dtype):
    """A layer above a ReLU in a chain: the reduced input gradient times the mask fraction is what the
    lower layer's filter would make of the masked full-resolution gradient (oracle: exactly that)."""
    N, Ci, Co, H, W, K, s, p, dl, g, r = case
    d = mk(N, Ci, Co, H, W, K, s, p, dl, g, r, dtype)
    od = odesc(oracle, d)
    Hy, Wy, Hp, Wp = B.gf_out_shape(d)
    x = (randn((N, Ci, H, W), 61, dtype) * 2.0 + 0.5).clamp(min=0.0)
    w = randn((Co, Ci // g, K, K), 62, dtype, scale=(2.0 / (Ci // g * K * K)) ** 0.5)
    gyu = randn((N, Co, Hp, Wp), 63, dtype, scale=1e-2)
    x_u, m_u = T.pool_activation_mask(d, x.cuda())
    g_w, g_xu = T.conv_bwd_chained(d, gyu.cuda(), x_u, w.cuda(), reduced_out=True, mask_u=m_u)
    g_w0, g_xu0 = T.conv_bwd_chained(d, gyu.cuda(), x_u, w.cuda(), reduced_out=True)
    torch.cuda.synchronize()
    assert torch.equal(g_w, g_w0)
    # oracle: full-resolution gradient of the upper layer, masked by the ReLU, filtered by the layer below
    gx_full = oracle.bwd_input(od, to64(gyu), to64(w))
    masked = gx_full * (to64(x) > 0)
    lower = oracle.Desc(N=N, C_in=1, C_out=Ci, H_in=H, W_in=W, K_h=1, K_w=1, r=r * s)
    ref = oracle.filter_grad(lower, masked)
    assert rel_err(g_xu, ref) <= TOL[dtype]
    # and it is the unmasked result times the fraction, rounded once
    prod = (g_xu0.float() * m_u.float()).to(g_xu0.dtype)
    assert torch.equal(g_xu, prod)


def test_r1_reductions_are_copies():
    d = mk(2, 3, 4, 14, 14, K=3, s=2, p=1, r=1, dtype="bf16")
    x = randn((2, 3, 14, 14), 1, "bf16").cuda()
    gy = randn((2, 4, 7, 7), 2, "bf16").cuda()
    assert torch.equal(T.pool_activation(d, x), x)
    assert torch.equal(T.filter_grad(d, gy), gy)


# ---------------------------------------------------------------------------
# S3 / S4 from given reduced maps
# ---------------------------------------------------------------------------
GF_CASES = [
    # N  Ci  Co  H   W  K  s  p  dl g   r
    (1, 16, 16, 16, 16, 3, 1, 1, 1, 1, 2),        # config 1
    (3, 24, 40, 12, 12, 1, 1, 0, 1, 1, 2),        # pointwise, channels not multiples of the tile
    (2, 70, 130, 7, 7, 3, 1, 1, 1, 1, 2),         # ragged 7x7, P = 16, several tiles with tails
    (5, 64, 96, 7, 7, 3, 1, 1, 1, 1, 4),          # P = 4
    (2, 32, 64, 14, 14, 3, 1, 1, 1, 1, 2),        # P = 49 (odd)
    (2, 32, 48, 14, 14, 3, 2, 1, 1, 1, 2),        # strided 14 -> 7, r_x = 4
    (2, 16, 16, 24, 24, 3, 1, 6, 6, 1, 4),        # dilated
    (3, 12, 18, 10, 10, 3, 1, 1, 1, 3, 2),        # grouped
    (4, 48, 48, 12, 12, 3, 1, 1, 1, 48, 2),       # depthwise
    (3, 40, 40, 7, 7, 3, 1, 1, 1, 40, 2),         # depthwise, ragged
    (3, 24, 24, 14, 14, 3, 2, 1, 1, 24, 2),       # depthwise, strided
    (2, 8, 8, 9, 9, 3, 1, 1, 1, 1, 3),            # r = 3
    (2, 8, 12, 7, 7, 3, 1, 1, 1, 1, 7),           # one patch per plane
    (2, 6, 6, 5, 5, 5, 1, 2, 1, 1, 8),            # r > H
    (1, 1, 1, 4, 4, 3, 1, 1, 1, 1, 2),            # the worked 4x4 example's shape
    (9, 200, 72, 8, 8, 1, 1, 0, 1, 1, 2),         # batch split across several slabs
    (2, 32, 24, 32, 32, 1, 1, 0, 1, 1, 8),        # r_x = 8: one patch spans whole 16-byte runs
    (2, 16, 32, 16, 16, 3, 2, 1, 1, 1, 2),        # strided with aligned rows, r_x = 4
    (2, 40, 24, 24, 16, 3, 1, 1, 1, 1, 4),        # H ragged (24 = 6 x 4), W aligned
    (1, 136, 264, 16, 16, 1, 1, 0, 1, 1, 2),      # several channel tiles in both directions
    (6, 72, 640, 7, 7, 1, 1, 0, 1, 1, 2),         # long K = C_out, few tiles: waves split K (P = 16)
    (3, 40, 600, 14, 14, 1, 1, 0, 1, 1, 2),       # same with P = 49 and uneven K split
    (2, 48, 512, 7, 7, 3, 1, 1, 1, 1, 4),         # P = 4: image blocks, 16 (bf16) / 8 (fp32) images per K chunk
    (2, 64, 544, 16, 16, 1, 1, 0, 1, 1, 2),       # K split with aligned rows (pixel-run store)
    (19, 24, 40, 7, 7, 3, 1, 1, 1, 1, 4),         # P = 4, batch not a multiple of the images per chunk
    (3, 72, 200, 6, 6, 1, 1, 0, 1, 1, 2),         # P = 9: seven images per chunk, blocks 16-byte aligned
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", GF_CASES)
def test_filtered_backward_steps(oracle, case, dtype):
    N, Ci, Co, H, W, K, s, p, dl, g, r = case
    d = mk(N, Ci, Co, H, W, K, s, p, dl, g, r, dtype)
    od = odesc(oracle, d)
    Hy, Wy, Hp, Wp = B.gf_out_shape(d)
    x = randn((N, Ci, H, W), 21, dtype, relu=True)
    w = randn((Co, Ci // g, K, K), 22, dtype, scale=(2.0 / (Ci // g * K * K)) ** 0.5)
    gy = randn((N, Co, Hy, Wy), 23, dtype, scale=1e-2)
    # reduced maps from the ORACLE, rounded once to the storage dtype, feed both sides
    x_u = rounded(oracle.pool_activation(od, to64(x)), dtype)
    gy_u = rounded(oracle.filter_grad(od, to64(gy)), dtype)
    ref_gw = oracle.bwd_weight(od, to64(x_u), to64(gy_u))
    ref_gx = oracle.bwd_input(od, to64(gy_u), to64(w))
    ref_gxu = oracle.bwd_input(od, to64(gy_u), to64(w), reduced_out=True)

    g_w = T.conv_bwd_weight(d, x_u.cuda(), gy_u.cuda())
    g_x = T.conv_bwd_input(d, gy_u.cuda(), w.cuda())
    g_xu = T.conv_bwd_input(d, gy_u.cuda(), w.cuda(), reduced_out=True)
    torch.cuda.synchronize()
    assert g_w.dtype == torch.float32
    assert rel_err(g_w, ref_gw) <= TOL[dtype]
    assert rel_err(g_x, ref_gx) <= TOL[dtype]
    assert rel_err(g_xu, ref_gxu) <= TOL[dtype]
    # structure with exactly one right answer: taps identical, patches constant, reduced == unique view
    gw = g_w.cpu()
    assert torch.equal(gw, gw[:, :, :1, :1].expand_as(gw))
    rx = r * s
    up = g_xu.repeat_interleave(rx, 2).repeat_interleave(rx, 3)[:, :, :H, :W]
    assert torch.equal(up, g_x)


FUSED_EXTRA = [
    (4, 48, 48, 56, 56, 3, 1, 1, 1, 48, 2),       # depthwise, aligned rows (register variant), 2 planes per block
    (3, 7, 7, 64, 64, 3, 1, 1, 1, 7, 4),          # odd plane count, r = 4
    (2, 6, 6, 32, 32, 3, 1, 1, 1, 6, 8),          # r = 8
    (2, 5, 5, 40, 120, 3, 1, 1, 1, 5, 2),         # more than one 256-item chunk per plane
    (5, 24, 24, 14, 14, 3, 1, 1, 1, 24, 2),       # depthwise 14x14 (LDS variant)
    (6, 33, 33, 7, 7, 3, 1, 1, 1, 33, 2),         # ragged 7x7, odd plane count: unaligned block runs
    (3, 10, 10, 7, 7, 3, 1, 1, 1, 10, 4),         # ragged, r = 4
    (2, 9, 9, 9, 9, 3, 1, 1, 1, 9, 3),            # r = 3 (run-time patch size)
    (1, 3, 3, 5, 5, 5, 1, 2, 1, 3, 8),            # one patch per plane, tiny tensor
    (5, 33, 33, 15, 13, 3, 2, 1, 1, 33, 2),       # depthwise, strided, odd map and odd plane count (one-pass strided variant)
    (2, 10, 10, 18, 18, 3, 3, 1, 1, 10, 2),       # depthwise, stride 3
    (3, 16, 16, 28, 28, 3, 2, 1, 1, 16, 4),       # depthwise, strided, ragged patches on g_y (14 = 3 x 4 + 2)
    (1, 3, 3, 6, 6, 3, 2, 1, 1, 3, 8),            # depthwise, strided, one patch per plane
    (3, 24, 144, 56, 56, 1, 1, 0, 1, 1, 2),       # MobileNetV2 expand shape
    (3, 144, 24, 56, 56, 1, 1, 0, 1, 1, 2),       # MobileNetV2 project shape
    (2, 40, 56, 32, 32, 3, 1, 1, 1, 1, 4),        # 3x3, r = 4, channels not multiples of 16
    (5, 16, 16, 16, 16, 3, 1, 1, 1, 1, 2),        # several units per block, W_p = 8
    (2, 20, 36, 64, 64, 1, 1, 0, 1, 1, 8),        # r = 8
    (1, 64, 64, 22, 24, 3, 1, 1, 1, 1, 2),        # ragged H (22 = 11 x 2), W_p = 12
    # pointwise layers with few input channels (one-pass kernel) and their mirror shapes
    (3, 8, 256, 15, 16, 1, 1, 0, 1, 1, 2),        # ragged H, tiles straddle images, eight chunks of C_y, C_x < 16
    (2, 160, 32, 6, 16, 1, 1, 0, 1, 1, 2),        # many input channels: the merged-launch path; three patch rows per image
    (1, 32, 72, 10, 128, 1, 1, 0, 1, 1, 2),       # W_p = 64: one patch row per tile; partial last chunk
    (5, 24, 48, 28, 28, 1, 1, 0, 1, 1, 2),        # W_p = 14 (narrow x_u loads), four patch rows per tile, tail tile
    (2, 96, 24, 8, 24, 1, 1, 0, 1, 1, 2),         # project shape, W_p = 12
    (7, 16, 40, 6, 8, 1, 1, 0, 1, 1, 2),          # W_p = 4: sixteen patch rows per tile, two images and a tail
    (2, 16, 48, 10, 16, 1, 1, 0, 1, 1, 4),        # one-pass kernel at r = 4: ragged H, tiles straddle images
    (1, 32, 272, 8, 64, 1, 1, 0, 1, 1, 4),        # ... many chunks of C_y (fp32: 17 chunks of 16 -> the merged-launch path)
    (3, 24, 144, 56, 56, 1, 1, 0, 1, 1, 4),       # expand / project shapes at r = 4: P = 196 is no vector multiple in bf16
    (3, 144, 24, 56, 56, 1, 1, 0, 1, 1, 4),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("want_gyu", [True, False])
@pytest.mark.parametrize("case", GF_CASES + FUSED_EXTRA)
def test_fused_entry_matches_separate_calls(oracle, case, dtype, want_gyu):
    """gf_conv_bwd_filtered against the oracle, and against the three separate entry
    points: g_x and gy_u bit for bit, g_w within the fp32 summation tolerance."""
    N, Ci, Co, H, W, K, s, p, dl, g, r = case
    d = mk(N, Ci, Co, H, W, K, s, p, dl, g, r, dtype)
    od = odesc(oracle, d)
    Hy, Wy, Hp, Wp = B.gf_out_shape(d)
    x = randn((N, Ci, H, W), 51, dtype, relu=True)
    w = randn((Co, Ci // g, K, K), 52, dtype, scale=(2.0 / (Ci // g * K * K)) ** 0.5)
    gy = randn((N, Co, Hy, Wy), 53, dtype, scale=1e-2)
    x_u = rounded(oracle.pool_activation(od, to64(x)), dtype).cuda()
    gyg, wg = gy.cuda(), w.cuda()
    g_w, g_x, gy_u = T.conv_bwd_filtered(d, gyg, x_u, wg, want_gyu=want_gyu)
    s_gyu = T.filter_grad(d, gyg)
    s_gw = T.conv_bwd_weight(d, x_u, s_gyu)
    s_gx = T.conv_bwd_input(d, s_gyu, wg)
    torch.cuda.synchronize()
    assert torch.equal(g_x, s_gx)
    if want_gyu:
        assert torch.equal(gy_u, s_gyu)
    else:
        assert gy_u is None
    gw_tol = 1e-5 if dtype == "f32" else 1e-5   # same rounded operands, only the fp32 summation order differs
    assert float((g_w - s_gw).abs().max()) <= gw_tol * float(s_gw.abs().max() + 1e-30)
    # and against the oracle: the filter from the same g_y; the two contractions from the oracle's own
    # filtered gradient rounded once to the storage type (where the library rounds it too)
    ref_gyu = oracle.filter_grad(od, to64(gy))
    ref_gyu_r = to64(rounded(ref_gyu, dtype))
    ref_gw = oracle.bwd_weight(od, to64(x_u), ref_gyu_r)
    ref_gx = oracle.bwd_input(od, ref_gyu_r, to64(w))
    assert rel_err(s_gyu, ref_gyu) <= TOL[dtype]
    assert rel_err(g_w, ref_gw) <= TOL[dtype]
    assert rel_err(g_x, ref_gx) <= TOL[dtype]


def _random_cases(count, seed):
    """Seeded random layers that satisfy the patch-grid rule ("same"-padded), mixing the properties that
    select kernels: aligned and odd map widths, channel counts that are / are not vector multiples, few
    and many channels, pointwise / 3x3 / 5x5, stride, dilation, depthwise and grouped."""
    rs = np.random.RandomState(seed)
    out = []
    while len(out) < count:
        K = int(rs.choice([1, 1, 3, 3, 5]))
        dl = int(rs.choice([1, 1, 2])) if K > 1 else 1
        s = int(rs.choice([1, 1, 1, 2]))
        r = int(rs.choice([2, 2, 2, 4, 3]))
        W = int(rs.choice([8, 12, 16, 24, 28, 32, 56, 7, 9, 14, 15, 20]))
        H = int(rs.choice([W, max(4, W - 3), W + 2, 6]))
        kind = rs.choice(["dense", "dense", "dense", "dw", "grouped"])
        if kind == "dw":
            Ci = Co = int(rs.choice([3, 8, 16, 24, 40]))
            g = Ci
        elif kind == "grouped":
            g = int(rs.choice([2, 4]))
            Ci, Co = g * int(rs.choice([2, 4, 6])), g * int(rs.choice([3, 4, 8]))
        else:
            g = 1
            Ci = int(rs.choice([8, 16, 24, 32, 40, 72, 96, 144, 10]))
            Co = int(rs.choice([8, 24, 32, 48, 80, 144, 160, 12]))
        p = dl * (K - 1) // 2
        N = int(rs.choice([1, 2, 3, 5]))
        if (H + 2 * p - dl * (K - 1) - 1) // s + 1 < 1:
            continue
        out.append((N, Ci, Co, H, W, K, s, p, dl, g, r))
    return out


RANDOM_CASES = _random_cases(48, 20230100)


def _random_pointwise_cases(count, seed):
    """Pointwise stride-1 layers on aligned maps: the shapes of the one-pass kernel (few input channels)
    and of the patch-row store epilogue, with odd heights, tiles that straddle images and tail tiles."""
    rs = np.random.RandomState(seed)
    out = []
    for _ in range(count):
        r = int(rs.choice([2, 2, 4]))
        W = int(rs.choice([8, 16, 24, 32, 40, 56, 64, 112]))
        H = int(rs.choice([r, 2 * r + 1, 3 * r, 9, 14, 28]))
        Ci = int(rs.choice([8, 16, 24, 32, 48, 144]))
        Co = int(rs.choice([8, 24, 40, 96, 144, 272]))
        N = int(rs.choice([1, 2, 3, 7]))
        out.append((N, Ci, Co, H, W, 1, 1, 0, 1, 1, r))
    return out


RANDOM_POINTWISE = _random_pointwise_cases(32, 330)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", RANDOM_CASES + RANDOM_POINTWISE)
def test_random_layers_one_call_and_chain(oracle, case, dtype):
    """gf_conv_bwd_filtered and gf_conv_bwd_chained (reduced and full output) on seeded random layers,
    each against the oracle on the same rounded inputs."""
    N, Ci, Co, H, W, K, s, p, dl, g, r = case
    d = mk(N, Ci, Co, H, W, K, s, p, dl, g, r, dtype)
    try:
        Hy, Wy, Hp, Wp = B.gf_out_shape(d)
    except B.GfError as e:          # the generator may produce a layer that breaks the patch-grid rule
        assert e.status == B.GF_ERR_SHAPE
        pytest.skip("patch grids of x and g_y differ")
    od = odesc(oracle, d)
    x = randn((N, Ci, H, W), 71, dtype, relu=True)
    w = randn((Co, Ci // g, K, K), 72, dtype, scale=(2.0 / (Ci // g * K * K)) ** 0.5)
    gy = randn((N, Co, Hy, Wy), 73, dtype, scale=1e-2)
    x_u = T.pool_activation(d, x.cuda())
    g_w, g_x, gy_u = T.conv_bwd_filtered(d, gy.cuda(), x_u, w.cuda(), want_gyu=True)
    n_gw, n_gx, _ = T.conv_bwd_filtered(d, gy.cuda(), x_u, w.cuda(), want_gyu=False)
    c_gw, c_gxu = T.conv_bwd_chained(d, gy_u, x_u, w.cuda(), reduced_out=True)
    f_gw, f_gx = T.conv_bwd_chained(d, gy_u, x_u, w.cuda(), reduced_out=False)
    torch.cuda.synchronize()
    assert torch.equal(n_gx, g_x) and torch.equal(n_gw, g_w)
    ref_gw, ref_gx, ref_xu, ref_gyu = oracle.gf_backward(od, to64(x), to64(w), to64(gy))
    tol = TOL[dtype]
    assert rel_err(x_u, ref_xu) <= tol, "x_u"
    assert rel_err(gy_u, ref_gyu) <= tol, "gy_u"
    assert rel_err(g_w, ref_gw) <= tol, "g_w"
    assert rel_err(g_x, ref_gx) <= tol, "g_x"
    assert rel_err(c_gw, ref_gw) <= tol and rel_err(f_gw, ref_gw) <= tol, "chained g_w"
    assert rel_err(f_gx, ref_gx) <= tol, "chained g_x"
    ref_red = oracle.bwd_input(od, to64(gy_u), to64(w), reduced_out=True)
    assert rel_err(c_gxu, ref_red) <= tol, "chained reduced g_x"


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", RANDOM_CASES[:24])
def test_random_layers_exact(oracle, case, dtype):
    """Vanilla BP on the same random layers (r = 1 lifts the patch-grid rule)."""
    N, Ci, Co, H, W, K, s, p, dl, g, r = case
    d = mk(N, Ci, Co, H, W, K, s, p, dl, g, 1, dtype)
    Hy, Wy, _, _ = B.gf_out_shape(d)
    od = odesc(oracle, d)
    x = randn((N, Ci, H, W), 81, dtype)
    w = randn((Co, Ci // g, K, K), 82, dtype, scale=(2.0 / (Ci // g * K * K)) ** 0.5)
    gy = randn((N, Co, Hy, Wy), 83, dtype, scale=1e-2)
    g_w, g_x = T.conv_bwd_exact(d, x.cuda(), w.cuda(), gy.cuda())
    torch.cuda.synchronize()
    ref_gw, ref_gx = oracle.bwd_exact(od, to64(x), to64(w), to64(gy))
    assert rel_err(g_w, ref_gw) <= TOL[dtype], "g_w"
    assert rel_err(g_x, ref_gx) <= TOL[dtype], "g_x"


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("reduced_out", [True, False])
@pytest.mark.parametrize("case", GF_CASES + FUSED_EXTRA)
def test_chained_entry_matches_separate_calls(oracle, case, dtype, reduced_out):
    """gf_conv_bwd_chained (the layer inside a chain: reduced gradient in, reduced or full
    gradient out) against the oracle and against gf_conv_bwd_weight + gf_conv_bwd_input:
    g_x bit for bit, g_w within the fp32 summation tolerance."""
    N, Ci, Co, H, W, K, s, p, dl, g, r = case
    d = mk(N, Ci, Co, H, W, K, s, p, dl, g, r, dtype)
    od = odesc(oracle, d)
    Hy, Wy, Hp, Wp = B.gf_out_shape(d)
    x = randn((N, Ci, H, W), 61, dtype, relu=True)
    w = randn((Co, Ci // g, K, K), 62, dtype, scale=(2.0 / (Ci // g * K * K)) ** 0.5)
    gyu = randn((N, Co, Hp, Wp), 63, dtype, scale=1e-2)
    x_u = rounded(oracle.pool_activation(od, to64(x)), dtype).cuda()
    gyug, wg = gyu.cuda(), w.cuda()
    g_w, g_x = T.conv_bwd_chained(d, gyug, x_u, wg, reduced_out=reduced_out)
    s_gw = T.conv_bwd_weight(d, x_u, gyug)
    s_gx = T.conv_bwd_input(d, gyug, wg, reduced_out=reduced_out)
    torch.cuda.synchronize()
    assert torch.equal(g_x, s_gx)
    assert float((g_w - s_gw).abs().max()) <= 1e-5 * float(s_gw.abs().max() + 1e-30)
    assert rel_err(g_w, oracle.bwd_weight(od, to64(x_u), to64(gyu))) <= TOL[dtype]
    assert rel_err(g_x, oracle.bwd_input(od, to64(gyu), to64(w), reduced_out=reduced_out)) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_chain_of_layers_equals_layer_by_layer(oracle, dtype):
    """The MobileNetV2 block of configuration 2, back to front (project, depthwise, expand), at a
    sub-batch.  Chained: one filter at the top, reduced maps handed down, full resolution only at
    the bottom.  Layer by layer: every layer gets the full-resolution gradient and filters it
    itself.  With r = 2 every patch mean of a patch-constant map is exact, so the two agree bit
    for bit on every g_x; the weight gradients agree to the summation tolerance; the fp32 run is
    also checked against the oracle run layer by layer in fp64."""
    cfg = WL.CONFIGS[2]
    N, r = 4, 2
    expand, dw, project = cfg.layers
    ds = [T.desc_for(L, N, r, dtype) for L in (project, dw, expand)]
    xs, ws = [], []
    for i, L in enumerate((project, dw, expand)):
        x, w, gy = WL.make_inputs(cfg, L, dtype, N=N, seed=900 + i)
        xs.append(x); ws.append(w)
        if i == 0:
            g_top = gy
    xus = [T.pool_activation(d, x.cuda()) for d, x in zip(ds, xs)]
    # layer by layer
    g = g_top.cuda()
    lbl_gw = []
    for d, xu, w in zip(ds, xus, ws):
        gw, g, _ = T.conv_bwd_filtered(d, g, xu, w.cuda())
        lbl_gw.append(gw)
    lbl_gx = g
    # chained
    gu = T.filter_grad(ds[0], g_top.cuda())
    ch_gw = []
    for i, (d, xu, w) in enumerate(zip(ds, xus, ws)):
        gw, gu = T.conv_bwd_chained(d, gu, xu, w.cuda(), reduced_out=(i < 2))
        ch_gw.append(gw)
    torch.cuda.synchronize()
    assert torch.equal(gu, lbl_gx)
    for a, b in zip(ch_gw, lbl_gw):
        assert float((a - b).abs().max()) <= 1e-5 * float(b.abs().max() + 1e-30)
    if dtype == "f32":
        ref = to64(g_top)
        for i, (d, x, w) in enumerate(zip(ds, xs, ws)):
            rgw, ref, _, _ = oracle.gf_backward(odesc(oracle, d), to64(x), to64(w), ref)
            assert rel_err(ch_gw[i], rgw) <= 5e-5     # three chained fp32 layers
        assert rel_err(gu, ref) <= 5e-5


def test_fused_entry_r1_is_vanilla_bp(oracle):
    d = mk(2, 6, 8, 9, 9, 3, 1, 1, 1, 1, 1, "f32")
    od = odesc(oracle, d)
    x, w, gy = randn((2, 6, 9, 9), 1, "f32"), randn((8, 6, 3, 3), 2, "f32"), randn((2, 8, 9, 9), 3, "f32")
    g_w, g_x, gy_u = T.conv_bwd_filtered(d, gy.cuda(), x.cuda(), w.cuda())
    ref_gw, ref_gx = oracle.bwd_exact(od, to64(x), to64(w), to64(gy))
    assert torch.equal(gy_u.cpu(), gy)
    assert rel_err(g_w, ref_gw) <= 1e-5 and rel_err(g_x, ref_gx) <= 1e-5


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("g,s", [(1, 1), (16, 1), (1, 2), (4, 1)])
def test_filtered_backward_bit_exact_on_integers(oracle, g, s, dtype):
    """Channel pairing, group ranges and the patch -> pixel map with integer-coded
    reduced maps and weights (power-of-two scale 1/s^2): every partial sum is an
    integer below 2^24, so any summation order gives the same bits."""
    N, Ci, Co, H, K, r = 4, 16, 16 if g != 4 else 32, 8 * s, 3, 2
    d = mk(N, Ci, Co, H, H, K, s, 1, 1, g, r, dtype)
    od = odesc(oracle, d)
    _, _, Hp, Wp = B.gf_out_shape(d)
    x_u = WL.integer_coded((N, Ci, Hp, Wp), 31, dtype=dtype)
    gy_u = WL.integer_coded((N, Co, Hp, Wp), 32, dtype=dtype)
    w = WL.integer_coded((Co, Ci // g, K, K), 33, lo=-2, hi=2, dtype=dtype)
    g_w = T.conv_bwd_weight(d, x_u.cuda(), gy_u.cuda())
    g_x = T.conv_bwd_input(d, gy_u.cuda(), w.cuda())
    assert np.array_equal(to64(g_w), oracle.bwd_weight(od, to64(x_u), to64(gy_u)))
    ref_gx = oracle.bwd_input(od, to64(gy_u), to64(w))
    # fp32 holds these integers exactly; bf16 storage rounds the exact value once
    assert np.array_equal(to64(g_x), to64(rounded(ref_gx, dtype)))


# ---------------------------------------------------------------------------
# S5 exact BP, and r == 1 through the filtered entries
# ---------------------------------------------------------------------------
EXACT_CASES = [
    (2, 6, 8, 9, 9, 3, 1, 1, 1, 1), (2, 8, 8, 14, 14, 3, 2, 1, 1, 1), (1, 8, 8, 12, 12, 3, 1, 4, 4, 1),
    (2, 12, 12, 10, 10, 3, 1, 1, 1, 12), (2, 8, 12, 14, 14, 3, 2, 1, 1, 4), (3, 10, 7, 6, 8, 1, 1, 0, 1, 1),
    (1, 4, 4, 11, 11, 5, 1, 2, 1, 1), (1, 5, 6, 8, 8, 3, 1, 0, 1, 1), (1, 16, 16, 16, 16, 3, 1, 1, 1, 1),
    (3, 72, 136, 14, 14, 3, 1, 1, 1, 1), (2, 64, 96, 7, 7, 3, 1, 1, 1, 1), (2, 40, 80, 14, 14, 3, 2, 1, 1, 1),
    (2, 32, 48, 24, 24, 3, 1, 6, 6, 1), (4, 130, 70, 8, 8, 1, 1, 0, 1, 1), (2, 256, 288, 16, 16, 3, 1, 1, 1, 1),
    (1, 24, 24, 56, 56, 1, 1, 0, 1, 1), (2, 16, 24, 9, 7, 3, 2, 1, 1, 1),
    # dense stride-1 "same"-size layers (implicit-GEMM kernels): odd maps, taps that leave the
    # image entirely, a tensor barely longer than one vector, planes that are not vector multiples
    (2, 8, 5, 9, 7, 3, 1, 1, 1, 1), (1, 8, 1, 3, 3, 3, 1, 1, 1, 1), (1, 8, 8, 6, 6, 3, 1, 7, 7, 1),
    (2, 16, 8, 10, 10, 5, 1, 4, 2, 1), (5, 24, 40, 7, 7, 3, 1, 1, 1, 1), (3, 136, 72, 14, 14, 3, 1, 1, 1, 1),
    (1, 8, 264, 20, 12, 3, 1, 2, 2, 1),
    # dense strided layers with ceil(W / s) == W_y (phase planes): odd maps, stride 3, a strided 1x1
    # (phases of g_x that no tap reaches), dilation, 5x5, many channels
    (2, 16, 16, 8, 8, 1, 2, 0, 1, 1), (2, 8, 16, 15, 13, 3, 2, 1, 1, 1), (1, 8, 8, 12, 12, 3, 3, 1, 1, 1),
    (2, 16, 8, 12, 12, 3, 2, 2, 2, 1), (1, 8, 8, 11, 9, 5, 2, 2, 1, 1), (3, 136, 72, 14, 14, 3, 2, 1, 1, 1),
    (3, 64, 128, 7, 7, 3, 2, 1, 1, 1),
    # depthwise layers (plane-staged kernels): a block per plane (56x56), a wave per plane with odd,
    # unaligned planes (7x7), stride 2 on an odd map, dilation, 5x5, no padding, stride 3,
    # 7x7 taps (weight gradient on the generic kernel), a plane too large for LDS in fp32
    (2, 16, 16, 56, 56, 3, 1, 1, 1, 16), (8, 40, 40, 7, 7, 3, 1, 1, 1, 40), (3, 10, 10, 15, 13, 3, 2, 1, 1, 10),
    (2, 6, 6, 12, 12, 3, 1, 2, 2, 6), (2, 5, 5, 11, 11, 5, 1, 2, 1, 5), (2, 7, 7, 9, 10, 3, 1, 0, 1, 7),
    (2, 9, 9, 14, 14, 3, 3, 1, 1, 9), (1, 4, 4, 10, 10, 7, 1, 3, 1, 4), (1, 3, 3, 100, 90, 3, 1, 1, 1, 3),
    (5, 33, 33, 14, 14, 5, 2, 2, 1, 33),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", EXACT_CASES)
def test_exact_backward(oracle, case, dtype):
    N, Ci, Co, H, W, K, s, p, dl, g = case
    d = mk(N, Ci, Co, H, W, K, s, p, dl, g, 1, dtype)
    od = odesc(oracle, d)
    Hy, Wy, _, _ = B.gf_out_shape(d)
    x = randn((N, Ci, H, W), 41, dtype, relu=True)
    w = randn((Co, Ci // g, K, K), 42, dtype, scale=0.3)
    gy = randn((N, Co, Hy, Wy), 43, dtype)
    ref_gw, ref_gx = oracle.bwd_exact(od, to64(x), to64(w), to64(gy))
    g_w, g_x = T.conv_bwd_exact(d.with_(r=3), x.cuda(), w.cuda(), gy.cuda())   # the exact entry ignores r
    assert rel_err(g_w, ref_gw) <= TOL[dtype]
    assert rel_err(g_x, ref_gx) <= TOL[dtype]
    # r == 1 through the filtered entry points is vanilla BP (Sec. 4.2)
    xu = T.pool_activation(d, x.cuda())
    gyu = T.filter_grad(d, gy.cuda())
    assert rel_err(T.conv_bwd_weight(d, xu, gyu), ref_gw) <= TOL[dtype]
    assert rel_err(T.conv_bwd_input(d, gyu, w.cuda()), ref_gx) <= TOL[dtype]
    only_w, none_x = T.conv_bwd_exact(d, x.cuda(), None, gy.cuda(), want_gx=False)
    assert none_x is None and torch.equal(only_w, g_w)


RECT_EXACT = [
    # N Ci Co  H   W  Kh Kw s p d g     kernels that are not square
    (2, 16, 24, 12, 12, 1, 3, 1, 1, 1, 1), (2, 8, 8, 10, 10, 3, 1, 1, 1, 1, 1), (2, 8, 8, 9, 9, 3, 2, 2, 1, 1, 1),
    (2, 6, 6, 12, 12, 3, 5, 1, 2, 1, 6), (2, 64, 72, 14, 14, 3, 1, 1, 1, 1, 1), (1, 8, 16, 11, 13, 2, 5, 1, 2, 2, 2),
    (3, 32, 32, 16, 16, 1, 5, 1, 2, 1, 1),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", RECT_EXACT)
def test_exact_backward_rectangular_kernels(oracle, case, dtype):
    N, Ci, Co, H, W, Kh, Kw, s, p, dl, g = case
    d = B.ConvDesc(N=N, C_in=Ci, C_out=Co, H_in=H, W_in=W, K_h=Kh, K_w=Kw, stride=s, pad=p, dilation=dl, groups=g,
                   r=1, dtype=B.GF_BF16 if dtype == "bf16" else B.GF_F32)
    od = odesc(oracle, d)
    Hy, Wy, _, _ = B.gf_out_shape(d)
    x = randn((N, Ci, H, W), 51, dtype, relu=True)
    w = randn((Co, Ci // g, Kh, Kw), 52, dtype, scale=0.3)
    gy = randn((N, Co, Hy, Wy), 53, dtype)
    ref_gw, ref_gx = oracle.bwd_exact(od, to64(x), to64(w), to64(gy))
    g_w, g_x = T.conv_bwd_exact(d, x.cuda(), w.cuda(), gy.cuda())
    assert rel_err(g_w, ref_gw) <= TOL[dtype]
    assert rel_err(g_x, ref_gx) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", [(2, 8, 12, 8, 7, 3, 2, 1, 1, 2), (2, 6, 6, 8, 7, 3, 2, 1, 6, 2),
                                  (2, 16, 16, 15, 16, 2, 3, 1, 1, 4), (2, 32, 48, 16, 16, 3, 4, 1, 1, 2)])
def test_filtered_backward_rectangular_kernels(oracle, case, dtype):
    """Eq. 3 / Eq. 5 read the kernel through its sum over BOTH tap indices and write all K_h x K_w taps."""
    N, Ci, Co, H, W, Kh, Kw, p, g, r = case
    d = B.ConvDesc(N=N, C_in=Ci, C_out=Co, H_in=H, W_in=W, K_h=Kh, K_w=Kw, stride=1, pad=p, dilation=1, groups=g,
                   r=r, dtype=B.GF_BF16 if dtype == "bf16" else B.GF_F32)
    od = odesc(oracle, d)
    Hy, Wy, _, _ = B.gf_out_shape(d)
    x = randn((N, Ci, H, W), 61, dtype, relu=True)
    w = randn((Co, Ci // g, Kh, Kw), 62, dtype, scale=0.3)
    gy = randn((N, Co, Hy, Wy), 63, dtype)
    x_u = T.pool_activation(d, x.cuda())
    g_w, g_x, gy_u = T.conv_bwd_filtered(d, gy.cuda(), x_u, w.cuda(), want_gyu=True)
    s_gw, s_gx = T.conv_bwd_weight(d, x_u, gy_u), T.conv_bwd_input(d, gy_u, w.cuda())
    torch.cuda.synchronize()
    ref_gw, ref_gx, _, _ = oracle.gf_backward(od, to64(x), to64(w), to64(gy))
    for got_w, got_x in ((g_w, g_x), (s_gw, s_gx)):
        assert rel_err(got_w, ref_gw) <= TOL[dtype] and rel_err(got_x, ref_gx) <= TOL[dtype]
    assert tuple(g_w.shape) == (Co, Ci // g, Kh, Kw)
    assert torch.equal(g_w, g_w[:, :, :1, :1].expand_as(g_w))   # every tap carries the same value


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", [(2, 8, 12, 12, 12, 3, 3, 1, 1, 2), (2, 16, 16, 24, 18, 3, 3, 1, 16, 2),
                                  (1, 8, 8, 16, 16, 1, 4, 0, 1, 2), (2, 6, 9, 18, 18, 5, 3, 2, 3, 3)])
def test_filtered_backward_large_strides(oracle, case, dtype):
    """Strides 3 and 4: the input-side patch is r * s (6, 8, 9 pixels) and both gradients carry 1 / s^2."""
    N, Ci, Co, H, W, K, s, p, g, r = case
    d = mk(N, Ci, Co, H, W, K=K, s=s, p=p, g=g, r=r, dtype=dtype)
    od = odesc(oracle, d)
    Hy, Wy, _, _ = B.gf_out_shape(d)
    x = randn((N, Ci, H, W), 71, dtype, relu=True)
    w = randn((Co, Ci // g, K, K), 72, dtype, scale=0.3)
    gy = randn((N, Co, Hy, Wy), 73, dtype)
    x_u = T.pool_activation(d, x.cuda())
    g_w, g_x, gy_u = T.conv_bwd_filtered(d, gy.cuda(), x_u, w.cuda(), want_gyu=True)
    s_gw, s_gx = T.conv_bwd_weight(d, x_u, gy_u), T.conv_bwd_input(d, gy_u, w.cuda())
    c_gw, c_gxu = T.conv_bwd_chained(d, gy_u, x_u, w.cuda(), reduced_out=True)
    torch.cuda.synchronize()
    ref_gw, ref_gx, ref_xu, ref_gyu = oracle.gf_backward(od, to64(x), to64(w), to64(gy))
    tol = TOL[dtype]
    assert rel_err(x_u, ref_xu) <= tol and rel_err(gy_u, ref_gyu) <= tol
    for got_w, got_x in ((g_w, g_x), (s_gw, s_gx)):
        assert rel_err(got_w, ref_gw) <= tol and rel_err(got_x, ref_gx) <= tol
    assert rel_err(c_gw, ref_gw) <= tol
    assert rel_err(c_gxu, oracle.bwd_input(od, ref_gyu, to64(w), reduced_out=True)) <= tol


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", [(2, 16, 24, 56, 56, 3, 1, 7), (2, 24, 24, 56, 56, 3, 24, 7), (2, 24, 144, 28, 28, 1, 1, 7),
                                  (2, 16, 16, 30, 44, 3, 1, 6), (1, 8, 8, 64, 64, 3, 1, 16), (2, 12, 12, 21, 21, 3, 12, 21)])
def test_large_and_odd_patch_sizes(oracle, case, dtype):
    """r = 7 (the size the paper's pooling figure uses), 6, 16 and a patch as large as the map."""
    N, Ci, Co, H, W, K, g, r = case
    d = mk(N, Ci, Co, H, W, K=K, p=K // 2, g=g, r=r, dtype=dtype)
    od = odesc(oracle, d)
    x = randn((N, Ci, H, W), 81, dtype, relu=True)
    w = randn((Co, Ci // g, K, K), 82, dtype, scale=0.3)
    gy = randn((N, Co, H, W), 83, dtype)
    x_u = T.pool_activation(d, x.cuda())
    g_w, g_x, gy_u = T.conv_bwd_filtered(d, gy.cuda(), x_u, w.cuda(), want_gyu=True)
    s_gw, s_gx = T.conv_bwd_weight(d, x_u, gy_u), T.conv_bwd_input(d, gy_u, w.cuda())
    torch.cuda.synchronize()
    ref_gw, ref_gx, ref_xu, ref_gyu = oracle.gf_backward(od, to64(x), to64(w), to64(gy))
    tol = TOL[dtype]
    assert rel_err(x_u, ref_xu) <= tol and rel_err(gy_u, ref_gyu) <= tol
    for got_w, got_x in ((g_w, g_x), (s_gw, s_gx)):
        assert rel_err(got_w, ref_gw) <= tol and rel_err(got_x, ref_gx) <= tol
    # the same on 8-bit codes: the library's codes against the oracle's, then the two contractions on
    # the ORACLE's codes, which must match the oracle's contractions bit for bit
    ref_ws = oracle.kernel_sum(od, to64(w))
    dx, dg = float(np.abs(ref_xu).max()) / 127.0, float(np.abs(ref_gyu).max()) / 127.0
    dw = float(np.abs(ref_ws).max()) / 127.0
    x_q, gy_q, w_q = T.pool_activation_q8(d, x.cuda(), 1 / dx), T.filter_grad_q8(d, gy.cuda(), 1 / dg), T.kernel_sum_q8(d, w.cuda(), 1 / dw)
    xq, gq, wq = oracle.quantize_q8(ref_xu, 1 / dx), oracle.quantize_q8(ref_gyu, 1 / dg), oracle.quantize_q8(ref_ws, 1 / dw)
    q_gw = T.conv_bwd_weight_q8(d, torch.from_numpy(xq).cuda(), torch.from_numpy(gq).cuda(), dx * dg)
    q_gx = T.conv_bwd_input_q8(d, torch.from_numpy(gq).cuda(), torch.from_numpy(wq).cuda(), dg * dw)
    torch.cuda.synchronize()
    check_codes(oracle, x_q, ref_xu, 1 / dx, "x_q")
    check_codes(oracle, gy_q, ref_gyu, 1 / dg, "gy_q")
    check_codes(oracle, w_q, ref_ws, 1 / dw, "w_q")
    assert torch.equal(q_gw.cpu(), torch.from_numpy(oracle.bwd_weight_q8(od, xq, gq, dx * dg)))
    assert torch.equal(q_gx.cpu(), rounded(oracle.bwd_input_q8(od, gq, wq, dg * dw), dtype))


# ---------------------------------------------------------------------------
# whole filtered backward on the benchmark configurations
# ---------------------------------------------------------------------------
def run_layer(d, x, w, gy):
    xg, wg, gyg = x.cuda(), w.cuda(), gy.cuda()
    x_u = T.pool_activation(d, xg)
    gy_u = T.filter_grad(d, gyg)
    g_w = T.conv_bwd_weight(d, x_u, gy_u)
    g_x = T.conv_bwd_input(d, gy_u, wg)
    torch.cuda.synchronize()
    return x_u, gy_u, g_w, g_x


def check_layer_full(oracle, cfg, layer, dtype, r, N=None):
    """End to end on one layer: the GPU chains its own (rounded) reduced maps, the
    oracle runs the whole path in fp64 from the same inputs."""
    N = cfg.N if N is None else N
    d = T.desc_for(layer, N, r, dtype)
    od = odesc(oracle, d)
    x, w, gy = WL.make_inputs(cfg, layer, dtype, N=N)
    x_u, gy_u, g_w, g_x = run_layer(d, x, w, gy)
    ref_gw, ref_gx, ref_xu, ref_gyu = oracle.gf_backward(od, to64(x), to64(w), to64(gy))
    tol = TOL[dtype]
    assert rel_err(x_u, ref_xu) <= tol, "x_u"
    assert rel_err(gy_u, ref_gyu) <= tol, "gy_u"
    assert rel_err(g_w, ref_gw) <= tol, "g_w"
    assert rel_err(g_x, ref_gx) <= tol, "g_x"


def test_config1_with_exact(oracle):
    cfg = WL.CONFIGS[1]
    layer = cfg.layers[0]
    check_layer_full(oracle, cfg, layer, "f32", 2)
    d = T.desc_for(layer, 1, 2, "f32")
    x, w, gy = WL.make_inputs(cfg, layer, "f32")
    g_w, g_x = T.conv_bwd_exact(d, x.cuda(), w.cuda(), gy.cuda())
    ref_gw, ref_gx = oracle.bwd_exact(odesc(oracle, d), to64(x), to64(w), to64(gy))
    assert rel_err(g_w, ref_gw) <= 1e-5 and rel_err(g_x, ref_gx) <= 1e-5


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("li", [0, 1, 2])
def test_config2_full_size(oracle, li, dtype):
    cfg = WL.CONFIGS[2]
    check_layer_full(oracle, cfg, cfg.layers[li], dtype, 2)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("r", [2, 4])
@pytest.mark.parametrize("li", [0, 1, 2])
def test_config2_full_size_one_call(oracle, li, r, dtype):
    """The call bench.py times (gf_conv_bwd_filtered at N = 32): at r = 2 one-pass kernels for the expand
    and the depthwise layer, filter + merged launch for the project layer; at r = 4 (P = 196, no vector
    multiple in bf16) filter + merged launch with element-aligned loads; against the oracle end to end."""
    cfg = WL.CONFIGS[2]
    layer = cfg.layers[li]
    d = T.desc_for(layer, cfg.N, r, dtype)
    od = odesc(oracle, d)
    x, w, gy = WL.make_inputs(cfg, layer, dtype)
    x_u = T.pool_activation(d, x.cuda())
    g_w, g_x, gy_u = T.conv_bwd_filtered(d, gy.cuda(), x_u, w.cuda(), want_gyu=True)
    g_w2, g_x2, none = T.conv_bwd_filtered(d, gy.cuda(), x_u, w.cuda(), want_gyu=False)
    torch.cuda.synchronize()
    assert none is None and torch.equal(g_x, g_x2) and torch.equal(g_w, g_w2)
    ref_gw, ref_gx, ref_xu, ref_gyu = oracle.gf_backward(od, to64(x), to64(w), to64(gy))
    tol = TOL[dtype]
    assert rel_err(gy_u, ref_gyu) <= tol, "gy_u"
    assert rel_err(g_w, ref_gw) <= tol, "g_w"
    assert rel_err(g_x, ref_gx) <= tol, "g_x"


@pytest.mark.parametrize("r", [2, 4])
@pytest.mark.parametrize("li", [0, 1, 2])
def test_config3_full_size(oracle, li, r):
    cfg = WL.CONFIGS[3]
    check_layer_full(oracle, cfg, cfg.layers[li], "bf16", r)


@pytest.mark.parametrize("r", [2, 4, 8])
@pytest.mark.parametrize("li", [0, 1, 3])
def test_config4_sub_batch(oracle, li, r):
    """Full layer shapes with a sub-batch of 2 images so the fp64 oracle stays within seconds."""
    cfg = WL.CONFIGS[4]
    check_layer_full(oracle, cfg, cfg.layers[li], "bf16", r, N=2)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("li", [0, 2, 4, 6, 7, 9])
def test_config5_sub_batch(oracle, li, dtype):
    cfg = WL.CONFIGS[5]
    check_layer_full(oracle, cfg, cfg.layers[li], dtype, 2, N=16)


@pytest.mark.parametrize("r", [2, 4])
@pytest.mark.parametrize("li", [0, 1, 2, 3, 5, 6])
def test_paper_cases_sub_batch(oracle, li, r):
    """The paper's own on-device test shapes (Supp. E, Table 7), fp32, one or two images."""
    cfg = WL.CONFIGS[7]
    check_layer_full(oracle, cfg, cfg.layers[li], "f32", r, N=1 if li < 2 else 2)


@pytest.mark.parametrize("li", [3, 4, 5])
def test_paper_cases_exact(oracle, li):
    """Vanilla BP (the paper's baseline) at the Table 7 shapes with small maps, fp32."""
    cfg = WL.CONFIGS[7]
    layer = cfg.layers[li]
    d = T.desc_for(layer, 2, 1, "f32")
    x, w, gy = WL.make_inputs(cfg, layer, "f32", N=2)
    g_w, g_x = T.conv_bwd_exact(d, x.cuda(), w.cuda(), gy.cuda())
    ref_gw, ref_gx = oracle.bwd_exact(odesc(oracle, d), to64(x), to64(w), to64(gy))
    assert rel_err(g_w, ref_gw) <= TOL["f32"] and rel_err(g_x, ref_gx) <= TOL["f32"]


def test_config4_full_size_sampled(oracle):
    """Config 4's largest layer at its full batch, in the launch configuration the
    benchmark uses; the oracle evaluates sampled outputs one by one: a weight
    gradient entry is a dot product over (n, patch) of two channel slices, and an
    input-gradient pixel is a dot product over c_o."""
    cfg = WL.CONFIGS[4]
    layer, r, dtype = cfg.layers[0], 2, "bf16"
    d = T.desc_for(layer, cfg.N, r, dtype)
    x, w, gy = WL.make_inputs(cfg, layer, dtype)
    x_u, gy_u, g_w, g_x = run_layer(d, x, w, gy)
    rs = np.random.default_rng(4)
    gw_c, gx_c = g_w.cpu(), g_x.cpu()
    gw_max = float(gw_c.abs().max())
    gx_max = float(gx_c.abs().float().max())
    cos = rs.choice(layer.C_out, 6, replace=False)
    cis = rs.choice(layer.C_in, 6, replace=False)
    for co, ci in zip(cos, cis):
        # slice one (c_o, c_i) pair: a 1 -> 1 channel layer seen by the oracle
        sd = oracle.Desc(N=cfg.N, C_in=1, C_out=1, H_in=layer.H, W_in=layer.W, r=r)
        xs, gs, ws = to64(x[:, ci:ci + 1]), to64(gy[:, co:co + 1]), to64(w[co:co + 1, ci:ci + 1])
        ref_gw, _, _, _ = oracle.gf_backward(sd, xs, ws, gs)
        assert abs(float(gw_c[co, ci, 0, 0]) - ref_gw[0, 0, 0, 0]) <= TOL[dtype] * gw_max
    # input gradient of one image, a slice of input channels (needs every c_o)
    n, c0 = 5, 1000
    sd = oracle.Desc(N=1, C_in=8, C_out=layer.C_out, H_in=layer.H, W_in=layer.W, r=r)
    ref = oracle.bwd_input(sd, oracle.filter_grad(sd, to64(gy[n:n + 1])), to64(w[:, c0:c0 + 8]))
    assert np.abs(to64(gx_c[n:n + 1, c0:c0 + 8]) - ref).max() <= TOL[dtype] * gx_max


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_fewer_unique_elements_only_variant(oracle, dtype):
    """Sec. 4.2, first saving only (the middle cost line of Fig. 3): the K x K backward on the
    r^2-smaller maps is the exact entry called with the reduced shape, fed by the two reductions."""
    N, Ci, Co, H, W, K, r = 2, 24, 16, 20, 28, 3, 2
    d = mk(N, Ci, Co, H, W, K=K, p=1, r=r, dtype=dtype)
    ds = mk(N, Ci, Co, H // r, W // r, K=K, p=1, r=1, dtype=dtype)
    x, w, gy = randn((N, Ci, H, W), 1, dtype, relu=True), randn((Co, Ci, K, K), 2, dtype, 0.1), randn((N, Co, H, W), 3, dtype)
    od, ods = odesc(oracle, d), odesc(oracle, ds)
    # the oracle's own reduced maps, rounded once to the storage type, are the reference's inputs
    ref_xu = rounded(oracle.pool_activation(od, to64(x)), dtype)
    ref_gyu = rounded(oracle.filter_grad(od, to64(gy)), dtype)
    ref_gw, ref_gx = oracle.bwd_exact(ods, to64(ref_xu), to64(w), to64(ref_gyu))
    x_u = T.pool_activation(d, x.cuda())
    gy_u = T.filter_grad(d, gy.cuda())
    g_w, g_x = T.conv_bwd_exact(ds, x_u, w.cuda(), gy_u)               # the composition as a user runs it
    o_gw, o_gx = T.conv_bwd_exact(ds, ref_xu.cuda(), w.cuda(), ref_gyu.cuda())   # the second half on the oracle's maps
    torch.cuda.synchronize()
    assert rel_err(x_u, to64(ref_xu)) <= TOL[dtype] and rel_err(gy_u, to64(ref_gyu)) <= TOL[dtype]
    assert rel_err(o_gw, ref_gw) <= TOL[dtype] and rel_err(o_gx, ref_gx) <= TOL[dtype]
    assert rel_err(g_w, ref_gw) <= TOL[dtype] and rel_err(g_x, ref_gx) <= TOL[dtype]


UNIQUE_CASES = [
    # N  Ci   Co   H   W  K  d   g  r
    (2, 24, 16, 20, 28, 3, 1, 1, 2),
    (2, 256, 256, 14, 14, 3, 1, 1, 2),     # ResNet-18 tail, 14 x 14 -> 7 x 7 patch grid
    (2, 512, 512, 7, 7, 3, 1, 1, 2),       # 7 x 7 -> 4 x 4, ragged patches
    (2, 512, 512, 7, 7, 3, 1, 1, 4),
    (1, 256, 256, 64, 64, 3, 12, 1, 2),    # DeepLabV3 head: dilation 12 on the 32 x 32 patch grid
    (1, 256, 256, 64, 64, 3, 12, 1, 4),    # ... on 16 x 16 (the taps reach past the map: padding only)
    (1, 2048, 256, 64, 64, 1, 1, 1, 2),    # 1 x 1: the same as the collapsed kernel
    (2, 32, 32, 15, 13, 3, 1, 32, 2),      # depthwise, ragged
    (2, 12, 18, 9, 11, 5, 1, 3, 3),        # groups, 5 x 5, r = 3
    (2, 16, 16, 12, 12, 3, 1, 1, 1),       # r = 1: vanilla BP
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", UNIQUE_CASES)
def test_unique_elements_only_entry(oracle, case, dtype):
    """gf_conv_bwd_unique (Sec. 4.2, middle cost line of Fig. 3) against the oracle's composition, full
    resolution and reduced, from the oracle's own reduced maps rounded once to the storage type; g_x is
    constant on patches and equal to the replicated reduced output."""
    N, Ci, Co, H, W, K, dl, g, r = case
    d = mk(N, Ci, Co, H, W, K=K, p=dl * (K - 1) // 2, dl=dl, g=g, r=r, dtype=dtype)
    od = odesc(oracle, d)
    x, gy = randn((N, Ci, H, W), 71, dtype, relu=True), randn((N, Co, H, W), 72, dtype)
    w = randn((Co, Ci // g, K, K), 73, dtype, scale=(2.0 / (Ci // g * K * K)) ** 0.5)
    x_u = rounded(oracle.pool_activation(od, to64(x)), dtype)
    gy_u = rounded(oracle.filter_grad(od, to64(gy)), dtype)
    ref_gw, ref_gx = oracle.bwd_unique(od, to64(x_u), to64(gy_u), to64(w))
    _, ref_gxu = oracle.bwd_unique(od, to64(x_u), to64(gy_u), to64(w), reduced_out=True)
    g_w, g_x = T.conv_bwd_unique(d, gy_u.cuda(), x_u.cuda(), w.cuda())
    g_w2, g_xu = T.conv_bwd_unique(d, gy_u.cuda(), x_u.cuda(), w.cuda(), reduced_out=True)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    assert rel_err(g_w, ref_gw) <= tol and rel_err(g_x, ref_gx) <= tol and rel_err(g_xu, ref_gxu) <= tol
    assert torch.equal(g_w, g_w2)
    if r > 1:
        up = g_xu.repeat_interleave(r, 2).repeat_interleave(r, 3)[:, :, :H, :W]
        assert torch.equal(g_x, up)


# ---------------------------------------------------------------------------
# Gradient filtering on 8-bit codes (reading of Supp. H)
# ---------------------------------------------------------------------------
def check_codes(oracle, q_gpu: torch.Tensor, v64: np.ndarray, inv_delta: float, what: str):
    """The code is decided in fp32 on both sides, but from sums added in different orders: codes
    must agree except where the scaled value sits within 1e-3 of a rounding boundary (there either
    neighbour is right), and never differ by more than one."""
    ref = oracle.quantize_q8(v64, inv_delta).astype(np.int64)
    got = q_gpu.detach().cpu().numpy().astype(np.int64)
    assert got.shape == ref.shape, what
    t = np.clip(v64 * float(np.float32(inv_delta)), -127.0, 127.0)
    near_tie = np.abs(np.abs(t - np.floor(t)) - 0.5) < 1e-3
    diff = np.abs(got - ref)
    assert diff.max() <= 1, what
    assert not np.any((diff > 0) & ~near_tie), what
    assert got.min() >= -127, what


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", REDUCE_CASES)
def test_q8_pool_and_filter_codes(oracle, case, dtype):
    N, C, H, W, r, s = case
    d = mk(N, C, C, H, W, K=3, s=s, p=1, r=r, dtype=dtype)
    Hy, Wy, Hp, Wp = B.gf_out_shape(d)
    x = randn((N, C, H, W), 21, dtype, relu=True)
    gy = randn((N, C, Hy, Wy), 22, dtype)
    od = odesc(oracle, d)
    ref_x, ref_g = oracle.pool_activation(od, to64(x)), oracle.filter_grad(od, to64(gy))
    inv_x, inv_g = 127.0 / float(np.abs(ref_x).max()), 127.0 / float(np.abs(ref_g).max())
    x_q = T.pool_activation_q8(d, x.cuda(), inv_x)
    gy_q = T.filter_grad_q8(d, gy.cuda(), inv_g)
    torch.cuda.synchronize()
    assert x_q.dtype == torch.int8 and tuple(x_q.shape) == (N, C, Hp, Wp)
    check_codes(oracle, x_q, ref_x, inv_x, "x_q")
    check_codes(oracle, gy_q, ref_g, inv_g, "gy_q")
    assert int(x_q.max()) == 127   # the largest value lands on the last code
    # values beyond the range are clipped to +-127, never -128
    g8 = T.filter_grad_q8(d, gy.cuda(), 1000.0 * inv_g)
    assert int(g8.min()) >= -127 and int(g8.to(torch.int32).abs().max()) == 127


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("H,W,r,s", [(8, 8, 2, 1), (56, 56, 2, 1), (64, 64, 8, 1), (16, 16, 2, 2), (7, 7, 2, 1),
                                     (14, 14, 4, 1)])
def test_q8_codes_bit_exact_on_integers(oracle, H, W, r, s, dtype):
    """Integer-coded maps (exact sums and means): the codes must match bit for bit, ties included."""
    N, C = 3, 5
    d = mk(N, C, C, H, W, K=3, s=s, p=1, r=r, dtype=dtype)
    Hy, Wy, Hp, Wp = B.gf_out_shape(d)
    x = WL.integer_coded((N, C, H, W), 5, dtype=dtype)
    gy = WL.integer_coded((N, C, Hy, Wy), 6, dtype=dtype) * (r * r)
    od = odesc(oracle, d)
    for inv in (0.5, 0.25, 1.0):   # halves and quarters of integers: many exact ties
        x_q = T.pool_activation_q8(d, x.cuda(), inv)
        gy_q = T.filter_grad_q8(d, gy.cuda(), inv)
        assert np.array_equal(x_q.cpu().numpy(), oracle.pool_activation_q8(od, to64(x), inv))
        assert np.array_equal(gy_q.cpu().numpy(), oracle.filter_grad_q8(od, to64(gy), inv))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_q8_codes_of_non_finite_values(oracle, dtype):
    d = mk(1, 2, 2, 8, 8, K=1, p=0, r=2, dtype=dtype)
    gy = randn((1, 2, 8, 8), 5, dtype)
    gy[0, 0, 0, 0], gy[0, 0, 2, 2], gy[0, 1, 4, 4] = float("nan"), float("inf"), float("-inf")
    q = T.filter_grad_q8(d, gy.cuda(), 3.0).cpu().numpy()
    assert np.array_equal(q, oracle.filter_grad_q8(odesc(oracle, d), to64(gy), 3.0))
    assert q[0, 0, 0, 0] == -127 and q[0, 0, 1, 1] == 127 and q[0, 1, 2, 2] == -127


Q8_LAYERS = [
    # N  Ci  Co   H   W  K  s  g   r     note
    (4, 24, 144, 56, 56, 1, 1, 1, 2),     # dense, plane of 784 codes: MFMA weight gradient
    (4, 144, 24, 56, 56, 1, 1, 1, 2),
    (3, 40, 72, 32, 32, 3, 1, 1, 2),      # ragged channel tiles, 3x3 (kernel sum of 9 taps)
    (2, 64, 64, 64, 64, 3, 1, 1, 4),      # r = 4
    (2, 32, 48, 32, 32, 3, 2, 1, 2),      # stride 2: plane 8 x 8, factor 1/4
    (4, 24, 144, 56, 56, 1, 1, 1, 4),     # plane of 196 codes: not a multiple of 16 -> pair kernel
    (3, 16, 24, 14, 14, 3, 1, 1, 2),      # 7 x 7 plane
    (3, 12, 18, 9, 11, 3, 1, 3, 2),       # groups, ragged patches
    (4, 144, 144, 56, 56, 3, 1, 144, 2),  # depthwise
    (2, 32, 32, 15, 15, 3, 2, 32, 2),     # depthwise, stride 2, ragged
    (8, 256, 32, 64, 64, 1, 1, 1, 2),     # many input channels: 4 x 4 register tiles in the input gradient
    (8, 256, 64, 64, 64, 1, 1, 4, 2),     # the same with groups
    (2, 8, 12, 30, 32, 3, 1, 1, 4),       # ragged last patch row under the fused full-resolution store
    (4, 128, 192, 32, 32, 1, 1, 1, 2),    # many channels on both sides: input gradient on the int8 matrix cores
    (2, 64, 80, 16, 48, 3, 1, 1, 2),      # ... with a ragged last K chunk (80 = 64 + 16) and 192 columns per image
    (3, 144, 64, 24, 24, 1, 1, 1, 2),     # ... with a ragged last c_i tile (144 = 2 * 64 + 16)
    (2, 256, 512, 14, 14, 3, 2, 1, 2),    # ... stride 2, 4 x 4 plane (16 codes: one vector per image and channel)
    (2, 64, 64, 30, 32, 1, 1, 1, 4),      # ... ragged last patch row under its full-resolution store
    (3, 96, 576, 14, 14, 1, 1, 1, 2),     # 7 x 7 planes (49 codes): runs that cross image boundaries, both MFMA kernels
    (3, 576, 96, 14, 14, 1, 1, 1, 2),
    (2, 128, 64, 30, 40, 3, 1, 1, 2),     # planes of 300 codes, full-resolution store after unaligned loads
    (5, 64, 64, 10, 6, 1, 1, 1, 2),       # planes of 15 codes: below one run, gathered code by code
    (6, 64, 96, 4, 4, 1, 1, 1, 2),        # planes of 4 codes
    (4, 512, 512, 7, 7, 3, 1, 1, 4),      # 7 x 7 maps at r = 4: 2 x 2 ragged patch grid
    (1, 16, 16, 4, 4, 1, 1, 1, 2),        # the whole K is four codes
    (5, 64, 64, 8, 8, 1, 1, 1, 2),        # planes of exactly 16 codes
    (1, 64, 64, 10, 8, 1, 1, 1, 2),       # a single image of 20 codes: the last run is cut by the end of the tensor
    (2, 64, 64, 64, 64, 3, 1, 1, 8),      # input-side patches of 8 pixels: matrix-core kernel ...
    (2, 16, 24, 64, 64, 1, 1, 1, 8),      # ... register-tile kernel ...
    (2, 32, 32, 32, 32, 3, 2, 1, 4),      # ... and r = 4 under stride 2
    (2, 24, 24, 60, 64, 3, 1, 24, 8),     # depthwise, ragged last patch row
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", Q8_LAYERS)
def test_q8_contractions_bit_exact(oracle, case, dtype):
    """Eq. 5 / Eq. 3 on given codes: the integer sums are exact and the one fp32 scaling is the same
    operation on both sides, so g_w and g_x (both forms) must match bit for bit."""
    N, Ci, Co, H, W, K, s, g, r = case
    d = mk(N, Ci, Co, H, W, K=K, s=s, p=K // 2, g=g, r=r, dtype=dtype)
    od = odesc(oracle, d)
    _, _, Hp, Wp = B.gf_out_shape(d)
    rs = np.random.default_rng(91)
    x_q = rs.integers(-127, 128, (N, Ci, Hp, Wp)).astype(np.int8)
    gy_q = rs.integers(-127, 128, (N, Co, Hp, Wp)).astype(np.int8)
    w_q = rs.integers(-127, 128, (Co, Ci // g)).astype(np.int8)
    scale = 3.1e-5
    tq = lambda a: torch.from_numpy(a).cuda()
    g_w = T.conv_bwd_weight_q8(d, tq(x_q), tq(gy_q), scale)
    g_x = T.conv_bwd_input_q8(d, tq(gy_q), tq(w_q), scale)
    g_xu = T.conv_bwd_input_q8(d, tq(gy_q), tq(w_q), scale, reduced_out=True)
    torch.cuda.synchronize()
    assert torch.equal(g_w.cpu(), torch.from_numpy(oracle.bwd_weight_q8(od, x_q, gy_q, scale)))
    assert torch.equal(g_x.cpu(), rounded(oracle.bwd_input_q8(od, gy_q, w_q, scale), dtype))
    assert torch.equal(g_xu.cpu(), rounded(oracle.bwd_input_q8(od, gy_q, w_q, scale, reduced_out=True), dtype))
    # the extreme codes everywhere: the largest sums the layer can produce
    big = lambda shape, v: np.full(shape, v, np.int8)
    g_w = T.conv_bwd_weight_q8(d, tq(big(x_q.shape, 127)), tq(big(gy_q.shape, -127)), 1.0)
    g_x = T.conv_bwd_input_q8(d, tq(big(gy_q.shape, -127)), tq(big(w_q.shape, -127)), 1.0, reduced_out=True)
    assert torch.equal(g_w.cpu(), torch.from_numpy(oracle.bwd_weight_q8(od, big(x_q.shape, 127), big(gy_q.shape, -127), 1.0)))
    assert torch.equal(g_x.cpu(), rounded(oracle.bwd_input_q8(od, big(gy_q.shape, -127), big(w_q.shape, -127), 1.0, True), dtype))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_q8_pool_batch_is_bit_identical(oracle, dtype):
    """gf_pool_activation_batch_q8: the codes of every layer equal gf_pool_activation_q8's bit for bit
    (REDUCE_CASES: all kernel variants, ragged maps, strips larger than LDS), and agree with the oracle's."""
    descs, xs, invs = [], [], []
    for k, (N, C, H, W, r, s) in enumerate(REDUCE_CASES):
        d = mk(N, C, C, H, W, K=3, s=s, p=1, r=r, dtype=dtype)
        x = randn((N, C, H, W), 200 + k, dtype, relu=True)
        ref = oracle.pool_activation(odesc(oracle, d), to64(x))
        descs.append(d); xs.append(x); invs.append(127.0 / float(np.abs(ref).max()))
    xg = [x.cuda() for x in xs]
    outs = T.pool_activation_batch_q8(descs, xg, invs)
    singles = [T.pool_activation_q8(d, x, inv) for d, x, inv in zip(descs, xg, invs)]
    torch.cuda.synchronize()
    for d, x, inv, o, s1 in zip(descs, xs, invs, outs, singles):
        assert torch.equal(o, s1)
        check_codes(oracle, o, oracle.pool_activation(odesc(oracle, d), to64(x)), inv, "x_q")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", Q8_LAYERS)
def test_q8_one_call_backward(oracle, case, dtype):
    """gf_conv_bwd_filtered_q8 = filter with code output (the kernel-sum codes riding along) + Eq. 5 + Eq. 3
    on codes.  Bit for bit the results of the four separate entry points; the codes against the oracle's;
    and, where the library's codes equal the oracle's (always on integer-coded inputs with whole patches),
    both gradients bit for bit against the oracle's contractions of ITS codes."""
    N, Ci, Co, H, W, K, s, g, r = case
    d = mk(N, Ci, Co, H, W, K=K, s=s, p=K // 2, g=g, r=r, dtype=dtype)
    od = odesc(oracle, d)
    Hy, Wy, Hp, Wp = B.gf_out_shape(d)
    rs = np.random.default_rng(97)
    x_q = torch.from_numpy(rs.integers(-127, 128, (N, Ci, Hp, Wp)).astype(np.int8)).cuda()
    whole = Hy % r == 0 and Wy % r == 0
    for integer in ([False, True] if whole else [False]):
        if integer:   # patch means are exact multiples of 1/4, kernel sums small integers: the codes do not
            # depend on the order of any sum (ties round to even on both sides)
            gy = WL.integer_coded((N, Co, Hy, Wy), 61, lo=-8, hi=8, dtype=dtype)
            w = WL.integer_coded((Co, Ci // g, K, K), 62, lo=-1, hi=1, dtype=dtype)
            inv_g, inv_w = 1.0, 1.0
        else:
            gy = randn((N, Co, Hy, Wy), 63, dtype)
            w = randn((Co, Ci // g, K, K), 64, dtype, scale=0.2)
            inv_g = 127.0 / float(np.abs(oracle.filter_grad(od, to64(gy))).max())
            inv_w = 127.0 / float(np.abs(oracle.kernel_sum(od, to64(w))).max())
        sw, sx = 2.0e-5 / inv_g, 1.0 / (inv_g * inv_w)
        g_w, g_x, gy_q = T.conv_bwd_filtered_q8(d, gy.cuda(), inv_g, x_q, w.cuda(), inv_w, sw, sx, want_gyq=True)
        g_w0, g_x0 = T.conv_bwd_filtered_q8(d, gy.cuda(), inv_g, x_q, w.cuda(), inv_w, sw, sx)   # codes in the workspace
        s_gyq, s_wq = T.filter_grad_q8(d, gy.cuda(), inv_g), T.kernel_sum_q8(d, w.cuda(), inv_w)
        s_gw, s_gx = T.conv_bwd_weight_q8(d, x_q, s_gyq, sw), T.conv_bwd_input_q8(d, s_gyq, s_wq, sx)
        torch.cuda.synchronize()
        assert torch.equal(gy_q, s_gyq) and torch.equal(g_w, s_gw) and torch.equal(g_x, s_gx)
        assert torch.equal(g_w0, s_gw) and torch.equal(g_x0, s_gx)
        ref_gq = oracle.filter_grad_q8(od, to64(gy), inv_g)
        ref_wq = oracle.quantize_q8(oracle.kernel_sum(od, to64(w)), inv_w)
        check_codes(oracle, gy_q, oracle.filter_grad(od, to64(gy)), inv_g, "gy_q")
        check_codes(oracle, s_wq, oracle.kernel_sum(od, to64(w)), inv_w, "w_q")
        same = np.array_equal(gy_q.cpu().numpy(), ref_gq) and np.array_equal(s_wq.cpu().numpy(), ref_wq)
        assert same or not integer
        if same:
            xq = x_q.cpu().numpy()
            assert torch.equal(g_w.cpu(), torch.from_numpy(oracle.bwd_weight_q8(od, xq, ref_gq, sw)))
            assert torch.equal(g_x.cpu(), rounded(oracle.bwd_input_q8(od, ref_gq, ref_wq, sx), dtype))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_q8_layer_end_to_end(oracle, dtype):
    """Config 2's layers, N = 4.  The library's codes are checked against the oracle's; the two
    contractions run on the ORACLE's codes and must match the oracle's contractions bit for bit; the
    whole chain on the library's own codes stays within a few per cent of the unquantised filtered
    gradients (codes at a rounding boundary may differ by one between the two sides, so that result
    is not compared bit for bit)."""
    cfg = WL.CONFIGS[2]
    for layer in cfg.layers:
        d = T.desc_for(layer, 4, 2, dtype)
        od = odesc(oracle, d)
        x, w, gy = WL.make_inputs(cfg, layer, dtype, N=4)
        ref_gw, ref_gx, ref_xu, ref_gyu = oracle.gf_backward(od, to64(x), to64(w), to64(gy))
        ref_ws = oracle.kernel_sum(od, to64(w))
        dx, dg, dw = (float(np.abs(t).max()) / 127.0 for t in (ref_xu, ref_gyu, ref_ws))
        x_q = T.pool_activation_q8(d, x.cuda(), 1.0 / dx)
        gy_q = T.filter_grad_q8(d, gy.cuda(), 1.0 / dg)
        w_q = T.kernel_sum_q8(d, w.cuda(), 1.0 / dw)
        g_w = T.conv_bwd_weight_q8(d, x_q, gy_q, dx * dg)
        g_x = T.conv_bwd_input_q8(d, gy_q, w_q, dg * dw)
        xq, gq, wq = (oracle.quantize_q8(t, 1.0 / dl) for t, dl in ((ref_xu, dx), (ref_gyu, dg), (ref_ws, dw)))
        o_gw = T.conv_bwd_weight_q8(d, torch.from_numpy(xq).cuda(), torch.from_numpy(gq).cuda(), dx * dg)
        o_gx = T.conv_bwd_input_q8(d, torch.from_numpy(gq).cuda(), torch.from_numpy(wq).cuda(), dg * dw)
        torch.cuda.synchronize()
        check_codes(oracle, x_q, ref_xu, 1.0 / dx, "x_q")
        check_codes(oracle, gy_q, ref_gyu, 1.0 / dg, "gy_q")
        check_codes(oracle, w_q, ref_ws, 1.0 / dw, "w_q")
        assert torch.equal(o_gw.cpu(), torch.from_numpy(oracle.bwd_weight_q8(od, xq, gq, dx * dg)))
        assert torch.equal(o_gx.cpu(), rounded(oracle.bwd_input_q8(od, gq, wq, dg * dw), dtype))
        assert np.abs(to64(g_w) - ref_gw).max() <= 0.05 * np.abs(ref_gw).max(), layer.name
        assert np.abs(to64(g_x) - ref_gx).max() <= 0.05 * np.abs(ref_gx).max(), layer.name


# Just under 2^31 elements per tensor: the most the entry points accept (the kernels index
# elements with 32 bits).  Sampled outputs at both ends of every tensor against the oracle.
MAX_CASES = [
    ("pointwise", dict(Ci=256, Co=256, H=256, W=256, K=1, p=0, g=1), 2),
    ("depthwise", dict(Ci=256, Co=256, H=256, W=256, K=3, p=1, g=256), 2),
    ("pointwise ragged", dict(Ci=256, Co=256, H=255, W=257, K=1, p=0, g=1), 4),
    ("depthwise ragged", dict(Ci=256, Co=256, H=255, W=257, K=3, p=1, g=256), 4),
]


@pytest.mark.parametrize("case", MAX_CASES, ids=[c[0] for c in MAX_CASES])
def test_largest_tensors_sampled(oracle, case):
    _, kw, r = case
    dtype, N = "bf16", 127
    d = mk(N, r=r, dtype=dtype, **kw)
    C, H, W, K, dw = kw["Ci"], kw["H"], kw["W"], kw["K"], kw["g"] > 1
    assert 2**31 - 2**25 < N * C * H * W < 2**31
    gen = torch.Generator(device="cuda").manual_seed(31)
    x = torch.randn((N, C, H, W), generator=gen, device="cuda", dtype=torch.bfloat16).abs_()
    gy = torch.randn((N, C, H, W), generator=gen, device="cuda", dtype=torch.bfloat16)
    w = (torch.randn((C, 1 if dw else C, K, K), generator=gen, device="cuda") * 0.05).to(torch.bfloat16)
    x_u = T.pool_activation(d, x)
    g_w, g_x, gy_u = T.conv_bwd_filtered(d, gy, x_u, w, want_gyu=True)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    gw_max, gx_max = float(g_w.abs().max()), float(g_x.abs().max())
    assert gw_max > 0 and gx_max > 0
    ends = [0, N - 1]
    chans = [slice(0, 4), slice(C - 4, C)]
    for n in ends:
        for cs in chans:  # reduced maps, first and last planes
            sd = oracle.Desc(N=1, C_in=4, C_out=4, H_in=H, W_in=W, r=r)
            assert rel_err(x_u[n:n + 1, cs], oracle.pool_activation(sd, to64(x[n:n + 1, cs]))) <= tol
            assert rel_err(gy_u[n:n + 1, cs], oracle.filter_grad(sd, to64(gy[n:n + 1, cs]))) <= tol
    if dw:
        for cs in chans:
            sd = oracle.Desc(N=N, C_in=4, C_out=4, H_in=H, W_in=W, K_h=K, K_w=K, pad=kw["p"], groups=4, r=r)
            ref_gw, ref_gx, _, _ = oracle.gf_backward(sd, to64(x[:, cs]), to64(w[cs]), to64(gy[:, cs]))
            assert np.abs(to64(g_w[cs]) - ref_gw).max() <= tol * gw_max
            assert np.abs(to64(g_x[:, cs]) - ref_gx).max() <= tol * gx_max
    else:
        for co, ci in [(0, 0), (C - 1, C - 1), (3, C - 2), (C - 5, 1)]:
            sd = oracle.Desc(N=N, C_in=1, C_out=1, H_in=H, W_in=W, r=r)
            ref_gw, _, _, _ = oracle.gf_backward(sd, to64(x[:, ci:ci + 1]), to64(w[co:co + 1, ci:ci + 1]),
                                                 to64(gy[:, co:co + 1]))
            assert abs(float(g_w[co, ci, 0, 0]) - ref_gw[0, 0, 0, 0]) <= tol * gw_max
        for n in ends:
            for cs in chans:
                sd = oracle.Desc(N=1, C_in=4, C_out=C, H_in=H, W_in=W, r=r)
                ref = oracle.bwd_input(sd, oracle.filter_grad(sd, to64(gy[n:n + 1])), to64(w[:, cs]))
                assert np.abs(to64(g_x[n:n + 1, cs]) - ref).max() <= tol * gx_max
    # the same tensors through the path on 8-bit codes: codes of the end planes, both contractions on slices
    del g_x
    inv_x, inv_g = 127.0 / float(x_u.float().abs().max()), 127.0 / float(gy_u.float().abs().max())
    x_q = T.pool_activation_q8(d, x, inv_x)
    gy_q = T.filter_grad_q8(d, gy, inv_g)
    w_q = T.kernel_sum_q8(d, w, 127.0 / float(w.float().sum(dim=(2, 3)).abs().max()))
    g_w8 = T.conv_bwd_weight_q8(d, x_q, gy_q, 1.0)
    g_x8 = T.conv_bwd_input_q8(d, gy_q, w_q, 1.0)
    torch.cuda.synchronize()
    for n in ends:
        for cs in chans:
            sd = oracle.Desc(N=1, C_in=4, C_out=4, H_in=H, W_in=W, r=r)
            check_codes(oracle, x_q[n:n + 1, cs], oracle.pool_activation(sd, to64(x[n:n + 1, cs])), inv_x, "x_q")
            check_codes(oracle, gy_q[n:n + 1, cs], oracle.filter_grad(sd, to64(gy[n:n + 1, cs])), inv_g, "gy_q")
    npq = lambda t: t.cpu().numpy()
    if dw:
        for cs in chans:
            sd = oracle.Desc(N=N, C_in=4, C_out=4, H_in=H, W_in=W, K_h=K, K_w=K, pad=kw["p"], groups=4, r=r)
            assert torch.equal(g_w8[cs].cpu(), torch.from_numpy(oracle.bwd_weight_q8(sd, npq(x_q[:, cs]), npq(gy_q[:, cs]), 1.0)))
            ref = oracle.bwd_input_q8(sd, npq(gy_q[:, cs]), npq(w_q[cs]), 1.0)
            assert torch.equal(g_x8[:, cs].cpu(), rounded(ref, dtype))
    else:
        for co, ci in [(0, 0), (C - 1, C - 1), (3, C - 2)]:
            sd = oracle.Desc(N=N, C_in=1, C_out=1, H_in=H, W_in=W, r=r)
            ref = oracle.bwd_weight_q8(sd, npq(x_q[:, ci:ci + 1]), npq(gy_q[:, co:co + 1]), 1.0)
            assert float(g_w8[co, ci, 0, 0]) == float(ref[0, 0, 0, 0])
        for n in ends:
            for cs in chans:
                sd = oracle.Desc(N=1, C_in=4, C_out=C, H_in=H, W_in=W, r=r)
                ref = oracle.bwd_input_q8(sd, npq(gy_q[n:n + 1]), npq(w_q[:, cs]), 1.0)
                assert torch.equal(g_x8[n:n + 1, cs].cpu(), rounded(ref, dtype))


WS_LAYERS = [
    # N  Ci  Co   H   W  K  s  g   r
    (4, 24, 144, 56, 56, 1, 1, 1, 2), (4, 144, 24, 56, 56, 1, 1, 1, 2), (4, 144, 144, 56, 56, 3, 1, 144, 2),
    (4, 24, 144, 56, 56, 1, 1, 1, 4), (4, 256, 256, 14, 14, 3, 1, 1, 2), (2, 512, 512, 7, 7, 3, 1, 1, 2),
    (2, 256, 512, 14, 14, 3, 2, 1, 2), (3, 96, 96, 7, 7, 3, 1, 96, 2), (2, 40, 72, 30, 40, 3, 1, 1, 2),
    (2, 12, 18, 9, 11, 3, 1, 3, 2), (2, 2048, 256, 16, 16, 1, 1, 1, 2), (2, 64, 64, 32, 32, 3, 1, 1, 8),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", WS_LAYERS)
def test_workspace_sizes_are_sufficient(case, dtype):
    """Every entry point is given exactly gf_workspace_bytes() of scratch, followed by guard bytes that
    must come back untouched (a kernel that writes past the reported size would corrupt the caller)."""
    N, Ci, Co, H, W, K, s, g, r = case
    d = mk(N, Ci, Co, H, W, K=K, s=s, p=K // 2, g=g, r=r, dtype=dtype)
    sh = T.shapes(d)
    td = WL.torch_dtype(dtype)
    P = B.ptr
    x = randn(sh["x"], 91, dtype, relu=True).cuda()
    w = randn(sh["w"], 92, dtype, scale=0.3).cuda()
    gy = randn(sh["g_y"], 93, dtype).cuda()
    x_u, gy_u = T.pool_activation(d, x), T.filter_grad(d, gy)
    x_q, gy_q, w_q = T.pool_activation_q8(d, x, 8.0), T.filter_grad_q8(d, gy, 40.0), T.kernel_sum_q8(d, w, 40.0)
    g_w = torch.empty(sh["w"], dtype=torch.float32, device="cuda")
    g_x = torch.empty(sh["x"], dtype=td, device="cuda")
    g_xu = torch.empty(sh["g_x_u"], dtype=td, device="cuda")
    stats = torch.zeros(2, dtype=torch.float64, device="cuda")
    GUARD = 4096

    def run(op, call, dd=d):
        n = B.gf_workspace_bytes(dd, op)
        buf = torch.full((n + GUARD,), 0xA5, dtype=torch.uint8, device="cuda")
        call(P(buf), n)
        torch.cuda.synchronize()
        assert bool((buf[n:] == 0xA5).all()), (op, n)

    run(B.GF_OP_BWD_WEIGHT, lambda p, n: B.gf_conv_bwd_weight(d, P(x_u), P(gy_u), P(g_w), p, n))
    run(B.GF_OP_BWD_INPUT, lambda p, n: B.gf_conv_bwd_input(d, P(gy_u), P(w), P(g_x), False, p, n))
    run(B.GF_OP_BWD_INPUT, lambda p, n: B.gf_conv_bwd_input(d, P(gy_u), P(w), P(g_xu), True, p, n))
    run(B.GF_OP_BWD_FILTERED, lambda p, n: B.gf_conv_bwd_filtered(d, P(gy), P(x_u), P(w), P(gy_u), P(g_w), P(g_x), p, n))
    run(B.GF_OP_BWD_FILTERED, lambda p, n: B.gf_conv_bwd_filtered(d, P(gy), P(x_u), P(w), 0, P(g_w), P(g_x), p, n))
    run(B.GF_OP_BWD_CHAINED, lambda p, n: B.gf_conv_bwd_chained(d, P(gy_u), P(x_u), P(w), P(g_w), P(g_xu), True, 0, p, n))
    run(B.GF_OP_BWD_CHAINED, lambda p, n: B.gf_conv_bwd_chained(d, P(gy_u), P(x_u), P(w), P(g_w), P(g_x), False, 0, p, n))
    run(B.GF_OP_FILTER_SNR, lambda p, n: B.gf_filter_grad_snr(d, P(gy), P(gy_u), P(stats), p, n))
    run(B.GF_OP_BWD_EXACT, lambda p, n: B.gf_conv_bwd_exact(d, P(x), P(w), P(gy), P(g_w), P(g_x), p, n))
    run(B.GF_OP_BWD_WEIGHT_Q8, lambda p, n: B.gf_conv_bwd_weight_q8(d, P(x_q), P(gy_q), 1e-3, P(g_w), p, n))
    run(B.GF_OP_BWD_INPUT_Q8, lambda p, n: B.gf_conv_bwd_input_q8(d, P(gy_q), P(w_q), 1e-3, P(g_x), False, p, n))
    # r = 1 through the filtered entries (vanilla BP)
    d1 = d.with_(r=1)
    run(B.GF_OP_BWD_WEIGHT, lambda p, n: B.gf_conv_bwd_weight(d1, P(x), P(gy), P(g_w), p, n), d1)
    run(B.GF_OP_BWD_INPUT, lambda p, n: B.gf_conv_bwd_input(d1, P(gy), P(w), P(g_x), False, p, n), d1)
    run(B.GF_OP_BWD_FILTERED, lambda p, n: B.gf_conv_bwd_filtered(d1, P(gy), P(x), P(w), 0, P(g_w), P(g_x), p, n), d1)


OOB_LAYERS = [
    # N  Ci  Co   H   W  K  s  g   r      odd and ragged shapes: vector stores must not run over the ends
    (3, 5, 7, 7, 7, 3, 1, 1, 2), (2, 12, 18, 9, 11, 3, 1, 3, 2), (3, 10, 10, 15, 13, 3, 2, 10, 2), (1, 8, 8, 5, 3, 3, 1, 1, 2),
    (2, 24, 40, 14, 14, 3, 1, 1, 2), (2, 40, 24, 7, 7, 1, 1, 1, 2), (1, 9, 9, 30, 41, 3, 1, 9, 4), (2, 16, 8, 13, 9, 3, 2, 1, 2),
    (1, 3, 3, 1, 1, 1, 1, 1, 2), (2, 64, 64, 7, 7, 3, 1, 1, 4), (3, 24, 144, 28, 28, 1, 1, 1, 2), (1, 130, 70, 6, 10, 1, 1, 1, 3),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", OOB_LAYERS)
def test_outputs_stay_in_bounds(case, dtype):
    """Every output tensor lies between two guard regions that must come back untouched."""
    N, Ci, Co, H, W, K, s, g, r = case
    d = mk(N, Ci, Co, H, W, K=K, s=s, p=K // 2, g=g, r=r, dtype=dtype)
    sh = T.shapes(d)
    td = WL.torch_dtype(dtype)
    P = B.ptr
    GUARD = 4096
    guarded = []

    def out(shape, dt):
        n = int(np.prod(shape)) * torch.empty(0, dtype=dt).element_size()
        pad = (-n) % 256
        buf = torch.full((GUARD + n + pad + GUARD,), 0xA5, dtype=torch.uint8, device="cuda")
        guarded.append((buf, n))
        return buf[GUARD:GUARD + n].view(dt).view(shape)

    def check(what):
        torch.cuda.synchronize()
        for buf, n in guarded:
            assert bool((buf[:GUARD] == 0xA5).all()) and bool((buf[GUARD + n:] == 0xA5).all()), what

    ws = T.Workspace()
    wsp = lambda op, dd=d: ws.get(B.gf_workspace_bytes(dd, op))
    x = randn(sh["x"], 95, dtype, relu=True).cuda()
    w = randn(sh["w"], 96, dtype, scale=0.3).cuda()
    gy = randn(sh["g_y"], 97, dtype).cuda()
    x_u, gy_u, m_u = out(sh["x_u"], td), out(sh["gy_u"], td), out(sh["x_u"], td)
    B.gf_pool_activation(d, P(x), P(x_u)); check("pool")
    B.gf_pool_activation_mask(d, P(x), 6.0, P(x_u), P(m_u)); check("pool mask")
    B.gf_filter_grad(d, P(gy), P(gy_u)); check("filter")
    stats = out((2,), torch.float64)
    B.gf_filter_grad_snr(d, P(gy), P(gy_u), P(stats), *wsp(B.GF_OP_FILTER_SNR)); check("snr")
    g_w, g_x, g_xu = out(sh["w"], torch.float32), out(sh["x"], td), out(sh["g_x_u"], td)
    B.gf_conv_bwd_weight(d, P(x_u), P(gy_u), P(g_w), *wsp(B.GF_OP_BWD_WEIGHT)); check("S3")
    B.gf_conv_bwd_input(d, P(gy_u), P(w), P(g_x), False, *wsp(B.GF_OP_BWD_INPUT)); check("S4")
    B.gf_conv_bwd_input(d, P(gy_u), P(w), P(g_xu), True, *wsp(B.GF_OP_BWD_INPUT)); check("S4 reduced")
    B.gf_conv_bwd_filtered(d, P(gy), P(x_u), P(w), P(gy_u), P(g_w), P(g_x), *wsp(B.GF_OP_BWD_FILTERED)); check("fused")
    B.gf_conv_bwd_chained(d, P(gy_u), P(x_u), P(w), P(g_w), P(g_xu), True, P(m_u), *wsp(B.GF_OP_BWD_CHAINED)); check("chained")
    B.gf_conv_bwd_chained(d, P(gy_u), P(x_u), P(w), P(g_w), P(g_x), False, 0, *wsp(B.GF_OP_BWD_CHAINED)); check("chained full")
    B.gf_conv_bwd_exact(d, P(x), P(w), P(gy), P(g_w), P(g_x), *wsp(B.GF_OP_BWD_EXACT)); check("exact")
    x_q, gy_q, w_q = out(sh["x_u"], torch.int8), out(sh["gy_u"], torch.int8), out(sh["w"][:2], torch.int8)
    B.gf_pool_activation_q8(d, P(x), 8.0, P(x_q)); check("pool q8")
    B.gf_filter_grad_q8(d, P(gy), 40.0, P(gy_q)); check("filter q8")
    B.gf_kernel_sum_q8(d, P(w), 40.0, P(w_q)); check("ksum q8")
    B.gf_conv_bwd_weight_q8(d, P(x_q), P(gy_q), 1e-3, P(g_w), *wsp(B.GF_OP_BWD_WEIGHT_Q8)); check("S3 q8")
    B.gf_conv_bwd_input_q8(d, P(gy_q), P(w_q), 1e-3, P(g_x), False, *wsp(B.GF_OP_BWD_INPUT_Q8)); check("S4 q8")
    B.gf_conv_bwd_input_q8(d, P(gy_q), P(w_q), 1e-3, P(g_xu), True, *wsp(B.GF_OP_BWD_INPUT_Q8)); check("S4 q8 reduced")


def test_entry_points_replay_from_a_hip_graph():
    """Every entry point only enqueues kernels (and device copies at r = 1), so a captured
    sequence must replay to the same bits as plain launches -- checked on three replays with
    new inputs written in place and eager work between them."""
    cfg = WL.CONFIGS[2]
    N, dtype = 4, "bf16"
    P = B.ptr
    jobs = []
    for layer in cfg.layers:
        for r in (2, 1):
            d = T.desc_for(layer, N, r, dtype)
            x, w, gy = (t.cuda() for t in WL.make_inputs(cfg, layer, dtype, N=N))
            sh = T.shapes(d)
            buf = dict(d=d, x=x, w=w, gy=gy)
            for name, key, dt in (("x_u", "x_u", x.dtype), ("gy_u", "gy_u", x.dtype), ("g_x", "x", x.dtype),
                                  ("g_xu", "g_x_u", x.dtype), ("e_x", "x", x.dtype),
                                  ("g_w", "w", torch.float32), ("c_w", "w", torch.float32), ("e_w", "w", torch.float32)):
                buf[name] = torch.zeros(sh[key], dtype=dt, device="cuda")
            buf["stats"] = torch.zeros(2, dtype=torch.float64, device="cuda")
            for op in (B.GF_OP_BWD_FILTERED, B.GF_OP_BWD_CHAINED, B.GF_OP_BWD_EXACT, B.GF_OP_FILTER_SNR):
                buf[op] = torch.empty(max(B.gf_workspace_bytes(d, op), 256), dtype=torch.uint8, device="cuda")
            jobs.append(buf)
    outs = ("x_u", "gy_u", "g_x", "g_xu", "e_x", "g_w", "c_w", "e_w", "stats")

    def enqueue(s):
        for b in jobs:
            d = b["d"]
            B.gf_pool_activation(d, P(b["x"]), P(b["x_u"]), s)
            B.gf_conv_bwd_filtered(d, P(b["gy"]), P(b["x_u"]), P(b["w"]), P(b["gy_u"]), P(b["g_w"]), P(b["g_x"]),
                                   P(b[B.GF_OP_BWD_FILTERED]), b[B.GF_OP_BWD_FILTERED].numel(), s)
            B.gf_conv_bwd_chained(d, P(b["gy_u"]), P(b["x_u"]), P(b["w"]), P(b["c_w"]), P(b["g_xu"]), True, 0,
                                  P(b[B.GF_OP_BWD_CHAINED]), b[B.GF_OP_BWD_CHAINED].numel(), s)
            B.gf_conv_bwd_exact(d, P(b["x"]), P(b["w"]), P(b["gy"]), P(b["e_w"]), P(b["e_x"]),
                                P(b[B.GF_OP_BWD_EXACT]), b[B.GF_OP_BWD_EXACT].numel(), s)
            if d.r > 1:
                B.gf_filter_grad_snr(d, P(b["gy"]), P(b["gy_u"]), P(b["stats"]), P(b[B.GF_OP_FILTER_SNR]),
                                     b[B.GF_OP_FILTER_SNR].numel(), s)

    def snapshot():
        torch.cuda.synchronize()
        return [[b[k].clone() for k in outs] for b in jobs]

    def clear():
        for b in jobs:
            for k in outs:
                b[k].zero_()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        enqueue(int(side.cuda_stream))      # warm-up outside the capture
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            enqueue(int(torch.cuda.current_stream().cuda_stream))
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        for b in jobs:   # new inputs, written in place (the graph holds the addresses)
            b["gy"].mul_(-1.5 - rep)
            b["x"].add_(0.25 * (rep + 1))
        clear()
        enqueue(int(torch.cuda.current_stream().cuda_stream))
        eager = snapshot()
        clear()
        g.replay()
        replay = snapshot()
        for je, jr in zip(eager, replay):
            for k, a, c in zip(outs, je, jr):
                assert torch.equal(a, c), (rep, k)


def test_repeat_runs_are_bit_identical():
    """No floating-point atomics anywhere: two runs must agree bit for bit."""
    cfg = WL.CONFIGS[2]
    for layer in cfg.layers:
        d = T.desc_for(layer, 8, 2, "bf16")
        x, w, gy = WL.make_inputs(cfg, layer, "bf16", N=8)
        a = run_layer(d, x, w, gy)
        b = run_layer(d, x, w, gy)
        for u, v in zip(a, b):
            assert torch.equal(u, v)


# ---------------------------------------------------------------------------
# the launch observer (tracing aid)
# ---------------------------------------------------------------------------
def test_launch_observer_lists_the_kernels_of_a_call():
    """gf_set_launch_observer reports every kernel a call enqueues, before and after the launch, and
    nothing once it is removed.  A dense fp32 layer on a small map is two launches: filter + relayout,
    then both contractions with their slab sums."""
    d = mk(4, 32, 48, 14, 14, K=3, p=1, r=2, dtype="f32")
    x_u = randn((4, 32, 7, 7), 1, "f32").cuda()
    w = randn((48, 32, 3, 3), 2, "f32", scale=0.1).cuda()
    gy = randn((4, 48, 14, 14), 3, "f32").cuda()
    seen = []
    B.gf_set_launch_observer(lambda name, phase, stream: seen.append((name, phase)))
    try:
        T.conv_bwd_filtered(d, gy, x_u, w)
    finally:
        B.gf_set_launch_observer(None)
    torch.cuda.synchronize()
    assert seen == [("dense_prep_k", 0), ("dense_prep_k", 1), ("dense_gemm_k", 0), ("dense_gemm_k", 1)]
    n = len(seen)
    T.conv_bwd_filtered(d, gy, x_u, w)
    assert len(seen) == n


@pytest.mark.parametrize("case", [
    # N  Ci  Co   H   W  K  s  r  dtype   two-launch dense path?
    (4, 32, 48, 14, 14, 1, 1, 2, "f32", True),     # 49 patches: one image per column tile
    (4, 32, 48, 14, 14, 3, 1, 2, "f32", True),     # ... also with a 3 x 3 kernel
    (4, 32, 48, 7, 7, 1, 1, 2, "f32", True),       # 16 patches, 1 x 1 kernel, r_x = 2
    (4, 32, 48, 7, 7, 3, 1, 2, "f32", True),       # ... with a 3 x 3 kernel
    (4, 32, 48, 14, 14, 3, 2, 2, "f32", True),     # 16 patches, r_x = 4 (stride 2)
    (4, 32, 48, 14, 14, 3, 1, 4, "f32", True),     # 16 patches, r_x = 4 (r = 4)
    (4, 32, 48, 7, 7, 1, 1, 4, "f32", True),       # 4 patches: 16 images per column tile
    (4, 32, 48, 7, 7, 1, 1, 7, "f32", False),      # 1 patch: 64 images per column tile
    (40, 256, 64, 14, 14, 3, 2, 4, "bf16", False), # 16 images per tile whose planes come to more than 256 KB
    (4, 32, 48, 14, 14, 1, 1, 2, "bf16", True),    # bf16 storage
    (4, 32, 48, 7, 7, 1, 1, 2, "bf16", True),
    (4, 32, 48, 14, 14, 3, 1, 2, "bf16", True),
    (4, 32, 48, 28, 28, 1, 1, 2, "f32", False),    # planes of more than 256 pixels
])
def test_which_layers_take_the_two_launch_path(oracle, case):
    """The dense small-map path is taken exactly for the shapes it was measured faster on; whichever path
    runs, the result is the oracle's."""
    N, Ci, Co, H, W, K, s, r, dtype, dense = case
    d = mk(N, Ci, Co, H, W, K=K, s=s, p=K // 2, r=r, dtype=dtype)
    od = odesc(oracle, d)
    Hy, Wy, Hp, Wp = B.gf_out_shape(d)
    x = randn((N, Ci, H, W), 5, dtype, relu=True)
    w = randn((Co, Ci, K, K), 6, dtype, scale=0.1)
    gy = randn((N, Co, Hy, Wy), 7, dtype)
    x_u = T.pool_activation(d, x.cuda())
    seen = []
    B.gf_set_launch_observer(lambda name, phase, stream: seen.append(name) if phase == 0 else None)
    try:
        g_w, g_x, _ = T.conv_bwd_filtered(d, gy.cuda(), x_u, w.cuda(), want_gyu=False)
    finally:
        B.gf_set_launch_observer(None)
    torch.cuda.synchronize()
    assert (seen == ["dense_prep_k", "dense_gemm_k"]) == dense, seen
    ref_gw, ref_gx, _, _ = oracle.gf_backward(od, to64(x), to64(w), to64(gy))
    assert rel_err(g_w, ref_gw) <= TOL[dtype] and rel_err(g_x, ref_gx) <= TOL[dtype]


def test_dense_fp32_products_are_fp32_products(oracle):
    """The dense small-map path multiplies fp32 operands as three bf16 terms each, six term products per
    product.  Operands on the grid (1 + a 2^-9 + b 2^-18) 2^e need all three terms, and a one-hot gy_u (one
    patch per output channel, each on a patch of its own) makes every output a single product, so a term
    product that is missing or misplaced shows as an error of 2^-9 ... 2^-19 of the value; what is allowed is
    the fp32 rounding of the product plus the three dropped products: 2^-22 of the value.  Zeros stay zeros."""
    N, Ci, Co, H = 8, 64, 64, 7
    d = mk(N, Ci, Co, H, H, K=1, r=2, dtype="f32")
    od = odesc(oracle, d)
    P = 16
    rng = np.random.default_rng(77)
    def grid(shape):
        a, b = rng.integers(0, 256, shape), rng.integers(0, 256, shape)
        e = rng.integers(-6, 7, shape)
        sign = rng.choice([-1.0, 1.0], shape)
        return sign * (1.0 + a * 2.0 ** -9 + b * 2.0 ** -18) * 2.0 ** e
    x_u = grid((N, Ci, 4, 4))
    w = grid((Co, Ci, 1, 1))
    gy_u = np.zeros((N, Co, 4, 4))
    slots = rng.permutation(N * P)[:Co]   # (image, patch) of the only non-zero of channel c_o
    gy_u.reshape(N, Co, P)[slots // P, np.arange(Co), slots % P] = grid((Co,))
    for arr in (x_u, w, gy_u):
        assert np.array_equal(arr.astype(np.float32).astype(np.float64), arr)   # exactly fp32
    tg = lambda a: torch.from_numpy(a.astype(np.float32)).cuda()
    seen = []
    B.gf_set_launch_observer(lambda name, phase, stream: seen.append(name) if phase == 0 else None)
    try:
        g_w = T.conv_bwd_weight(d, tg(x_u), tg(gy_u))
        g_x = T.conv_bwd_input(d, tg(gy_u), tg(w), reduced_out=True)
    finally:
        B.gf_set_launch_observer(None)
    torch.cuda.synchronize()
    assert seen == ["dense_prep_k", "dense_gemm_k"] * 2, seen
    for got, ref in ((g_w, oracle.bwd_weight(od, x_u, gy_u)), (g_x, oracle.bwd_input(od, gy_u, w, reduced_out=True))):
        got = to64(got)
        assert np.array_equal(got == 0, ref == 0)
        nz = ref != 0
        assert nz.sum() >= Co * Ci
        assert (np.abs(got[nz] - ref[nz]) / np.abs(ref[nz])).max() <= 2.0 ** -22


# ---------------------------------------------------------------------------
# activation pooling of several layers in one launch
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_pool_activation_batch_is_bit_identical(oracle, dtype):
    """gf_pool_activation_batch against gf_pool_activation layer by layer (bit for bit) and against the
    oracle: register and LDS variants of every patch size, ragged maps, a strided layer (r_x = 4), a
    layer with r = 1 (copied), a strip too large for LDS (launch of its own in the middle of the list)
    and more layers than one launch holds."""
    cases = [(2, 3, 8, 8, 2, 1), (3, 5, 7, 7, 2, 1), (3, 5, 7, 7, 4, 1), (2, 4, 14, 14, 2, 2), (1, 2, 56, 56, 2, 1),
             (2, 3, 64, 64, 8, 1), (1, 3, 9, 5, 3, 1), (2, 2, 7, 7, 7, 1), (2, 3, 9, 9, 1, 1), (1, 1, 12, 9000, 8, 1),
             (4, 37, 7, 7, 2, 1), (2, 3, 30, 40, 4, 1), (1, 2, 160, 120, 2, 1), (2, 24, 56, 56, 4, 1), (1, 1, 1, 1, 2, 1),
             (2, 3, 16, 16, 2, 1), (3, 4, 28, 28, 2, 1), (2, 8, 14, 14, 4, 1), (1, 2, 32, 32, 8, 1), (2, 6, 15, 13, 2, 2)]
    descs, xs = [], []
    for k, (N, C, H, W, r, s) in enumerate(cases):
        descs.append(mk(N, C, C, H, W, K=3, s=s, p=1, r=r, dtype=dtype))
        xs.append(randn((N, C, H, W), 100 + k, dtype).cuda())
    outs = T.pool_activation_batch(descs, xs)
    torch.cuda.synchronize()
    assert len(outs) == len(cases)
    for d, x, got in zip(descs, xs, outs):
        one = T.pool_activation(d, x)
        assert torch.equal(got, one)
        assert rel_err(got, oracle.pool_activation(odesc(oracle, d), to64(x))) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_pool_activation_batch_walks_large_jobs(oracle, dtype):
    """A register-variant job with more blocks of work than the launch gives it (1024 planes of 111x112,
    ragged in height: 3136 blocks of work in bf16, 6272 in fp32, 2048 launched), beside a small job and an
    LDS job; floats against the oracle, codes bit for bit against the single-tensor entry."""
    cases = [(2, 3, 16, 16, 2, 1), (16, 64, 111, 112, 2, 1), (3, 5, 7, 7, 2, 1), (4, 32, 56, 56, 4, 1)]
    descs, xs, invs = [], [], []
    for k, (N, C, H, W, r, s) in enumerate(cases):
        descs.append(mk(N, C, C, H, W, K=3, s=s, p=1, r=r, dtype=dtype))
        xs.append(randn((N, C, H, W), 300 + k, dtype, relu=True))
    xg = [x.cuda() for x in xs]
    outs = T.pool_activation_batch(descs, xg)
    refs = [oracle.pool_activation(odesc(oracle, d), to64(x)) for d, x in zip(descs, xs)]
    invs = [127.0 / float(np.abs(ref).max()) for ref in refs]
    codes = T.pool_activation_batch_q8(descs, xg, invs)
    singles = [T.pool_activation_q8(d, x, inv) for d, x, inv in zip(descs, xg, invs)]
    torch.cuda.synchronize()
    for got, ref, c, s1 in zip(outs, refs, codes, singles):
        assert tuple(got.shape) == ref.shape
        assert rel_err(got, ref) <= TOL[dtype]
        assert torch.equal(c, s1)


def test_pool_activation_batch_full_config5(oracle):
    """The call bench.py times: all ten layers of configuration 5 at N = 128, fp32, in one launch."""
    cfg = WL.CONFIGS[5]
    descs = [T.desc_for(L, cfg.N, 2, "f32") for L in cfg.layers]
    xs = [WL.make_inputs(cfg, L, "f32")[0] for L in cfg.layers]
    outs = T.pool_activation_batch(descs, [x.cuda() for x in xs])
    torch.cuda.synchronize()
    for d, x, got in zip(descs, xs, outs):
        assert rel_err(got, oracle.pool_activation(odesc(oracle, d), to64(x))) <= 1e-5
