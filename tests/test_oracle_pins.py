"""Pins of the CPU oracle against things other than itself (no GPU needed).

Each test cites what fixes the expected value: a library routine that computes
the same textbook quantity (torch autograd / pooling in fp64), a hand-worked
fixture, an identity that follows from the paper's equations, or a number the
paper prints.  They are chosen so that a dropped term, a wrong sign or index, a
transposed operand or a mis-scaled factor in ``oracle/gf_ref.c`` fails at least
one of them.
"""
import itertools
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def D(o, **kw):
    return o.Desc(**kw)


RECT_CASES = [
    # N Ci Co H  W  Kh Kw s p d g      kernels that are not square: the two tap loops must not be swapped
    (2, 3, 4, 7, 6, 1, 3, 1, 1, 1, 1),
    (1, 4, 6, 9, 9, 3, 1, 2, 1, 1, 2),
    (2, 4, 4, 8, 8, 2, 3, 1, 2, 2, 4),
    (1, 2, 3, 6, 7, 5, 2, 1, 2, 1, 1),
]


@pytest.mark.parametrize("case", RECT_CASES)
def test_exact_bp_rectangular_kernels_match_torch_autograd(oracle, case):
    N, Ci, Co, H, W, Kh, Kw, s, p, dl, g = case
    d = D(oracle, N=N, C_in=Ci, C_out=Co, H_in=H, W_in=W, K_h=Kh, K_w=Kw, stride=s, pad=p, dilation=dl, groups=g, r=1)
    r = rng(hash(case) % 2**31)
    x = r.standard_normal((N, Ci, H, W))
    w = r.standard_normal((Co, Ci // g, Kh, Kw))
    xt, wt = torch.tensor(x, requires_grad=True), torch.tensor(w, requires_grad=True)
    y = F.conv2d(xt, wt, None, s, p, dl, g)
    gy = r.standard_normal(tuple(y.shape))
    y.backward(torch.tensor(gy))
    assert oracle.out_shape(d)[:2] == tuple(y.shape[2:])
    np.testing.assert_allclose(oracle.conv_fwd(d, x, w), y.detach().numpy(), rtol=1e-12, atol=1e-12)
    g_w, g_x = oracle.bwd_exact(d, x, w, gy)
    np.testing.assert_allclose(g_w, wt.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(g_x, xt.grad.numpy(), rtol=1e-11, atol=1e-11)
    # the kernel sum runs over both tap indices
    np.testing.assert_allclose(oracle.kernel_sum(d, w), w.sum(axis=(2, 3)), rtol=1e-13)


# ----------------------------------------------------------------------------
# exact BP (Sec. 3.1) against torch's fp64 autograd, a library routine
# ----------------------------------------------------------------------------
EXACT_CASES = [
    # N Ci Co H  W  K s p d g
    (2, 3, 4, 7, 6, 3, 1, 1, 1, 1),
    (1, 4, 6, 9, 9, 3, 2, 1, 1, 2),
    (2, 4, 4, 8, 8, 3, 1, 2, 2, 4),   # depthwise, dilated
    (1, 2, 3, 5, 7, 1, 1, 0, 1, 1),   # pointwise
    (1, 2, 2, 11, 10, 5, 2, 2, 1, 1),
    (2, 6, 3, 10, 10, 3, 1, 3, 3, 3),
    (1, 3, 5, 6, 6, 3, 1, 0, 1, 1),   # no padding: H_y < H_x
]


@pytest.mark.parametrize("case", EXACT_CASES)
def test_exact_bp_matches_torch_autograd(oracle, case):
    N, Ci, Co, H, W, K, s, p, dl, g = case
    d = D(oracle, N=N, C_in=Ci, C_out=Co, H_in=H, W_in=W, K_h=K, K_w=K, stride=s, pad=p,
          dilation=dl, groups=g, r=1)
    r = rng(hash(case) % 2**31)
    x = r.standard_normal((N, Ci, H, W))
    w = r.standard_normal((Co, Ci // g, K, K))
    xt = torch.tensor(x, requires_grad=True)
    wt = torch.tensor(w, requires_grad=True)
    y = F.conv2d(xt, wt, None, s, p, dl, g)
    gy = r.standard_normal(tuple(y.shape))
    y.backward(torch.tensor(gy))
    np.testing.assert_allclose(oracle.conv_fwd(d, x, w), y.detach().numpy(), rtol=1e-12, atol=1e-12)
    g_w, g_x = oracle.bwd_exact(d, x, w, gy)
    np.testing.assert_allclose(g_w, wt.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(g_x, xt.grad.numpy(), rtol=1e-11, atol=1e-11)
    # r == 1 through the filtered entry points is vanilla BP (Sec. 4.2)
    x_u = oracle.pool_activation(d, x)
    gy_u = oracle.filter_grad(d, gy)
    assert np.array_equal(x_u, x) and np.array_equal(gy_u, gy)
    np.testing.assert_allclose(oracle.bwd_weight(d, x_u, gy_u), wt.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(oracle.bwd_input(d, gy_u, w), xt.grad.numpy(), rtol=1e-11, atol=1e-11)


def test_exact_bp_brute_force_gather_form(oracle):
    """g_x written the other way round (gather over taps that land on the pixel)
    and g_theta by the definition, in pure Python on a tiny layer."""
    N, Ci, Co, H, W, K, s, p, dl = 1, 2, 2, 5, 4, 3, 2, 1, 1
    d = D(oracle, N=N, C_in=Ci, C_out=Co, H_in=H, W_in=W, K_h=K, K_w=K, stride=s, pad=p, r=1)
    Hy, Wy, _, _ = oracle.out_shape(d)
    r = rng(7)
    x, w, gy = r.standard_normal((N, Ci, H, W)), r.standard_normal((Co, Ci, K, K)), r.standard_normal((N, Co, Hy, Wy))
    gx = np.zeros_like(x)
    gw = np.zeros_like(w)
    for n, ci, h, ww in itertools.product(range(N), range(Ci), range(H), range(W)):
        for co, u, v in itertools.product(range(Co), range(K), range(K)):
            ni, nj = h + p - u * dl, ww + p - v * dl
            if ni % s or nj % s:
                continue
            i, j = ni // s, nj // s
            if 0 <= i < Hy and 0 <= j < Wy:
                gx[n, ci, h, ww] += w[co, ci, u, v] * gy[n, co, i, j]
    for co, ci, u, v in itertools.product(range(Co), range(Ci), range(K), range(K)):
        for n, i, j in itertools.product(range(N), range(Hy), range(Wy)):
            h, ww = i * s - p + u * dl, j * s - p + v * dl
            if 0 <= h < H and 0 <= ww < W:
                gw[co, ci, u, v] += x[n, ci, h, ww] * gy[n, co, i, j]
    g_w, g_x = oracle.bwd_exact(d, x, w, gy)
    np.testing.assert_allclose(g_w, gw, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(g_x, gx, rtol=1e-12, atol=1e-12)


# ----------------------------------------------------------------------------
# the gradient filter and the activation pooling (Eq. 2; text after Eq. 5)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("H,W,r", [(8, 8, 2), (7, 7, 2), (7, 7, 4), (14, 14, 4), (9, 5, 3), (6, 10, 7),
                                   (5, 5, 8), (16, 12, 4), (7, 7, 7)])
def test_filter_and_pool_match_library_pooling(oracle, H, W, r):
    """ceil-mode average pooling that divides by the in-bounds count is the
    patch mean with ragged last patches; with divisor 1 it is the patch sum."""
    d = D(oracle, N=2, C_in=3, C_out=3, H_in=H, W_in=W, r=r)
    g = rng(H * 100 + W * 10 + r).standard_normal((2, 3, H, W))
    ref_mean = F.avg_pool2d(torch.tensor(g), r, r, 0, ceil_mode=True, count_include_pad=False).numpy()
    ref_sum = F.avg_pool2d(torch.tensor(g), r, r, 0, ceil_mode=True, divisor_override=1).numpy()
    np.testing.assert_allclose(oracle.filter_grad(d, g), ref_mean, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oracle.pool_activation(d, g), ref_sum, rtol=1e-13, atol=1e-13)
    Hy, Wy, Hp, Wp = oracle.out_shape(d)
    assert (Hp, Wp) == (-(-H // r), -(-W // r))   # ceil(H/r) x ceil(W/r) blocks, Sec. 3.3


def _read_fixture(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, *v = line.split()
                out[k] = [float(t) for t in v]
    return out


def test_worked_example_4x4(oracle):
    fx = _read_fixture("worked_example_4x4.txt")
    d = D(oracle, N=1, C_in=1, C_out=1, H_in=4, W_in=4, K_h=3, K_w=3, pad=1, r=2)
    a = np.arange(1.0, 17.0).reshape(1, 1, 4, 4)
    w = np.arange(1.0, 10.0).reshape(1, 1, 3, 3)
    g_w, g_x, x_u, gy_u = oracle.gf_backward(d, a, w, a)
    assert gy_u.ravel().tolist() == fx["gy_u"]
    assert x_u.ravel().tolist() == fx["x_u"]
    assert oracle.kernel_sum(d, w).ravel().tolist() == fx["w_sum"]
    assert g_w.ravel().tolist() == fx["g_w"] * 9
    assert oracle.bwd_input(d, gy_u, w, reduced_out=True).ravel().tolist() == fx["g_x_u"]
    up = np.kron(np.array(fx["g_x_u"]).reshape(2, 2), np.ones((2, 2)))
    assert np.array_equal(g_x[0, 0], up)


def upsample(a, q, H, W):
    """every pixel takes the value of its q x q patch (Supp. B, the 'p' view)"""
    return np.repeat(np.repeat(a, q, axis=2), q, axis=3)[:, :, :H, :W]


@pytest.mark.parametrize("H,W,r", [(8, 8, 2), (7, 7, 2), (7, 9, 4), (10, 10, 3), (5, 5, 8)])
def test_filter_fixed_point_and_idempotence(oracle, H, W, r):
    """A map that is constant on each patch passes through the filter unchanged
    (Supp. B: all offsets of a patch share the unique value)."""
    d = D(oracle, N=2, C_in=2, C_out=2, H_in=H, W_in=W, r=r)
    _, _, Hp, Wp = oracle.out_shape(d)
    u = rng(r + H).standard_normal((2, 2, Hp, Wp))
    pc = upsample(u, r, H, W)
    f = oracle.filter_grad(d, pc)
    np.testing.assert_allclose(f, u, rtol=1e-15, atol=0)
    g = rng(99).standard_normal((2, 2, H, W))
    f1 = oracle.filter_grad(d, g)
    f2 = oracle.filter_grad(d, upsample(f1, r, H, W))
    np.testing.assert_allclose(f2, f1, rtol=1e-15, atol=0)
    # the filter keeps the total of every full patch: mean * count == sum
    if H % r == 0 and W % r == 0:
        np.testing.assert_allclose(f1 * r * r, oracle.pool_activation(d, g), rtol=1e-13)


@pytest.mark.parametrize("s,r,K,p", [(1, 2, 3, 1), (1, 4, 1, 0), (2, 2, 3, 1), (1, 3, 3, 1)])
def test_chain_of_filtered_layers_can_pass_reduced_maps(oracle, s, r, K, p):
    """Two stacked layers, nothing between them.  The upper layer's input gradient (Eq. 3) is
    constant on its input-side patches (size r * stride), so the lower layer's gradient filter
    (Eq. 2) with that patch size returns exactly the upper layer's one value per patch: the
    reduced map can be handed down instead of the full-resolution gradient, and every
    gradient of the lower layer comes out the same."""
    H = W = 12
    up = D(oracle, N=2, C_in=3, C_out=4, H_in=H, W_in=W, K_h=K, K_w=K, stride=s, pad=p, r=r)
    lo = D(oracle, N=2, C_in=2, C_out=3, H_in=H, W_in=W, K_h=3, K_w=3, pad=1, r=r * s)  # its output is the upper input
    g = rng(5 + s + r)
    Hy, Wy, _, _ = oracle.out_shape(up)
    g_y = g.standard_normal((2, 4, Hy, Wy))
    w_up = g.standard_normal((4, 3, K, K))
    w_lo = g.standard_normal((3, 2, 3, 3))
    x_lo = g.standard_normal((2, 2, H, W))
    gyu_up = oracle.filter_grad(up, g_y)
    gx_full = oracle.bwd_input(up, gyu_up, w_up)                      # [2, 3, H, W]
    gx_red = oracle.bwd_input(up, gyu_up, w_up, reduced_out=True)     # [2, 3, H/(r s), W/(r s)]
    np.testing.assert_allclose(oracle.filter_grad(lo, gx_full), gx_red, rtol=1e-14, atol=1e-300)
    xu_lo = oracle.pool_activation(lo, x_lo)
    # lower layer fed the full gradient (filters it itself) vs fed the reduced map directly
    ref = oracle.gf_backward(lo, x_lo, w_lo, gx_full)
    np.testing.assert_allclose(oracle.bwd_weight(lo, xu_lo, gx_red), ref[0], rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(oracle.bwd_input(lo, gx_red, w_lo), ref[1], rtol=1e-12, atol=1e-300)


@pytest.mark.parametrize("act", ["relu", "relu6"])
@pytest.mark.parametrize("s,r,H", [(1, 2, 12), (1, 4, 10), (2, 2, 14), (1, 3, 7)])
def test_chain_across_a_relu_needs_the_mask_fraction_only(oracle, s, r, H, act):
    """Two stacked layers with a (clipped) ReLU between them.  torch's autograd of the
    non-linearity (a library routine) turns the upper layer's patch-constant input gradient into
    the lower layer's g_y; the lower layer's filter (Eq. 2, patch r * stride) of it equals the
    reduced input gradient times the fraction of each patch that the non-linearity lets through,
    which is what the masked activation pooling returns beside x_u."""
    W = H
    q = r * s
    up = D(oracle, N=2, C_in=3, C_out=4, H_in=H, W_in=W, K_h=3, K_w=3, stride=s, pad=1, r=r)
    lo = D(oracle, N=2, C_in=2, C_out=3, H_in=H, W_in=W, K_h=3, K_w=3, pad=1, r=q)
    g = rng(40 + s + r + H)
    Hy, Wy, _, _ = oracle.out_shape(up)
    pre = torch.tensor(g.standard_normal((2, 3, H, W)) * 4.0 + 2.0, requires_grad=True)   # output of the lower layer (+BN)
    post = F.relu(pre) if act == "relu" else F.relu6(pre)                                    # input of the upper layer
    hi = float("inf") if act == "relu" else 6.0
    x_up = post.detach().numpy()
    gyu_up = oracle.filter_grad(up, g.standard_normal((2, 4, Hy, Wy)))
    w_up = g.standard_normal((4, 3, 3, 3))
    gx_full = oracle.bwd_input(up, gyu_up, w_up)                      # gradient w.r.t. `post`
    gx_red = oracle.bwd_input(up, gyu_up, w_up, reduced_out=True)
    post.backward(torch.tensor(gx_full))
    g_pre = pre.grad.numpy()                                          # what reaches the lower layer
    x_u, m_u = oracle.pool_activation_mask(up, x_up, hi)
    np.testing.assert_allclose(x_u, oracle.pool_activation(up, x_up), rtol=0, atol=0)
    np.testing.assert_allclose(oracle.filter_grad(lo, g_pre), gx_red * m_u, rtol=1e-13, atol=1e-300)
    # the fraction itself: average pooling of the 0/1 mask over in-bounds pixels (library routine)
    mask = torch.tensor(((x_up > 0) & (x_up < hi)).astype(np.float64))
    ref = F.avg_pool2d(mask, q, ceil_mode=True, count_include_pad=False).numpy()
    np.testing.assert_allclose(m_u, ref, rtol=1e-15, atol=0)
    assert 0.0 < m_u.mean() < 1.0 and ((m_u > 0) & (m_u < 1)).any()


def test_mask_fraction_hand_example(oracle):
    d = D(oracle, N=1, C_in=1, C_out=1, H_in=3, W_in=3, K_h=1, K_w=1, r=2)
    x = np.array([[-1.0, 2.0, 7.0], [0.0, 3.0, 5.0], [6.5, 0.5, -2.0]]).reshape(1, 1, 3, 3)
    x_u, m = oracle.pool_activation_mask(d, x)
    # patches {-1, 2, 0, 3}, {7, 5}, {6.5, 0.5}, {-2}: x = 0 passes nothing
    assert m.reshape(-1).tolist() == [0.5, 1.0, 1.0, 0.0]
    assert x_u.reshape(-1).tolist() == [4.0, 12.0, 7.0, -2.0]
    _, m6 = oracle.pool_activation_mask(d, x, 6.0)
    assert m6.reshape(-1).tolist() == [0.5, 0.5, 0.5, 0.0]


GF_CASES = [
    # N Ci Co H  W  K s p d g r
    (2, 3, 4, 8, 8, 3, 1, 1, 1, 1, 2),
    (2, 4, 6, 7, 7, 3, 1, 1, 1, 2, 2),    # ragged, grouped
    (1, 4, 4, 7, 7, 3, 1, 1, 1, 4, 4),    # ragged, depthwise
    (2, 2, 3, 12, 12, 3, 1, 2, 2, 1, 4),  # dilated
    (1, 3, 2, 14, 14, 3, 2, 1, 1, 1, 2),  # strided 14 -> 7
    (2, 4, 4, 14, 14, 3, 2, 1, 1, 4, 4),  # strided depthwise, r_x = 8
    (1, 5, 3, 9, 6, 1, 1, 0, 1, 1, 3),    # pointwise
    (1, 2, 2, 6, 6, 5, 1, 2, 1, 1, 7),    # one patch per plane (r >= H)
]


@pytest.mark.parametrize("case", GF_CASES)
def test_gf_equals_pointwise_bp_of_the_filtered_gradient(oracle, case):
    """Eq. (3) and Eq. (5), read through Supp. B: with every patch 'padded
    sufficiently' the K x K layer acts on the filtered gradient like a 1x1,
    stride-1 layer whose weight is the spatial kernel sum.  So
      g_theta~ = <x, up(gy_u)> / s^2   and   g_x~ = sum_co up(gy_u) * w_sum / s^2,
    which are the exact gradients (already pinned to torch above) of that 1x1
    layer fed x and the upsampled filtered gradient."""
    N, Ci, Co, H, W, K, s, p, dl, g, r = case
    d = D(oracle, N=N, C_in=Ci, C_out=Co, H_in=H, W_in=W, K_h=K, K_w=K, stride=s, pad=p,
          dilation=dl, groups=g, r=r)
    Hy, Wy, Hp, Wp = oracle.out_shape(d)
    rr = rng(hash(case) % 2**31)
    x = rr.standard_normal((N, Ci, H, W))
    w = rr.standard_normal((Co, Ci // g, K, K))
    gy = rr.standard_normal((N, Co, Hy, Wy))
    g_w, g_x, x_u, gy_u = oracle.gf_backward(d, x, w, gy)

    up = upsample(gy_u, r * s, H, W) / (s * s)
    pw = D(oracle, N=N, C_in=Ci, C_out=Co, H_in=H, W_in=W, groups=g, r=1)
    w_sum = w.sum(axis=(2, 3))
    np.testing.assert_allclose(oracle.kernel_sum(d, w), w_sum, rtol=1e-13, atol=1e-13)
    ref_gw, ref_gx = oracle.bwd_exact(pw, x, w_sum[:, :, None, None], up)
    np.testing.assert_allclose(g_x, ref_gx, rtol=1e-12, atol=1e-12)
    for u, v in itertools.product(range(K), range(K)):       # same value for every tap
        np.testing.assert_allclose(g_w[:, :, u, v], ref_gw[:, :, 0, 0], rtol=1e-12, atol=1e-12)
        assert np.array_equal(g_w[:, :, u, v], g_w[:, :, 0, 0])
    # and the same two numbers from torch directly
    xt = torch.tensor(x, requires_grad=True)
    wt = torch.tensor(w_sum[:, :, None, None].copy(), requires_grad=True)
    F.conv2d(xt, wt, groups=g).backward(torch.tensor(up))
    np.testing.assert_allclose(g_x, xt.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(g_w[:, :, 0, 0], wt.grad.numpy()[:, :, 0, 0], rtol=1e-11, atol=1e-11)
    # layout: reduced output is the unique-value view of the full output
    g_x_u = oracle.bwd_input(d, gy_u, w, reduced_out=True)
    assert g_x_u.shape == (N, Ci, Hp, Wp)
    assert np.array_equal(upsample(g_x_u, r * s, H, W), g_x)


@pytest.mark.parametrize("r,g", [(2, 1), (4, 1), (3, 2), (2, 4)])
def test_pointwise_layer_with_patch_constant_gradient_is_exact(oracle, r, g):
    """For a 1x1 stride-1 layer no tap leaves its patch, so if g_y is already
    constant on each patch the filtered gradients ARE the exact ones."""
    N, Ci, Co, H, W = 2, 4, 8, 9, 8
    d = D(oracle, N=N, C_in=Ci, C_out=Co, H_in=H, W_in=W, groups=g, r=r)
    _, _, Hp, Wp = oracle.out_shape(d)
    rr = rng(31 + r)
    x = rr.standard_normal((N, Ci, H, W))
    w = rr.standard_normal((Co, Ci // g, 1, 1))
    gy = upsample(rr.standard_normal((N, Co, Hp, Wp)), r, H, W)
    g_w, g_x, _, _ = oracle.gf_backward(d, x, w, gy)
    e_w, e_x = oracle.bwd_exact(d, x, w, gy)
    np.testing.assert_allclose(g_w, e_w, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(g_x, e_x, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("K,dl", [(3, 1), (3, 2), (5, 1)])
def test_constant_gradient_interior_exactness(oracle, K, dl):
    """Sec. 3.2 (ii): if every element of g_y is the same value v the
    convolution with the rotated kernel is (sum theta') v, boundary elements
    aside.  The filtered g_x must equal exact g_x wherever the whole (dilated)
    window stays inside the image."""
    N, Ci, Co, H, W, r = 1, 2, 3, 12, 12, 2
    p = dl * (K - 1) // 2
    d = D(oracle, N=N, C_in=Ci, C_out=Co, H_in=H, W_in=W, K_h=K, K_w=K, pad=p, dilation=dl, r=r)
    rr = rng(K * 10 + dl)
    w = rr.standard_normal((Co, Ci, K, K))
    v = rr.standard_normal((N, Co, 1, 1))
    gy = np.broadcast_to(v, (N, Co, H, W)).copy()
    gf = oracle.bwd_input(d, oracle.filter_grad(d, gy), w)
    _, ex = oracle.bwd_exact(d, np.zeros((N, Ci, H, W)), w, gy, want_gw=False)
    m = p
    np.testing.assert_allclose(gf[:, :, m:H - m, m:W - m], ex[:, :, m:H - m, m:W - m], rtol=1e-12, atol=1e-12)
    assert not np.allclose(gf, ex)        # border pixels differ: no border correction


@pytest.mark.parametrize("g,r,s", [(1, 2, 2), (4, 2, 2), (1, 1 + 1, 3)])
def test_stride_rule_zero_insertion(oracle, g, r, s):
    """A stride-s layer is a stride-1 layer followed by subsampling; the
    subsampling back-propagates by zero insertion.  Applying the paper's method
    with patch r*s to that stride-1 layer must give the strided result
    (this is where the 1/s^2 factor and the r*s activation patch come from)."""
    N, Ci, Co, K, p = 2, 4, 4, 3, 1
    Hy = 7 if s == 2 else 4
    H = Hy * s
    ds = D(oracle, N=N, C_in=Ci, C_out=Co, H_in=H, W_in=H, K_h=K, K_w=K, stride=s, pad=p, groups=g, r=r)
    d1 = D(oracle, N=N, C_in=Ci, C_out=Co, H_in=H, W_in=H, K_h=K, K_w=K, stride=1, pad=p, groups=g, r=r * s)
    assert oracle.out_shape(ds)[0] == Hy and oracle.out_shape(d1)[0] == H
    rr = rng(5 + s)
    x = rr.standard_normal((N, Ci, H, H))
    w = rr.standard_normal((Co, Ci // g, K, K))
    gy = rr.standard_normal((N, Co, Hy, Hy))
    gy1 = np.zeros((N, Co, H, H))
    gy1[:, :, ::s, ::s] = gy
    a_w, a_x, a_xu, _ = oracle.gf_backward(ds, x, w, gy)
    b_w, b_x, b_xu, _ = oracle.gf_backward(d1, x, w, gy1)
    assert np.array_equal(a_xu, b_xu)
    np.testing.assert_allclose(a_w, b_w, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(a_x, b_x, rtol=1e-12, atol=1e-12)


def test_linearity_and_structure(oracle):
    d = D(oracle, N=2, C_in=4, C_out=6, H_in=7, W_in=7, K_h=3, K_w=3, pad=1, groups=2, r=2)
    rr = rng(3)
    x1, x2 = rr.standard_normal((2, 2, 4, 7, 7))
    g1, g2 = rr.standard_normal((2, 2, 6, 7, 7))
    w = rr.standard_normal((6, 2, 3, 3))
    a, b = 0.75, -1.5
    f = oracle.filter_grad
    np.testing.assert_allclose(f(d, a * g1 + b * g2), a * f(d, g1) + b * f(d, g2), rtol=1e-12, atol=1e-12)
    pa = oracle.pool_activation
    np.testing.assert_allclose(pa(d, a * x1 + b * x2), a * pa(d, x1) + b * pa(d, x2), rtol=1e-12, atol=1e-12)
    gw = lambda x, g: oracle.bwd_weight(d, pa(d, x), f(d, g))
    np.testing.assert_allclose(gw(a * x1 + b * x2, g1), a * gw(x1, g1) + b * gw(x2, g1), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(gw(x1, a * g1 + b * g2), a * gw(x1, g1) + b * gw(x1, g2), rtol=1e-12, atol=1e-12)
    gx = lambda g, ww: oracle.bwd_input(d, f(d, g), ww)
    np.testing.assert_allclose(gx(a * g1 + b * g2, w), a * gx(g1, w) + b * gx(g2, w), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(gx(g1, a * w), a * gx(g1, w), rtol=1e-12, atol=1e-12)
    # group structure: output channels of group 1 never reach input channels of group 0
    g0 = g1.copy()
    g0[:, :3] = 0.0
    assert np.all(gx(g0, w)[:, :2] == 0.0) and np.any(gx(g0, w)[:, 2:] != 0.0)
    assert np.all(gw(x1, g0)[:3] == 0.0)
    # transposed-operand check: weight-gradient entry [co, ci] pairs gy channel co with x channel ci
    e = np.zeros((2, 6, 7, 7)); e[:, 1] = 1.0
    xx = np.zeros((2, 4, 7, 7)); xx[:, 1] = 1.0
    gwe = gw(xx, e)
    assert gwe[1, 1, 0, 0] == 2 * 49 and np.count_nonzero(gwe[:, :, 0, 0]) == 1


# ----------------------------------------------------------------------------
# numbers and closed forms the paper prints
# ----------------------------------------------------------------------------
def _layers(net, k):
    """(C_in, C_out, K, stride, pad, groups, H_in) of the last k conv layers."""
    r18 = [(256, 512, 3, 2, 1, 1, 14), (512, 512, 3, 1, 1, 1, 7), (512, 512, 3, 1, 1, 1, 7), (512, 512, 3, 1, 1, 1, 7)]
    r34 = [(512, 512, 3, 1, 1, 1, 7)] * 4
    mb2 = [(160, 960, 1, 1, 0, 1, 7), (960, 960, 3, 1, 1, 960, 7), (960, 320, 1, 1, 0, 1, 7), (320, 1280, 1, 1, 0, 1, 7)]
    return {"ResNet-18": r18, "ResNet-34": r34, "MobileNetV2": mb2}[net][-k:]


def test_table1_activation_memory(oracle):
    rows = []
    with open(os.path.join(GOLDEN, "table1_activation_memory.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                rows.append((line[0], int(line[1]), float(line[2]), float(line[3])))
    assert len(rows) == 6
    for net, k, kb_exact, kb_gf in rows:
        ex = gf = 0.0
        for ci, co, K, s, p, g, H in _layers(net, k):
            c = oracle.cost_model(D(oracle, N=1, C_in=ci, C_out=co, H_in=H, W_in=H, K_h=K, K_w=K,
                                    stride=s, pad=p, groups=g, r=2))
            ex += c["act_elems_exact"] * 4 / 1024
            gf += c["act_elems_gf"] * 4 / 1024
        assert abs(ex - kb_exact) < 0.005, (net, k, ex)
        assert abs(gf - kb_gf) < 0.005, (net, k, gf)


def test_closed_forms(oracle):
    fx = _read_fixture("closed_forms.txt")
    unet = dict(N=1, C_in=192, C_out=64, H_in=160, W_in=120, K_h=3, K_w=3, pad=1)   # footnote of Fig. 3
    c1 = oracle.cost_model(D(oracle, r=1, **unet))
    assert c1["flops_exact_gx"] == 2 * 192 * 64 * 120 * 160 * 9                      # Eq. (1)
    for r in (2, 4, 8):
        c = oracle.cost_model(D(oracle, r=r, **unet))
        assert c["flops_gf_gx"] == (160 // r) * (120 // r) * 192 * (2 * 64 - 1)      # Eq. (12)
        ratio = c["flops_exact_gx"] / c["flops_gf_gx"]
        assert abs(ratio / (r * r * 9) - 1) < 0.01                                   # Supp. D: about 1/(r^2 H_th W_th)
        assert c["flops_gf_min"] == 2 * 192 * 64 - 192                               # Eq. (13)
    # patch as large as the map reaches the minimum (Sec. 4.2)
    c = oracle.cost_model(D(oracle, r=160, **unet))
    assert c["flops_gf_gx"] == c["flops_gf_min"]
    # kernel collapse alone: (K^2 - 1)/K^2 of the work removed
    for K, key in ((3, "kernel_collapse_3x3_removed"), (5, "kernel_collapse_5x5_removed")):
        removed = 1 - 1 / (K * K)
        assert abs(removed - fx[key][0]) <= fx[key][1]
        cK = oracle.cost_model(D(oracle, N=1, C_in=8, C_out=8, H_in=16, W_in=16, K_h=K, K_w=K, pad=K // 2, r=1))
        # r = 1 in Eq. (12) is the structured map alone
        assert abs(1 - (cK["flops_gf_gx"] + 8 * 16 * 16) / cK["flops_exact_gx"] - removed) < 1e-12
    c2 = oracle.cost_model(D(oracle, r=2, **unet))
    assert c2["overhead_fwd"] == 1 / (2 * 64 * 9) and c2["overhead_bwd"] == 3 / (2 * 192)
    assert c2["overhead_fwd"] < fx["unet_overhead_upper_bound"][0]
    assert c2["overhead_bwd"] < fx["unet_overhead_upper_bound"][0]
    # Sec. 4.3: about 1 - 1/r^2 of the activation memory saved
    for r in (2, 4):
        c = oracle.cost_model(D(oracle, r=r, **unet))
        assert c["act_elems_gf"] / c["act_elems_exact"] == 1 / (r * r)


# ----------------------------------------------------------------------------
# noise of the filter (Sec. 3.4, first line of Eq. 8)
# ----------------------------------------------------------------------------
def test_filter_snr_hand_example(oracle):
    # one 2x2 patch {1, 2, 3, 6}: mean 3, energy 1 + 4 + 9 + 36 = 50, noise 4 + 1 + 0 + 9 = 14
    d = D(oracle, N=1, C_in=1, C_out=1, H_in=2, W_in=2, K_h=1, K_w=1, r=2)
    e, v = oracle.filter_snr(d, np.array([1.0, 2.0, 3.0, 6.0]).reshape(1, 1, 2, 2))
    assert e == 50.0 and v == 14.0
    # ragged 3x3 map with r = 2: patches {1,2,4,5}, {3,6}, {7,8}, {9}; means 3, 4.5, 7.5, 9
    g = np.arange(1.0, 10.0).reshape(1, 1, 3, 3)
    d = D(oracle, N=1, C_in=1, C_out=1, H_in=3, W_in=3, K_h=1, K_w=1, r=2)
    e, v = oracle.filter_snr(d, g)
    assert e == 285.0
    assert v == (4 + 1 + 1 + 4) + 2 * 1.5 ** 2 + 2 * 0.5 ** 2 + 0.0


def test_filter_snr_is_the_spectral_ratio_of_eq8(oracle):
    # Eq. (8), first line, is written on the patch's DFT.  Per patch the filtered signal is
    # constant, so its DFT keeps the DC bin of G_y and nothing else: the noise is the AC energy
    # and the signal the total energy, both r^2 times their pixel-domain sums (numpy's fft2).
    r_ = rng(21)
    for r in (2, 4):
        N, C, H, W = 2, 3, 4 * r, 3 * r
        g = r_.standard_normal((N, C, H, W)) + 0.7
        d = D(oracle, N=N, C_in=C, C_out=C, H_in=H, W_in=W, K_h=1, K_w=1, r=r)
        e, v = oracle.filter_snr(d, g)
        tot = ac = 0.0
        for n, c, hp, wp in itertools.product(range(N), range(C), range(H // r), range(W // r)):
            G = np.fft.fft2(g[n, c, hp * r:(hp + 1) * r, wp * r:(wp + 1) * r])
            P = np.abs(G) ** 2
            tot += P.sum()
            ac += P.sum() - P[0, 0]
        np.testing.assert_allclose(e * r * r, tot, rtol=1e-12)
        np.testing.assert_allclose(v * r * r, ac, rtol=1e-12)
        assert e / v > 1.0


def test_filter_snr_identities(oracle):
    r_ = rng(22)
    N, C, H, W, r = 2, 2, 7, 10, 4   # ragged in both directions
    d = D(oracle, N=N, C_in=C, C_out=C, H_in=H, W_in=W, K_h=1, K_w=1, r=r)
    g = r_.standard_normal((N, C, H, W))
    e, v = oracle.filter_snr(d, g)
    # energy is the plain sum of squares; the means split it: energy = noise + sum cnt * mean^2
    np.testing.assert_allclose(e, (g ** 2).sum(), rtol=1e-13)
    m = oracle.filter_grad(d, g)
    cnt = F.avg_pool2d(torch.ones(1, 1, H, W, dtype=torch.float64), r, ceil_mode=True,
                       divisor_override=1).numpy()
    np.testing.assert_allclose(e - v, (cnt * m ** 2).sum(), rtol=1e-12)
    # scaling g scales both sums by the square: the ratio does not move
    e3, v3 = oracle.filter_snr(d, 3.0 * g)
    np.testing.assert_allclose([e3, v3], [9 * e, 9 * v], rtol=1e-13)
    # a patch-constant gradient passes the filter unchanged: no noise
    gc = np.kron(r_.standard_normal((N, C, 2, 3)), np.ones((r, r)))[:, :, :H, :W]
    ec, vc = oracle.filter_snr(d, gc)
    assert vc <= 1e-28 * ec
    # r = 1: the filter is the identity
    d1 = D(oracle, N=N, C_in=C, C_out=C, H_in=H, W_in=W, K_h=1, K_w=1, r=1)
    assert oracle.filter_snr(d1, g)[1] == 0.0
    # a larger patch removes more (nested patches): noise(r = 4) >= noise(r = 2)
    d2 = D(oracle, N=N, C_in=C, C_out=C, H_in=8, W_in=8, K_h=1, K_w=1, r=2)
    d4 = D(oracle, N=N, C_in=C, C_out=C, H_in=8, W_in=8, K_h=1, K_w=1, r=4)
    g8 = r_.standard_normal((N, C, 8, 8))
    assert oracle.filter_snr(d4, g8)[1] >= oracle.filter_snr(d2, g8)[1]


def test_descriptor_rejection(oracle):
    ok = dict(N=1, C_in=4, C_out=4, H_in=8, W_in=8, K_h=3, K_w=3, pad=1, r=2)
    oracle.out_shape(D(oracle, **ok))
    for bad in (dict(r=0), dict(groups=3), dict(N=0), dict(stride=0), dict(dilation=0), dict(pad=-1),
                dict(pad=0),              # 8 -> 6: patch grids of x and g_y differ (3 vs 4)...
                dict(K_h=11, K_w=11)):    # kernel larger than padded input
        kw = {**ok, **bad}
        if bad == dict(pad=0):
            # 6x6 output, r=2 -> 3x3 grid; 8x8 input -> 4x4 grid: rejected
            pass
        with pytest.raises(oracle.OracleError):
            oracle.out_shape(D(oracle, **kw))
    # with r == 1 the unpadded layer is legal (exact BP has no grid rule)
    oracle.out_shape(D(oracle, **{**ok, "pad": 0, "r": 1}))


# ---------------------------------------------------------------------------
# gradient filtering on 8-bit codes (reading of Supp. H: per-tensor step size, round half to even,
# clip to +-127, exact integer contractions)
# ---------------------------------------------------------------------------
def test_q8_codes_by_hand(oracle):
    v = np.array([0.5, 1.5, -2.5, 2.5, 1000.0, -1000.0, 0.49, 126.5, 127.5, -0.5, 3.0])
    #            ties go to the even code; values beyond the range are clipped, never -128
    want = np.array([0, 2, -2, 2, 127, -127, 0, 126, 127, 0, 3], np.int8)
    assert np.array_equal(oracle.quantize_q8(v, 1.0), want)
    # the step size enters as its reciprocal: delta = 0.25
    assert np.array_equal(oracle.quantize_q8(np.array([0.25, 0.3, -0.4, 40.0]), 4.0), np.array([1, 1, -2, 127], np.int8))
    with pytest.raises(oracle.OracleError):
        oracle.quantize_q8(v, 0.0)
    # infinities are clipped; a NaN fails every comparison of the clip and lands on -127
    assert np.array_equal(oracle.quantize_q8(np.array([np.inf, -np.inf, np.nan]), 1.0), np.array([127, -127, -127], np.int8))


def test_q8_round_trip_error_is_half_a_step(oracle):
    r_ = rng(81)
    v = r_.standard_normal(5000) * 3.0
    delta = float(np.abs(v).max() / 127.0)
    q = oracle.quantize_q8(v, 1.0 / delta)
    assert q.min() >= -127 and q.max() <= 127 and max(int(q.max()), -int(q.min())) == 127
    assert np.abs(q.astype(np.float64) * delta - v).max() <= 0.5 * delta * (1 + 1e-5)


@pytest.mark.parametrize("g,s", [(1, 1), (2, 1), (1, 2), (6, 1)])
def test_q8_contractions_are_the_float_formulas_on_the_codes(oracle, g, s):
    """Integer sums of products of small integers are exact in fp64 too: Eq. 5 / Eq. 3 of the
    (independently pinned) fp64 oracle, fed the codes as numbers, must give the same integers."""
    r_ = rng(82 + g + s)
    N, Ci, Co, H, W, r = 2, 6, 12, 8, 12, 2
    d = D(oracle, N=N, C_in=Ci, C_out=Co, H_in=H, W_in=W, K_h=3, K_w=3, stride=s, pad=1, groups=g, r=r)
    _, _, Hp, Wp = oracle.out_shape(d)
    x_q = r_.integers(-127, 128, (N, Ci, Hp, Wp)).astype(np.int8)
    gy_q = r_.integers(-127, 128, (N, Co, Hp, Wp)).astype(np.int8)
    w_q = r_.integers(-127, 128, (Co, Ci // g)).astype(np.int8)
    s2 = float(s * s)
    gw8 = oracle.bwd_weight_q8(d, x_q, gy_q, 1.0)
    ref = oracle.bwd_weight(d, x_q.astype(np.float64), gy_q.astype(np.float64))   # carries 1/s^2 already
    assert gw8.dtype == np.float32 and np.array_equal(gw8.astype(np.float64), ref)
    # Eq. 3 reads the kernel through its spatial sum only: a 1x1 layer whose kernel is the codes
    d1 = D(oracle, N=N, C_in=Ci, C_out=Co, H_in=H, W_in=W, K_h=1, K_w=1, stride=s, pad=0, groups=g, r=r)
    for reduced in (True, False):
        gx8 = oracle.bwd_input_q8(d, gy_q, w_q, 1.0, reduced_out=reduced)
        ref = oracle.bwd_input(d1, gy_q.astype(np.float64), w_q.astype(np.float64)[:, :, None, None], reduced_out=reduced)
        assert np.array_equal(gx8.astype(np.float64), ref), reduced
    # the step-size product is one binary32 factor on the integer
    gw_s = oracle.bwd_weight_q8(d, x_q, gy_q, 0.375)
    assert np.array_equal(gw_s, (gw8 * np.float32(s2)) * (np.float32(0.375) / np.float32(s2)))


def test_q8_contractions_brute_force(oracle):
    r_ = rng(85)
    N, Ci, Co, H, W, r, g = 1, 4, 6, 4, 6, 2, 2
    d = D(oracle, N=N, C_in=Ci, C_out=Co, H_in=H, W_in=W, K_h=1, K_w=1, groups=g, r=r)
    Hp, Wp, Cg, Og = 2, 3, Ci // g, Co // g
    x_q = r_.integers(-127, 128, (N, Ci, Hp, Wp)).astype(np.int8)
    gy_q = r_.integers(-127, 128, (N, Co, Hp, Wp)).astype(np.int8)
    w_q = r_.integers(-127, 128, (Co, Cg)).astype(np.int8)
    gw = oracle.bwd_weight_q8(d, x_q, gy_q, 1.0)
    gx = oracle.bwd_input_q8(d, gy_q, w_q, 1.0, reduced_out=True)
    for co in range(Co):
        for cl in range(Cg):
            ci = (co // Og) * Cg + cl
            want = sum(int(x_q[0, ci, i, j]) * int(gy_q[0, co, i, j]) for i in range(Hp) for j in range(Wp))
            assert int(gw[co, cl, 0, 0]) == want
    for ci in range(Ci):
        grp, cl = ci // Cg, ci % Cg
        for i in range(Hp):
            for j in range(Wp):
                want = sum(int(gy_q[0, grp * Og + ol, i, j]) * int(w_q[grp * Og + ol, cl]) for ol in range(Og))
                assert int(gx[0, ci, i, j]) == want


def test_q8_path_approaches_the_float_path(oracle):
    """With the step sizes at max|.| / 127 the two gradients stay within a few step sizes' worth of
    the unquantised Eq. 5 / Eq. 3 (errors of single codes are <= half a step and average out)."""
    r_ = rng(86)
    d = D(oracle, N=4, C_in=16, C_out=24, H_in=16, W_in=16, K_h=3, K_w=3, pad=1, r=2)
    x = np.abs(r_.standard_normal((4, 16, 16, 16)))
    gy = r_.standard_normal((4, 24, 16, 16))
    w = r_.standard_normal((24, 16, 3, 3)) * 0.1
    x_u, gy_u, ws = oracle.pool_activation(d, x), oracle.filter_grad(d, gy), oracle.kernel_sum(d, w)
    dx, dg, dw = (float(np.abs(t).max() / 127.0) for t in (x_u, gy_u, ws))
    x_q = oracle.pool_activation_q8(d, x, 1.0 / dx)
    gy_q = oracle.filter_grad_q8(d, gy, 1.0 / dg)
    w_q = oracle.kernel_sum_q8(d, w, 1.0 / dw)
    assert np.array_equal(x_q, oracle.quantize_q8(x_u, 1.0 / dx))
    gw8, gx8 = oracle.bwd_weight_q8(d, x_q, gy_q, dx * dg), oracle.bwd_input_q8(d, gy_q, w_q, dg * dw)
    gw, gx = oracle.bwd_weight(d, x_u, gy_u), oracle.bwd_input(d, gy_u, w)
    assert np.abs(gw8 - gw).max() <= 0.02 * np.abs(gw).max()
    assert np.abs(gx8 - gx).max() <= 0.03 * np.abs(gx).max()


# ---------------------------------------------------------------------------
# 'fewer unique elements' alone (Sec. 4.2, middle cost line of Fig. 3)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("case", [
    # N  Ci  Co  H   W  K  d  g  r
    (2, 3, 4, 8, 8, 3, 1, 1, 2), (1, 4, 6, 9, 7, 3, 1, 2, 2), (2, 2, 3, 12, 12, 3, 2, 1, 4),
    (1, 3, 3, 10, 14, 5, 1, 3, 2), (2, 2, 2, 7, 7, 1, 1, 1, 4),
])
def test_unique_elements_only_against_torch(oracle, case):
    """bwd_unique against library routines: torch's fp64 convolution backward on the reduced maps,
    and repeat_interleave for the replication to full resolution."""
    N, Ci, Co, H, W, K, dl, g, r = case
    p = dl * (K - 1) // 2
    d = oracle.Desc(N=N, C_in=Ci, C_out=Co, H_in=H, W_in=W, K_h=K, K_w=K, stride=1, pad=p, dilation=dl, groups=g, r=r)
    _, _, Hp, Wp = oracle.out_shape(d)
    rr = np.random.default_rng(7)
    x_u, gy_u = rr.standard_normal((N, Ci, Hp, Wp)), rr.standard_normal((N, Co, Hp, Wp))
    w = rr.standard_normal((Co, Ci // g, K, K))
    g_w, g_x = oracle.bwd_unique(d, x_u, gy_u, w)
    _, g_xu = oracle.bwd_unique(d, x_u, gy_u, w, reduced_out=True)
    xt = torch.from_numpy(x_u).requires_grad_(True)
    wt = torch.from_numpy(w).requires_grad_(True)
    y = torch.nn.functional.conv2d(xt, wt, None, 1, p, dl, g)
    t_gx, t_gw = torch.autograd.grad(y, (xt, wt), torch.from_numpy(gy_u))
    assert np.allclose(g_w, t_gw.numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(g_xu, t_gx.numpy(), rtol=1e-12, atol=1e-12)
    up = t_gx.repeat_interleave(r, 2).repeat_interleave(r, 3)[:, :, :H, :W].numpy()
    assert g_x.shape == (N, Ci, H, W) and np.allclose(g_x, up, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("r", [2, 3, 4])
@pytest.mark.parametrize("g", [1, 2])
def test_unique_elements_only_equals_filtering_for_1x1_kernels(oracle, r, g):
    """With a 1 x 1 kernel there is nothing left to collapse: the reduced-map backward is Eq. 5 / Eq. 3
    (ragged maps included), and with r = 1 it is vanilla BP."""
    N, Ci, Co, H, W = 2, 4, 6, 9, 11
    d = oracle.Desc(N=N, C_in=Ci, C_out=Co, H_in=H, W_in=W, groups=g, r=r)
    rr = np.random.default_rng(8)
    x, gy, w = rr.standard_normal((N, Ci, H, W)), rr.standard_normal((N, Co, H, W)), rr.standard_normal((Co, Ci // g, 1, 1))
    x_u, gy_u = oracle.pool_activation(d, x), oracle.filter_grad(d, gy)
    g_w, g_x = oracle.bwd_unique(d, x_u, gy_u, w)
    assert np.allclose(g_w, oracle.bwd_weight(d, x_u, gy_u), rtol=1e-12, atol=1e-13)
    assert np.allclose(g_x, oracle.bwd_input(d, gy_u, w), rtol=1e-12, atol=1e-13)
    d1 = oracle.Desc(N=N, C_in=Ci, C_out=Co, H_in=H, W_in=W, K_h=3, K_w=3, pad=1, groups=g, r=1)
    w3 = rr.standard_normal((Co, Ci // g, 3, 3))
    e_w, e_x = oracle.bwd_exact(d1, x, w3, gy)
    u_w, u_x = oracle.bwd_unique(d1, x, gy, w3)
    assert np.array_equal(e_w, u_w) and np.array_equal(e_x, u_x)


def test_unique_elements_only_by_hand(oracle):
    """4 x 4 map, r = 2, one channel, 3 x 3 kernel, padding 1: the patch grid is 2 x 2, so every tap of
    the kernel meets at most the four patch values; written out from the definition."""
    d = oracle.Desc(N=1, C_in=1, C_out=1, H_in=4, W_in=4, K_h=3, K_w=3, pad=1, r=2)
    x_u = np.array([[[[1., 2.], [3., 4.]]]])
    gy_u = np.array([[[[0.5, -1.], [2., 0.25]]]])
    w = np.arange(1., 10.).reshape(1, 1, 3, 3)
    g_w, g_x = oracle.bwd_unique(d, x_u, gy_u, w)
    xp = np.pad(x_u[0, 0], 1)
    for u in range(3):
        for v in range(3):
            want = sum(xp[hp + u, wp + v] * gy_u[0, 0, hp, wp] for hp in range(2) for wp in range(2))
            assert abs(g_w[0, 0, u, v] - want) < 1e-13
    for hp in range(2):
        for wp in range(2):
            want = 0.0
            for u in range(3):
                for v in range(3):
                    i, j = hp - u + 1, wp - v + 1
                    if 0 <= i < 2 and 0 <= j < 2:
                        want += w[0, 0, u, v] * gy_u[0, 0, i, j]
            assert np.allclose(g_x[0, 0, 2 * hp:2 * hp + 2, 2 * wp:2 * wp + 2], want, atol=1e-13)
    with pytest.raises(oracle.OracleError):
        oracle.bwd_unique(oracle.Desc(N=1, C_in=1, C_out=1, H_in=4, W_in=4, K_h=3, K_w=3, stride=2, pad=1, r=2),
                          np.zeros((1, 1, 1, 1)), np.zeros((1, 1, 1, 1)), w)
