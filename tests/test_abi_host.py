"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol include/gf.h declares, and rejects bad calls before any launch."""
import numpy as np
import ctypes as C
import os
import re

import pytest

import paper_2301_00330_amd.binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2301_00330_amd.build import build
        build()
    return B.lib()


def test_exports_match_header(lib):
    hdr = open(os.path.join(ROOT, "include", "gf.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(gf_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert B.gf_version() >= 100


def test_largest_accepted_tensor(lib):
    """Kernels index elements with 32 bits: a tensor may hold up to 2^31 - 2^20 elements."""
    big = dict(N=1, C_in=2047, C_out=2047, H_in=1024, W_in=1024, K_h=1, K_w=1, pad=0, r=2)
    assert B.gf_out_shape(B.ConvDesc(**big)) == (1024, 1024, 512, 512)
    for over in (dict(W_in=1025), dict(C_in=2048), dict(C_out=2048)):
        with pytest.raises(B.GfError) as ei:
            B.gf_out_shape(B.ConvDesc(**{**big, **over}))
        assert ei.value.status == B.GF_ERR_UNSUPPORTED


def test_element_count_cannot_wrap(lib):
    """Extents whose product passes 2^64 (16 * 4096 * 2^24 * 2^24 = 2^64 wraps to 0 in 64 bits) and
    other products beyond 2^63 are refused like any tensor that is too large."""
    for kw in (dict(N=16, C_in=4096, C_out=4096, H_in=1 << 24, W_in=1 << 24, K_h=3, K_w=3, pad=1, groups=4096),
               dict(N=1 << 15, C_in=1 << 16, C_out=1 << 16, H_in=1 << 16, W_in=1 << 16, K_h=1, K_w=1, pad=0),
               dict(N=1, C_in=1 << 20, C_out=1 << 20, H_in=1 << 12, W_in=1 << 12, K_h=1 << 11, K_w=1 << 11, pad=1023),
               dict(N=1, C_in=1, C_out=1, H_in=(1 << 31) - 1, W_in=(1 << 31) - 1, K_h=1, K_w=1, pad=0)):
        d = B.ConvDesc(r=2, **kw)
        for call in (lambda: B.gf_out_shape(d), lambda: B.gf_workspace_bytes(d, B.GF_OP_FILTER_SNR),
                     lambda: B.gf_filter_grad(d, FAKE, FAKE)):
            with pytest.raises(B.GfError) as ei:
                call()
            assert ei.value.status == B.GF_ERR_UNSUPPORTED


def test_static_scratch_entry_host_checks(lib):
    """gf_conv_bwd_filtered_static: descriptor, pointer and size errors come before any device call."""
    d = B.ConvDesc(**OK)
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_filtered_static(d, 0, FAKE, FAKE, FAKE, FAKE, FAKE)
    assert ei.value.status == B.GF_ERR_NULL
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_filtered_static(d, FAKE, FAKE, FAKE + 8, FAKE, FAKE, FAKE)
    assert ei.value.status == B.GF_ERR_UNSUPPORTED
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_filtered_static(d.with_(r=0), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE)
    assert ei.value.status == B.GF_ERR_BAD_DESC
    big = B.ConvDesc(N=8, C_in=2048, C_out=256, H_in=64, W_in=64, r=2, dtype=B.GF_BF16)
    assert B.gf_workspace_bytes(big, B.GF_OP_BWD_FILTERED) > B.GF_STATIC_SCRATCH_BYTES
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_filtered_static(big, FAKE, FAKE, FAKE, 0, FAKE, FAKE)
    assert ei.value.status == B.GF_ERR_WORKSPACE
    hdr = open(os.path.join(ROOT, "include", "gf.h")).read()
    m = re.search(r"#define\s+GF_STATIC_SCRATCH_BYTES\s+\((\d+)u\s*<<\s*(\d+)\)", hdr)
    assert m and int(m.group(1)) << int(m.group(2)) == B.GF_STATIC_SCRATCH_BYTES


OK = dict(N=2, C_in=4, C_out=8, H_in=8, W_in=8, K_h=3, K_w=3, pad=1, r=2)
FAKE = 0x1000  # non-null, 16-byte aligned; never dereferenced because validation fails first


@pytest.mark.parametrize("bad,status", [
    (dict(r=0), B.GF_ERR_BAD_DESC), (dict(groups=3), B.GF_ERR_BAD_DESC), (dict(N=0), B.GF_ERR_BAD_DESC),
    (dict(stride=0), B.GF_ERR_BAD_DESC), (dict(dilation=0), B.GF_ERR_BAD_DESC), (dict(pad=-1), B.GF_ERR_BAD_DESC),
    (dict(dtype=7), B.GF_ERR_BAD_DESC), (dict(pad=0), B.GF_ERR_SHAPE), (dict(K_h=19, K_w=19), B.GF_ERR_SHAPE),
    (dict(N=1 << 20, C_in=1 << 10, H_in=64, W_in=64), B.GF_ERR_UNSUPPORTED),
])
def test_descriptor_errors(lib, bad, status):  # the last case: 2^36 elements
    d = B.ConvDesc(**{**OK, **bad})
    for call in (lambda: B.gf_out_shape(d),
                 lambda: B.gf_workspace_bytes(d, B.GF_OP_BWD_WEIGHT),
                 lambda: B.gf_filter_grad(d, FAKE, FAKE),
                 lambda: B.gf_pool_activation(d, FAKE, FAKE),
                 lambda: B.gf_conv_bwd_weight(d, FAKE, FAKE, FAKE, FAKE, 1 << 30),
                 lambda: B.gf_conv_bwd_input(d, FAKE, FAKE, FAKE, False, FAKE, 1 << 30),
                 lambda: B.gf_cost_model(d)):
        with pytest.raises(B.GfError) as ei:
            call()
        assert ei.value.status == status


def test_exact_entry_ignores_patch_grid_rule(lib):
    # an unpadded 3x3 layer is illegal for r = 2 (grids differ) but fine for the exact entry
    d = B.ConvDesc(**{**OK, "pad": 0})
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_exact(d, FAKE, FAKE, 0, FAKE, FAKE, 0, 0)
    assert ei.value.status == B.GF_ERR_NULL        # g_y is NULL: shape accepted, pointer rejected


def test_pointer_and_workspace_errors(lib):
    d = B.ConvDesc(**OK)
    with pytest.raises(B.GfError) as ei:
        B.gf_filter_grad(d, 0, FAKE)
    assert ei.value.status == B.GF_ERR_NULL
    with pytest.raises(B.GfError) as ei:
        B.gf_pool_activation(d, FAKE, 0)
    assert ei.value.status == B.GF_ERR_NULL
    with pytest.raises(B.GfError) as ei:
        B.gf_filter_grad(d, FAKE + 4, FAKE)
    assert ei.value.status == B.GF_ERR_UNSUPPORTED
    need = B.gf_workspace_bytes(d, B.GF_OP_BWD_WEIGHT)
    assert need > 0
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_weight(d, FAKE, FAKE, FAKE, FAKE, need - 1)
    assert ei.value.status == B.GF_ERR_WORKSPACE
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_input(d, FAKE, FAKE, FAKE, False, 0, 0)
    assert ei.value.status == B.GF_ERR_WORKSPACE
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_exact(d, 0, 0, FAKE, 0, 0, 0, 0)
    assert ei.value.status == B.GF_ERR_NULL
    # the chained and the fused entry: null pointers, then the workspace, before anything is enqueued
    for reduced in (True, False):
        with pytest.raises(B.GfError) as ei:
            B.gf_conv_bwd_chained(d, 0, FAKE, FAKE, FAKE, FAKE, reduced, 0, FAKE, 1 << 30)
        assert ei.value.status == B.GF_ERR_NULL
        need_c = B.gf_workspace_bytes(d, B.GF_OP_BWD_CHAINED)
        assert need_c > 0
        with pytest.raises(B.GfError) as ei:
            B.gf_conv_bwd_chained(d, FAKE, FAKE, FAKE, FAKE, FAKE, reduced, 0, FAKE, need_c - 1)
        assert ei.value.status == B.GF_ERR_WORKSPACE
        with pytest.raises(B.GfError) as ei:
            B.gf_conv_bwd_chained(d, FAKE, FAKE + 2, FAKE, FAKE, FAKE, reduced, 0, FAKE, need_c)
        assert ei.value.status == B.GF_ERR_UNSUPPORTED
    # a mask on a full-resolution output of a filtered layer is refused; so is a misaligned mask
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_chained(d, FAKE, FAKE, FAKE, FAKE, FAKE, False, FAKE, FAKE, 1 << 30)
    assert ei.value.status == B.GF_ERR_UNSUPPORTED
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_chained(d, FAKE, FAKE, FAKE, FAKE, FAKE, True, FAKE + 4, FAKE, 1 << 30)
    assert ei.value.status == B.GF_ERR_UNSUPPORTED
    # masked activation pooling
    with pytest.raises(B.GfError) as ei:
        B.gf_pool_activation_mask(d, FAKE, 6.0, FAKE, 0)
    assert ei.value.status == B.GF_ERR_NULL
    for bad_hi in (0.0, -1.0, float("nan")):
        with pytest.raises(B.GfError) as ei:
            B.gf_pool_activation_mask(d, FAKE, bad_hi, FAKE, FAKE)
        assert ei.value.status == B.GF_ERR_BAD_DESC
    # the filter with its noise figures
    need_s = B.gf_workspace_bytes(d, B.GF_OP_FILTER_SNR)
    assert need_s >= 8
    with pytest.raises(B.GfError) as ei:
        B.gf_filter_grad_snr(d, FAKE, FAKE, 0, FAKE, need_s)
    assert ei.value.status == B.GF_ERR_NULL
    with pytest.raises(B.GfError) as ei:
        B.gf_filter_grad_snr(d, FAKE, FAKE, FAKE, FAKE, need_s - 1)
    assert ei.value.status == B.GF_ERR_WORKSPACE
    with pytest.raises(B.GfError) as ei:
        B.gf_filter_grad_snr(d, FAKE, FAKE, FAKE + 8, FAKE, need_s)
    assert ei.value.status == B.GF_ERR_UNSUPPORTED
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_filtered(d, FAKE, FAKE, FAKE, 0, FAKE, FAKE, FAKE, 0)
    assert ei.value.status == B.GF_ERR_WORKSPACE
    with pytest.raises(B.GfError) as ei:
        B.gf_workspace_bytes(d, 99)
    assert ei.value.status == B.GF_ERR_BAD_DESC
    # wrong struct_size
    cd = d.c()
    cd.struct_size = 8
    assert lib.gf_out_shape(C.byref(cd), None, None, None, None) == B.GF_ERR_BAD_DESC
    assert lib.gf_out_shape(None, None, None, None, None) == B.GF_ERR_NULL
    assert "GF_ERR_SHAPE" in B.status_string(B.GF_ERR_SHAPE)


def test_shapes_and_cost_model_against_oracle(lib, oracle):
    """The library's host-side shape rule and closed forms agree with the oracle's
    (two independent implementations of Sec. 3.2 / 3.3 / 4.2 / 4.3)."""
    cases = [dict(N=32, C_in=24, C_out=144, H_in=56, W_in=56, r=2),
             dict(N=64, C_in=256, C_out=512, H_in=14, W_in=14, K_h=3, K_w=3, stride=2, pad=1, r=2),
             dict(N=64, C_in=512, C_out=512, H_in=7, W_in=7, K_h=3, K_w=3, pad=1, r=4),
             dict(N=8, C_in=256, C_out=256, H_in=64, W_in=64, K_h=3, K_w=3, pad=36, dilation=36, r=8),
             dict(N=1, C_in=192, C_out=64, H_in=160, W_in=120, K_h=3, K_w=3, pad=1, r=1),
             dict(N=2, C_in=8, C_out=8, H_in=14, W_in=14, K_h=3, K_w=3, stride=2, pad=1, groups=8, r=1)]
    for kw in cases:
        d, o = B.ConvDesc(**kw), oracle.Desc(**kw)
        assert B.gf_out_shape(d) == oracle.out_shape(o)
        c, oc = B.gf_cost_model(d), oracle.cost_model(o)
        for k, v in oc.items():
            assert c[k] == pytest.approx(v, rel=1e-12), k


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; --gpus above 1 must exit with a message, before touching the GPU."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stderr + r.stdout)


def test_header_is_plain_c(tmp_path):
    """include/gf.h must compile as C99 on its own (the boundary is a C ABI) and a C program that
    only takes the addresses of the declared entry points must link against libgf.so."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    names = re.findall(r"\b(gf_[a-z0-9_]+)\s*\(", open(os.path.join(root, "include", "gf.h")).read())
    names = sorted(set(n for n in names if n in B.EXPORTS))
    assert len(names) == len(B.EXPORTS)
    src = tmp_path / "use_gf.c"
    src.write_text('#include "gf.h"\n#include <stdio.h>\ntypedef void (*fn_t)(void);\nint main(void) {\n  fn_t p[] = {'
                   + ", ".join(f"(fn_t){n}" for n in names)
                   + '};\n  printf("%d %d\\n", (int)(sizeof p / sizeof p[0]), gf_version());\n  return 0;\n}\n')
    exe = tmp_path / "use_gf"
    libdir = os.path.join(root, "paper_2301_00330_amd")
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-pedantic", f"-I{os.path.join(root, 'include')}", str(src),
                        f"-L{libdir}", "-lgf", f"-Wl,-rpath,{libdir}", "-o", str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_q8_entry_errors(lib):
    d = B.ConvDesc(**OK)
    for bad in (0.0, -1.0, float("nan"), float("inf")):
        for call in (lambda: B.gf_filter_grad_q8(d, FAKE, bad, FAKE),
                     lambda: B.gf_pool_activation_q8(d, FAKE, bad, FAKE),
                     lambda: B.gf_kernel_sum_q8(d, FAKE, bad, FAKE),
                     lambda: B.gf_conv_bwd_weight_q8(d, FAKE, FAKE, bad, FAKE, FAKE, 1 << 30),
                     lambda: B.gf_conv_bwd_input_q8(d, FAKE, FAKE, bad, FAKE, True, FAKE, 1 << 30)):
            with pytest.raises(B.GfError) as ei:
                call()
            assert ei.value.status == B.GF_ERR_BAD_DESC
    # the one-call entry checks each of its four factors the same way, then pointers, then the workspace
    for k in range(4):
        for bad in (0.0, -1.0, float("nan"), float("inf")):
            f = [1.0, 1.0, 1.0, 1.0]
            f[k] = bad
            with pytest.raises(B.GfError) as ei:
                B.gf_conv_bwd_filtered_q8(d, FAKE, f[0], FAKE, FAKE, f[1], f[2], f[3], 0, FAKE, FAKE, FAKE, 1 << 30)
            assert ei.value.status == B.GF_ERR_BAD_DESC
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_filtered_q8(d, FAKE, 1.0, 0, FAKE, 1.0, 1.0, 1.0, 0, FAKE, FAKE, FAKE, 1 << 30)
    assert ei.value.status == B.GF_ERR_NULL
    need = B.gf_workspace_bytes(d, B.GF_OP_BWD_FILTERED_Q8)
    Hy, Wy, Hp, Wp = B.gf_out_shape(d)
    assert need >= d.N * d.C_out * Hp * Wp + d.C_out * (d.C_in // d.groups)   # codes of g_y and of the kernel sums
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_filtered_q8(d, FAKE, 1.0, FAKE, FAKE, 1.0, 1.0, 1.0, 0, FAKE, FAKE, FAKE, need - 1)
    assert ei.value.status == B.GF_ERR_WORKSPACE
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_filtered_q8(d.with_(r=1), FAKE, 1.0, FAKE, FAKE, 1.0, 1.0, 1.0, 0, FAKE, FAKE, FAKE, 1 << 30)
    assert ei.value.status == B.GF_ERR_UNSUPPORTED
    # codes stand for reduced maps: r = 1 has none
    with pytest.raises(B.GfError) as ei:
        B.gf_filter_grad_q8(d.with_(r=1), FAKE, 1.0, FAKE)
    assert ei.value.status == B.GF_ERR_UNSUPPORTED
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_weight_q8(d, 0, FAKE, 1.0, FAKE, FAKE, 1 << 30)
    assert ei.value.status == B.GF_ERR_NULL
    with pytest.raises(B.GfError) as ei:
        B.gf_filter_grad_q8(d, FAKE + 4, 1.0, FAKE)
    assert ei.value.status == B.GF_ERR_UNSUPPORTED
    # full-resolution input gradient: no workspace when the kernel stores the pixel runs itself
    # (patch rows of 4 k patches), else the fp32 reduced map
    assert B.gf_workspace_bytes(d, B.GF_OP_BWD_INPUT_Q8) == 0
    d12 = d.with_(H_in=12, W_in=12)
    need = B.gf_workspace_bytes(d12, B.GF_OP_BWD_INPUT_Q8)
    assert need == d12.N * d12.C_in * 6 * 6 * 4
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_input_q8(d12, FAKE, FAKE, 1.0, FAKE, False, FAKE, need - 1)
    assert ei.value.status == B.GF_ERR_WORKSPACE


def test_probe_library_builds_and_exports(lib):
    """The measurement probes of bench.py --ceilings are a library of their own, built by the same build step."""
    import ctypes as C
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    path = os.path.join(root, "paper_2301_00330_amd", "libgf_probe.so")
    assert os.path.exists(path), "run the build step first"
    L = C.CDLL(path)
    for name in ("gfp_read", "gfp_write", "gfp_copy", "gfp_mfma", "gfp_mfma_out_floats"):
        assert getattr(L, name) is not None
    # argument checks happen on the host before any launch
    L.gfp_mfma.argtypes = [C.c_int, C.c_int, C.c_void_p, C.POINTER(C.c_double), C.c_void_p]
    ops = C.c_double(0.0)
    assert L.gfp_mfma(7, 10, FAKE, C.byref(ops), None) == 1 and L.gfp_mfma(0, 0, FAKE, C.byref(ops), None) == 1
    L.gfp_read.argtypes = [C.c_void_p, C.c_void_p, C.c_long, C.c_void_p]
    assert L.gfp_read(None, FAKE, 1024, None) == 1 and L.gfp_read(FAKE, FAKE, 8, None) == 1


def test_pool_batch_host_checks(lib):
    """gf_pool_activation_batch validates every layer before anything is enqueued."""
    d = B.ConvDesc(**OK)
    with pytest.raises(B.GfError) as ei:
        B.gf_pool_activation_batch(B.PoolBatch([], [], []))
    assert ei.value.status == B.GF_ERR_BAD_DESC
    with pytest.raises(B.GfError) as ei:
        B.gf_pool_activation_batch(B.PoolBatch([d, d], [FAKE, 0], [FAKE, FAKE]))
    assert ei.value.status == B.GF_ERR_NULL
    with pytest.raises(B.GfError) as ei:
        B.gf_pool_activation_batch(B.PoolBatch([d, d.with_(r=0)], [FAKE, FAKE], [FAKE, FAKE]))
    assert ei.value.status == B.GF_ERR_BAD_DESC
    with pytest.raises(B.GfError) as ei:
        B.gf_pool_activation_batch(B.PoolBatch([d, d.with_(dtype=B.GF_BF16)], [FAKE, FAKE], [FAKE, FAKE]))
    assert ei.value.status == B.GF_ERR_UNSUPPORTED
    with pytest.raises(B.GfError) as ei:
        B.gf_pool_activation_batch(B.PoolBatch([d, d], [FAKE, FAKE + 4], [FAKE, FAKE]))
    assert ei.value.status == B.GF_ERR_UNSUPPORTED
    # the same on 8-bit codes, plus the step-size reciprocal of every layer
    Q = B.PoolBatchQ8
    for batch, want in ((Q([], [], [], []), B.GF_ERR_BAD_DESC),
                        (Q([d, d], [FAKE, 0], [1.0, 1.0], [FAKE, FAKE]), B.GF_ERR_NULL),
                        (Q([d, d], [FAKE, FAKE], [1.0, 0.0], [FAKE, FAKE]), B.GF_ERR_BAD_DESC),
                        (Q([d, d], [FAKE, FAKE], [1.0, float("nan")], [FAKE, FAKE]), B.GF_ERR_BAD_DESC),
                        (Q([d, d.with_(dtype=B.GF_BF16)], [FAKE, FAKE], [1.0, 1.0], [FAKE, FAKE]), B.GF_ERR_UNSUPPORTED),
                        (Q([d, d.with_(r=1)], [FAKE, FAKE], [1.0, 1.0], [FAKE, FAKE]), B.GF_ERR_UNSUPPORTED),
                        (Q([d, d], [FAKE, FAKE], [1.0, 1.0], [FAKE, FAKE + 4]), B.GF_ERR_UNSUPPORTED)):
        with pytest.raises(B.GfError) as ei:
            B.gf_pool_activation_batch_q8(batch)
        assert ei.value.status == want


def test_unique_elements_entry_host_checks(lib):
    """gf_conv_bwd_unique: stride-1 layers whose padding keeps the map size; workspace = vanilla BP on
    the patch grid plus the reduced g_x."""
    d = B.ConvDesc(**OK)
    need = B.gf_workspace_bytes(d, B.GF_OP_BWD_UNIQUE)
    Hy, Wy, Hp, Wp = B.gf_out_shape(d)
    assert need >= d.N * d.C_in * Hp * Wp * 4
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_unique(d.with_(stride=2, H_in=16, W_in=16), FAKE, FAKE, FAKE, FAKE, FAKE, False, FAKE, 1 << 30)
    assert ei.value.status == B.GF_ERR_UNSUPPORTED
    with pytest.raises(B.GfError) as ei:   # 3 x 3 kernel without padding: the patch grid would shrink
        B.gf_conv_bwd_unique(d.with_(pad=0, H_in=18, W_in=18), FAKE, FAKE, FAKE, FAKE, FAKE, False, FAKE, 1 << 30)
    assert ei.value.status == B.GF_ERR_SHAPE
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_unique(d, 0, FAKE, FAKE, FAKE, FAKE, False, FAKE, 1 << 30)
    assert ei.value.status == B.GF_ERR_NULL
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_unique(d, FAKE, FAKE, FAKE, 0, 0, False, FAKE, 1 << 30)
    assert ei.value.status == B.GF_ERR_NULL
    with pytest.raises(B.GfError) as ei:
        B.gf_conv_bwd_unique(d, FAKE, FAKE, FAKE, FAKE, FAKE, False, FAKE, need - 1)
    assert ei.value.status == B.GF_ERR_WORKSPACE


# ---------------------------------------------------------------------------
# arithmetic of the fp32 contraction on the bf16 matrix pipe (dense small-map path), checked on the host
# ---------------------------------------------------------------------------
def _bf16_rne(x):
    """float32 array -> nearest bfloat16 (ties to even), returned as float32."""
    u = np.asarray(x, np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def test_three_term_bf16_split_is_exact_and_six_products_suffice():
    """The dense small-map kernels split every fp32 operand as t0 = bf16(x), t1 = bf16(x - t0), t2 = x - t0 - t1 and
    form x*y from the six term products of order <= 2.  Emulated here with numpy: both remainders are exact fp32
    values, t2 is a bf16 value, the three terms add up to x exactly, and the three dropped products (at most
    2^-23 |x y| in theory: |t1| <= 2^-8 |x|, |t2| <= 2^-16 |x|) stay below 2^-24 |x y| on these operands."""
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(200000).astype(np.float32) * np.float32(10.0) ** rng.integers(-6, 7, 200000).astype(np.float32),
                        np.float32([1.0, -1.0, 1.0 + 2.0 ** -23, 1.0 - 2.0 ** -24, 255.0 / 256.0, 3.0e38, 1.2e-30, 0.0])])
    y = np.roll(x, 7)
    def split(v):
        t0 = _bf16_rne(v)
        r1 = v - t0                                   # float32 arithmetic
        assert np.array_equal(r1.astype(np.float64), v.astype(np.float64) - t0.astype(np.float64))
        t1 = _bf16_rne(r1)
        r2 = r1 - t1
        assert np.array_equal(r2.astype(np.float64), r1.astype(np.float64) - t1.astype(np.float64))
        assert np.array_equal(_bf16_rne(r2), r2)      # the second remainder is a bf16 value
        return t0.astype(np.float64), t1.astype(np.float64), r2.astype(np.float64)
    a, b = split(x), split(y)
    assert np.array_equal(a[0] + a[1] + a[2], x.astype(np.float64))
    kept = a[0] * b[0] + a[0] * b[1] + a[1] * b[0] + a[1] * b[1] + a[0] * b[2] + a[2] * b[0]
    exact = x.astype(np.float64) * y.astype(np.float64)
    nz = exact != 0
    assert (np.abs(kept - exact)[nz] / np.abs(exact)[nz]).max() <= 2.0 ** -24
