#!/usr/bin/env python3
"""Benchmark of the gradient-filtered conv backward hot path on one MI355X.

A "step" is one pass of the whole filtered path over one batch of the workload:
for every conv layer of the block, the forward-time activation pooling, the
gradient filter, the kernel sum, the filtered weight gradient and the filtered
input gradient.  The default workload is the MobileNetV2 inverted-residual block
backward (N=32, 56x56, expand 24->144, depthwise 3x3, project 144->24, r=2).
Inputs are seeded synthetic tensors resident in HBM before the timed region; the
buffer sets rotate so that no step finds its tensors in the last-level cache.

Prints one JSON line (see the keys below); everything else goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0
MFMA_F32_PEAK_TFLOPS = 157.3


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--dtype", choices=["bf16", "f32"], default="f32",
                    help="storage dtype of the headline number (fp32 is the paper's precision); the other\n"
                         "dtype of the configuration is measured too and reported under 'other_dtype'")
    ap.add_argument("--single-dtype", action="store_true", help="skip the second dtype")
    ap.add_argument("--config", type=int, default=2, help="workload: configuration id in workloads.CONFIGS")
    ap.add_argument("--r", type=int, default=0, help="patch size (default: the configuration's first)")
    ap.add_argument("--sets", type=int, default=0, help="rotating buffer sets (default: enough for > 768 MB)")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of HIP-graph replays")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-exact", action="store_true")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="end with five plain 256 MiB device copies (a kernel of known traffic, used to\n"
                         "scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--table", action="store_true", help="also print a per-layer table to stderr")
    ap.add_argument("--ceilings", action="store_true",
                    help="instead of the benchmark: what this GPU sustains in plain probes -- streaming reads,\n"
                         "writes and copies (HBM) and register-only loops of matrix instructions (MFMA)")
    ap.add_argument("--fig3", action="store_true",
                    help="instead of the benchmark: the three cost lines of the paper's Fig. 3 (vanilla BP, fewer\n"
                         "unique elements only, gradient filtering) as measured time on the layer of its footnote")
    return ap.parse_args()


class LayerBufs:
    """Device tensors of one layer in one buffer set, plus raw pointers for the C ABI."""

    def __init__(self, T, B, d, x, w, gy, torch):
        s = T.shapes(d)
        self.d = d
        self.x, self.w, self.gy = x.cuda(), w.cuda(), gy.cuda()
        dt = self.x.dtype
        self.x_u = torch.empty(s["x_u"], dtype=dt, device="cuda")
        self.gy_u = torch.empty(s["gy_u"], dtype=dt, device="cuda")
        self.g_w = torch.empty(s["w"], dtype=torch.float32, device="cuda")
        self.g_x = torch.empty(s["x"], dtype=dt, device="cuda")
        self.ws_w_bytes = B.gf_workspace_bytes(d, B.GF_OP_BWD_WEIGHT)
        self.ws_i_bytes = B.gf_workspace_bytes(d, B.GF_OP_BWD_INPUT)
        self.ws_e_bytes = B.gf_workspace_bytes(d, B.GF_OP_BWD_EXACT)
        self.ws_w = torch.empty(max(self.ws_w_bytes, 256), dtype=torch.uint8, device="cuda")
        self.ws_i = torch.empty(max(self.ws_i_bytes, 256), dtype=torch.uint8, device="cuda")
        self.ws_e = torch.empty(max(self.ws_e_bytes, 256), dtype=torch.uint8, device="cuda")
        self.ws_f_bytes = B.gf_workspace_bytes(d, B.GF_OP_BWD_FILTERED)
        self.ws_f = torch.empty(max(self.ws_f_bytes, 256), dtype=torch.uint8, device="cuda")
        self.ws_s = torch.empty(max(B.gf_workspace_bytes(d, B.GF_OP_FILTER_SNR), 256), dtype=torch.uint8, device="cuda")
        self.stats = torch.zeros(2, dtype=torch.float64, device="cuda")
        self.e_w = None
        self.e_x = None
        self.g_xu = None   # reduced input gradient (chained mode)
        self.ws_c = None

    def nbytes(self):
        ts = [self.x, self.w, self.gy, self.x_u, self.gy_u, self.g_w, self.g_x, self.ws_w, self.ws_i, self.ws_f]
        return sum(t.numel() * t.element_size() for t in ts)


def main():
    args = parse()
    if args.gpus != 1:
        log("bench.py: this build measures ONE GPU only (the path has no multi-GPU part); "
            "run with --gpus 1")
        sys.exit(2)
    if args.fig3:
        print(json.dumps(fig3(args)), flush=True)
        return
    if args.ceilings:
        print(json.dumps(ceilings()), flush=True)
        return
    out = measure(args, args.dtype, full=True)
    from paper_2301_00330_amd import workloads as WL
    others = [d for d in WL.CONFIGS[args.config].dtypes if d != out["dtype"]]
    if others and not args.single_dtype:
        o = measure(args, others[0], full=False)
        out["other_dtype"] = {k: o[k] for k in ("dtype", "value", "unit", "ms_per_step", "roofline", "per_layer",
                                                "chained_block", "q8_block") if k in o}
    print(json.dumps(out), flush=True)


def ceilings():
    """Measured ceilings of the two resources the kernels are bound by, from the probes of
    paper_2301_00330_amd/csrc_probe (a library of their own): cold streaming reads / writes / copies with
    16-byte vectors over rotating buffers (> 1.2 GB in rotation, so the 256 MB memory-side cache cannot
    serve them), and register-only loops of independent matrix instructions at 8 waves per SIMD."""
    import ctypes as C
    import torch
    lib_path = os.path.join(ROOT, "paper_2301_00330_amd", "libgf_probe.so")
    if not os.path.exists(lib_path):
        raise ImportError(f"{lib_path} is missing: build it with `python -m paper_2301_00330_amd.build`")
    L = C.CDLL(lib_path)
    vp = C.c_void_p
    L.gfp_read.argtypes = [vp, vp, C.c_long, vp]
    L.gfp_write.argtypes = [vp, C.c_long, vp]
    L.gfp_copy.argtypes = [vp, vp, C.c_long, vp]
    L.gfp_mfma.argtypes = [C.c_int, C.c_int, vp, C.POINTER(C.c_double), vp]
    L.gfp_mfma_out_floats.restype = C.c_long
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    st = lambda: int(torch.cuda.current_stream().cuda_stream)

    def timeit(fn, n):
        fn(0)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(n):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / n   # us per launch

    def ok(rc):
        if rc != 0:
            raise RuntimeError(f"probe failed with code {rc}")

    flag = torch.zeros(64, dtype=torch.int32, device="cuda")
    hbm = []
    for mb in (36, 72, 256):
        nb = mb * 1000 * 1000 // 16 * 16
        nbuf = max(3, int(1.2e9 // nb) + 1)
        bufs = [torch.empty(nb, dtype=torch.uint8, device="cuda").random_(0, 255) for _ in range(nbuf)]
        outs = [torch.empty(nb, dtype=torch.uint8, device="cuda") for _ in range(nbuf)]
        rd = timeit(lambda i: ok(L.gfp_read(bufs[i % nbuf].data_ptr(), flag.data_ptr(), nb, st())), 4 * nbuf)
        wr = timeit(lambda i: ok(L.gfp_write(outs[i % nbuf].data_ptr(), nb, st())), 4 * nbuf)
        cp = timeit(lambda i: ok(L.gfp_copy(bufs[i % nbuf].data_ptr(), outs[i % nbuf].data_ptr(), nb, st())), 4 * nbuf)
        hbm.append({"MB": mb, "read_us": round(rd, 2), "read_GBps": round(nb / rd * 1e-3, 1),
                    "write_us": round(wr, 2), "write_GBps": round(nb / wr * 1e-3, 1),
                    "copy_us": round(cp, 2), "copy_GBps_read_plus_write": round(2 * nb / cp * 1e-3, 1)})
        log(f"HBM {mb:4d} MB: read {nb / rd * 1e-6:.2f} TB/s, write {nb / wr * 1e-6:.2f} TB/s, copy {2 * nb / cp * 1e-6:.2f} TB/s (read + write)")
        del bufs, outs
    mout = torch.empty(int(L.gfp_mfma_out_floats()), dtype=torch.float32, device="cuda")
    mfma = []
    for kind, name, iters, peak in ((0, "v_mfma_f32_32x32x16_bf16", 20000, 2500.0), (1, "v_mfma_f32_16x16x32_bf16", 20000, 2500.0),
                                    (2, "v_mfma_f32_16x16x4_f32", 5000, 157.3), (3, "v_mfma_i32_16x16x64_i8", 20000, 5000.0)):
        ops = C.c_double(0.0)
        us = timeit(lambda i: ok(L.gfp_mfma(kind, iters, mout.data_ptr(), C.byref(ops), st())), 3)
        tops = ops.value / (us * 1e-6) * 1e-12
        mfma.append({"instruction": name, "T(FL)OPs": round(tops, 1), "datasheet": peak, "frac": round(tops / peak, 3)})
        log(f"MFMA {name}: {tops:.1f} T(FL)OP/s ({100 * tops / peak:.0f} % of the datasheet figure)")
    return {"what": "measured ceilings (probes, not library kernels)", "n_gpus": 1, "hbm": hbm, "mfma": mfma}


def fig3(args):
    """Sec. 4.2 / Fig. 3 on this GPU: the layer of the figure's footnote (3x3, 192 -> 64 channels, 120 x 160
    map) under the three cost lines of the analysis -- vanilla BP; 'fewer unique elements' only, i.e. the
    same K x K backward run on the r^2-smaller maps (gf_conv_bwd_exact on the reduced shape); and gradient
    filtering with the collapsed kernel (Eq. 3 / Eq. 5).  Times are per call, cold (rotating buffer sets),
    from HIP events around back-to-back launches; FLOPs are the closed forms of Eq. 1 and Eq. 12."""
    import torch
    import paper_2301_00330_amd.binding as B
    import paper_2301_00330_amd.torch_api as T
    from paper_2301_00330_amd import workloads as WL

    B.lib()
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    dtype = args.dtype
    td = WL.torch_dtype(dtype)
    N, Ci, Co, H, W, K = 8, 192, 64, 120, 160, 3
    code = B.GF_BF16 if dtype == "bf16" else B.GF_F32
    P = B.ptr
    gen = torch.Generator(device="cpu").manual_seed(230100330 + 3)
    hx = torch.randn((N, Ci, H, W), generator=gen).abs().to(td)
    hw = (torch.randn((Co, Ci, K, K), generator=gen) * (2.0 / (Ci * K * K)) ** 0.5).to(td)
    hg = (torch.randn((N, Co, H, W), generator=gen) * 1e-2).to(td)
    nsets = 8   # 118 MB of x (fp32) per set: rotation keeps every call out of the 256 MB memory-side cache

    def ws_for(d, op):
        return torch.empty(max(B.gf_workspace_bytes(d, op), 256), dtype=torch.uint8, device="cuda")

    def timed(fn, reps=5):
        s = int(torch.cuda.current_stream().cuda_stream)
        for k in range(nsets):
            fn(k, s)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            for k in range(nsets):
                fn(k, s)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (reps * nsets)

    xs = [hx.cuda() for _ in range(nsets)]
    gs = [hg.cuda() for _ in range(nsets)]
    w = hw.cuda()
    gws = [torch.empty((Co, Ci, K, K), dtype=torch.float32, device="cuda") for _ in range(nsets)]
    gxs = [torch.empty_like(xs[0]) for _ in range(nsets)]
    d1 = B.ConvDesc(N=N, C_in=Ci, C_out=Co, H_in=H, W_in=W, K_h=K, K_w=K, stride=1, pad=1, dilation=1, groups=1,
                    r=1, dtype=code)
    ws1 = ws_for(d1, B.GF_OP_BWD_EXACT)
    cost1 = B.gf_cost_model(d1)
    rows = []
    t_gx = timed(lambda k, s: B.gf_conv_bwd_exact(d1, 0, P(w), P(gs[k]), 0, P(gxs[k]), P(ws1), ws1.numel(), s))
    t_all = timed(lambda k, s: B.gf_conv_bwd_exact(d1, P(xs[k]), P(w), P(gs[k]), P(gws[k]), P(gxs[k]), P(ws1),
                                                   ws1.numel(), s))
    rows.append({"line": "vanilla BP", "r": 1, "flops_gx_per_image": cost1["flops_exact_gx"],
                 "gx_us": round(t_gx, 1), "backward_us": round(t_all, 1)})
    for r in (2, 4, 8):
        d = d1.with_(r=r)
        sh = T.shapes(d)
        xus = [torch.empty(sh["x_u"], dtype=td, device="cuda") for _ in range(nsets)]
        gus = [torch.empty(sh["gy_u"], dtype=td, device="cuda") for _ in range(nsets)]
        for k in range(nsets):
            B.gf_pool_activation(d, P(xs[k]), P(xus[k]), 0)
        cost = B.gf_cost_model(d)
        # fewer unique elements only: the exact K x K backward on the reduced maps
        ds = d1.with_(H_in=sh["x_u"][2], W_in=sh["x_u"][3])
        wss = ws_for(ds, B.GF_OP_BWD_EXACT)
        gxr = [torch.empty(sh["x_u"], dtype=td, device="cuda") for _ in range(nsets)]

        def small_gx(k, s):
            B.gf_filter_grad(d, P(gs[k]), P(gus[k]), s)
            B.gf_conv_bwd_exact(ds, 0, P(w), P(gus[k]), 0, P(gxr[k]), P(wss), wss.numel(), s)

        def small_all(k, s):
            B.gf_filter_grad(d, P(gs[k]), P(gus[k]), s)
            B.gf_conv_bwd_exact(ds, P(xus[k]), P(w), P(gus[k]), P(gws[k]), P(gxr[k]), P(wss), wss.numel(), s)

        rows.append({"line": "fewer unique elements only", "r": r,
                     "flops_gx_per_image": cost1["flops_exact_gx"] / (r * r),
                     "gx_us": round(timed(small_gx), 1), "backward_us": round(timed(small_all), 1)})
        # gradient filtering: Eq. 2, then Eq. 3 (and Eq. 5)
        wsi, wsf = ws_for(d, B.GF_OP_BWD_INPUT), ws_for(d, B.GF_OP_BWD_FILTERED)

        def gf_gx(k, s):
            B.gf_filter_grad(d, P(gs[k]), P(gus[k]), s)
            B.gf_conv_bwd_input(d, P(gus[k]), P(w), P(gxs[k]), False, P(wsi), wsi.numel(), s)

        def gf_all(k, s):
            B.gf_conv_bwd_filtered(d, P(gs[k]), P(xus[k]), P(w), 0, P(gws[k]), P(gxs[k]), P(wsf), wsf.numel(), s)

        rows.append({"line": "gradient filtering", "r": r, "flops_gx_per_image": cost["flops_gf_gx"],
                     "gx_us": round(timed(gf_gx), 1), "backward_us": round(timed(gf_all), 1)})
        del xus, gus, gxr
    log(f"Fig. 3 layer: 3x3, {Ci} -> {Co} channels, {H} x {W}, N={N}, {dtype}; times per call in us")
    log(f"{'line':30s} {'r':>2s} {'MFLOP g_x / image':>18s} {'g_x us':>9s} {'g_w + g_x us':>13s}")
    for q in rows:
        log(f"{q['line']:30s} {q['r']:2d} {q['flops_gx_per_image'] / 1e6:18.1f} {q['gx_us']:9.1f} {q['backward_us']:13.1f}")
    return {"figure": "Fig. 3 (Sec. 4.2) as measured time", "n_gpus": 1, "dtype": dtype, "data": "synthetic",
            "layer": {"N": N, "C_in": Ci, "C_out": Co, "H": H, "W": W, "K": K}, "unit": "us per call",
            "note": "g_x columns include the gradient filter (Eq. 2) where it applies; the pooling of x is forward-time work",
            "lines": rows}


def measure(args, dtype, full):
    import torch
    import paper_2301_00330_amd.binding as B
    import paper_2301_00330_amd.torch_api as T
    from paper_2301_00330_amd import workloads as WL

    B.lib()  # no fallback: fail here if libgf.so is missing
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    cfg = WL.CONFIGS[args.config]
    r = args.r or cfg.rs[0]
    if dtype not in cfg.dtypes:
        dtype = cfg.dtypes[0]
    N = cfg.N
    layers = list(cfg.layers)

    # ---- inputs: seeded on the host, copied once into several HBM-resident buffer sets ----
    host = [WL.make_inputs(cfg, L, dtype) for L in layers]
    descs = [T.desc_for(L, N, r, dtype) for L in layers]
    one = [LayerBufs(T, B, d, *h, torch) for d, h in zip(descs, host)]
    set_bytes = sum(lb.nbytes() for lb in one)
    # enough sets that (a) a step never finds its inputs in the 256 MB memory-side cache and (b) the
    # per-stage timings, which rotate over ONE layer's tensors only, do not either (>= 1 GB of the
    # largest tensor), within 12 GB in total and 48 sets (tiny workloads stay cache-resident)
    largest = max(max(lb.x.numel() * lb.x.element_size(), lb.gy.numel() * lb.gy.element_size()) for lb in one)
    nsets = args.sets or min(48, max(3, int(768e6 // set_bytes) + 1,
                                     min(int(1.0e9 // largest) + 1, max(1, int(12e9 // set_bytes)))))
    sets = [one] + [[LayerBufs(T, B, d, *h, torch) for d, h in zip(descs, host)] for _ in range(nsets - 1)]
    log(f"workload cfg{cfg.cfg_id} '{cfg.name}' N={N} r={r} dtype={dtype}: {set_bytes / 1e6:.1f} MB per set x {nsets} sets")

    def st():
        return int(torch.cuda.current_stream().cuda_stream)

    P = B.ptr

    def enqueue_pool(lb, s): B.gf_pool_activation(lb.d, P(lb.x), P(lb.x_u), s)
    def enqueue_filter(lb, s): B.gf_filter_grad(lb.d, P(lb.gy), P(lb.gy_u), s)
    def enqueue_filter_snr(lb, s):
        B.gf_filter_grad_snr(lb.d, P(lb.gy), P(lb.gy_u), P(lb.stats), P(lb.ws_s), lb.ws_s.numel(), s)
    def enqueue_bww(lb, s): B.gf_conv_bwd_weight(lb.d, P(lb.x_u), P(lb.gy_u), P(lb.g_w), P(lb.ws_w), lb.ws_w.numel(), s)
    def enqueue_bwi(lb, s): B.gf_conv_bwd_input(lb.d, P(lb.gy_u), P(lb.w), P(lb.g_x), False, P(lb.ws_i), lb.ws_i.numel(), s)

    def enqueue_fused(lb, s):   # filter + weight gradient + input gradient in one call
        B.gf_conv_bwd_filtered(lb.d, P(lb.gy), P(lb.x_u), P(lb.w), 0, P(lb.g_w), P(lb.g_x), P(lb.ws_f), lb.ws_f.numel(), s)

    def enqueue_exact(lb, s):
        if lb.e_w is None:
            lb.e_w = torch.empty_like(lb.g_w)
            lb.e_x = torch.empty_like(lb.g_x)
        B.gf_conv_bwd_exact(lb.d, P(lb.x), P(lb.w), P(lb.gy), P(lb.e_w), P(lb.e_x), P(lb.ws_e), lb.ws_e.numel(), s)

    STAGES = (("pool_activation", enqueue_pool), ("filter_grad", enqueue_filter),
              ("bwd_weight", enqueue_bww), ("bwd_input", enqueue_bwi))

    def step(bufset):
        # the order of a training step: the activations are pooled on the way forward (first layer
        # first), the backward pass then walks the layers from the last to the first
        s = st()
        for lb in bufset:
            enqueue_pool(lb, s)      # forward-time S0
        for lb in reversed(bufset):
            enqueue_fused(lb, s)     # S1 + S2 + S3 + S4

    # ---- warm-up (eager), then optional graph capture of one step per buffer set ----
    for i in range(max(args.warmup, 1)):
        step(sets[i % nsets])
    torch.cuda.synchronize()

    graphs = None
    if not args.no_graph:
        graphs = []
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for bs in sets:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    step(bs)
                graphs.append(g)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        for g in graphs:   # one untimed replay each
            g.replay()
        torch.cuda.synchronize()

    def run_steps(k, use_graph):
        for i in range(k):
            if use_graph:
                graphs[i % nsets].replay()
            else:
                step(sets[i % nsets])

    def timed(k, use_graph):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(k, use_graph)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / k

    # ---- untimed calibration: graph replay or plain launches, whichever runs the step faster
    # (replays win when the host cannot keep up with short kernels, plain launches when it can) ----
    use_graph = graphs is not None
    calib = None
    if graphs is not None:
        k = max(5, min(20, args.steps))
        calib = {"hip-graph replay": round(timed(k, True), 5), "eager": round(timed(k, False), 5)}
        use_graph = calib["hip-graph replay"] <= calib["eager"]

    # ---- the timed region: exactly --steps steps ----
    ms_per_step = timed(args.steps, use_graph)
    value = N / (ms_per_step * 1e-3)

    # ---- secondary: the layers as a chain that hands reduced maps from layer to layer ----
    chained = None
    if cfg.chain and r > 1:
        order = list(cfg.chain)                       # back to front
        for bs in sets:
            for lb in bs:
                s_ = T.shapes(lb.d)
                lb.g_xu = torch.empty(s_["g_x_u"], dtype=lb.x.dtype, device="cuda")
                nb = B.gf_workspace_bytes(lb.d, B.GF_OP_BWD_CHAINED)
                lb.ws_c = torch.empty(max(nb, 256), dtype=torch.uint8, device="cuda")

        clip = list(cfg.chain_clip) if cfg.chain_clip else [0.0] * len(layers)
        for bs in sets:
            for li, lb in enumerate(bs):
                lb.m_u = torch.empty_like(lb.x_u) if clip[li] > 0 else None

        def step_chained(bufset, masked=False):
            s = st()
            for li, lb in enumerate(bufset):          # forward-time S0 (with the mask fraction below a ReLU)
                if masked and lb.m_u is not None:
                    B.gf_pool_activation_mask(lb.d, P(lb.x), clip[li], P(lb.x_u), P(lb.m_u), s)
                else:
                    enqueue_pool(lb, s)
            top = bufset[order[0]]
            B.gf_filter_grad(top.d, P(top.gy), P(top.gy_u), s)
            gin = top.gy_u
            for k, li in enumerate(order):
                lb = bufset[li]
                last = k == len(order) - 1
                gout = lb.g_x if last else lb.g_xu
                m = P(lb.m_u) if (masked and not last and lb.m_u is not None) else 0
                B.gf_conv_bwd_chained(lb.d, P(gin), P(lb.x_u), P(lb.w), P(lb.g_w), P(gout), not last, m,
                                      P(lb.ws_c), lb.ws_c.numel(), s)
                gin = gout

        for i in range(max(args.warmup, 1)):
            step_chained(sets[i % nsets])
        torch.cuda.synchronize()
        cgraphs = None
        if not args.no_graph:
            cgraphs = []
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for bs in sets:
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g, stream=side):
                        step_chained(bs)
                    cgraphs.append(g)
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            for g in cgraphs:
                g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            if cgraphs is not None:
                cgraphs[i % nsets].replay()
            else:
                step_chained(sets[i % nsets])
        torch.cuda.synchronize()
        cms = (time.perf_counter() - t0) * 1e3 / args.steps
        mms = None
        if any(c > 0 for c in clip):   # the same chain with the clipped ReLUs of the block between the layers
            for i in range(max(args.warmup, 1)):
                step_chained(sets[i % nsets], True)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(args.steps):
                step_chained(sets[i % nsets], True)
            torch.cuda.synchronize()
            mms = (time.perf_counter() - t0) * 1e3 / args.steps
        chained = {"ms_per_step": round(cms, 5), "value": round(N / (cms * 1e-3), 1), "unit": "images/s",
                   "with_relu6_masks_ms_per_step": None if mms is None else round(mms, 5),
                   "with_relu6_masks_note": "plain launches; S0 of the layers below a ReLU6 also writes the mask "
                                            "fraction (gf_pool_activation_mask), the reduced input gradient is "
                                            "multiplied by it inside the chained call",
                   "note": "same layers and S0 launches, but only the top layer's g_y is filtered: "
                           "gf_conv_bwd_chained hands the reduced input gradient of a layer to the layer below "
                           "(valid for a stack of stride-1 convolutions with nothing between them); full "
                           "resolution is written only at the bottom"}

    # ---- secondary: the same step on signed 8-bit codes (reading of Supp. H) ----
    q8 = None
    if r > 1:
        for bs in sets:
            for lb in bs:
                s_ = T.shapes(lb.d)
                lb.x_q = torch.empty(s_["x_u"], dtype=torch.int8, device="cuda")
                lb.gy_q = torch.empty(s_["gy_u"], dtype=torch.int8, device="cuda")
                lb.w_q = torch.empty(s_["w"][:2], dtype=torch.int8, device="cuda")
                lb.ws_q = torch.empty(max(B.gf_workspace_bytes(lb.d, B.GF_OP_BWD_WEIGHT_Q8),
                                          B.gf_workspace_bytes(lb.d, B.GF_OP_BWD_INPUT_Q8), 256),
                                      dtype=torch.uint8, device="cuda")
        # step sizes: max|.| / 127 of the reduced maps and of the kernel sum (the caller's choice; formed
        # once here from the floating-point maps of the first buffer set, outside the timed region)
        deltas = []
        for lb in one:
            enqueue_pool(lb, st())
            enqueue_filter(lb, st())
            torch.cuda.synchronize()
            dx = float(lb.x_u.float().abs().max()) / 127.0
            dg = float(lb.gy_u.float().abs().max()) / 127.0
            dw = float(lb.w.float().sum(dim=(2, 3)).abs().max()) / 127.0
            deltas.append((dx or 1.0, dg or 1.0, dw or 1.0))

        def q8_pool(lb, s, li): B.gf_pool_activation_q8(lb.d, P(lb.x), 1.0 / deltas[li][0], P(lb.x_q), s)
        def q8_filter(lb, s, li): B.gf_filter_grad_q8(lb.d, P(lb.gy), 1.0 / deltas[li][1], P(lb.gy_q), s)
        def q8_ksum(lb, s, li): B.gf_kernel_sum_q8(lb.d, P(lb.w), 1.0 / deltas[li][2], P(lb.w_q), s)
        def q8_bww(lb, s, li):
            B.gf_conv_bwd_weight_q8(lb.d, P(lb.x_q), P(lb.gy_q), deltas[li][0] * deltas[li][1], P(lb.g_w),
                                    P(lb.ws_q), lb.ws_q.numel(), s)
        def q8_bwi(lb, s, li):
            B.gf_conv_bwd_input_q8(lb.d, P(lb.gy_q), P(lb.w_q), deltas[li][1] * deltas[li][2], P(lb.g_x), False,
                                   P(lb.ws_q), lb.ws_q.numel(), s)

        def step_q8(bufset):
            s = st()
            for li, lb in enumerate(bufset):
                q8_pool(lb, s, li)
            for li in reversed(range(len(bufset))):
                lb = bufset[li]
                q8_filter(lb, s, li)
                q8_ksum(lb, s, li)
                q8_bww(lb, s, li)
                q8_bwi(lb, s, li)

        for i in range(max(args.warmup, 1)):
            step_q8(sets[i % nsets])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step_q8(sets[i % nsets])
        torch.cuda.synchronize()
        qms = (time.perf_counter() - t0) * 1e3 / args.steps
        q8 = {"ms_per_step": round(qms, 5), "value": round(N / (qms * 1e-3), 1), "unit": "images/s",
              "arithmetic": "int8 codes, int32 / int64 sums, one fp32 scaling",
              "stored_activation_bytes_per_step": int(sum(lb.x_q.numel() for lb in one)),
              "stored_activation_bytes_per_step_float_path": int(sum(lb.x_u.numel() * lb.x_u.element_size() for lb in one)),
              "note": "plain launches; per layer gf_pool_activation_q8, then gf_filter_grad_q8, gf_kernel_sum_q8, "
                      "gf_conv_bwd_weight_q8 and gf_conv_bwd_input_q8 (full-resolution g_x in the storage type); "
                      "the step is bound by reading g_y and writing g_x, which the codes do not shrink"}

    # the other launch mode for comparison (eager includes the host's launch overhead)
    other_ms = timed(args.steps, not use_graph) if graphs is not None else None

    # ---- per-kernel durations with HIP events on the launch stream (cold, rotating sets) ----
    def time_stage(fn, li, reps=8):
        """Average GPU time of one launch of stage `fn` on layer `li`, cold: a HIP graph holding
        one launch per buffer set (twice over) is replayed `reps` times between two events on
        the launch stream, so neither host launch latency nor cache reuse enters the figure."""
        per_graph = 2 * nsets
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            s = int(side.cuda_stream)
            for k in range(nsets):
                fn(sets[k][li], s)
            side.synchronize()
            with torch.cuda.graph(g, stream=side):
                s = int(torch.cuda.current_stream().cuda_stream)
                for k in range(per_graph):
                    fn(sets[k % nsets][li], s)
        torch.cuda.current_stream().wait_stream(side)
        g.replay()
        torch.cuda.synchronize()
        ev0 = torch.cuda.Event(enable_timing=True)
        ev1 = torch.cuda.Event(enable_timing=True)
        ev0.record()
        for rep in range(reps):
            g.replay()
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) * 1e3 / (reps * per_graph)   # microseconds per launch

    def time_isolated(fn, li, reps=6):
        """Average duration of ONE launch, each bracketed by its own pair of events on the launch
        stream (eager, cold buffers).  This is the figure rocprofv3 reports per dispatch; it
        includes the launch ramp-up and drain that back-to-back launches overlap."""
        s = st()
        evs = []
        for k in range(nsets):
            fn(sets[k][li], s)
        torch.cuda.synchronize()
        for rep in range(reps):
            for k in range(nsets):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                fn(sets[k][li], s)
                e1.record()
                evs.append((e0, e1))
        torch.cuda.synchronize()
        return sum(a.elapsed_time(b) for a, b in evs) * 1e3 / len(evs)

    cost = [B.gf_cost_model(d) for d in descs]
    stage_bytes = {"pool_activation": "bytes_pool", "filter_grad": "bytes_filter",
                   "bwd_weight": "bytes_bwd_weight", "bwd_input": "bytes_bwd_input"}
    per_layer = []
    for li, L in enumerate(layers):
        row = {"layer": L.name}
        tot_us = 0.0
        for name, fn in STAGES:
            us = time_stage(fn, li)
            by = cost[li][stage_bytes[name]]
            row[name] = {"us": round(us, 2), "GBps": round(by / us * 1e-3, 1), "bytes": by}
            if name != "pool_activation":
                tot_us += us
        if r > 1:   # the filter with its by-product, the noise figures of Eq. (8)
            us = time_stage(enqueue_filter_snr, li)
            e_, v_ = sets[0][li].stats.tolist()
            row["filter_grad_snr"] = {"us": round(us, 2), "snr": round(e_ / v_, 4) if v_ > 0 else None}
        if q8 is not None:   # the stages of the same layer on 8-bit codes
            row["q8_us"] = {name: round(time_stage(lambda lb, s, f=fn: f(lb, s, li), li), 2)
                            for name, fn in (("pool_activation_q8", q8_pool), ("filter_grad_q8", q8_filter),
                                             ("kernel_sum_q8", q8_ksum), ("bwd_weight_q8", q8_bww),
                                             ("bwd_input_q8", q8_bwi))}
        fl = cost[li]["flops_bwd_weight"] + cost[li]["flops_bwd_input"]
        row["separate_calls_us"] = round(tot_us, 2)     # gf_filter_grad + gf_conv_bwd_weight + gf_conv_bwd_input
        tot_us = time_stage(enqueue_fused, li)
        row["backward_us"] = round(tot_us, 2)           # S1 + S2 + S3 + S4 in one call (pooling is forward-time)
        by = cost[li]["bytes_filter"] + cost[li]["bytes_bwd_weight"] + cost[li]["bytes_bwd_input"]
        row["backward_GBps"] = round(by / tot_us * 1e-3, 1)
        row["images_per_s"] = round(N / (tot_us * 1e-6), 1)
        row["tflops"] = round(fl / tot_us * 1e-6, 3)
        per_layer.append(row)

    # the reduction kernel (patch_reduce_rows) runs 2x per layer and moves most of the bytes
    red_us = [per_layer[li][k]["us"] for li in range(len(layers)) for k in ("pool_activation", "filter_grad")]
    red_by = [per_layer[li][k]["bytes"] for li in range(len(layers)) for k in ("pool_activation", "filter_grad")]
    iso_us = [time_isolated(fn, li) for li in range(len(layers)) for fn in (enqueue_pool, enqueue_filter)]
    achieved = sum(red_by) / sum(iso_us) * 1e-3      # GB/s, algorithmic bytes / per-launch duration
    pipelined = sum(red_by) / sum(red_us) * 1e-3     # same launches back to back in a graph
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_patch_reduce_rows_cfg{cfg.cfg_id}_{dtype}.txt")
    if os.path.exists(tpath):   # HBM bytes per launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch="):
                traffic = float(line.split("=")[1])
    # `achieved`: the kernel's six launch shapes of a step, each replayed back to back from a graph
    # over rotating cold buffers between two events on the launch stream; this average launch
    # duration is the one rocprofv3's kernel trace reports for the same command.  The figures with
    # one event pair around every single eager launch (which adds the events' own cost of ~3 us
    # to each launch) are kept beside it.
    roofline = {"kernel": "patch_reduce_rows", "bound": "hbm", "achieved": round(pipelined, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(pipelined / HBM_PEAK_GBS, 4),
                "avg_launch_us": round(sum(red_us) / len(red_us), 2),
                "achieved_event_pair_per_launch": round(achieved, 1),
                "frac_event_pair_per_launch": round(achieved / HBM_PEAK_GBS, 4),
                "avg_launch_us_event_pair_per_launch": round(sum(iso_us) / len(iso_us), 2),
                "bytes_per_launch": sum(red_by) / len(red_by), "traffic": traffic}

    # ---- exact BP at the same shapes (speed-up denominator) ----
    exact = None
    if full and not args.no_exact:
        import torch.nn.functional as F
        ex_us, mi_us = [], []
        for li, L in enumerate(layers):
            ex_us.append(time_stage(enqueue_exact, li, reps=1))
            # context: PyTorch-ROCm's (MIOpen) conv backward, both gradients, same tensors
            lb = sets[0][li]
            xg = lb.x.detach().clone().requires_grad_(True)
            wg = lb.w.detach().clone().requires_grad_(True)
            y = F.conv2d(xg, wg, None, L.stride, L.pad, L.dilation, L.groups)
            for _ in range(3):
                torch.autograd.grad(y, (xg, wg), lb.gy, retain_graph=True)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                torch.autograd.grad(y, (xg, wg), lb.gy, retain_graph=True)
            e1.record()
            torch.cuda.synchronize()
            mi_us.append(e0.elapsed_time(e1) * 1e3 / 10)
            del xg, wg, y
        gf_us = [row["backward_us"] for row in per_layer]
        exact = {"own_entry_us": [round(u, 1) for u in ex_us],
                 "torch_miopen_us": [round(u, 1) for u in mi_us],
                 "speedup_vs_torch_miopen": [round(e / g, 2) for e, g in zip(mi_us, gf_us)],
                 "speedup_vs_torch_miopen_block": round(sum(mi_us) / sum(gf_us), 2),
                 "speedup_vs_own_entry_block": round(sum(ex_us) / sum(gf_us), 2),
                 "note": "filtered = gf_conv_bwd_filtered (S1+S2+S3+S4) per layer; own entry = gf_conv_bwd_exact "
                         "(dense stride-1: implicit MFMA GEMMs; other dense: column tensor + MFMA GEMMs; depthwise: plane-staged "
                         "kernels), cold; torch = autograd of "
                         "F.conv2d (MIOpen), hot cache, for context"}

    # ---- CPU oracle on the host cores (reported baseline only) ----
    cpu = None
    if full and not args.no_cpu_baseline:
        import oracle
        f64 = lambda t: t.to(torch.float64).numpy()
        prep = []
        for L, d, (x, w, gy) in zip(layers, descs, host):
            od = oracle.Desc(N=N, C_in=L.C_in, C_out=L.C_out, H_in=L.H, W_in=L.W, K_h=L.K, K_w=L.K,
                             stride=L.stride, pad=L.pad, dilation=L.dilation, groups=L.groups, r=r)
            prep.append((od, f64(x), f64(w), f64(gy)))
        oracle.gf_backward(*prep[0])     # build + warm
        reps, t_cpu = 0, 0.0
        while t_cpu < 10.0 and reps < 5:
            t0 = time.perf_counter()
            for od, x, w, gy in prep:
                oracle.gf_backward(od, x, w, gy)
            t_cpu += time.perf_counter() - t0
            reps += 1
        cpu = {"value": round(N / (t_cpu / reps), 2), "unit": "images/s", "cores": oracle.num_threads(),
               "kind": "oracle", "sample": f"the full workload (all {len(layers)} layers, N={N}), fp64, mean of {reps} passes"}

    if args.table:
        for row in per_layer:
            log(json.dumps(row))

    out = {
        "metric": "filtered_conv_backward_images_per_sec", "value": round(value, 1), "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": f"cfg{cfg.cfg_id}: {cfg.name}, N={N}, r={r}, "
                               + " + ".join(L.name for L in layers),
                   "step": "gf_pool_activation + gf_conv_bwd_filtered (filter, kernel sum, weight and input gradient) for every layer",
                   "launch": "hip-graph replay" if use_graph else "eager", "buffer_sets": nsets,
                   "cache": "cold (rotating sets)"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "other_launch_mode_ms_per_step": None if other_ms is None else round(other_ms, 5),
        "launch_calibration_ms_per_step": calib,
        "per_layer": per_layer,
        "exact_bp": exact,
    }
    if chained is not None:
        out["chained_block"] = chained
    if q8 is not None:
        out["q8_block"] = q8
    del sets, one, graphs
    torch.cuda.empty_cache()
    if full and args.pmc_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    return out


if __name__ == "__main__":
    main()
