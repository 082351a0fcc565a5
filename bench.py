#!/usr/bin/env python3
"""Benchmark of the gradient-filtered conv backward hot path on one MI355X.

A "step" is one pass of the whole filtered path over one batch of a workload:
for every conv layer, the forward-time activation pooling (gf_pool_activation),
then the gradient filter, the kernel sum, the filtered weight gradient and the
filtered input gradient in one call (gf_conv_bwd_filtered).  The default run
times ALL five benchmark configurations (each dtype and patch size of each) and
prints one JSON line: the headline is the largest workload (configuration 5:
the last conv layers of a MobileNetV2-shaped net, N=128, fp32, r=2), the others
are listed under "per_config".  Inputs are seeded synthetic tensors resident in
HBM before the timed region; buffer sets rotate so that no step finds its
tensors in the last-level cache.

Everything except the JSON line goes to stderr.
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
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}   # dense matrix-core peaks
HEADLINE = (5, "f32", 2)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--configs", default="5,1,2,3,4",
                    help="configuration ids to time (the first (config, dtype, r) of the list that matches the\n"
                         "headline workload (5, f32, 2) is the headline; without it the first one measured is)")
    ap.add_argument("--only", default="", help="CFG:DTYPE:R -- time this one combination only")
    ap.add_argument("--sets", type=int, default=0, help="rotating buffer sets (default: enough for > 768 MB)")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches only (no HIP-graph replays)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-exact", action="store_true", help="skip vanilla BP at the same shapes (speed-up denominator)")
    ap.add_argument("--miopen", action="store_true", help="also time torch's conv backward (MIOpen) as context")
    ap.add_argument("--extras", action="store_true",
                    help="also time the chained block (configuration 2) and the step on 8-bit codes")
    ap.add_argument("--step-only", default="",
                    help="CFG:DTYPE:R -- run only warm-up + steps of that step with plain launches and print a\n"
                         "short JSON line (the command the rocprofv3 summaries under profiles/ are made with)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="with --step-only: end with five plain 256 MiB device copies (a kernel of known traffic,\n"
                         "used to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--ceilings", action="store_true",
                    help="instead of the benchmark: what this GPU sustains in plain probes -- streaming reads,\n"
                         "writes and copies (HBM) and register-only loops of matrix instructions (MFMA)")
    ap.add_argument("--fig3", action="store_true",
                    help="instead of the benchmark: the three cost lines of the paper's Fig. 3 (vanilla BP, fewer\n"
                         "unique elements only, gradient filtering) as measured time on the layer of its footnote")
    ap.add_argument("--dtype", choices=["bf16", "f32"], default="f32", help="storage type for --fig3")
    return ap.parse_args()


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
    same K x K backward run on the r^2-smaller maps (gf_conv_bwd_unique, g_x at full resolution); and gradient
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
        # fewer unique elements only: the K x K backward on the reduced maps, g_x replicated to full resolution
        wss = ws_for(d, B.GF_OP_BWD_UNIQUE)

        def small_gx(k, s):
            B.gf_filter_grad(d, P(gs[k]), P(gus[k]), s)
            B.gf_conv_bwd_unique(d, P(gus[k]), 0, P(w), 0, P(gxs[k]), False, P(wss), wss.numel(), s)

        def small_all(k, s):
            B.gf_filter_grad(d, P(gs[k]), P(gus[k]), s)
            B.gf_conv_bwd_unique(d, P(gus[k]), P(xus[k]), P(w), P(gws[k]), P(gxs[k]), False, P(wss), wss.numel(), s)

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
        del xus, gus
    log(f"Fig. 3 layer: 3x3, {Ci} -> {Co} channels, {H} x {W}, N={N}, {dtype}; times per call in us")
    log(f"{'line':30s} {'r':>2s} {'MFLOP g_x / image':>18s} {'g_x us':>9s} {'g_w + g_x us':>13s}")
    for q in rows:
        log(f"{q['line']:30s} {q['r']:2d} {q['flops_gx_per_image'] / 1e6:18.1f} {q['gx_us']:9.1f} {q['backward_us']:13.1f}")
    return {"figure": "Fig. 3 (Sec. 4.2) as measured time", "n_gpus": 1, "dtype": dtype, "data": "synthetic",
            "layer": {"N": N, "C_in": Ci, "C_out": Co, "H": H, "W": W, "K": K}, "unit": "us per call",
            "note": "g_x columns include the gradient filter (Eq. 2) where it applies; the pooling of x is forward-time work",
            "lines": rows}



class LayerBufs:
    """Device tensors of one layer in one buffer set, plus raw pointers for the C ABI."""

    def __init__(self, T, B, d, x, w, gy, torch):
        s = T.shapes(d)
        self.d = d
        self.x, self.w, self.gy = x.cuda(), w.cuda(), gy.cuda()
        dt = self.x.dtype
        self.x_u = torch.empty(s["x_u"], dtype=dt, device="cuda")
        self.g_w = torch.empty(s["w"], dtype=torch.float32, device="cuda")
        self.g_x = torch.empty(s["x"], dtype=dt, device="cuda")
        self.ws_f = torch.empty(max(B.gf_workspace_bytes(d, B.GF_OP_BWD_FILTERED), 256), dtype=torch.uint8, device="cuda")
        self.ws_e = None
        self.e_w = self.e_x = None

    def nbytes(self):
        ts = [self.x, self.w, self.gy, self.x_u, self.g_w, self.g_x, self.ws_f]
        return sum(t.numel() * t.element_size() for t in ts)


# Which algorithmic quantities a kernel of the library moves, by name (the names the launch observer
# reports).  Values: keys of layer_costs() below; "mfma" marks the contraction kernels.
KERNEL_RULES = (
    ("dense_gemm_k", ("bytes_bwd_weight", "bytes_bwd_input"), True),
    ("s3s4_", ("bytes_bwd_weight", "bytes_bwd_input"), True),
    ("wgrad_", ("bytes_bwd_weight",), True), ("xwgrad_k", ("bytes_bwd_weight",), True),
    ("dgrad_", ("bytes_bwd_input",), True),
    ("dense_prep_k", ("bytes_filter",), False),
    ("onepass_k", ("bytes_fused",), False), ("dw_fused", ("bytes_fused",), False),
    ("dw_dot", ("bytes_bwd_weight",), False), ("expand", ("bytes_bwd_input",), False),
    ("patch_reduce", ("bytes_reduce",), False),
)


def layer_costs(B, d):
    """Algorithmic HBM bytes and FLOPs of one layer: gf_cost_model's figures (each tensor read or written
    once by the step that owns it), plus `bytes_fused`, what a single pass over the layer must move: read
    g_y, x_u and the kernel, write g_x and g_w."""
    c = B.gf_cost_model(d)
    Hy, Wy, Hp, Wp = B.gf_out_shape(d)
    b = 2 if d.dtype == B.GF_BF16 else 4
    wel = d.C_out * (d.C_in // d.groups) * d.K_h * d.K_w
    c["bytes_fused"] = (b * d.N * (d.C_out * Hy * Wy + d.C_in * Hp * Wp + d.C_in * d.H_in * d.W_in) + (b + 4) * wel)
    c["bytes_backward"] = c["bytes_filter"] + c["bytes_bwd_weight"] + c["bytes_bwd_input"]
    c["flops_backward"] = c["flops_bwd_weight"] + c["flops_bwd_input"]
    return c


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
    from paper_2301_00330_amd import workloads as WL
    if args.step_only:
        c, dt, r = args.step_only.split(":")
        print(json.dumps(step_only(args, int(c), dt, int(r))), flush=True)
        return
    if args.only:
        c, dt, r = args.only.split(":")
        combos = [(int(c), dt, int(r))]
    else:
        combos = []
        for c in (int(v) for v in args.configs.split(",")):
            cfg = WL.CONFIGS[c]
            combos += [(c, dt, r) for dt in cfg.dtypes for r in cfg.rs]
        if HEADLINE in combos:   # headline first
            combos.remove(HEADLINE)
            combos.insert(0, HEADLINE)
    t_start = time.time()
    results = []
    exact_cache = {}
    for (c, dt, r) in combos:
        results.append(measure(args, c, dt, r, exact_cache))
        log(f"  [{time.time() - t_start:6.1f} s] cfg{c} {dt} r={r}: {results[-1]['ms_per_step'] * 1e3:.1f} us per step, "
            f"{results[-1]['images_per_s']:.0f} images/s, step at {100 * results[-1]['step_roofline']['frac']:.0f} % of HBM peak, "
            f"dominant kernel {results[-1]['roofline']['kernel']} at {100 * results[-1]['roofline']['frac']:.0f} % of its "
            f"{results[-1]['roofline']['bound']} peak")
    head = results[0]
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(head["cfg"], head["dtype"], head["r"])
    out = {
        "metric": "filtered_conv_backward_images_per_sec", "value": head["images_per_s"], "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": head["workload"],
                   "step": "gf_pool_activation_batch over all layers (one launch), then for every layer gf_conv_bwd_filtered "
                           "(gradient filter, kernel sum, weight and input gradient)",
                   "launch": head["launch"], "buffer_sets": head["buffer_sets"], "cache": "cold (rotating sets)"},
        "roofline": head["roofline"],
        "step_roofline": head["step_roofline"],
        "cpu_baseline": cpu,
        "speedup_vs_exact_bp": head.get("speedup_vs_exact_bp"),
        "per_config": results,
    }
    print(json.dumps(out), flush=True)


def build_sets(args, cfg, dtype, r, torch, B, T, WL):
    host = [WL.make_inputs(cfg, L, dtype) for L in cfg.layers]
    descs = [T.desc_for(L, cfg.N, r, dtype) for L in cfg.layers]
    one = [LayerBufs(T, B, d, *h, torch) for d, h in zip(descs, host)]
    set_bytes = sum(lb.nbytes() for lb in one)
    # enough sets that (a) a step never finds its inputs in the 256 MB memory-side cache and (b) the
    # per-call timings, which rotate over ONE layer's tensors only, do not either (>= 1 GB of the
    # largest tensor), within 12 GB in total and 48 sets (tiny workloads stay cache-resident)
    largest = max(max(lb.x.numel() * lb.x.element_size(), lb.gy.numel() * lb.gy.element_size()) for lb in one)
    nsets = args.sets or min(48, max(3, int(768e6 // set_bytes) + 1,
                                     min(int(1.0e9 // largest) + 1, max(1, int(12e9 // set_bytes)))))
    sets = [one] + [[LayerBufs(T, B, d, *h, torch) for d, h in zip(descs, host)] for _ in range(nsets - 1)]
    return host, descs, sets, set_bytes


def step_only(args, c, dtype, r):
    """Warm-up + exactly --steps steps with plain launches, nothing else: the command behind the
    rocprofv3 kernel-trace and counter summaries under profiles/."""
    import torch
    import paper_2301_00330_amd.binding as B
    import paper_2301_00330_amd.torch_api as T
    from paper_2301_00330_amd import workloads as WL
    B.lib()
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    cfg = WL.CONFIGS[c]
    host, descs, sets, set_bytes = build_sets(args, cfg, dtype, r, torch, B, T, WL)
    P = B.ptr
    s = int(torch.cuda.current_stream().cuda_stream)

    pool_batches = [B.PoolBatch([lb.d for lb in bs], [P(lb.x) for lb in bs], [P(lb.x_u) for lb in bs]) for bs in sets]

    def step(bufset):
        B.gf_pool_activation_batch(pool_batches[sets.index(bufset)], s)
        for lb in reversed(bufset):
            B.gf_conv_bwd_filtered(lb.d, P(lb.gy), P(lb.x_u), P(lb.w), 0, P(lb.g_w), P(lb.g_x), P(lb.ws_f), lb.ws_f.numel(), s)

    for i in range(max(args.warmup, 1)):
        step(sets[i % len(sets)])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(sets[i % len(sets)])
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    if args.pmc_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
    return {"step_only": f"cfg{c}:{dtype}:r{r}", "steps": args.steps, "warmup": args.warmup, "launch": "eager",
            "ms_per_step": round(ms, 5), "buffer_sets": len(sets)}


def measure(args, c, dtype, r, exact_cache):
    import torch
    import paper_2301_00330_amd.binding as B
    import paper_2301_00330_amd.torch_api as T
    from paper_2301_00330_amd import workloads as WL

    B.lib()  # no fallback: fail here if libgf.so is missing
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    cfg = WL.CONFIGS[c]
    N = cfg.N
    layers = list(cfg.layers)
    host, descs, sets, set_bytes = build_sets(args, cfg, dtype, r, torch, B, T, WL)
    nsets = len(sets)
    log(f"workload cfg{cfg.cfg_id} '{cfg.name}' N={N} r={r} dtype={dtype}: {set_bytes / 1e6:.1f} MB per set x {nsets} sets")

    def st():
        return int(torch.cuda.current_stream().cuda_stream)

    P = B.ptr

    def enqueue_pool(lb, s): B.gf_pool_activation(lb.d, P(lb.x), P(lb.x_u), s)

    def enqueue_fused(lb, s):   # filter + weight gradient + input gradient in one call
        B.gf_conv_bwd_filtered(lb.d, P(lb.gy), P(lb.x_u), P(lb.w), 0, P(lb.g_w), P(lb.g_x), P(lb.ws_f), lb.ws_f.numel(), s)

    def enqueue_exact(lb, s):
        if lb.e_w is None:
            lb.e_w = torch.empty_like(lb.g_w)
            lb.e_x = torch.empty_like(lb.g_x)
            lb.ws_e = torch.empty(max(B.gf_workspace_bytes(lb.d, B.GF_OP_BWD_EXACT), 256), dtype=torch.uint8, device="cuda")
        B.gf_conv_bwd_exact(lb.d, P(lb.x), P(lb.w), P(lb.gy), P(lb.e_w), P(lb.e_x), P(lb.ws_e), lb.ws_e.numel(), s)

    # forward-time S0 of all layers of the step in one launch
    pool_batches = [B.PoolBatch([lb.d for lb in bs], [P(lb.x) for lb in bs], [P(lb.x_u) for lb in bs]) for bs in sets]

    def step(k):
        # the activations are pooled on the way forward, the backward pass then walks the layers
        # from the last to the first
        s = st()
        B.gf_pool_activation_batch(pool_batches[k], s)     # S0
        for lb in reversed(sets[k]):
            enqueue_fused(lb, s)                            # S1 + S2 + S3 + S4

    # ---- warm-up (eager), then optional graph capture of one step per buffer set ----
    for i in range(max(args.warmup, 1)):
        step(i % nsets)
    torch.cuda.synchronize()

    graphs = None
    if not args.no_graph:
        graphs = []
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for k in range(nsets):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    step(k)
                graphs.append(g)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        for g in graphs:   # one untimed replay each
            g.replay()
        torch.cuda.synchronize()

    def timed(k, use_graph):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(k):
            if use_graph:
                graphs[i % nsets].replay()
            else:
                step(i % nsets)
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

    # ---- per-call durations with HIP events on the launch stream (cold, rotating sets) ----
    def time_call(fn, li, reps=6):
        """Average GPU time of one call `fn` on layer `li`, cold: a HIP graph holding one call per
        buffer set (twice over) is replayed between two events on the launch stream, so neither
        host launch latency nor cache reuse enters the figure."""
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
        return ev0.elapsed_time(ev1) * 1e3 / (reps * per_graph)   # microseconds per call

    cost = [layer_costs(B, d) for d in descs]

    # ---- which kernels the step launches, and how long each runs: the launch observer of the library
    # brackets every launch of a few eager steps with a pair of events on the launch stream ----
    trace = []            # (kind, layer, kernel, ev0, ev1)
    cur = {"kind": None, "li": -1, "ev": None}

    def observer(name, phase, stream):
        if phase == 0:
            cur["ev"] = torch.cuda.Event(enable_timing=True)
            cur["ev"].record()
        else:
            e1 = torch.cuda.Event(enable_timing=True)
            e1.record()
            trace.append((cur["kind"], cur["li"], name, cur["ev"], e1))

    # The events must measure the GPU, not the host: recording two events and a launch from Python takes
    # longer than a short kernel runs, and a kernel that finds the queue empty is timed from the moment
    # the event before it completed.  Ahead of every traced step the stream therefore gets a kernel that
    # only waits (torch's device sleep, ~1.7 ms, no memory traffic), so that the step's launches and
    # events are all queued behind it before the first of them runs.
    def block_gpu():
        sleep = getattr(torch.cuda, "_sleep", None)
        if sleep is not None:
            sleep(4_000_000)

    traced_steps = 3 * nsets if nsets <= 8 else nsets
    B.gf_set_launch_observer(observer)
    try:
        for i in range(traced_steps):
            bs = sets[i % nsets]
            s = st()
            block_gpu()
            cur["kind"], cur["li"] = "pool", -1
            B.gf_pool_activation_batch(pool_batches[i % nsets], s)
            for li in reversed(range(len(bs))):
                cur["kind"], cur["li"] = "backward", li
                enqueue_fused(bs[li], s)
    finally:
        B.gf_set_launch_observer(None)
    torch.cuda.synchronize()
    # what a pair of events adds to a launch: the same single-launch call, once as event pairs around eager
    # launches (above) and once replayed back to back from a graph between two events
    def enqueue_pool_batch(lb, s):   # (time_call hands over layer 0 of a set: look the set up)
        B.gf_pool_activation_batch(pool_batches[set_of[id(lb)]], s)

    set_of = {id(bs[0]): k for k, bs in enumerate(sets)}
    pool_replay_us = time_call(enqueue_pool_batch, 0)
    # what a pair of events adds to a launch: one single-launch call (the pooling of the layer with the
    # smallest input, so that the difference is not lost in the kernel's own run-to-run spread), once as
    # event pairs around eager launches and once replayed back to back from a graph between two events
    li_cal = min(range(len(layers)), key=lambda i: cost[i]["bytes_pool"])
    cal_replay_us = time_call(enqueue_pool, li_cal)
    pairs = []
    for rep in range(4):
        for k in range(nsets):
            if k % 8 == 0:
                block_gpu()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            enqueue_pool(sets[k][li_cal], st())
            e1.record()
            pairs.append((e0, e1))
    torch.cuda.synchronize()
    cal_pair_us = sorted(a.elapsed_time(b) * 1e3 for a, b in pairs)[len(pairs) // 2]
    pair_overhead_us = max(0.0, cal_pair_us - cal_replay_us)
    # Every traced step issues the same launches in the same order: the duration of launch number p of a
    # step is the MEDIAN over the traced steps (a single disturbed step -- the box is shared with a
    # host that does other things -- must not move a mean over 77 samples by a factor), and a kernel's
    # average is the mean of those medians over its launches of a step.
    per_step = len(trace) // traced_steps
    assert per_step * traced_steps == len(trace), "every traced step must issue the same launches"
    dur = [e0.elapsed_time(e1) * 1e3 for _, _, _, e0, e1 in trace]
    med = []
    for pos in range(per_step):
        v = sorted(dur[pos::per_step])
        med.append(v[len(v) // 2])
        assert all(trace[pos + k * per_step][2] == trace[pos][2] for k in range(traced_steps))
        worst = v[-1]
        if worst > 3.0 * med[-1] + 20.0:
            log(f"    note: launch {pos} of the step ({trace[pos][2]}) took {worst:.0f} us in one traced step, "
                f"median {med[-1]:.1f} us over {traced_steps} steps; the median is reported")
    kernels = {}
    for pos in range(per_step):
        kind, li, name, _, _ = trace[pos]
        k = kernels.setdefault(name, {"us": 0.0, "launches": 0, "bytes": 0.0, "flops": 0.0, "mfma": False})
        k["us"] += med[pos] * traced_steps
        k["launches"] += traced_steps
        for prefix, keys, mfma in KERNEL_RULES:
            if name.startswith(prefix):
                for key in keys:
                    if key == "bytes_reduce" and kind == "pool":     # the batch launch pools every layer
                        k["bytes"] += traced_steps * sum(q["bytes_pool"] for q in cost)
                    else:
                        k["bytes"] += traced_steps * cost[li]["bytes_filter" if key == "bytes_reduce" else key]
                if mfma:
                    k["mfma"] = True
                    k["flops"] += traced_steps * (cost[li]["flops_backward"] if len(keys) == 2 else cost[li]["flops_bwd_weight"])
                break
    klist = []
    for name, k in kernels.items():
        avg = k["us"] / k["launches"]
        corr = max(avg - pair_overhead_us, 0.1)
        klist.append({"kernel": name, "launches_per_step": round(k["launches"] / traced_steps, 2),
                      "avg_launch_us_event_pair": round(avg, 2), "avg_launch_us": round(corr, 2),
                      "bytes_per_launch": k["bytes"] / k["launches"], "flops_per_launch": k["flops"] / k["launches"],
                      "mfma": k["mfma"], "step_share_us": round(corr * k["launches"] / traced_steps, 2)})
    klist.sort(key=lambda q: -q["step_share_us"])
    dom = klist[0]
    ridge = MFMA_PEAK_TFLOPS[dtype] * 1e12 / (HBM_PEAK_GBS * 1e9)
    if dom["mfma"] and dom["bytes_per_launch"] > 0 and dom["flops_per_launch"] / dom["bytes_per_launch"] > ridge:
        ach = dom["flops_per_launch"] / dom["avg_launch_us"] * 1e-6      # TFLOP/s
        roofline = {"kernel": dom["kernel"], "bound": "mfma", "achieved": round(ach, 2), "peak": MFMA_PEAK_TFLOPS[dtype],
                    "unit": "TFLOP/s", "frac": round(ach / MFMA_PEAK_TFLOPS[dtype], 4)}
        if dtype == "f32" and dom["kernel"] == "dense_gemm_k":
            # an fp32 contraction, priced against the fp32 matrix peak; the kernel forms every fp32 product from six
            # bf16 matrix-instruction products (operands split into three bf16 terms), so the instructions it issues
            # run at six times the algorithmic rate
            roofline["executed"] = {"what": "bf16 matrix instructions issued: 6 x the algorithmic FLOPs",
                                    "achieved": round(6 * ach, 1), "peak": MFMA_PEAK_TFLOPS["bf16"], "unit": "TFLOP/s",
                                    "frac": round(6 * ach / MFMA_PEAK_TFLOPS["bf16"], 4)}
    else:
        ach = dom["bytes_per_launch"] / dom["avg_launch_us"] * 1e-3      # GB/s
        roofline = {"kernel": dom["kernel"], "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4)}
    roofline.update({"avg_launch_us": dom["avg_launch_us"], "launches_per_step": dom["launches_per_step"],
                     "bytes_per_launch": dom["bytes_per_launch"], "flops_per_launch": dom["flops_per_launch"],
                     "method": "events around every launch of the step's kernels (launch observer; per launch of the step the "
                               "median over the traced steps), minus what an event "
                               "pair adds to a launch (the same single-launch call timed as event pairs and as back-to-back "
                               "graph replays)", "event_pair_overhead_us": round(pair_overhead_us, 2),
                     "traffic": traffic_from_profile(cfg.cfg_id, dtype, r, dom["kernel"])})
    step_bytes = sum(q["bytes_pool"] + q["bytes_backward"] for q in cost)
    step_flops = sum(q["flops_backward"] for q in cost)
    step_roofline = {"bytes": step_bytes, "flops": step_flops,
                     "achieved": round(step_bytes / (ms_per_step * 1e-3) * 1e-9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(step_bytes / (ms_per_step * 1e-3) * 1e-9 / HBM_PEAK_GBS, 4),
                     "note": "algorithmic bytes of all calls of the step (each tensor read or written once by the step that "
                             "owns it) over the step time"}

    # ---- per layer: the two calls of the step, cold, and vanilla BP at the same shape ----
    per_layer = []
    ekey = (c, dtype)
    if not args.no_exact and ekey not in exact_cache:
        exact_cache[ekey] = [time_call(enqueue_exact, li, reps=1) for li in range(len(layers))]
    ex_us = exact_cache.get(ekey)
    mi_us = None
    if args.miopen:
        import torch.nn.functional as F
        mi_us = []
        for li, L in enumerate(layers):
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
    for li, L in enumerate(layers):
        s0 = time_call(enqueue_pool, li)
        bw = time_call(enqueue_fused, li)
        q = cost[li]
        row = {"layer": L.name, "pool_us": round(s0, 2), "pool_GBps": round(q["bytes_pool"] / s0 * 1e-3, 1),
               "backward_us": round(bw, 2), "backward_bytes": q["bytes_backward"],
               "backward_GBps": round(q["bytes_backward"] / bw * 1e-3, 1),
               "backward_hbm_frac": round(q["bytes_backward"] / bw * 1e-3 / HBM_PEAK_GBS, 4),
               "backward_TFLOPs": round(q["flops_backward"] / bw * 1e-6, 3),
               "images_per_s": round(N / (bw * 1e-6), 1)}
        # the launches of one backward call (the trace repeats them every step)
        names = [name for kind, l2, name, _, _ in trace if kind == "backward" and l2 == li]
        row["kernels"] = names[:len(names) // traced_steps]
        if ex_us is not None:
            row["exact_bp_us"] = round(ex_us[li], 1)
            row["speedup_vs_exact_bp"] = round(ex_us[li] / bw, 2)
        if mi_us is not None:
            row["torch_miopen_us"] = round(mi_us[li], 1)
            row["speedup_vs_torch_miopen"] = round(mi_us[li] / bw, 2)
        per_layer.append(row)

    out = {"cfg": c, "dtype": dtype, "r": r, "N": N,
           "workload": f"cfg{cfg.cfg_id}: {cfg.name}, N={N}, r={r}, {dtype}: " + " + ".join(L.name for L in layers),
           "ms_per_step": round(ms_per_step, 5), "images_per_s": round(N / (ms_per_step * 1e-3), 1),
           "launch": "hip-graph replay" if use_graph else "eager", "launch_calibration_ms_per_step": calib,
           "buffer_sets": nsets, "pool_batch_us": round(pool_replay_us, 2), "roofline": roofline, "step_roofline": step_roofline,
           "kernels": klist, "per_layer": per_layer}
    if ex_us is not None:
        tot_b = sum(row["backward_us"] for row in per_layer)
        out["speedup_vs_exact_bp"] = round(sum(ex_us) / tot_b, 2)
        out["exact_bp_note"] = "gf_conv_bwd_exact (both gradients) per layer, cold, against gf_conv_bwd_filtered per layer"
    if mi_us is not None:
        out["speedup_vs_torch_miopen"] = round(sum(mi_us) / sum(row["backward_us"] for row in per_layer), 2)
    if args.extras:
        out.update(extras(args, cfg, dtype, r, sets, torch, B, T))
    del sets, graphs
    torch.cuda.empty_cache()
    return out


def traffic_from_profile(cfg_id, dtype, r, kernel):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE runs
    (profiles/traffic_<kernel>_cfg<id>_<dtype>_r<r>.txt, line 'traffic_bytes_per_launch=...'), or None."""
    path = os.path.join(ROOT, "profiles", f"traffic_{kernel}_cfg{cfg_id}_{dtype}_r{r}.txt")
    if os.path.exists(path):
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch="):
                return float(line.split("=")[1])
    return None


def cpu_baseline(c, dtype, r):
    """The CPU oracle as it stands on this machine's host cores, on a bounded sample of the headline
    workload: filtered backward and vanilla BP, all threads and one thread (reported baseline only)."""
    import ctypes
    import torch
    import oracle
    from paper_2301_00330_amd import workloads as WL
    cfg = WL.CONFIGS[c]
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    f64 = lambda t: t.to(torch.float64).numpy()

    def prep(n):
        out = []
        for L in cfg.layers:
            x, w, gy = WL.make_inputs(cfg, L, dtype, N=n)
            od = oracle.Desc(N=n, C_in=L.C_in, C_out=L.C_out, H_in=L.H, W_in=L.W, K_h=L.K, K_w=L.K,
                             stride=L.stride, pad=L.pad, dilation=L.dilation, groups=L.groups, r=r)
            out.append((od, f64(x), f64(w), f64(gy)))
        return out

    def run(items, exact):
        t0 = time.perf_counter()
        for od, x, w, gy in items:
            if exact:
                oracle.bwd_exact(od, x, w, gy)
            else:
                oracle.gf_backward(od, x, w, gy)
        return time.perf_counter() - t0

    threads = oracle.num_threads()
    gomp = ctypes.CDLL("libgomp.so.1")
    n_all, n_one, n_ex, n_ex1 = min(cfg.N, 32), min(cfg.N, 8), min(cfg.N, 8), min(cfg.N, 1)
    oracle.gf_backward(*prep(1)[0])     # build + warm
    items = prep(n_all)
    t_f = min(run(items, False) for _ in range(2))
    t_e = run(prep(n_ex), True)
    gomp.omp_set_num_threads(1)
    try:
        t_f1 = run(prep(n_one), False)
        t_e1 = run(prep(n_ex1), True)
    finally:
        gomp.omp_set_num_threads(threads)
    return {"value": round(n_all / t_f, 2), "unit": "images/s", "cores": threads, "kind": "oracle",
            "sample": f"filtered backward (all {len(cfg.layers)} layers of cfg{c}, {dtype} inputs, fp64 arithmetic) on "
                      f"{n_all} of {cfg.N} images, best of 2 passes",
            "cpu_model": model,
            "single_thread": {"value": round(n_one / t_f1, 2), "unit": "images/s", "cores": 1, "sample": f"{n_one} images, one pass"},
            "exact_bp": {"value": round(n_ex / t_e, 2), "unit": "images/s", "cores": threads,
                         "sample": f"gf_ref_bwd_exact (brute-force direct convolution) on {n_ex} images, one pass"},
            "exact_bp_single_thread": {"value": round(n_ex1 / t_e1, 2), "unit": "images/s", "cores": 1,
                                       "sample": f"{n_ex1} image(s), one pass"}}



def extras(args, cfg, dtype, r, sets, torch, B, T):
    """Secondary measurements (--extras): the layers as a chain that hands reduced maps from layer to layer
    (configurations whose layers form a stack), and the same step on signed 8-bit codes."""
    P = B.ptr
    nsets = len(sets)
    N = cfg.N
    out = {}

    def st():
        return int(torch.cuda.current_stream().cuda_stream)

    def run(fn):
        for i in range(max(args.warmup, 1)):
            fn(sets[i % nsets])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            fn(sets[i % nsets])
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    if cfg.chain and r > 1:
        order = list(cfg.chain)                       # back to front
        clip = list(cfg.chain_clip) if cfg.chain_clip else [0.0] * len(cfg.layers)
        for bs in sets:
            for li, lb in enumerate(bs):
                s_ = T.shapes(lb.d)
                lb.gy_u = torch.empty(s_["gy_u"], dtype=lb.x.dtype, device="cuda")
                lb.g_xu = torch.empty(s_["g_x_u"], dtype=lb.x.dtype, device="cuda")
                lb.ws_c = torch.empty(max(B.gf_workspace_bytes(lb.d, B.GF_OP_BWD_CHAINED), 256), dtype=torch.uint8, device="cuda")
                lb.m_u = torch.empty_like(lb.x_u) if clip[li] > 0 else None

        def step_chained(bufset, masked=False):
            s = st()
            for li, lb in enumerate(bufset):          # forward-time S0 (with the mask fraction below a ReLU)
                if masked and lb.m_u is not None:
                    B.gf_pool_activation_mask(lb.d, P(lb.x), clip[li], P(lb.x_u), P(lb.m_u), s)
                else:
                    B.gf_pool_activation(lb.d, P(lb.x), P(lb.x_u), s)
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

        cms = run(step_chained)
        mms = run(lambda bs: step_chained(bs, True)) if any(v > 0 for v in clip) else None
        out["chained_block"] = {
            "ms_per_step": round(cms, 5), "images_per_s": round(N / (cms * 1e-3), 1),
            "with_relu6_masks_ms_per_step": None if mms is None else round(mms, 5),
            "note": "plain launches; same layers and S0 launches, but only the top layer's g_y is filtered: "
                    "gf_conv_bwd_chained hands the reduced input gradient of a layer to the layer below; full "
                    "resolution is written only at the bottom; with masks, S0 of the layers below a ReLU6 also writes "
                    "the mask fraction and the reduced input gradient is multiplied by it inside the chained call"}
    if r > 1:
        one = sets[0]
        for bs in sets:
            for lb in bs:
                s_ = T.shapes(lb.d)
                lb.x_q = torch.empty(s_["x_u"], dtype=torch.int8, device="cuda")
                lb.gy_q = torch.empty(s_["gy_u"], dtype=torch.int8, device="cuda")
                lb.w_q = torch.empty(s_["w"][:2], dtype=torch.int8, device="cuda")
                lb.ws_q = torch.empty(max(B.gf_workspace_bytes(lb.d, B.GF_OP_BWD_FILTERED_Q8), 256),
                                      dtype=torch.uint8, device="cuda")
        # step sizes: max|.| / 127 of the reduced maps and of the kernel sum (the caller's choice; formed
        # once here from the floating-point maps of the first buffer set, outside the timed region)
        deltas = []
        for lb in one:
            gy_u = T.filter_grad(lb.d, lb.gy)
            x_u = T.pool_activation(lb.d, lb.x)
            torch.cuda.synchronize()
            dx = float(x_u.float().abs().max()) / 127.0
            dg = float(gy_u.float().abs().max()) / 127.0
            dw = float(lb.w.float().sum(dim=(2, 3)).abs().max()) / 127.0
            deltas.append((dx or 1.0, dg or 1.0, dw or 1.0))
        pool_q = {id(bs): B.PoolBatchQ8([lb.d for lb in bs], [P(lb.x) for lb in bs], [1.0 / dl[0] for dl in deltas],
                                        [P(lb.x_q) for lb in bs]) for bs in sets}

        def step_q8(bufset):
            s = st()
            B.gf_pool_activation_batch_q8(pool_q[id(bufset)], s)
            for li in reversed(range(len(bufset))):
                lb = bufset[li]
                dx, dg, dw = deltas[li]
                B.gf_conv_bwd_filtered_q8(lb.d, P(lb.gy), 1.0 / dg, P(lb.x_q), P(lb.w), 1.0 / dw, dx * dg, dg * dw, 0,
                                          P(lb.g_w), P(lb.g_x), P(lb.ws_q), lb.ws_q.numel(), s)

        qms = run(step_q8)
        out["q8_block"] = {
            "ms_per_step": round(qms, 5), "images_per_s": round(N / (qms * 1e-3), 1),
            "arithmetic": "int8 codes, int32 / int64 sums, one fp32 scaling",
            "stored_activation_bytes_per_step": int(sum(lb.x_q.numel() for lb in one)),
            "stored_activation_bytes_per_step_float_path": int(sum(lb.x_u.numel() * lb.x_u.element_size() for lb in one)),
            "note": "plain launches; gf_pool_activation_batch_q8 over all layers, then per layer gf_conv_bwd_filtered_q8 "
                    "(filter and kernel-sum codes in one launch, Eq. 5 and Eq. 3 on codes; full-resolution g_x in the "
                    "storage type)"}
    return out


if __name__ == "__main__":
    main()
