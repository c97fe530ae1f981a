#!/usr/bin/env python3
"""Benchmark of the FP4 linear hot path on one MI355X.

A step is one pass of the whole path -- forward (OCC + quantize + FP4 GEMM + residual),
activation gradient and weight gradient (with DGE) -- over every linear layer of the
workload, on synthetic inputs already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3|c2|c4|c5|c1]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP4_MFMA_PEAK_TFLOPS = 10100.0   # MI355X dense FP4 (published)
FP32_VECTOR_PEAK_TFLOPS = 157.3  # MI355X fp32 vector (published; counts packed FMAs)


def build_layers(cfg, torch, b):
    """Per-layer device tensors, drawn on the GPU with the workload's recipe."""
    layers = []
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    for li, l in enumerate(cfg.layers):
        g = torch.Generator(device="cuda")
        g.manual_seed(20250117 + 1000 * cfg.idx + 10 * li)
        A = torch.randn(l.M, l.K, generator=g, device="cuda", dtype=torch.float32)
        if cfg.act == "gauss_outlier":
            n_out = max(1, int(round(cfg.outlier_frac * l.K)))
            ch = torch.randperm(l.K, generator=g, device="cuda")[:n_out]
            A[:, ch] *= cfg.outlier_scale
        else:  # student-t, nu = 3
            chi = torch.zeros_like(A)
            for _ in range(3):
                chi += torch.randn(l.M, l.K, generator=g, device="cuda", dtype=torch.float32) ** 2
            A = A / torch.sqrt(chi / 3.0)
            del chi
        A = A.to(tdt)
        W = (torch.randn(l.K, l.N, generator=g, device="cuda", dtype=torch.float32) * 0.02).to(tdt)
        dY = (torch.randn(l.M, l.N, generator=g, device="cuda", dtype=torch.float32) * 1e-2).to(tdt)
        layers.append(dict(shape=l, A=A, W=W, dY=dY,
                           Y=torch.empty(l.M, l.N, device="cuda", dtype=tdt),
                           dA=torch.empty(l.M, l.K, device="cuda", dtype=tdt),
                           dW=torch.empty(l.K, l.N, device="cuda", dtype=torch.float32),
                           ctx=b.FwdCtx(l.M, l.K, l.N, cfg.alpha)))
    return layers


def run_step(cfg, layers, b, ws, ctx_key="ctx", alpha=None, cached=False, combined=True):
    """One pass of the whole path over every layer: forward, activation gradient, weight gradient.
    ctx_key picks the saved-state buffers (their capacity and threshold scope go with an operating
    point); cached = W's quantizations come from the per-layer weight cache (valid between optimizer
    steps) instead of being redone; combined = both gradients through fp4_linear_bwd (dY read once for
    its two quantizations) instead of the two separate entry points -- same results bit for bit."""
    alpha = cfg.alpha if alpha is None else alpha
    for L in layers:
        wq = L["wq"] if cached else None
        if cached:
            b.fp4_linear_fwd_cached(L["A"], L["W"], wq, alpha, ctx=L[ctx_key], Y=L["Y"], ws=ws)
        else:
            b.fp4_linear_fwd(L["A"], L["W"], alpha, ctx=L[ctx_key], Y=L["Y"], ws=ws)
        if combined:
            b.fp4_linear_bwd(L["dY"], L["A"], L["W"], L[ctx_key], cfg.dge_k, cfg.dge_cap, wq=wq, dA=L["dA"], dW=L["dW"], ws=ws)
        else:
            if cached:
                b.fp4_linear_bwd_dgrad_cached(L["dY"], wq, dA=L["dA"], ws=ws)
            else:
                b.fp4_linear_bwd_dgrad(L["dY"], L["W"], dA=L["dA"], ws=ws)
            b.fp4_linear_bwd_wgrad(L["A"], L["dY"], L["W"], L[ctx_key], cfg.dge_k, cfg.dge_cap, dW=L["dW"], ws=ws)


def time_steps(fn, torch, steps, warmup=1):
    for _ in range(warmup):
        fn()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def cpu_baseline(cfg):
    """The oracle, as it stands, on a bounded slice of the same workload."""
    import numpy as np
    from oracle import fp4_oracle as o
    from paper_2501_17116_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:   # the BLAS pool's size cannot be read: what the process may run on
        cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    l = min(cfg.layers, key=lambda s: s.K * s.N)
    Ms = min(l.M, 8192)   # 10-20 s of oracle work on the GPU machine's 16 host threads
    A, W, dY = synth.make_layer(cfg, l, M=Ms)
    A, W, dY = A.numpy(), W.numpy(), dY.numpy()
    t0 = time.perf_counter()
    o.fp4_linear_fwd(A, W, cfg.alpha, cfg.dtype)
    o.fp4_linear_bwd_dgrad(dY, W, cfg.dtype)
    o.fp4_linear_bwd_wgrad(A, dY, W, cfg.alpha, cfg.dge_k, cfg.dge_cap)
    dt = time.perf_counter() - t0
    flops = 3 * 2.0 * Ms * l.K * l.N
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": "layer %s (K=%d, N=%d) with %d of its %d tokens, fwd+dgrad+wgrad, %.1f s" %
                      (l.name, l.K, l.N, Ms, l.M, dt)}


HBM_PEAK_GBS = 8000.0   # MI355X HBM3E (published)


def _time(fn, torch, n=10, warm=2):
    for _ in range(warm):
        fn()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(n):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n * 1e-3


def _rotating(t, torch, min_bytes=320 << 20):
    """Copies of t whose total size exceeds the 256 MB memory-side cache, so that a kernel timed
    on them in turn reads HBM, not cache."""
    n = max(2, -(-min_bytes // (t.numel() * t.element_size())))
    return [t] + [t.clone() for _ in range(n - 1)]


def kernel_report(cfg, layers, b, torch, ws):
    """Stand-alone rates of the bandwidth-bound entry points on the workload's first layer
    (algorithmic bytes -- what the operation must read and write once -- over time, inputs rotated
    through more copies than the last-level cache holds), the cost of the fused pieces (DGE in the
    weight-gradient GEMM, the residual in the forward pass) and a bf16 GEMM chain of the same
    shapes through torch.matmul (the vendor BLAS: a yardstick, not part of the library)."""
    L = layers[0]
    l = L["shape"]
    eb = 2 if cfg.dtype == "bf16" else 4
    rep = {}

    def add(name, fn, nbytes):
        t = _time(fn, torch)
        rep[name] = {"GB/s": nbytes / t / 1e9, "frac_of_hbm_peak": nbytes / t / 1e9 / HBM_PEAK_GBS, "us": t * 1e6}

    def cyc(fn, tensors):
        state = {"i": 0}

        def run():
            state["i"] += 1
            return fn(tensors[state["i"] % len(tensors)])
        return run

    MK, KN, MN = l.M * l.K, l.K * l.N, l.M * l.N
    As, Ws, dYs = _rotating(L["A"], torch), _rotating(L["W"], torch), _rotating(L["dY"], torch)
    add("quantize_rows(dY)", cyc(lambda x: b.fp4_quantize(x, b.FP4_AXIS_ROW, ws=ws), dYs), MN * (eb + 0.5) + 4 * l.M)
    add("quantize_rows(A)", cyc(lambda x: b.fp4_quantize(x, b.FP4_AXIS_ROW, ws=ws), As), MK * (eb + 0.5) + 4 * l.M)
    # a column scale spans all rows: the tensor has to be read twice
    add("quantize_cols(W)", cyc(lambda x: b.fp4_quantize(x, b.FP4_AXIS_COL, ws=ws), Ws), KN * (2 * eb + 0.5) + 4 * l.N)
    add("quantize_cols(dY)", cyc(lambda x: b.fp4_quantize(x, b.FP4_AXIS_COL, ws=ws), dYs), MN * (2 * eb + 0.5) + 4 * l.N)
    # OCC: thresholds cannot be applied in the pass that finds them: two reads, codes, CSR entries
    dens = 2 * (1 - cfg.alpha)
    add("occ_clamp_residual(A)", cyc(lambda x: b.occ_clamp_residual(x, cfg.alpha, ws=ws), As),
        MK * (2 * eb + 0.5 + 8 * dens) + 12 * l.M)
    G = torch.empty(l.K, l.N, device="cuda", dtype=torch.float32).normal_()
    add("dge_apply(W)", cyc(lambda x: b.fp4_dge_apply(G, x, L["ctx"].gamma_W, cfg.dge_k, cfg.dge_cap, dW=L["dW"]), Ws),
        KN * (eb + 8))
    del As, Ws, dYs
    nnz = int(L["ctx"].nnz.item())
    R = torch.empty(l.M, l.N, device="cuda", dtype=torch.float32)
    t = _time(lambda: b.fp4_residual_spmm(L["ctx"].row_ptr, L["ctx"].col_idx, L["ctx"].val, l.K, L["W"], R=R, ws=ws),
              torch)
    # bound by the vector ALUs (fp32 FMAs): against the published fp32 vector peak, which counts
    # packed FMAs the kernel does not use (one FMA per lane and cycle is half of it)
    rep["residual_spmm(fwd)"] = {"nnz": nnz, "us": t * 1e6, "GFLOP/s": 2.0 * nnz * l.N / t / 1e9, "bound": "alu",
                                 "frac_of_fp32_vector_peak": 2.0 * nnz * l.N / t / 157.3e12}
    del R
    # what the fused pieces cost: forward with and without the outlier residual, weight gradient
    # with the DGE factor and with the straight-through estimator (dge_k = 0)
    ctx1 = b.FwdCtx(l.M, l.K, l.N, 1.0)
    t_occ = _time(lambda: b.fp4_linear_fwd(L["A"], L["W"], cfg.alpha, ctx=L["ctx"], Y=L["Y"], ws=ws), torch)
    t_plain = _time(lambda: b.fp4_linear_fwd(L["A"], L["W"], 1.0, ctx=ctx1, Y=L["Y"], ws=ws), torch)
    rep["fwd(layer 0)"] = {"us_with_residual": t_occ * 1e6, "us_without": t_plain * 1e6, "nnz": nnz}
    t_dge = _time(lambda: b.fp4_linear_bwd_wgrad(L["A"], L["dY"], L["W"], ctx1, cfg.dge_k, cfg.dge_cap, dW=L["dW"],
                                                 ws=ws), torch)
    t_ste = _time(lambda: b.fp4_linear_bwd_wgrad(L["A"], L["dY"], L["W"], ctx1, 0.0, cfg.dge_cap, dW=L["dW"], ws=ws),
                  torch)
    rep["wgrad(layer 0, no residual)"] = {"us_with_dge": t_dge * 1e6, "us_ste": t_ste * 1e6}
    b.fp4_linear_fwd(L["A"], L["W"], cfg.alpha, ctx=L["ctx"], Y=L["Y"], ws=ws)   # restore the saved state

    def bf16_chain():
        for X in layers:
            torch.matmul(X["A"], X["W"], out=X["Y"])
            torch.matmul(X["dY"], X["W"].t(), out=X["dA"])
            torch.matmul(X["A"].t(), X["dY"])
    if cfg.dtype == "bf16":
        t = _time(bf16_chain, torch, n=5, warm=2)
        flops = sum(3 * 2.0 * X["shape"].M * X["shape"].K * X["shape"].N for X in layers)
        rep["bf16_gemm_chain(torch.matmul)"] = {"ms": t * 1e3, "TFLOP/s": flops / t / 1e12}
    return rep


def operating_points(cfg, layers, b, torch, ws, step_flops, steps=3):
    """The same step at the other residual densities of Sec. 4.3 (alpha = 0.999 / 0.97: 0.2 % / 6 %), with the
    compensation off, under the per-token reading of the clamp, and with W's quantizations cached across
    micro-batches.  Whole-path ms per step and TFLOP/s on the dense GEMM FLOPs, like the headline."""
    out = {}

    def leg(name, **kw):
        ms = time_steps(lambda: run_step(cfg, layers, b, ws, **kw), torch, steps)
        out[name] = {"ms_per_step": ms, "TFLOP/s": step_flops / (ms * 1e-3) / 1e12}

    for a in (0.999, 0.97, 1.0):
        if a == cfg.alpha:
            continue
        key = "ctx_a%g" % a
        for L in layers:
            l = L["shape"]
            L[key] = b.FwdCtx(l.M, l.K, l.N, a)
        leg("alpha=%g" % a if a < 1.0 else "occ_off", ctx_key=key, alpha=a)
        for L in layers:
            del L[key]
    if all(L["shape"].K <= 16384 for L in layers):
        for L in layers:
            l = L["shape"]
            L["ctx_tok"] = b.FwdCtx(l.M, l.K, l.N, cfg.alpha, scope=b.FP4_OCC_TOKEN)
        leg("per_token_thresholds(alpha=%g)" % cfg.alpha, ctx_key="ctx_tok")
        L0 = layers[0]
        l = L0["shape"]
        eb = 2 if cfg.dtype == "bf16" else 4
        As = _rotating(L0["A"], torch)
        st = {"i": 0}

        def occ_tok():
            st["i"] += 1
            b.occ_clamp_residual(As[st["i"] % len(As)], cfg.alpha, ws=ws, scope=b.FP4_OCC_TOKEN)
        t = _time(occ_tok, torch)
        nbytes = l.M * l.K * (eb + 0.5 + 8 * 2 * (1 - cfg.alpha)) + 20 * l.M   # one read: the row holds its own thresholds
        out["occ_clamp_residual_token(A)"] = {"us": t * 1e6, "GB/s": nbytes / t / 1e9,
                                              "frac_of_hbm_peak": nbytes / t / 1e9 / HBM_PEAK_GBS}
        del As
        c = L0["ctx_tok"]
        R = torch.empty(l.M, l.N, device="cuda", dtype=torch.float32)
        t = _time(lambda: b.fp4_residual_spmm(c.row_ptr, c.col_idx, c.val, l.K, L0["W"], R=R, ws=ws), torch)
        nnz = int(c.nnz.item())
        out["residual_spmm(fwd, per-token rows)"] = {"nnz": nnz, "us": t * 1e6, "GFLOP/s": 2.0 * nnz * l.N / t / 1e9}
        del R
        for L in layers:
            del L["ctx_tok"]
    # the mixed-format GEMM of the W4A8 / W8A4 ablations on the first layer's forward shape (8-bit operands
    # run the matrix cores at the FP8 rate: 5 PFLOP/s published)
    L0 = layers[0]
    l = L0["shape"]
    if l.K % 128 == 0:
        a8, ga8 = b.fp8_quantize(L0["A"], b.FP4_AXIS_ROW, ws=ws)
        w4, gw4 = b.fp4_quantize(L0["W"], b.FP4_AXIS_COL, ws=ws)
        t = _time(lambda: b.fp4_gemm_mixed(a8, b.FP4_FMT_E4M3, ga8, w4, b.FP4_FMT_E2M1, gw4, out_dtype=L0["Y"].dtype), torch,
                  n=5)
        fl = 2.0 * l.M * l.K * l.N
        out["mixed_gemm(W4A8, layer 0 fwd)"] = {"us": t * 1e6, "TFLOP/s": fl / t / 1e12, "frac_of_fp8_mfma_peak": fl / t / 5.0e15}
        del a8, w4
        ctx8 = b.FwdCtx(l.M, l.K, l.N, 1.0)
        t = _time(lambda: b.fp4_linear_fwd_mixed(L0["A"], L0["W"], b.FP4_FMT_E4M3, b.FP4_FMT_E2M1, 1.0, ctx=ctx8, Y=L0["Y"],
                                                 ws=ws), torch, n=5)
        out["fwd_mixed(W4A8, layer 0)"] = {"us": t * 1e6, "TFLOP/s": fl / t / 1e12}
    # the granularity ablation's forward pass (tensor-wise scales on both operands) beside the vector-wise one
    L0 = layers[0]
    l = L0["shape"]
    fl = 2.0 * l.M * l.K * l.N
    ctxg = b.FwdCtx(l.M, l.K, l.N, cfg.alpha)
    t = _time(lambda: b.fp4_linear_fwd_granularity(L0["A"], L0["W"], True, True, cfg.alpha, ctx=ctxg, Y=L0["Y"], ws=ws), torch, n=5)
    out["fwd_tensorwise_scales(layer 0)"] = {"us": t * 1e6, "TFLOP/s": fl / t / 1e12}
    del ctxg
    for L in layers:
        L["wq"] = b.fp4_prepare_weights(L["W"], ws=ws)
    leg("cached_W_quantizations", cached=True)
    leg("separate_dgrad_and_wgrad_calls", combined=False)
    for L in layers:
        del L["wq"]
    run_step(cfg, layers, b, ws)   # leave the default saved state behind
    # the same step recorded once in a HIP graph and replayed: the entry points only enqueue kernels
    # on the caller's stream, so the whole step is capturable (tests/test_gpu_graph.py checks the results)
    try:
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run_step(cfg, layers, b, ws)
        ms = time_steps(graph.replay, torch, steps)
        out["step_replayed_from_hip_graph"] = {"ms_per_step": ms, "TFLOP/s": step_flops / (ms * 1e-3) / 1e12}
        del graph
    except Exception as e:   # reported, never fatal: the headline does not depend on it
        out["step_replayed_from_hip_graph"] = {"error": str(e)[:200]}
    torch.cuda.synchronize()
    return out


def ceilings(b, torch):
    """What this part sustains: FP4 MFMA issue loop (constant and random operand data) and a
    streaming copy.  Context for the roofline fractions, which stay quoted against the
    published peaks."""
    out = {}
    wgs, iters = 256, 20000
    sink = torch.empty(wgs * 512, device="cuda", dtype=torch.float32)
    flop = wgs * 8.0 * iters * 8 * 131072
    for name, data in (("constant", torch.full((1 << 20,), 0x21, dtype=torch.uint8, device="cuda")),
                       ("random", torch.randint(0, 256, (1 << 20,), dtype=torch.uint8, device="cuda"))):
        t = _time(lambda: b.fp4_probe_mfma(data, wgs, iters, sink), torch, n=3, warm=1)
        out["fp4_mfma_issue_loop_%s_operands_TFLOPs" % name] = flop / t / 1e12
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").zero_()
    dst = torch.empty_like(src)
    t = _time(lambda: b.fp4_probe_copy(src, dst), torch, n=5, warm=1)
    out["stream_copy_GBs_read_plus_write"] = 2.0 * src.numel() / t / 1e9
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3")
    ap.add_argument("--alpha", type=float, default=None,
                    help="OCC quantile instead of the workload's (1.0 switches the residual off)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device copy (gives hardware counters a kernel of known traffic)")
    ap.add_argument("--no-kernel-report", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.stderr.write("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
                         "--gpus %d is not supported\n" % args.gpus)
        sys.exit(2)

    import torch
    from paper_2501_17116_amd import binding as b
    from paper_2501_17116_amd import synth

    b.lib()   # fail loudly if the HIP library is missing
    cfg = synth.CONFIGS[args.workload]
    if args.alpha is not None:
        import dataclasses
        cfg = dataclasses.replace(cfg, alpha=args.alpha)
    torch.cuda.set_device(0)
    layers = build_layers(cfg, torch, b)
    ws = b.Workspace()
    n_gemm = 3 * len(layers)
    gemm_flops = []
    for L in layers:
        l = L["shape"]
        gemm_flops += [2.0 * l.M * l.K * l.N] * 3
    step_flops = sum(gemm_flops)

    for _ in range(args.warmup):
        run_step(cfg, layers, b, ws)
    torch.cuda.synchronize()

    n_spmm = 2 * len(layers) if cfg.alpha < 1.0 else 0
    n_trace = (n_gemm + n_spmm) * args.steps
    b.fp4_trace_begin(n_trace)
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t_wall0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        run_step(cfg, layers, b, ws)
    e1.record()
    torch.cuda.synchronize()
    t_wall = time.perf_counter() - t_wall0
    ms_total = e0.elapsed_time(e1)
    trace = b.fp4_trace_end(n_trace)
    gemm_ms = [ms for kind, ms in trace if kind == b.FP4_TRACE_GEMM]
    spmm_ms = [ms for kind, ms in trace if kind == b.FP4_TRACE_SPMM]
    ms_per_step = ms_total / args.steps
    value = step_flops / (ms_per_step * 1e-3) / 1e12

    avg_gemm_ms = sum(gemm_ms) / max(len(gemm_ms), 1)
    avg_gemm_flops = step_flops / n_gemm
    achieved = avg_gemm_flops / (avg_gemm_ms * 1e-3) / 1e12 if gemm_ms else 0.0
    out = {
        "metric": "FP4 linear fwd+bwd TFLOP/s and % of FP4 MFMA peak; quantize GB/s",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp4-e2m1 x fp4-e2m1 -> f32", "data": "synthetic",
        "config": {"workload": "%s (%s): %s; M=%d tokens, %s masters, OCC alpha=%g, DGE k=%g; "
                               "fwd+dgrad+wgrad per layer" %
                               (args.workload, cfg.name,
                                ", ".join("%s %dx%d" % (l.name, l.K, l.N) for l in cfg.layers),
                                cfg.layers[0].M, cfg.dtype, cfg.alpha, cfg.dge_k),
                   "gemm_flop_per_step": step_flops, "wall_ms_per_step": t_wall / args.steps * 1e3},
        # the contraction the metric names: the FP4 GEMM against the FP4 matrix-core peak
        "roofline": {"bound": "mfma", "kernel": "fp4_gemm_nt_kernel", "achieved": achieved,
                     "peak": FP4_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / FP4_MFMA_PEAK_TFLOPS,
                     "traffic": None, "avg_launch_ms": avg_gemm_ms, "launches": len(gemm_ms),
                     "share_of_step": sum(gemm_ms) / ms_total if ms_total else None},
    }
    if spmm_ms:
        # the kernel the step spends most of its time in: the residual product, plain fp32 FMAs on the
        # vector ALUs (2 nnz N FLOP per launch), against the published fp32 vector peak
        nnz = [int(L["ctx"].nnz.item()) for L in layers]
        spmm_flops = sum(2 * 2.0 * n * L["shape"].N for n, L in zip(nnz, layers))   # forward + weight gradient
        avg_spmm_ms = sum(spmm_ms) / len(spmm_ms)
        ach = spmm_flops / n_spmm / (avg_spmm_ms * 1e-3) / 1e12
        out["roofline_residual"] = {"bound": "alu", "kernel": "spmm_tile_kernel", "achieved": ach,
                                    "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                                    "frac": ach / FP32_VECTOR_PEAK_TFLOPS, "traffic": None,
                                    "avg_launch_ms": avg_spmm_ms, "launches": len(spmm_ms),
                                    "share_of_step": sum(spmm_ms) / ms_total if ms_total else None,
                                    "nnz_per_layer": nnz}
    tfile = os.path.join(ROOT, "profiles", "fp4_gemm_nt_kernel_%s_hbm_traffic.txt" % args.workload)
    if os.path.exists(tfile):   # hardware counters cannot be read from inside the run: the committed PMC summary
        for line in open(tfile):
            if line.startswith("TRAFFIC_BYTES_PER_LAUNCH="):
                out["roofline"]["traffic"] = float(line.split("=", 1)[1])
                out["roofline"]["traffic_source"] = os.path.relpath(tfile, ROOT)
    mfile = os.path.join(ROOT, "profiles", "fp4_gemm_nt_kernel_%s_mfma_busy.md" % args.workload)
    if os.path.exists(mfile):   # likewise: share of the kernel's CU-cycles in which the matrix cores were busy
        for line in open(mfile):
            if line.startswith("MFMA_BUSY_FRACTION="):
                out["roofline"]["matrix_core_busy"] = float(line.split("=", 1)[1])
                out["roofline"]["matrix_core_busy_source"] = os.path.relpath(mfile, ROOT)
    if not args.no_kernel_report:
        out["kernels"] = kernel_report(cfg, layers, b, torch, ws)
        if cfg.alpha < 1.0 and args.alpha is None:
            out["operating_points"] = operating_points(cfg, layers, b, torch, ws, step_flops)
        out["ceilings"] = ceilings(b, torch)
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").zero_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
