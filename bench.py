"""Benchmark of the tile-operation hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2]

A step is one forward + backward pass (+ Adam step for the configurations that
take one) of a GPT-2 block through the C-ABI library, on seed-generated inputs
that are resident in HBM before the timed region starts.  Prints ONE JSON line:
whole-job TFLOP/s, the roofline figures of the dominant kernel measured with HIP
events inside the timed region (per-task timing of the executor), and the fp64
CPU oracle timed on the host cores of the same box over a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2516.6}     # dense MFMA peaks of MI355X
PEAK_HBM_GBS = 8000.0


def cpu_baseline(cfg, sample_batch):
    """The oracle as it stands, forward + backward, on a batch-reduced sample of the workload."""
    import numpy as np
    import threadpoolctl
    import workload
    from oracle import definition as D
    scfg = cfg.replace(N_b=sample_batch)
    inp = workload.generate(scfg)
    p64 = {k: np.asarray(inp[k], np.float64) for k in workload.PARAM_NAMES}
    t0 = time.perf_counter()
    Out, cache = D.block_forward(p64, inp["X"], scfg.N_h, scfg.eps, scfg.gelu)
    D.block_backward(p64, cache, inp["dOut"], scfg.N_h, scfg.gelu)
    dt = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] or [1])
    flops = workload.model_flops(scfg, tile_skip=False)      # the oracle computes every score
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": "%s with N_b=%d of %d (fp64 numpy oracle, forward+backward, %.1f s)" % (cfg.name, sample_batch, cfg.N_b, dt),
            "seconds": dt}


def model_ops(cfg, capi, tiled, torch):
    """Embedding lookup, its adjoint and the cross-entropy loss over vocabulary tiles at the config's token
    count and a GPT-2-sized vocabulary (50304 = 50257 padded to a multiple of 128), timed per operation."""
    import numpy as np
    N_v, tv = 50304, 8192
    T = cfg.N_s * cfg.N_b
    w = 4 if cfg.dtype == "f32" else 2
    out = []
    with tiled.Context(n_streams=1) as ctx:
        base_e, base_s = min(cfg.tile, cfg.N_e), min(cfg.tile, cfg.N_s)
        W = tiled.TiledTensor(ctx, "f32", (cfg.N_e, N_v), (base_e, tv))
        dW = tiled.TiledTensor.zeros(ctx, (cfg.N_e, N_v), (base_e, tv))
        Y = tiled.TiledTensor(ctx, cfg.dtype, (cfg.N_e, cfg.N_s, cfg.N_b), (base_e, base_s, cfg.N_b))
        X = tiled.TiledTensor(ctx, cfg.dtype, (N_v, cfg.N_s, cfg.N_b), (tv, base_s, cfg.N_b))
        S = tiled.TiledTensor(ctx, "f32", (2, cfg.N_s, cfg.N_b), (2, base_s, cfg.N_b))
        for t in (W, Y, X):
            for k in range(len(t.tile_index)):
                t.tile_view(k).normal_()
        g = torch.Generator(device="cuda").manual_seed(1)
        tok = torch.randint(0, N_v, (T,), device="cuda", dtype=torch.int32, generator=g)
        col, tot = torch.empty(T, device="cuda"), torch.empty(1, device="cuda")

        def run(call, reps=6):
            call()
            ctx.wait()
            ctx.profile(True)
            for _ in range(reps):
                call()
            ctx.wait()
            rec = ctx.profile_read()
            ctx.profile(False)
            return rec
        for name, call in (("embedding_fwd", lambda: capi.nnt_embedding_fwd(ctx.h, tok.data_ptr(), W.h, Y.h)),
                           ("embedding_bwd", lambda: capi.nnt_embedding_bwd(ctx.h, tok.data_ptr(), Y.h, dW.h)),
                           ("cross_entropy", lambda: capi.nnt_cross_entropy(ctx.h, X.h, tok.data_ptr(), S.h, col.data_ptr(), tot.data_ptr()))):
            for label, e in run(call).items():
                ms = e["ms"] / max(e["tasks"], 1)
                gbs = e["work"] / max(e["tasks"], 1) / ms / 1e6
                out.append({"operation": name, "kernel": label, "N_v": N_v, "tokens": T, "median_free_ms": ms, "GB/s": gbs,
                            "frac_hbm_peak": gbs / PEAK_HBM_GBS})
    return out


def tile_kernels(cfg, capi, torch):
    """Single-kernel figures through the nnt_tile_* entry points at the shapes of `cfg`."""
    dt = capi.NNT_F32 if cfg.dtype == "f32" else capi.NNT_BF16
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    w = 4 if cfg.dtype == "f32" else 2
    st = torch.cuda.current_stream().cuda_stream
    T = cfg.N_s * cfg.N_b

    def timed(call, nsets, iters=24, warm=3):
        for i in range(warm):
            call(i % nsets)
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
        ev[0].record()
        for i in range(iters):
            call(i % nsets)
            ev[i + 1].record()
        torch.cuda.synchronize()
        ts = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(iters))
        return ts[len(ts) // 2], ts[0]

    out = {"products": [], "memory_bound": []}
    # products: the whole operations of the block (what one launch covers) and the paper's tile task
    t = cfg.tile
    shapes = [("qkv / fc1-like  W X", "N", "N", 3 * cfg.N_e, T, cfg.N_e), ("fc1  W X", "N", "N", cfg.N_m, T, cfg.N_e),
              ("fc2  W X", "N", "N", cfg.N_e, T, cfg.N_m), ("dX = W^T dY", "T", "N", cfg.N_e, T, cfg.N_m),
              ("dW = dY X^T", "N", "T", cfg.N_m, cfg.N_e, T), ("one tile task (paper's granularity)", "N", "N", min(t, cfg.N_e), min(t, cfg.N_s) * cfg.N_b, min(t, cfg.N_e))]
    for name, opA, opB, m, n, k in shapes:
        A = torch.randn(m * k, device="cuda").to(tdt)
        B = torch.randn(k * n, device="cuda").to(tdt)
        Cm = torch.zeros(m * n, device="cuda").to(tdt)
        lda = m if opA == "N" else k
        ldb = k if opB == "N" else n
        med, mn = timed(lambda i: capi.nnt_tile_gemm(st, dt, dt, 0 if opA == "N" else 1, 0 if opB == "N" else 1, m, n, k, 1, 1.0,
                                                     A.data_ptr(), lda, m * k, B.data_ptr(), ldb, k * n, 0.0, Cm.data_ptr(), m, m * n), 1)
        tf = 2.0 * m * n * k / med / 1e9
        out["products"].append({"name": name, "op": opA + opB, "m": m, "n": n, "k": k, "median_us": med * 1e3, "min_us": mn * 1e3,
                                "TFLOP/s": tf, "frac_mfma_peak": tf / PEAK_TFLOPS[cfg.dtype]})
    # the weight-gradient shape again through the tensor-level operation, whose plan may cut the long
    # contraction into slices (the stateless tile call has no workspace and leaves most CUs idle here)
    from paper_2504_13236_amd import tiled as _tiled
    with _tiled.Context(n_streams=1) as ctx:
        m, n, k = cfg.N_m, cfg.N_e, T
        tA = _tiled.TiledTensor(ctx, cfg.dtype, (m, k), (m, k))
        tB = _tiled.TiledTensor(ctx, cfg.dtype, (n, k), (n, k))
        tC = _tiled.TiledTensor(ctx, "f32", (m, n), (m, n))
        for t_ in (tA, tB):
            t_.tile_view(0).normal_()
        for _ in range(3):
            capi.nnt_gemm(ctx.h, 1.0, 0, tA.h, 1, tB.h, 0.0, tC.h, 1, 0, None)
        ctx.wait()
        ctx.profile(True)
        for _ in range(12):
            capi.nnt_gemm(ctx.h, 1.0, 0, tA.h, 1, tB.h, 0.0, tC.h, 1, 0, None)
        ctx.wait()
        rec = ctx.profile_read()
        ms = sum(e["ms"] for e in rec.values()) / 12
        tf = 2.0 * m * n * k / ms / 1e9
        out["products"].append({"name": "dW = dY X^T through nnt_gemm (k cut into slices, sum kernel included)", "op": "NT", "m": m, "n": n,
                                "k": k, "median_us": ms * 1e3, "min_us": ms * 1e3, "TFLOP/s": tf,
                                "frac_mfma_peak": tf / PEAK_TFLOPS[cfg.dtype]})
    # attention products, batched over (batch, head), one sequence-tile pair
    ts_ = min(t, cfg.N_s)
    h, nb = cfg.N_e // cfg.N_h, cfg.N_b * cfg.N_h
    for name, opA, opB, m, n, k in (("scores K^T Q", "T", "N", ts_, ts_, h), ("V P", "N", "N", h, ts_, ts_), ("dV = dB P^T", "N", "T", h, ts_, ts_)):
        A = torch.randn(m * k * nb, device="cuda").to(tdt)
        B = torch.randn(k * n * nb, device="cuda").to(tdt)
        Cm = torch.zeros(m * n * nb, device="cuda").to(tdt)
        lda = m if opA == "N" else k
        ldb = k if opB == "N" else n
        med, mn = timed(lambda i: capi.nnt_tile_gemm(st, dt, dt, 0 if opA == "N" else 1, 0 if opB == "N" else 1, m, n, k, nb, 1.0,
                                                     A.data_ptr(), lda, m * k, B.data_ptr(), ldb, k * n, 0.0, Cm.data_ptr(), m, m * n), 1)
        tf = 2.0 * m * n * k * nb / med / 1e9
        gb = w * nb * (m * k + k * n + m * n) / med / 1e6
        out["products"].append({"name": name, "op": opA + opB, "m": m, "n": n, "k": k, "batch": nb, "median_us": med * 1e3,
                                "min_us": mn * 1e3, "TFLOP/s": tf, "frac_mfma_peak": tf / PEAK_TFLOPS[cfg.dtype], "GB/s": gb,
                                "frac_hbm_peak": gb / PEAK_HBM_GBS})

    # memory-bound kernels on one activation-sized tile set (N_m x T elements), warm and cold
    n_el = cfg.N_m * T
    nsets = max(3, -(-(640 << 20) // (3 * n_el * w)))

    def bufs(count, dtype=tdt):
        return [[torch.randn(n_el, device="cuda").to(dtype) for _ in range(count)] for _ in range(nsets)]

    def report(name, bytes_per_el, call, sets):
        rec = {"name": name, "elements": n_el, "bytes_per_element": bytes_per_el}
        for label, ns in (("warm", 1), ("cold", sets)):
            med, mn = timed(call, ns)
            rec[label] = {"median_us": med * 1e3, "GB/s": bytes_per_el * n_el / med / 1e6, "frac_hbm_peak": bytes_per_el * n_el / med / 1e6 / PEAK_HBM_GBS}
        out["memory_bound"].append(rec)

    b = bufs(3)
    report("gelu", 2 * w, lambda i: capi.nnt_tile_gelu(st, dt, 0, n_el, b[i][0].data_ptr(), b[i][1].data_ptr()), nsets)
    report("gelu_bwd", 3 * w, lambda i: capi.nnt_tile_gelu_bwd(st, dt, 0, n_el, b[i][0].data_ptr(), b[i][1].data_ptr(), b[i][2].data_ptr()), nsets)
    report("add (y = a x + b y)", 3 * w, lambda i: capi.nnt_tile_add(st, dt, n_el, 1.0, b[i][0].data_ptr(), 1.0, b[i][1].data_ptr()), nsets)
    bias = torch.randn(cfg.N_m, device="cuda")
    report("bias_add", 2 * w, lambda i: capi.nnt_tile_bias_add(st, dt, cfg.N_m, T, bias.data_ptr(), b[i][0].data_ptr()), nsets)
    scratch = torch.empty(int(capi.nnt_tile_bias_grad_scratch(cfg.N_m, T)), device="cuda")
    db = torch.empty(cfg.N_m, device="cuda")
    report("bias_grad (column sums)", w, lambda i: capi.nnt_tile_bias_grad(st, dt, cfg.N_m, T, b[i][0].data_ptr(), db.data_ptr(), 0, scratch.data_ptr()), nsets)
    if cfg.dtype == "bf16":
        f32b = [torch.randn(n_el, device="cuda") for _ in range(nsets)]
        report("cast fp32 -> bf16", 6, lambda i: capi.nnt_tile_cast(st, capi.NNT_F32, capi.NNT_BF16, n_el, f32b[i].data_ptr(), b[i][0].data_ptr()), nsets)
        del f32b
    del b
    # Adam on an fp32 parameter set of the same size
    pa = [[torch.randn(n_el, device="cuda").abs() * 0.01 for _ in range(4)] for _ in range(nsets)]
    import workload
    a = workload.ADAM
    report("adam (fp32 p, g, m, v)", 28, lambda i: capi.nnt_tile_adam(st, n_el, 1, a["lr"], a["beta1"], a["beta2"], a["eps"], a["weight_decay"],
                                                                    pa[i][0].data_ptr(), pa[i][1].data_ptr(), pa[i][2].data_ptr(), pa[i][3].data_ptr(), None), nsets)
    report("sgd with momentum (fp32 p, g, v)", 20, lambda i: capi.nnt_tile_sgd(st, n_el, 0.05, 0.9, 0.0, 0, pa[i][1].data_ptr(), pa[i][0].data_ptr(),
                                                                                pa[i][2].data_ptr(), None), nsets)
    del pa
    return out


def gemm_ceiling(capi, torch):
    """What bounds the product kernels on the box at hand: the matrix-core issue rate on register
    operands (constants / values that change from instruction to instruction), and one large product
    per type through nnt_tile_gemm on operands of different content (the clock drops with the power the
    operands' bit toggling draws, so the same kernel runs at different rates on zeros and on noise)."""
    import ctypes as C
    st = torch.cuda.current_stream().cuda_stream
    sink = torch.zeros(1, device="cuda")

    def timed(call, iters=5):
        call()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            call()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    out = {"mfma_only": [], "products_8192_cubed": []}
    for dt, name in ((capi.NNT_F32, "f32"), (capi.NNT_BF16, "bf16")):
        for rnd in (0, 1):
            for occ in (1, 2):
                fl = C.c_double()
                wgs, iters = 256 * occ, 1 << 15
                ms = timed(lambda: capi.nnt_probe_mfma_rate(st, dt, rnd, iters, wgs, sink.data_ptr(), C.byref(fl)))
                out["mfma_only"].append({"dtype": name, "operands": "random" if rnd else "constant", "waves_per_simd": occ,
                                         "TFLOP/s": fl.value / ms / 1e9, "frac_mfma_peak": fl.value / ms / 1e9 / PEAK_TFLOPS[name]})
    m = n = k = 8192
    content = {"zeros": lambda t: t.zero_(), "ones": lambda t: t.fill_(1.0), "normal(0,1)": lambda t: t.normal_(),
               "normal(0,0.02)": lambda t: t.normal_(0.0, 0.02)}
    for dt, name, tdt in ((capi.NNT_F32, "f32", torch.float32), (capi.NNT_BF16, "bf16", torch.bfloat16)):
        A = torch.empty(m * k, device="cuda", dtype=tdt)
        B = torch.empty(k * n, device="cuda", dtype=tdt)
        Cm = torch.empty(m * n, device="cuda", dtype=tdt)
        for cname, fill in content.items():
            fill(A)
            fill(B)
            for opA, opB, on in ((1, 0, "TN"), (0, 0, "NN")):
                ms = timed(lambda: capi.nnt_tile_gemm(st, dt, dt, opA, opB, m, n, k, 1, 1.0, A.data_ptr(), k if opA else m, m * k,
                                                      B.data_ptr(), k, k * n, 0.0, Cm.data_ptr(), m, m * n))
                tf = 2.0 * m * n * k / ms / 1e9
                out["products_8192_cubed"].append({"dtype": name, "op": on, "operands": cname, "TFLOP/s": tf,
                                                   "frac_mfma_peak": tf / PEAK_TFLOPS[name]})
    return out


def measure(args, cfg, inp, attention, capi, tiled, torch, workload):
    """Times K steps of the block (forward + backward [+ Adam]) with the given attention flow and
    returns the bench record."""
    gran = capi.NNT_GRAN_OP if args.granularity == "op" else capi.NNT_GRAN_TILE
    ctx = tiled.Context(n_streams=args.streams, granularity=gran)
    nblk = max(1, args.blocks)
    tiles = workload.base_tiles(cfg)
    if args.batch_tile:
        tiles = dict(tiles, b=min(args.batch_tile, cfg.N_b))
    blks = [tiled.Gpt2Block(ctx, cfg.N_e, cfg.N_h, cfg.N_m, cfg.N_s, cfg.N_b, tiles, dtype=cfg.dtype,
                            eps=cfg.eps, gelu=cfg.gelu, adam=cfg.adam, fused_attention=attention == "fused") for _ in range(nblk)]
    for b in blks:
        b.set_params({k: inp[k] for k in workload.PARAM_NAMES})
    blk = blks[0]
    step_no = [0]
    if nblk == 1:
        X, dOut = blk.activation(inp["X"]), blk.activation(inp["dOut"])
        Out, dX = blk.activation(), blk.activation()

        def step():
            blk.forward(X, Out)
            blk.backward(dOut, dX)
            if cfg.adam:
                step_no[0] += 1
                blk.adam(step_no[0], **workload.ADAM)
    else:
        # a chain of identical blocks as one flow of tasks
        stack = tiled.Gpt2Stack(ctx, blks)
        stack.acts[0].upload(inp["X"])
        stack.dacts[nblk].upload(inp["dOut"])

        def step():
            stack.forward()
            stack.backward()
            if cfg.adam:
                step_no[0] += 1
                stack.adam(step_no[0], **workload.ADAM)

    for _ in range(max(args.warmup, 1)):
        step()
    ctx.wait()
    graph = None
    if args.graph:
        import ctypes as C
        graph = C.c_void_p()
        capi.nnt_capture_begin(ctx.h)
        step()
        capi.nnt_capture_end(ctx.h, C.byref(graph))
        capi.nnt_graph_launch(graph)
        ctx.wait()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        if graph is not None:
            capi.nnt_graph_launch(graph)
        else:
            step()
    dt_submit = time.perf_counter() - t0      # the host's share: all tasks handed to the streams, none waited for
    ctx.wait()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # Second timed pass of the same K steps for the per-kernel figures: one stream, every task
    # bracketed by HIP events on that stream, so that a kernel's duration is its own and not
    # shared with kernels that overlap it on other streams.
    ctx.set_serial(True)
    step()
    ctx.profile(True)
    for _ in range(args.steps):
        step()
    prof = ctx.profile_read()
    ctx.profile(False)
    ctx.set_serial(False)
    # what a pair of timing events reads with nothing between them (median of 50): every per-kernel duration of
    # the serial pass contains about this much marker time on top of launch gaps
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(50)]
    with torch.cuda.stream(ctx.streams[0]):
        for a, b in pairs:
            a.record()
            b.record()
    torch.cuda.synchronize()
    empty_pair_us = sorted(a.elapsed_time(b) for a, b in pairs)[25] * 1e3
    ms_per_step = dt / args.steps * 1e3
    flops = nblk * workload.model_flops(cfg, tile_skip=True, visible_only=attention == "fused")
    value = flops / (dt / args.steps) / 1e12

    # per-operation figures from the executor's event pairs
    kernels = {}
    for label, e in prof.items():
        if e["ms"] <= 0:
            continue
        rate = e["work"] / (e["ms"] * 1e-3)
        if e["unit"] == "flops":
            kernels[label] = {"ms_per_step": e["ms"] / args.steps, "launches_per_step": e["launches"] / args.steps,
                              "avg_launch_us": e["ms"] / max(e["launches"], 1) * 1e3,
                              "TFLOP/s": rate / 1e12, "frac_mfma_peak": rate / 1e12 / PEAK_TFLOPS[cfg.dtype]}
        else:
            kernels[label] = {"ms_per_step": e["ms"] / args.steps, "launches_per_step": e["launches"] / args.steps,
                              "avg_launch_us": e["ms"] / max(e["launches"], 1) * 1e3,
                              "GB/s": rate / 1e9, "frac_hbm_peak": rate / 1e9 / PEAK_HBM_GBS}
    roofline = None
    gemms = {k: v for k, v in kernels.items() if "TFLOP/s" in v}
    if gemms:
        dom = max(gemms, key=lambda k: gemms[k]["ms_per_step"])
        e = prof[dom]
        roofline = {"bound": "mfma", "kernel": dom, "achieved": gemms[dom]["TFLOP/s"], "peak": PEAK_TFLOPS[cfg.dtype],
                    "unit": "TFLOP/s", "frac": gemms[dom]["TFLOP/s"] / PEAK_TFLOPS[cfg.dtype], "traffic": None,
                    "avg_launch_us": gemms[dom]["avg_launch_us"], "launches": e["launches"],
                    "flops_per_launch": e["work"] / max(e["launches"], 1)}
        # HBM bytes per launch of that kernel, as measured by the committed rocprofv3 --pmc runs
        # (FETCH_SIZE and WRITE_SIZE scaled by a plain copy kernel); null when no such run is on file
        tpath = os.path.join(ROOT, "profiles", "hbm_traffic_C%d.txt" % args.config)
        if os.path.exists(tpath):
            for line in open(tpath):
                parts = line.rstrip("\n").split("\t")
                if len(parts) == 3 and parts[0] == dom.replace(" batched", ""):
                    roofline["traffic"] = float(parts[1]) + float(parts[2])      # HBM bytes per launch, read + written
                    roofline["traffic_detail"] = {"read_bytes_per_launch": float(parts[1]), "written_bytes_per_launch": float(parts[2]),
                                                  "source": "profiles/" + os.path.basename(tpath),
                                                  "note": "stored figure of the named rocprofv3 --pmc runs of this command "
                                                          "(hardware counters cannot be read from inside the run); not measured now"}
        wg = [v for k, v in gemms.items()]
        tot_ms = sum(v["ms_per_step"] for v in wg)
        tot_fl = sum(v["TFLOP/s"] * v["ms_per_step"] for v in wg)
        roofline["all_products_TFLOP/s"] = tot_fl / tot_ms if tot_ms else None

    # the metric's other two figures, as time-weighted aggregates of the serial per-kernel pass
    def aggregate(items, key, peak):
        ms = sum(v["ms_per_step"] for v in items)
        work = sum(v[key] * v["ms_per_step"] for v in items)
        return {"ms_per_step": ms, key: work / ms if ms else None, "frac_of_peak": work / ms / peak if ms else None}
    summary = {
        "tile_gemm_weights": aggregate([v for k, v in gemms.items() if "batched" not in k and not k.startswith("attention")],
                                       "TFLOP/s", PEAK_TFLOPS[cfg.dtype]),
        "tile_gemm_attention": aggregate([v for k, v in gemms.items() if "batched" in k or k.startswith("attention")],
                                         "TFLOP/s", PEAK_TFLOPS[cfg.dtype]),
        "memory_bound_kernels": aggregate([v for k, v in kernels.items() if "GB/s" in v], "GB/s", PEAK_HBM_GBS),
    }
    # time the step would take if every kernel ran at its roofline, over the measured step
    bound_ms = sum(v["ms_per_step"] * v.get("frac_mfma_peak", v.get("frac_hbm_peak", 0.0)) for v in kernels.values())
    summary["time_weighted_roofline"] = bound_ms / ms_per_step if ms_per_step else None

    out = {"metric": "GPT-2 block fwd+bwd TFLOP/s on 1 MI355X", "value": value, "unit": "TFLOP/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
           "host_submit_ms_per_step": dt_submit / args.steps * 1e3, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32" if cfg.dtype == "f32" else "bf16", "data": "synthetic",
           "config": {"workload": "%s: one GPT-2 block %s N_e=%d N_h=%d N_m=%d N_s=%d N_b=%d tile=%d, forward+backward%s, causal"
                                  % (cfg.name, cfg.dtype, cfg.N_e, cfg.N_h, cfg.N_m, cfg.N_s, cfg.N_b, cfg.tile,
                                     "+Adam" if cfg.adam else ""),
                      "streams": args.streams, "granularity": args.granularity, "batch_tile": tiles["b"], "graph_replay": bool(args.graph),
                      "attention": attention, "blocks": nblk,
                      "flops_per_step": flops,
                      "attention_flops": "visible (key, query) pairs only, no recomputation" if attention == "fused"
                                         else "computed sequence-tile pairs only"},
           # the metric's second and third figure (time-weighted over the serial per-kernel pass)
           "tile_gemm_pct_mfma_peak": 100.0 * (summary["tile_gemm_weights"]["frac_of_peak"] or 0.0),
           "elementwise_GBps": summary["memory_bound_kernels"]["GB/s"],
           "roofline": roofline, "summary": summary, "kernels": kernels, "executor": ctx.stats(),
           "empty_event_pair_us": empty_pair_us}
    if nblk > 1:
        stack.close()
    for b in blks:
        b.close()
    ctx.close()
    return out


def model_iteration(args, cfg, capi, tiled, torch, workload):
    """A whole training iteration of a GPT-2-shaped language model built from the block of `cfg`: token and
    position embeddings, `--blocks` blocks (12 when not given), final layer norm, tied head over a
    50304-item vocabulary, cross-entropy loss, backward, Adam on every parameter; one flow of tasks."""
    import numpy as np
    nblk = args.blocks if args.blocks > 1 else 12
    N_v, tile_v = 50304, 8192
    ctx = tiled.Context(n_streams=args.streams)
    inp = workload.generate(cfg)
    blks = [tiled.Gpt2Block(ctx, cfg.N_e, cfg.N_h, cfg.N_m, cfg.N_s, cfg.N_b, workload.base_tiles(cfg), dtype=cfg.dtype,
                            eps=cfg.eps, gelu=cfg.gelu, adam=True, fused_attention=args.attention == "fused") for _ in range(nblk)]
    for b in blks:
        b.set_params({k: inp[k] for k in workload.PARAM_NAMES})
    model = tiled.Gpt2Model(ctx, blks, N_v, tile_v)
    r = np.random.Generator(np.random.Philox(workload.SEED_BASE + 100 * cfg.index + 50))
    model.set_params(0.02 * r.standard_normal((cfg.N_e, N_v)), 0.01 * r.standard_normal((cfg.N_e, cfg.N_s)),
                     np.ones(cfg.N_e), np.zeros(cfg.N_e))
    tok = r.integers(0, N_v, (cfg.N_s, cfg.N_b))
    model.set_batch(tok, np.roll(tok, -1, axis=0))            # next-token labels of a random sequence
    step_no = [0]
    losses = []

    def step():
        step_no[0] += 1
        model.forward()
        model.backward()
        model.adam(step_no[0], **workload.ADAM)
    for _ in range(max(args.warmup, 1)):
        step()
        ctx.wait()
        losses.append(model.loss.item())
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    dt_submit = time.perf_counter() - t0
    ctx.wait()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    losses.append(model.loss.item())
    T = cfg.N_s * cfg.N_b
    head = 3.0 * 2.0 * N_v * T * cfg.N_e
    flops = nblk * workload.model_flops(cfg, tile_skip=True, visible_only=args.attention == "fused") + head
    sec = dt / args.steps
    per_block = 4 * cfg.N_e ** 2 + 2 * cfg.N_e * cfg.N_m + 9 * cfg.N_e + cfg.N_m
    nparams = nblk * per_block + cfg.N_e * (N_v + cfg.N_s) + 2 * cfg.N_e
    out = {"metric": "GPT-2 language-model training iteration on 1 MI355X", "value": flops / sec / 1e12, "unit": "TFLOP/s",
           "tokens_per_s": T / sec, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": sec * 1e3,
           "host_submit_ms_per_step": dt_submit / args.steps * 1e3, "higher_is_better": True, "vs_baseline": None,
           "dtype": "f32" if cfg.dtype == "f32" else "bf16", "data": "synthetic",
           "config": {"workload": "%d blocks of %s (N_e=%d N_h=%d N_m=%d N_s=%d N_b=%d tile=%d), vocabulary %d in tiles of %d, "
                                  "tied head, cross-entropy, forward+backward+Adam" % (nblk, cfg.name, cfg.N_e, cfg.N_h, cfg.N_m,
                                                                                       cfg.N_s, cfg.N_b, cfg.tile, N_v, tile_v),
                      "parameters": int(nparams), "streams": args.streams, "attention": args.attention, "flops_per_step": flops},
           "loss_per_token_warmup_steps": [l / T for l in losses[:-1]], "loss_per_token_after_timed_steps": losses[-1] / T,
           "executor": ctx.stats()}
    model.close()
    for b in blks:
        b.close()
    ctx.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="workload number 1..5 (default: the fp32 GPT-2-small-shaped block)")
    ap.add_argument("--streams", type=int, default=2)
    ap.add_argument("--granularity", choices=["op", "tile"], default="op")
    ap.add_argument("--batch-tile", type=int, default=0, metavar="N",
                    help="cut the batch axis every N members (default: whole; 1 with --granularity tile is the stress "
                         "case of the executor: every tile of every batch member a task of its own)")
    ap.add_argument("--graph", action="store_true", help="replay the step from a captured HIP graph")
    ap.add_argument("--blocks", type=int, default=1, help="chain this many identical blocks into one flow of tasks")
    ap.add_argument("--attention", choices=["tiles", "fused"], default="tiles",
                    help="tiles: scores, softmax and the product with V as three operations on the stored N_s x N_s "
                         "tensor (the paper's flow, the default); fused: one kernel per direction that never stores it")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-next-rows", action="store_true", help="skip the extra pass with the fused attention kernels")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="default run only: skip the bf16 configurations C3, C4 and C5 that are timed beside the headline")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark, copy MIB MiB of fp32 a few times with the library's cast kernel "
                         "(a plain copy kernel of known size, for scaling HBM counters)")
    ap.add_argument("--cpu-sample-batch", type=int, default=0)
    ap.add_argument("--tile-kernels", action="store_true",
                    help="instead of the block benchmark, time single calls of the tile kernels at the config's shapes: "
                         "products against the MFMA peak, memory-bound kernels against HBM, warm (one buffer set) and "
                         "cold (rotating over > 512 MB of buffer sets, more than the 256 MB Infinity Cache)")
    ap.add_argument("--gemm-ceiling", action="store_true",
                    help="instead of the block benchmark, measure the matrix-core issue rate on register operands (constant / "
                         "random) and one 8192^3 product per type on operands of different content")
    ap.add_argument("--model", action="store_true",
                    help="instead of the block benchmark, time whole training iterations of a language model made of "
                         "--blocks blocks (default 12) of the config: embeddings, blocks, final layer norm, tied head, loss, "
                         "backward, Adam")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (--gpus %d refused)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import workload
    from paper_2504_13236_amd import capi, tiled

    if not torch.cuda.is_available():
        print("bench.py needs a GPU: the HIP library is the only execution path", file=sys.stderr)
        sys.exit(3)
    if args.copy_calibration:
        n = args.copy_calibration * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        st = torch.cuda.current_stream().cuda_stream
        for _ in range(3):
            capi.nnt_tile_cast(st, capi.NNT_F32, capi.NNT_F32, n, src.data_ptr(), dst.data_ptr())
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            capi.nnt_tile_cast(st, capi.NNT_F32, capi.NNT_F32, n, src.data_ptr(), dst.data_ptr())
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 5
        print(json.dumps({"copy_calibration": {"bytes_read": 4 * n, "bytes_written": 4 * n, "launches": 8, "ms": ms,
                                               "GB/s": 8.0 * n / ms / 1e6,
                                               "kernel": "ew_kernel<CastF<float, float>>"}}))
        return
    if args.gemm_ceiling:
        print(json.dumps({"gemm_ceiling": gemm_ceiling(capi, torch)}))
        return
    if args.tile_kernels:
        res = tile_kernels(workload.CONFIGS[args.config], capi, torch)
        res["model_ops"] = model_ops(workload.CONFIGS[args.config], capi, tiled, torch)
        print(json.dumps({"tile_kernels": res}))
        return
    cfg = workload.CONFIGS[args.config]
    if args.model:
        print(json.dumps(model_iteration(args, cfg, capi, tiled, torch, workload)))
        return
    inp = workload.generate(cfg)
    out = measure(args, cfg, inp, args.attention, capi, tiled, torch, workload)
    if args.attention == "tiles" and cfg.h in (64, 128) and not args.no_next_rows and args.blocks == 1:
        # the first of the "next" rows beside the headline: the same block with the fused attention kernels
        f = measure(args, cfg, inp, "fused", capi, tiled, torch, workload)
        out["next_rows"] = {"fused_attention": {k: f[k] for k in ("value", "unit", "ms_per_step", "config", "summary")}}
        out["next_rows"]["fused_attention"]["kernels"] = {k: v for k, v in f["kernels"].items() if k.startswith("attention")}
    if args.config == 2 and args.blocks == 1 and args.granularity == "op" and not args.graph and not args.batch_tile and not args.no_other_configs:
        # the bf16 configurations beside the headline (same run, same launch configuration, fewer steps for the
        # largest one): the metric's second figure, tile-GEMM share of the MFMA peak, for bf16
        out["other_configs"] = {}
        for number in (3, 4, 5):
            ocfg = workload.CONFIGS[number]
            oargs = argparse.Namespace(**vars(args))
            oargs.config = number
            oargs.steps = args.steps if number < 5 else max(3, args.steps // 4)
            oargs.warmup = min(args.warmup, 2)
            oinp = workload.generate(ocfg)
            o = measure(oargs, ocfg, oinp, "tiles", capi, tiled, torch, workload)
            rec = {k: o[k] for k in ("value", "unit", "steps", "ms_per_step", "dtype", "config",
                                     "tile_gemm_pct_mfma_peak", "elementwise_GBps", "roofline", "summary")}
            # the same block with the fused attention kernels (a "next" row; flops credited for visible pairs only)
            f = measure(oargs, ocfg, oinp, "fused", capi, tiled, torch, workload)
            rec["fused_attention"] = {k: f[k] for k in ("value", "unit", "ms_per_step")}
            del oinp
            out["other_configs"][ocfg.name] = rec
            torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        # the whole workload takes the oracle a few seconds up to C4; C5 is sampled on one batch member
        sb = args.cpu_sample_batch or (cfg.N_b if args.config <= 4 else 1)
        out["cpu_baseline"] = cpu_baseline(cfg, sb)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
