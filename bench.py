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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="workload number 1..5 (default: the fp32 GPT-2-small-shaped block)")
    ap.add_argument("--streams", type=int, default=4)
    ap.add_argument("--granularity", choices=["op", "tile"], default="op")
    ap.add_argument("--graph", action="store_true", help="replay the step from a captured HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark, copy MIB MiB of fp32 a few times with the library's cast kernel "
                         "(a plain copy kernel of known size, for scaling HBM counters)")
    ap.add_argument("--cpu-sample-batch", type=int, default=0)
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
    cfg = workload.CONFIGS[args.config]
    inp = workload.generate(cfg)
    gran = capi.NNT_GRAN_OP if args.granularity == "op" else capi.NNT_GRAN_TILE
    ctx = tiled.Context(n_streams=args.streams, granularity=gran)
    blk = tiled.Gpt2Block(ctx, cfg.N_e, cfg.N_h, cfg.N_m, cfg.N_s, cfg.N_b, workload.base_tiles(cfg), dtype=cfg.dtype,
                          eps=cfg.eps, gelu=cfg.gelu, adam=cfg.adam)
    blk.set_params({k: inp[k] for k in workload.PARAM_NAMES})
    X, dOut = blk.activation(inp["X"]), blk.activation(inp["dOut"])
    Out, dX = blk.activation(), blk.activation()
    step_no = [0]

    def step():
        blk.forward(X, Out)
        blk.backward(dOut, dX)
        if cfg.adam:
            step_no[0] += 1
            blk.adam(step_no[0], **workload.ADAM)

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
    ms_per_step = dt / args.steps * 1e3
    flops = workload.model_flops(cfg, tile_skip=True)
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
                    roofline["traffic"] = {"read_bytes_per_launch": float(parts[1]), "written_bytes_per_launch": float(parts[2]),
                                           "source": "profiles/" + os.path.basename(tpath)}
        wg = [v for k, v in gemms.items()]
        tot_ms = sum(v["ms_per_step"] for v in wg)
        tot_fl = sum(v["TFLOP/s"] * v["ms_per_step"] for v in wg)
        roofline["all_products_TFLOP/s"] = tot_fl / tot_ms if tot_ms else None

    out = {"metric": "GPT-2 block fwd+bwd TFLOP/s on 1 MI355X", "value": value, "unit": "TFLOP/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32" if cfg.dtype == "f32" else "bf16", "data": "synthetic",
           "config": {"workload": "%s: one GPT-2 block %s N_e=%d N_h=%d N_m=%d N_s=%d N_b=%d tile=%d, forward+backward%s, causal"
                                  % (cfg.name, cfg.dtype, cfg.N_e, cfg.N_h, cfg.N_m, cfg.N_s, cfg.N_b, cfg.tile,
                                     "+Adam" if cfg.adam else ""),
                      "streams": args.streams, "granularity": args.granularity, "graph_replay": bool(args.graph),
                      "flops_per_step": flops, "attention_flops": "computed sequence-tile pairs only"},
           "roofline": roofline, "kernels": kernels, "executor": ctx.stats()}
    if not args.no_cpu_baseline:
        # the whole workload takes the oracle a few seconds up to C4; C5 is sampled on one batch member
        sb = args.cpu_sample_batch or (cfg.N_b if args.config <= 4 else 1)
        out["cpu_baseline"] = cpu_baseline(cfg, sb)
    blk.close()
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
