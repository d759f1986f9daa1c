#!/usr/bin/env python3
"""Benchmark of the UBP sparse x dense product on one MI355X.

A step is one ubp_spmm call (the whole hot path: the packed weights times one batch of
synthetic activations) with all inputs already resident in HBM.  Steps rotate through
enough distinct (X, Y, packed W) buffer sets that more than twice the 256 MB Infinity
Cache is touched between two uses of a set ("cold"), so the time is an HBM time.  The K
timed steps are recorded once into a HIP graph and replayed, which removes the host's
launch cost from the measurement; HIP events on the launch stream bracket the replay.

Prints ONE JSON line: the headline workload (default c4) plus, under "per_config", the
same measurement for the other layers.  `value` counts flops on kept weights only
(2 * nb * bh * bw * N per step).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = 2500.0        # dense bf16 / fp16 MFMA, published
INFINITY_CACHE_BYTES = 256 << 20


def algorithmic_bytes(cfg, nb, N, y_bytes):
    """Bytes the method must move once per step: packed values + indptr + indices, X, Y."""
    esz = 4 if cfg.dtype == "f32" else 2
    w = nb * cfg.bh * cfg.bw * esz + (cfg.M - cfg.bh + 2) * 4 + nb * 4
    return w + cfg.K * N * esz + cfg.M * N * y_bytes


def measure(cfg_name, steps, warmup, y_dtype, plan_kw, use_graph, hot):
    import torch
    import paper_2407_19644_amd as ubp
    from synthetic import get_config, make_layer

    cfg = get_config(cfg_name)
    blocks, W, X = make_layer(cfg)
    nb = len(blocks)
    N = cfg.N
    y_dtype = y_dtype or cfg.dtype
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
    y_bytes = 4 if y_dtype == "f32" else 2
    abytes = algorithmic_bytes(cfg, nb, N, y_bytes)
    set_bytes = abytes
    nsets = 1 if hot else int(np.ceil(2.0 * INFINITY_CACHE_BYTES / set_bytes)) + 1
    nsets = max(1, min(nsets, 192))

    Xt = torch.from_numpy(X)
    if cfg.dtype == "bf16":
        Xt = Xt.view(torch.bfloat16)
    Xs, Ys, Ps = [], [], []
    for s in range(nsets):
        Xs.append(Xt.cuda() if s == 0 else Xs[0].clone())
        Ys.append(torch.empty((cfg.M, N), dtype=tdt[y_dtype], device="cuda"))
        Ps.append(ubp.pack(W, cfg.dtype, cfg.bh, cfg.bw, blocks, device=0))
    plan = None
    if plan_kw:
        plan = ubp.Plan()
        for k, v in plan_kw.items():
            setattr(plan, k, v)

    def step(i, stream):
        s = i % nsets
        ubp.spmm(Ps[s], Xs[s].data_ptr(), N, N, Ys[s].data_ptr(), N, y_dtype, stream, plan)

    stream = torch.cuda.Stream()          # default priority; every launch and event is on it
    with torch.cuda.stream(stream):
        sp = stream.cuda_stream
        for i in range(warmup):
            step(i, sp)
        stream.synchronize()
        graph = None
        if use_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for i in range(steps):
                    step(warmup + i, stream.cuda_stream)
            graph.replay()                # one untimed replay (graph upload)
            stream.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record(stream)
        if graph is not None:
            graph.replay()
        else:
            for i in range(steps):
                step(warmup + i, sp)
        e1.record(stream)
        stream.synchronize()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    ev_ms = e0.elapsed_time(e1)
    ms_per_step = wall * 1e3 / steps
    kernel_us = ev_ms * 1e3 / steps        # average launch duration inside the timed region
    flops = 2.0 * nb * cfg.bh * cfg.bw * N
    t_hbm = abytes / (HBM_PEAK_GBS * 1e9)
    t_mfma = flops / (MFMA_PEAK_TFLOPS * 1e12) if cfg.dtype != "f32" else 0.0
    res = {
        "workload": cfg.name, "what": cfg.what, "M": cfg.M, "K": cfg.K, "N": N, "block": "%dx%d" % (cfg.bh, cfg.bw),
        "density": cfg.density, "nb": nb, "in_dtype": cfg.dtype, "y_dtype": y_dtype,
        "gflops_kept": flops / (ms_per_step * 1e-3) / 1e9,
        "ms_per_step": ms_per_step, "kernel_us": kernel_us,
        "algorithmic_bytes": abytes, "achieved_GBs": abytes / (kernel_us * 1e-6) / 1e9,
        "hbm_frac": (abytes / (kernel_us * 1e-6) / 1e9) / HBM_PEAK_GBS,
        "t_roof_us": max(t_hbm, t_mfma) * 1e6, "cache": "hot" if hot else "cold", "buffer_sets": nsets,
        "graph": bool(use_graph),
    }
    for p in Ps:
        p.free()
    del Xs, Ys
    torch.cuda.empty_cache()
    return res, (cfg, blocks, W, X)


def cpu_baseline(cfg, blocks, W, X, budget_s=15.0):
    """The oracle as it stands (densify + naive double-precision loops, one thread) on a
    bounded sample of the same workload: the first R output rows, all columns."""
    import oracle
    from synthetic import decode_f64
    W64 = decode_f64(W, cfg.dtype)
    X64 = decode_f64(X, cfg.dtype)
    probe = min(4, cfg.M)
    t = time.perf_counter()
    oracle.spmm(W64, cfg.bh, cfg.bw, blocks, X64, rows=np.arange(probe))
    per_row = max((time.perf_counter() - t) / probe, 1e-6)
    R = int(max(probe, min(cfg.M, budget_s / per_row)))
    rows = np.arange(R)
    t = time.perf_counter()
    oracle.spmm(W64, cfg.bh, cfg.bw, blocks, X64, rows=rows)
    dt = time.perf_counter() - t
    Wd = oracle.densify(W64, cfg.bh, cfg.bw, blocks)
    kept = int(np.count_nonzero(Wd[:R]))
    return {"value": 2.0 * kept * cfg.N / dt / 1e9, "unit": "GFLOP/s (kept weights)", "cores": 1, "kind": "oracle",
            "sample": "first %d of %d output rows, all %d columns, %.1f s; dense work %.2f GFLOP/s"
                      % (R, cfg.M, cfg.N, dt, 2.0 * R * cfg.K * cfg.N / dt / 1e9)}


def kernel_name(cfg, pinned):
    """The kernel ubp_spmm runs for this layer (same rule as the library's), or the pinned one."""
    if cfg.dtype == "f32" or pinned == 1:
        return "wros_kernel"
    if pinned == 3:
        return "tile_kernel"
    if pinned == 4 or (pinned == 0 and cfg.K <= 256 and cfg.N % 8 == 0):
        return "xstat_kernel"
    tiles_mb = ((cfg.M + 15) // 16) * 8 * ((cfg.K + 255) // 256) / 1024.0   # zero-filled W as operand tiles
    if pinned == 5 or (pinned == 0 and cfg.N % 8 == 0 and tiles_mb <= 8 and cfg.density >= 0.2):
        return "xchunk_kernel"
    return "stripe_kernel"


def load_traffic(workload, y_dtype):
    """HBM bytes per launch from the committed rocprofv3 --pmc summaries, if present."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            t = json.load(f)
        return t.get("%s/%s" % (workload, y_dtype))
    except (OSError, ValueError):
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="c4", help="headline workload (c0..c4)")
    ap.add_argument("--y-dtype", default=None, help="f32, or the layer's input dtype (default)")
    ap.add_argument("--only", action="store_true", help="skip the per_config table of the other layers")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-graph", action="store_true", help="launch step by step instead of replaying a HIP graph")
    ap.add_argument("--hot", action="store_true", help="reuse one buffer set (cache-resident timing)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain elementwise kernel over 256 MiB 3 times (reads 256 MiB, writes 256 MiB: "
                         "known traffic, to scale rocprofv3 byte counters)")
    ap.add_argument("--kernel", type=int, default=0)
    ap.add_argument("--G", type=int, default=0)
    ap.add_argument("--CT", type=int, default=0)
    ap.add_argument("--waves", type=int, default=0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the product path has no multi-GPU part); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    import paper_2407_19644_amd as ubp
    ubp.load_library()                      # fails loudly if the native library is missing
    plan_kw = {k: v for k, v in (("kernel", args.kernel), ("sub_stripes", args.G), ("col_tiles", args.CT),
                                 ("waves", args.waves)) if v}
    use_graph = not args.no_graph
    if args.copy_calibration:
        src = torch.empty(128 << 20, dtype=torch.bfloat16, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    head, data = measure(args.config, args.steps, args.warmup, args.y_dtype, plan_kw, use_graph, args.hot)
    per = {}
    if not args.only:
        for name in ("c1", "c2", "c3", "c4"):
            for yd in (None, "f32"):
                if name == args.config and (yd or None) == (args.y_dtype or None):
                    r = head
                else:
                    r, _ = measure(name, args.steps, args.warmup, yd, plan_kw, use_graph, args.hot)
                per["%s/y_%s" % (name, r["y_dtype"])] = {k: r[k] for k in (
                    "gflops_kept", "kernel_us", "achieved_GBs", "hbm_frac", "t_roof_us", "algorithmic_bytes")}
    cfg = data[0]
    out = {
        "metric": "UBP SpMM effective GFLOP/s (kept-weight FLOPs) + % of HBM/MFMA roofline",
        "value": head["gflops_kept"], "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype,          # multiplications in this type on the matrix cores, sums in f32
        "data": "synthetic",
        "config": {k: head[k] for k in ("workload", "what", "M", "K", "N", "block", "density", "nb", "in_dtype",
                                        "y_dtype", "cache", "buffer_sets", "graph")},
        "roofline": {"bound": "hbm", "achieved": head["achieved_GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": head["hbm_frac"], "traffic": load_traffic(head["workload"], head["y_dtype"]),
                     "kernel": kernel_name(cfg, args.kernel),
                     "kernel_us": head["kernel_us"], "algorithmic_bytes": head["algorithmic_bytes"],
                     "t_roof_us": head["t_roof_us"]},
    }
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(*data)
    if per:
        out["per_config"] = per
    print(json.dumps(out))


if __name__ == "__main__":
    main()
