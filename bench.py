#!/usr/bin/env python3
"""Benchmark of the UBP sparse x dense product on one MI355X.

A step is one ubp_spmm call (the whole hot path: the packed weights times one batch of
synthetic activations) with all inputs already resident in HBM.  Steps rotate through
enough distinct (X, Y, packed W) buffer sets that more than twice the 256 MB Infinity
Cache is touched between two uses of a set ("cold"), so the time is an HBM time.  The K
timed steps are recorded once into a HIP graph, which removes the host's launch cost from
the measurement; the graph is replayed until at least 50 ms have been timed (the first
milliseconds of a burst run at a lower clock), HIP events on the launch stream bracket every
replay, and the per-launch kernel time is the median replay divided by K.

After timing, every handle's error flags are read and the last Y of the headline layer is
compared with the CPU oracle on a sample of rows: a kernel that produced wrong numbers makes
the run fail instead of being reported.

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
MIN_TIMED_MS = 50.0
KERNEL_NAMES = {1: "wros_kernel", 2: "stripe_kernel", 3: "naive_kernel", 4: "xstat_kernel", 5: "xchunk_kernel", 6: "blk_kernel",
                7: "gemm_kernel"}


def algorithmic_bytes(cfg, nb, N, y_bytes):
    """Bytes the method must move once per step: packed values + indptr + indices, X, Y."""
    esz = 4 if cfg.dtype == "f32" else 2
    w = nb * cfg.bh * cfg.bw * esz + (cfg.M - cfg.bh + 2) * 4 + nb * 4
    return w + cfg.K * N * esz + cfg.M * N * y_bytes


PROFILING = False      # --profile: one replay per measurement, no launch-floor / copy-bandwidth legs


def timed_replays(run_once, stream, est_ms):
    """Replays until MIN_TIMED_MS are covered.  Returns (wall seconds of all replays, list of
    per-replay event milliseconds)."""
    import torch
    reps = 1 if PROFILING else int(min(2000, max(3, np.ceil(MIN_TIMED_MS / max(est_ms, 1e-3)))))
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for e0, e1 in ev:
        e0.record(stream)
        run_once()
        e1.record(stream)
    stream.synchronize()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, [e0.elapsed_time(e1) for e0, e1 in ev]


def measure(cfg, layer, steps, warmup, y_dtype, plan_kw, use_graph, hot, verify_rows=0, fused=False):
    import torch
    import paper_2407_19644_amd as ubp

    blocks, W, X = layer
    nb = len(blocks)
    N = X.shape[1]
    y_dtype = y_dtype or cfg.dtype
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
    y_bytes = 4 if y_dtype == "f32" else 2
    abytes = algorithmic_bytes(cfg, nb, N, y_bytes)
    want_sets = int(np.ceil(2.0 * INFINITY_CACHE_BYTES / abytes)) + 1
    nsets = 1 if hot else max(1, min(want_sets, steps, 192))   # a set no step touches would only cost memory
    cold = (not hot) and nsets >= want_sets

    Xt = torch.from_numpy(X)
    if cfg.dtype == "bf16":
        Xt = Xt.view(torch.bfloat16)
    Xs, Ys, Ps = [], [], []
    for s in range(nsets):
        Xs.append(Xt.cuda() if s == 0 else Xs[0].clone())
        Ys.append(torch.full((cfg.M, N), float("nan"), dtype=tdt[y_dtype], device="cuda"))
        Ps.append(ubp.pack(W, cfg.dtype, cfg.bh, cfg.bw, blocks, device=0))
    plan = None
    if plan_kw:
        plan = ubp.Plan()
        for k, v in plan_kw.items():
            setattr(plan, k, v)
    # everything a first call would allocate or build is done here, outside any timing or capture
    for s in range(nsets):
        chosen = ubp.spmm_prepare(Ps[s], Xs[s].data_ptr(), N, N, Ys[s].data_ptr(), N, y_dtype, plan)

    bias = None
    if fused:                              # bias per output row + ReLU, fused into the stores
        bias = (np.random.default_rng(5).standard_normal(cfg.M) * 0.1).astype(np.float32)
        bias_d = torch.from_numpy(bias).cuda()

    def step(i, stream):
        s = i % nsets
        if fused:
            ubp.spmm_fused(Ps[s], Xs[s].data_ptr(), N, N, Ys[s].data_ptr(), N, y_dtype, bias_d.data_ptr(), "relu", 0.0, 0.0,
                           stream, plan)
        else:
            ubp.spmm(Ps[s], Xs[s].data_ptr(), N, N, Ys[s].data_ptr(), N, y_dtype, stream, plan)

    stream = torch.cuda.Stream()          # default priority; every launch and event is on it
    with torch.cuda.stream(stream):
        sp = stream.cuda_stream
        for i in range(warmup):
            step(i, sp)
        stream.synchronize()
        if use_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for i in range(steps):
                    step(warmup + i, stream.cuda_stream)
            run_once = graph.replay
        else:
            def run_once():
                for i in range(steps):
                    step(warmup + i, sp)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        run_once()                        # one untimed replay (graph upload) that also sizes the timed region
        e1.record(stream)
        stream.synchronize()
        wall, ev_ms = timed_replays(run_once, stream, e0.elapsed_time(e1))
    reps = len(ev_ms)
    ms_per_step = wall * 1e3 / (reps * steps)
    kernel_us = float(np.median(ev_ms)) * 1e3 / steps      # per launch, median replay
    flops = 2.0 * nb * cfg.bh * cfg.bw * N
    t_hbm = abytes / (HBM_PEAK_GBS * 1e9)
    t_mfma = flops / (MFMA_PEAK_TFLOPS * 1e12) if cfg.dtype != "f32" else 0.0

    flags = [p.device_error() for p in Ps]
    if any(flags):
        raise RuntimeError("%s: a bounded wait inside a kernel ran out (flags %s): the timing is void" % (cfg.name, flags))
    checked = 0
    if verify_rows:
        checked = verify(cfg, layer, Ys[(warmup + steps - 1) % nsets], y_dtype, verify_rows, bias)

    issued = {2: 100 + ubp.layout_slot(chosen.sub_stripes, chosen.col_tiles) if chosen.kernel == 2 else -1,
              4: 10, 5: 10, 6: 300 + {2: 0, 4: 1, 5: 2}.get(chosen.sub_stripes, 1)}.get(chosen.kernel, -1)
    res = {
        "workload": cfg.name, "what": cfg.what, "M": cfg.M, "K": cfg.K, "N": N, "block": "%dx%d" % (cfg.bh, cfg.bw),
        "density": cfg.density, "nb": nb, "in_dtype": cfg.dtype, "y_dtype": y_dtype,
        "gflops_kept": flops / (ms_per_step * 1e-3) / 1e9,
        "ms_per_step": ms_per_step, "kernel_us": kernel_us, "kernel_us_min": float(min(ev_ms)) * 1e3 / steps,
        "algorithmic_bytes": abytes, "achieved_GBs": abytes / (kernel_us * 1e-6) / 1e9,
        "hbm_frac": (abytes / (kernel_us * 1e-6) / 1e9) / HBM_PEAK_GBS,
        "t_roof_us": max(t_hbm, t_mfma) * 1e6, "cache": "cold" if cold else ("hot" if hot else "warm"), "buffer_sets": nsets,
        "graph": bool(use_graph), "replays": reps,
        "kernel": KERNEL_NAMES.get(chosen.kernel, "?"),
        "shape": {"sub_stripes": chosen.sub_stripes, "col_tiles": chosen.col_tiles, "waves": chosen.waves,
                  "producers": chosen.producers, "wg_rows": chosen.wg_rows},
        "mfma_needed": Ps[0].info(9) if cfg.dtype != "f32" else None,
        "mfma_issued": Ps[0].info(issued) if issued >= 0 else None,
        "device_bytes_per_handle": Ps[0].info(8), "canonical_bytes": Ps[0].info(7),
        "rows_checked_against_oracle": checked,
    }
    for p in Ps:
        p.free()
    del Xs, Ys
    torch.cuda.empty_cache()
    return res


def verify(cfg, layer, Yt, y_dtype, nrows, bias=None):
    """Rows of the timed run's last Y against the oracle (first, last, stripe borders and a seeded
    draw); raises on a mismatch.  Tolerances as in the parity tests."""
    import torch
    import oracle
    from synthetic import decode_f64
    blocks, W, X = layer
    rng = np.random.default_rng(7)
    rows = sorted(set([0, 15, 16, cfg.M - 16, cfg.M - 1]) | set(int(r) for r in rng.integers(0, cfg.M, size=max(0, nrows - 5))))
    Yref = oracle.spmm(decode_f64(W, cfg.dtype), cfg.bh, cfg.bw, blocks, decode_f64(X, cfg.dtype), rows=rows)
    if bias is not None:
        Yref = oracle.fused(Yref, bias.astype(np.float64), "relu", rows=rows)
    t = Yt[torch.tensor(rows, device=Yt.device)].detach().cpu()
    Y = decode_f64(t.view(torch.uint16).numpy(), "bf16") if y_dtype == "bf16" else t.numpy().astype(np.float64)
    if not np.isfinite(Y).all():
        raise RuntimeError("%s: Y holds NaN/Inf after the timed run" % cfg.name)
    scale = np.abs(Yref).max()
    err = np.abs(Y - Yref)
    if cfg.dtype == "f32":
        ok = err.max() <= 1e-5 * scale
    elif y_dtype == "f32":
        ok = err.max() <= 2e-3 * scale
    else:
        mant, emin = (10, -24) if y_dtype == "f16" else (7, -133)
        a = np.maximum(np.abs(Yref), 2.0 ** (emin + mant))
        half_ulp = 0.5 * np.maximum(2.0 ** (np.floor(np.log2(a)) - mant), 2.0 ** emin)
        ok = bool((err <= 1.01 * half_ulp + 1e-4 * scale).all())
    if not ok:
        raise RuntimeError("%s: the timed run's Y does not match the oracle (max err %.3e, max |Y| %.3e)" % (cfg.name, err.max(), scale))
    return len(rows)


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


def launch_floor_us():
    """Per-launch time of an empty kernel, graph-replayed like the layers: what no layer can beat."""
    import torch
    import paper_2407_19644_amd as ubp
    stream = torch.cuda.Stream()
    n = 200
    with torch.cuda.stream(stream):
        for _ in range(10):
            ubp.launch_floor(stream.cuda_stream)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for _ in range(n):
                ubp.launch_floor(stream.cuda_stream)
        graph.replay()
        stream.synchronize()
        _, ev = timed_replays(graph.replay, stream, 1.0)
    return float(np.median(ev)) * 1e3 / n


def copy_bandwidth_GBs():
    """Bytes read plus bytes written per second of a plain device copy, on rotating buffers larger
    than the Infinity Cache: what a kernel with no arithmetic gets out of this box's memory."""
    import torch
    stream = torch.cuda.Stream()
    n = 256 << 20
    bufs = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(4)]
    with torch.cuda.stream(stream):
        for b in bufs:
            b.zero_()
        stream.synchronize()

        def once():
            for i in range(4):
                bufs[(i + 1) % 4].copy_(bufs[i])
        once()
        stream.synchronize()
        _, ev = timed_replays(once, stream, 1.0)
    return 4 * 2.0 * n / (float(np.median(ev)) * 1e-3) / 1e9


def load_traffic(workload, y_dtype):
    """HBM bytes per launch from the committed rocprofv3 --pmc summaries (profiles/traffic.json), if present."""
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
    ap.add_argument("--config", default="c4", help="headline workload (a name from synthetic/configs.py)")
    ap.add_argument("--y-dtype", default=None, help="f32, or the layer's input dtype (default)")
    ap.add_argument("--only", action="store_true", help="skip the per_config table of the other layers")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-graph", action="store_true", help="launch step by step instead of replaying a HIP graph")
    ap.add_argument("--hot", action="store_true", help="reuse one buffer set (cache-resident timing)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain elementwise kernel over 256 MiB 3 times (reads 256 MiB, writes 256 MiB: "
                         "known traffic, to scale rocprofv3 byte counters)")
    ap.add_argument("--profile", action="store_true",
                    help="for runs under rocprofv3, where every dispatch is slow: one replay per measurement and no "
                         "launch-floor / copy-bandwidth legs (their fields are null)")
    ap.add_argument("--kernel", type=int, default=0)
    ap.add_argument("--G", type=int, default=0)
    ap.add_argument("--CT", type=int, default=0)
    ap.add_argument("--waves", type=int, default=0)
    args = ap.parse_args()
    global PROFILING
    PROFILING = args.profile
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the product path has no multi-GPU part); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    import paper_2407_19644_amd as ubp
    from synthetic import CONFIGS, EXTRA_CONFIGS, aligned_twin, get_config, make_layer
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
    cfg = get_config(args.config)
    layer = make_layer(cfg)
    head = measure(cfg, layer, args.steps, args.warmup, args.y_dtype, plan_kw, use_graph, args.hot, verify_rows=32)
    per = {}
    keys = ("gflops_kept", "kernel_us", "achieved_GBs", "hbm_frac", "t_roof_us", "algorithmic_bytes", "kernel", "cache",
            "mfma_needed", "mfma_issued")
    if not args.only:
        for c in CONFIGS[1:]:
            for yd in (None, "f32"):
                if c.name == cfg.name and (yd or None) == (args.y_dtype or None):
                    r = head
                else:
                    lay = layer if c.name == cfg.name else make_layer(c)
                    want = int(np.ceil(2.0 * INFINITY_CACHE_BYTES / algorithmic_bytes(c, len(lay[0]), c.N, 4 if yd else 2))) + 1
                    # (small layers: enough steps per replay to rotate through a cold number of sets)
                    r = measure(c, lay, max(args.steps, min(want, 192)), args.warmup, yd, plan_kw, use_graph, args.hot,
                                verify_rows=8)
                per["%s/y_%s" % (c.name, r["y_dtype"])] = {k: r[k] for k in keys}
        # the paper's own block shapes (N x 1 and N x (h w)) on MobileNetV1-shaped layers: unaligned
        # (UBP) beside the same number of blocks at aligned origins (ABP), as in the paper's Fig. 6
        for c in EXTRA_CONFIGS:
            lay = make_layer(c)
            want = int(np.ceil(2.0 * INFINITY_CACHE_BYTES / algorithmic_bytes(c, len(lay[0]), c.N, 2))) + 1
            st = max(args.steps, min(want, 192))
            r = measure(c, lay, st, args.warmup, None, plan_kw, use_graph, args.hot, verify_rows=8)
            ca = aligned_twin(c)
            ra = measure(ca, make_layer(ca), st, args.warmup, None, plan_kw, use_graph, args.hot, verify_rows=8)
            e = {k: r[k] for k in keys}
            e.update({"abp_kernel_us": ra["kernel_us"], "abp_kernel": ra["kernel"], "ubp_over_abp": r["kernel_us"] / ra["kernel_us"],
                      "block": r["block"], "density": c.density})
            per["%s/y_%s" % (c.name, r["y_dtype"])] = e
            # the vector kernel's two dataflows on the same layer (Section 5.2): weights rotated and
            # outputs stationary, on unaligned and on aligned origins, against the register-shifting one
            if c.bw == 1:
                vw = measure(c, lay, st, args.warmup, None, {"kernel": 1}, use_graph, args.hot, verify_rows=8)
                va = measure(ca, make_layer(ca), st, args.warmup, None, {"kernel": 1}, use_graph, args.hot, verify_rows=8)
                vn = measure(c, lay, st, args.warmup, None, {"kernel": 3}, use_graph, args.hot, verify_rows=8)
                e["vector_dataflows_us"] = {"ubp_wros": vw["kernel_us"], "abp": va["kernel_us"], "ubp_naive": vn["kernel_us"],
                                            "wros_over_abp": vw["kernel_us"] / va["kernel_us"],
                                            "naive_over_wros": vn["kernel_us"] / vw["kernel_us"]}
    out = {
        "metric": "UBP SpMM effective GFLOP/s (kept-weight FLOPs) + % of HBM/MFMA roofline",
        "value": head["gflops_kept"], "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype,          # multiplications in this type on the matrix cores, sums in f32
        "data": "synthetic",
        "config": {k: head[k] for k in ("workload", "what", "M", "K", "N", "block", "density", "nb", "in_dtype",
                                        "y_dtype", "cache", "buffer_sets", "graph", "replays", "shape",
                                        "rows_checked_against_oracle", "device_bytes_per_handle", "canonical_bytes")},
        "roofline": {"bound": "hbm", "achieved": head["achieved_GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": head["hbm_frac"], "traffic": load_traffic(head["workload"], head["y_dtype"]),
                     "traffic_source": "profiles/traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a copy kernel)",
                     "kernel": head["kernel"],
                     "kernel_us": head["kernel_us"], "kernel_us_min": head["kernel_us_min"],
                     "algorithmic_bytes": head["algorithmic_bytes"], "t_roof_us": head["t_roof_us"],
                     "mfma_needed": head["mfma_needed"], "mfma_issued": head["mfma_issued"],
                     "launch_floor_us": None if PROFILING else launch_floor_us(),
                     "copy_GBs": None if PROFILING else copy_bandwidth_GBs()},
    }
    if not args.only:
        fe = measure(cfg, layer, args.steps, args.warmup, args.y_dtype, plan_kw, use_graph, args.hot, verify_rows=8, fused=True)
        out["fused_epilogue"] = {"what": "ubp_spmm_fused on the headline layer: bias per output row + ReLU in the stores",
                                 "kernel_us": fe["kernel_us"], "over_plain": fe["kernel_us"] / head["kernel_us"]}
    out["roofline"]["frac_of_copy"] = None if PROFILING else head["achieved_GBs"] / out["roofline"]["copy_GBs"]
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(cfg, *layer)
    if per:
        out["per_config"] = per
    print(json.dumps(out))


if __name__ == "__main__":
    main()
