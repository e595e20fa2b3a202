#!/usr/bin/env python3
"""Benchmark of the STWQ + GPS quantized linear hot path on one MI355X.

A step is one pass of the online path (activation quantize -> int8 MFMA linear with the
dequantizing epilogue) over the four linears of a VAR-d16-shaped transformer block at W8A8:
batch 32 (16 x 2 for classifier-free guidance) x 680 token positions = 21760 rows,
qkv 1024->3072, proj 1024->1024, fc1 1024->4096, fc2 4096->1024.  Inputs are seeded synthetic
tensors (workloads.py), calibrated through the library's own offline calls (statistics, GPS scale,
fold, per-position parameters) before timing; every timed input is resident in HBM.

Prints ONE JSON line.  `value` is int8 tera-operations per second over whole steps
(2 M K N per linear; quantize time included).  `roofline` is for the dominant kernel, the prefill
linear, timed with HIP events on the launch stream inside the timed region.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5033.0     # 256 CUs x 4 SIMDs x 1024 MAC/clk x 2 x 2.4 GHz (dense)
HBM_PEAK_GBS = 8000.0


def recorded_traffic(key: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this same command (FETCH_SIZE and
    WRITE_SIZE runs, scaled by the reference copy); None when the summary is absent."""
    path = os.path.join(ROOT, "profiles", "bench_hbm_traffic_pmc.md")
    try:
        for line in open(path):
            if line.startswith(key + ":"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def calibrate_block(specs, device):
    """Offline stage for every linear of the block, all through the library."""
    import torch
    import workloads as wl
    from paper_2601_21238_amd.layer import StwqLinear

    layers = []
    for spec in specs:
        t0 = time.time()
        w, b = wl.make_weights(spec)
        layer = StwqLinear(spec.N, spec.K, spec.L, spec.a_bits, spec.w_bits, device)
        wd = torch.from_numpy(w).to(device)
        bd = torch.from_numpy(b).to(device)
        if spec.gps:
            xc = torch.from_numpy(wl.make_calibration(spec)).to(device)
            s = layer.solve_scale(xc, wd)
            layer.fold(wd, s, bd)
            layer.accumulate_position_stats(xc)
            del xc
        else:
            layer.fold(wd, None, bd)
            for chunk in wl.activation_chunks(spec, spec.n_calib, wl.ROLE_CALIB):
                layer.accumulate_position_stats(torch.from_numpy(chunk).to(device))
        layer.finalize()
        layers.append(layer)
        log(f"calibrated {spec.name} {spec.K}->{spec.N} in {time.time() - t0:.1f} s")
    return layers


def time_launches(fn, n_warm, n_iter, batch=1):
    """Median and mean duration (seconds) of fn() measured with events on the current stream.  With batch > 1 each
    event pair brackets `batch` back-to-back calls and the time is per call: for kernels of a few microseconds, whose
    single launches would be timed with the event's own cost and the host's launch path on top."""
    import torch
    for _ in range(n_warm):
        fn()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_iter)]
    for a, b in evs:
        a.record()
        for _ in range(batch):
            fn()
        b.record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) * 1e-3 / batch for a, b in evs)
    return ts[len(ts) // 2], sum(ts) / len(ts)


def decode_step(device, n_iter=30, rowmajor_too=False):
    """Configuration 4: one RAR-XXL-shaped decode step, 24 layers x (qkv, fc1, fc2), M = 128 rows at one token
    position per layer, 432.5 MB of distinct int8 weights streamed once per step by ONE grouped launch.  The
    weights are in the panel layout (repacked once, with the fold); with rowmajor_too the row-major launch is timed
    beside it (off by default: both run the same kernel, and a profile of the default run should hold one kind)."""
    import torch
    import workloads as wl
    import paper_2601_21238_amd as P
    from paper_2601_21238_amd.layer import StwqLinear

    specs = wl.config_linears(4)
    t0 = time.time()
    problems, keep, qproblems = [], [], []
    for spec in specs:
        w, b = wl.make_weights(spec)
        layer = StwqLinear(spec.N, spec.K, spec.L, spec.a_bits, spec.w_bits, device)
        wd, bd = torch.from_numpy(w).to(device), torch.from_numpy(b).to(device)
        xc = torch.from_numpy(wl.make_calibration(spec)).to(device)
        s = layer.solve_scale(xc, wd) if spec.gps else None
        layer.calibrate(xc, wd, s, bd)
        pos = wl.decode_position(spec)
        x = torch.from_numpy(wl.make_test_input(spec)).to(device)
        q = layer.quantize(x, t0=pos)
        y = torch.empty((spec.M, spec.N), dtype=torch.bfloat16, device=device)
        problems.append(dict(q=q, wq=layer.wq, dw=layer.dw, wsum=layer.wsum, delta=layer.delta[pos:pos + 1],
                             zp=layer.zp[pos:pos + 1], a_bits=spec.a_bits, bias=layer.bias, y=y, L=1))
        qproblems.append(dict(x=x, L=1, inv_s=layer.inv_s, inv_delta=layer.inv_delta[pos:pos + 1], zp=layer.zp[pos:pos + 1],
                              a_bits=spec.a_bits, q=q))
        keep.append((layer, x, pos))
        del wd, xc
    torch.cuda.synchronize()
    log(f"decode step: 72 linears calibrated in {time.time() - t0:.1f} s")
    rmed = None
    if rowmajor_too:
        rowmajor_group = P.LinearGroup(problems)
        rmed, _ = time_launches(rowmajor_group.run, 5, n_iter)
    packed_problems = []
    for spec, pr in zip(specs, problems):
        packed = torch.empty(P.stwq_packed_weight_bytes(spec.N, spec.K), dtype=torch.int8, device=device)
        P.stwq_pack_weights(pr["wq"], packed)
        packed_problems.append(dict(pr, wq=packed, N=spec.N, w_layout=P.LAYOUT_PANEL32))
    group = P.LinearGroup(packed_problems)
    med, mean = time_launches(group.run, 5, n_iter)
    w_bytes = float(sum(s.N * s.K for s in specs))
    all_bytes = float(sum(s.N * s.K + s.M * s.K + 2 * s.M * s.N + 12 * s.N + 8 for s in specs))
    ops = float(sum(2.0 * s.M * s.K * s.N for s in specs))

    def quantize_all():
        for (layer, x, pos), pr in zip(keep, problems):
            layer.quantize(x, pr["q"], t0=pos)
    qmed, _ = time_launches(quantize_all, 3, 10)
    qgroup = P.QuantizeGroup(qproblems)
    qgmed, _ = time_launches(qgroup.run, 3, n_iter)

    def whole_step():
        qgroup.run()
        group.run()
    smed, _ = time_launches(whole_step, 3, n_iter)
    graph = torch.cuda.CUDAGraph()                 # the same two launches as one HIP graph
    with torch.cuda.graph(graph):
        whole_step()
    gmed, _ = time_launches(graph.replay, 3, n_iter)
    q_bytes = float(sum(5.0 * s.M * s.K for s in specs))
    return {"workload": "config 4: RAR-XXL-shaped decode step, 72 linears, M = 128, one grouped launch",
            "us": med * 1e6, "gbs": all_bytes / med / 1e9, "weight_gbs": w_bytes / med / 1e9,
            "frac_hbm_peak": all_bytes / med / 1e9 / HBM_PEAK_GBS, "tops": ops / med / 1e12,
            "roofline": {"bound": "hbm", "achieved": all_bytes / mean / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": all_bytes / mean / 1e9 / HBM_PEAK_GBS,
                         "traffic": recorded_traffic("decode_linear_traffic_bytes_per_launch"),
                         "kernel": "stwq::linear_stream_kernel", "avg_launch_us": mean * 1e6},
            "rowmajor_weights_us": None if rmed is None else rmed * 1e6,
            "quantize_72_launches_us": qmed * 1e6, "quantize_grouped_us": qgmed * 1e6,
            "step_us": smed * 1e6, "step_graph_replay_us": gmed * 1e6, "step_gbs": (all_bytes + q_bytes) / smed / 1e9,
            "step_frac_hbm_peak": (all_bytes + q_bytes) / smed / 1e9 / HBM_PEAK_GBS}


def cpu_baseline(specs, sample_rows=21760, repeats=3):
    """The oracle as it stands, timed on this host on a bounded sample: the first `sample_rows`
    rows of every linear of the block (quantize, exact integer product, dequantize)."""
    import workloads as wl
    from oracle import stwq_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    ops, secs = 0.0, 0.0
    rng = np.random.default_rng(0)
    for spec in specs:
        small = wl.shrink(spec, n_calib=2)
        w, b = wl.make_weights(small)
        xc = wl.make_calibration(small)
        x = wl.make_test_input(small)[:sample_rows]
        s = rng.uniform(1.0, 20.0, spec.K).astype(np.float32) if spec.gps else None   # scale values do not change the cost
        pack = O.calibrate_layer(xc, w, b, spec.L, spec.a_bits, spec.w_bits, False, s=s)
        for _ in range(repeats):
            t0 = time.perf_counter()
            O.forward(pack, x)
            secs += time.perf_counter() - t0
            ops += 2.0 * x.shape[0] * spec.K * spec.N
    return {"value": ops / secs / 1e12, "unit": "TOPS", "cores": int(cores), "kind": "oracle",
            "sample": f"{repeats} passes over the first {sample_rows} rows of each of the 4 linears (quantize + exact integer "
                      f"product via fp64 matmul + fp64 dequantize), {secs:.1f} s of CPU work"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--skip-cpu-baseline", action="store_true")
    ap.add_argument("--decode-rowmajor", action="store_true", help="also time the decode step on row-major weights")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus must be 1. "
              "Rows shard with no exchange; see DESIGN.md.", file=sys.stderr)
        return 2

    import torch
    import workloads as wl
    import paper_2601_21238_amd as P
    from paper_2601_21238_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    device = "cuda:0"
    torch.cuda.set_device(0)
    log(f"library {P.version()} on {torch.cuda.get_device_name(0)}")

    specs = wl.config_linears(2)
    layers = calibrate_block(specs, device)
    xs, qs, ys = [], [], []
    for spec in specs:
        x = torch.from_numpy(wl.make_test_input(spec)).to(device)
        xs.append(x)
        qs.append(torch.empty((spec.M, spec.K), dtype=torch.int8, device=device))
        ys.append(torch.empty((spec.M, spec.N), dtype=torch.bfloat16, device=device))
    torch.cuda.synchronize()
    log("inputs resident; timing")

    n = len(specs)
    lin_events = []

    def step(sampled: int):
        """One pass over the block; the linear with index `sampled` (if any) is bracketed by events.  An event on the
        stream costs about 5.6 us of idle GPU (kernel trace), so a step times ONE of its linears, in turn, rather than
        all four: every linear is still sampled inside the timed region, and the region loses 11 us per step, not 45."""
        for i in range(n):
            layers[i].quantize(xs[i], qs[i])
            if i == sampled:
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                layers[i].linear(qs[i], ys[i])
                b.record()
                lin_events.append((i, a, b))
            else:
                layers[i].linear(qs[i], ys[i])

    for _ in range(args.warmup):
        step(-1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(k % n)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    step_ops = sum(2.0 * s.M * s.K * s.N for s in specs)
    value = step_ops * args.steps / elapsed / 1e12
    lin_time, lin_count = [0.0] * n, [0] * n
    for i, a, b in lin_events:
        lin_time[i] += a.elapsed_time(b) * 1e-3
        lin_count[i] += 1
    if min(lin_count) == 0:          # fewer steps than linears: time the missing ones once, after the region
        for i in range(n):
            if lin_count[i] == 0:
                med, _ = time_launches(lambda i=i: layers[i].linear(qs[i], ys[i]), 1, 3)
                lin_time[i], lin_count[i] = med, 1
    lin_avg = [t / c for t, c in zip(lin_time, lin_count)]
    lin_total_avg = sum(lin_avg) / n                       # average duration of one linear launch
    achieved = step_ops / n / lin_total_avg / 1e12         # average ops per launch / average duration

    # the other rows of the hot path, each timed on its own (not part of `value`)
    extra = {"linear": {}, "quantize": {}}
    for i, spec in enumerate(specs):
        ops = 2.0 * spec.M * spec.K * spec.N
        extra["linear"][spec.name] = {"us": lin_avg[i] * 1e6, "tops": ops / lin_avg[i] / 1e12,
                                      "frac_mfma_peak": ops / lin_avg[i] / 1e12 / INT8_MFMA_PEAK_TOPS}
        med, _ = time_launches(lambda i=i: layers[i].quantize(xs[i], qs[i]), 3, 20)
        gbs = 5.0 * spec.M * spec.K / med / 1e9
        extra["quantize"][spec.name] = {"us": med * 1e6, "gbs": gbs, "frac_hbm_peak": gbs / HBM_PEAK_GBS}
    # calibration statistics and fold on the fc1-shaped linear (4 B read per element; 4 B + 1 B per weight)
    spec = specs[2]
    xc = torch.from_numpy(wl.make_calibration(wl.shrink(spec, n_calib=32))).to(device)
    lay = layers[2]
    pm = torch.full((spec.L,), float("inf"), device=device)
    px = torch.full((spec.L,), float("-inf"), device=device)
    med, _ = time_launches(lambda: B.stwq_calibrate_stats(xc, spec.L, inv_s=lay.inv_s, pos_min=pm, pos_max=px), 3, 10, batch=8)
    extra["stats_position"] = {"us": med * 1e6, "gbs": 4.0 * xc.numel() / med / 1e9,
                               "frac_hbm_peak": 4.0 * xc.numel() / med / 1e9 / HBM_PEAK_GBS}
    cm = torch.full((spec.K,), float("inf"), device=device)
    cx = torch.full((spec.K,), float("-inf"), device=device)
    ca = torch.zeros(spec.K, device=device)
    med, _ = time_launches(lambda: B.stwq_calibrate_stats(xc, spec.L, ch_min=cm, ch_max=cx, ch_absmax=ca), 3, 10, batch=8)
    extra["stats_channel"] = {"us": med * 1e6, "gbs": 4.0 * xc.numel() / med / 1e9,
                              "frac_hbm_peak": 4.0 * xc.numel() / med / 1e9 / HBM_PEAK_GBS}
    wd = torch.from_numpy(wl.make_weights(spec)[0]).to(device)
    sd = lay.s
    tmp = StwqScratch(spec, device)
    med, _ = time_launches(lambda: B.gps_fold_weights(wd, sd, 8, tmp.wq, tmp.dw, tmp.wsum, tmp.inv_s), 3, 10, batch=8)
    extra["fold"] = {"us": med * 1e6, "gbs": 5.0 * wd.numel() / med / 1e9,
                     "frac_hbm_peak": 5.0 * wd.numel() / med / 1e9 / HBM_PEAK_GBS}
    del xc, wd, tmp
    extra["decode"] = decode_step(device, rowmajor_too=args.decode_rowmajor)
    # a plain device-to-device copy of known size: the reference that scales the FETCH_SIZE / WRITE_SIZE counters
    cal_src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device=device).normal_()
    cal_dst = torch.empty_like(cal_src)
    for _ in range(3):
        cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    extra["pmc_reference_copy_bytes"] = int(cal_src.numel() * 4)
    del cal_src, cal_dst

    out = {
        "metric": "stwq_w8a8_linear_int8_tops",
        "value": value,
        "unit": "TOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": "config 2: VAR-d16-shaped block linears (qkv, proj, fc1, fc2), W8A8, M = 32 x 680 = 21760 rows, "
                               "step = quantize + linear for all four"},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                     "frac": achieved / INT8_MFMA_PEAK_TOPS,
                     "traffic": recorded_traffic("prefill_linear_traffic_bytes_per_launch"),
                     "kernel": "stwq::linear_prefill_kernel and stwq::linear_prefill_pair_kernel (the same tile loop; the pair "
                               "kernel runs the full rounds in wide tiles and the remaining rows in narrow tiles)",
                     "avg_launch_us": lin_total_avg * 1e6},
        "extra": extra,
    }
    if not args.skip_cpu_baseline:
        log("timing the CPU oracle on a bounded sample")
        out["cpu_baseline"] = cpu_baseline(specs)
    print(json.dumps(out), flush=True)
    return 0


class StwqScratch:
    """Output buffers for a stand-alone fold timing."""

    def __init__(self, spec, device):
        import torch
        self.wq = torch.empty((spec.N, spec.K), dtype=torch.int8, device=device)
        self.dw = torch.empty(spec.N, dtype=torch.float32, device=device)
        self.wsum = torch.empty(spec.N, dtype=torch.int32, device=device)
        self.inv_s = torch.empty(spec.K, dtype=torch.float32, device=device)


if __name__ == "__main__":
    sys.exit(main())
