#!/usr/bin/env python3
"""Benchmark of the lognormal gradient-compression hot path on one MI355X.

One step = one pass of the whole path over one batch of gradient tensors already resident in HBM:

    lgn_stats -> lgn_threshold -> lgn_fp_params -> lgn_prune_quantize_fused

By default the first three run as ONE launch (lgn_stats_solve: the last workgroup of the statistics
pass runs both solvers; results identical to the separate calls), so a step is two launches;
--launches separate times the calls one by one.

Workload (default, "c4"): the ResNet-50-style activation gradient of the benchmark configurations,
256x256x56x56 = 205 520 896 fp32 elements, 40 % exact zeros, ln|g| ~ N(-13, 2^2) (seeded
synthetic data standing in for ImageNet gradients); target sparsity 0.85, FP6 with the
closed-form exponent/mantissa split and quantile scale, stochastic rounding, one byte per code.
Other workloads: c1 (2^20 elements), c2 (51.4 M elements, one statistics pass and four pruning
passes at four sparsities), c3 (20 tensors of ResNet-18 shapes, batched: one statistics+solve
launch and one fused launch for all of them), c5 (10^9 bf16 elements, packed 6-bit codes);
--workload all runs them one after the other and reports them in one table.

Metric: GB/s of ALGORITHMIC bytes (for c4: 2 reads of the tensor + 1 write of the codes) / time.

Protocol.  The device clocks dip for some tens of milliseconds after every idle period (a step that
takes 0.31 ms in the steady state takes up to 0.41 ms between the 2nd and the 15th millisecond
of a burst).  So the run is:  (1) a cold pass, `warmup` + `steps` steps straight after the idle
period of data generation, reported as cold_ms_per_step;  (2) a pre-conditioning phase of the same
launches for --precondition-ms of wall time, outside any timed region and reported as
preconditioning_ms;  (3) `warmup` untimed steps and EXACTLY `steps` timed steps between two
synchronisations: their wall-clock mean is ms_per_step and `value`; HIP events on the stream
around every launch of every N-th of those same steps (--event-every) give the per-kernel times
and the median and minimum per step.  Prints exactly one JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
METRIC = "GB/s and % HBM peak for fused lognormal-stats+prune+FP-n quantize"
DTYPE = "u32 (bit-level prune/quantize) + f64 (statistics, solver)"
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hot_path_c4_hbm_traffic.txt")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c3", "c4", "c5", "all"])
    ap.add_argument("--n", type=int, default=None, help="override the element count")
    ap.add_argument("--out-kind", default=None, choices=["code8", "packed", "value"],
                    help="default: code8 (packed for c5, value for c2)")
    ap.add_argument("--rounding", default="stochastic", choices=["stochastic", "nearest"])
    ap.add_argument("--launches", default="merged", choices=["merged", "separate"],
                    help="merged: lgn_stats_solve + lgn_prune_quantize_fused (two launches per step); "
                         "separate: lgn_stats, lgn_threshold, lgn_fp_params, lgn_prune_quantize_fused")
    ap.add_argument("--precondition-ms", type=float, default=150.0,
                    help="wall time of the untimed pre-conditioning phase before warm-up (0 = none, and no cold pass)")
    ap.add_argument("--event-every", type=int, default=0,
                    help="record the per-kernel HIP events on every N-th timed step (each record costs the stream "
                         "3-4 us: a step with its three records runs ~4 %% longer than one without); 0 = steps // 10, "
                         "at least 1 and at most 10, i.e. every 2nd of 20 steps, every 10th of 500")
    ap.add_argument("--c3-mode", default="batched", choices=["batched", "streams"],
                    help="workload c3: one batched statistics+solve launch and one batched fused launch "
                         "for all tensors, or one chain per tensor dealt to --streams streams")
    ap.add_argument("--streams", type=int, default=1, help="workload c3, --c3-mode streams: number of HIP streams")
    ap.add_argument("--evict", action="store_true",
                    help="cache-evicting variant: a 512 MB buffer is read before every timed step (outside the "
                         "events), so nothing of the tensor is left in the memory-side cache from the step before; "
                         "per-step times then come from the events alone")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-beyond", action="store_true", help="skip the timings of the rows beyond the hot path")
    ap.add_argument("--no-keep0", action="store_true", help="skip the extra loop with the statistics pass all streaming")
    ap.add_argument("--table-out", default=None, help="--workload all: also write the table as text to this file")
    ap.add_argument("--cold-trace", default=None, metavar="FILE",
                    help="one-tensor workloads: instead of the plain cold pass, run 300 steps straight after the idle "
                         "period with events on every step and write the per-step kernel times to FILE")
    ap.add_argument("--touch-outputs", action="store_true",
                    help="write the output and struct buffers once before anything is timed (to tell first-touch "
                         "effects from clock effects in a cold trace)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="run one plain elementwise copy of the tensor before the timed region "
                         "(known traffic, to calibrate rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured_traffic(key):
    """HBM bytes per launch of a kernel, from the tracked rocprofv3 counter summary (lines of the
    form `traffic_bytes_per_launch <key> = <bytes>`); None if the file has no such line."""
    try:
        for line in open(TRAFFIC_FILE):
            m = re.match(r"\s*traffic_bytes_per_launch\s+(\S+)\s*=\s*(\d+)", line)
            if m and m.group(1) == key:
                return int(m.group(2))
    except OSError:
        pass
    return None


class Runner:
    """Timing protocol shared by all workloads: `step(marks)` enqueues one step and, if `marks` is a
    list, appends a recorded event before the first launch and after every launch."""

    def __init__(self, torch, args, step, n_marks):
        self.torch, self.args, self.step, self.n_marks = torch, args, step, n_marks
        self.evict_buf = None
        if args.evict:
            self.evict_buf = torch.zeros(128 << 20, dtype=torch.int32, device="cuda")   # 512 MB

    def _wall(self, warmup, steps):
        t = self.torch
        for _ in range(warmup):
            self.step(None)
        t.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step(None)
        t.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    def cold(self):
        return self._wall(self.args.warmup, self.args.steps)

    def precondition(self):
        t, target = self.torch, self.args.precondition_ms
        done, t0 = 0, time.perf_counter()
        while (time.perf_counter() - t0) * 1e3 < target:
            for _ in range(50):
                self.step(None)
            t.cuda.synchronize()
            done += 50
        return (time.perf_counter() - t0) * 1e3, done

    def timed(self):
        """warmup + exactly `steps` timed steps; returns (wall ms per step, list of per-step mark times)."""
        t, args = self.torch, self.args
        for _ in range(args.warmup):
            self.step(None)
        every = args.event_every if args.event_every > 0 else max(1, min(10, args.steps // 10))
        marks = [[] if (k % every == 0 or self.evict_buf is not None) else None for k in range(args.steps)]
        t.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            if self.evict_buf is not None:
                self.evict_buf.sum()     # ordinary loads over 512 MB replace what the 256 MB cache held and
                                         # leave nothing dirty behind that the next kernel would have to wait for
            self.step(marks[k])
        t.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / args.steps
        spans = []
        for m in marks:
            if m:
                spans.append([m[i].elapsed_time(m[i + 1]) for i in range(len(m) - 1)])
        if self.evict_buf is not None:   # the wall clock contains the evicting kernel: use the events
            wall = statistics.fmean(sum(s) for s in spans)
        return wall, spans


def mark(torch, marks):
    if marks is not None:
        e = torch.cuda.Event(enable_timing=True)
        e.record()
        marks.append(e)


def summarize(spans):
    totals = [sum(s) for s in spans]
    cols = list(zip(*spans))
    return {"events_on_steps": len(spans), "median_ms": round(statistics.median(totals), 4),
            "min_ms": round(min(totals), 4), "mean_ms": round(statistics.fmean(totals), 4),
            "per_launch_mean_ms": [round(statistics.fmean(c), 4) for c in cols],
            "per_launch_median_ms": [round(statistics.median(c), 4) for c in cols]}


def cold_trace(torch, args, step, path):
    """300 steps from cold with events around every launch; writes a table, returns the mean of the
    first warmup + steps step spans (what a cold pass of the requested size would have seen)."""
    k = 300
    marks = [[] for _ in range(k)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for m in marks:
        step(m)
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / k
    spans = [[m[i].elapsed_time(m[i + 1]) * 1e3 for i in range(len(m) - 1)] for m in marks]
    tot = [sum(s) for s in spans]
    with open(path, "w") as f:
        f.write("python3 bench.py " + " ".join(sys.argv[1:]) + "\n")
        f.write(f"{k} steps straight after the idle period of data generation, HIP events around every launch "
                f"(wall clock {wall * 1e3:.1f} us per step including the event records)\n")
        f.write("step | " + " | ".join(f"launch {i + 1} us" for i in range(len(spans[0]))) + " | step us\n")
        for i in list(range(40)) + list(range(40, k, 10)):
            f.write(f"{i} | " + " | ".join(f"{x:.1f}" for x in spans[i]) + f" | {tot[i]:.1f}\n")
        for lo, hi in ((0, 5), (5, 25), (25, 100), (100, 200), (200, 300)):
            seg = tot[lo:hi]
            cols = list(zip(*spans[lo:hi]))
            f.write(f"steps [{lo},{hi}): mean step {statistics.fmean(seg):.1f} us, median {statistics.median(seg):.1f}, "
                    f"min {min(seg):.1f}; per launch mean " + ", ".join(f"{statistics.fmean(c):.1f}" for c in cols) + "\n")
    w, s_ = args.warmup, args.steps
    seg = tot[min(w, k - 1):min(w + s_, k)]
    return statistics.fmean(seg) * 1e-3


def protocol(torch, args, step, n_marks):
    r = Runner(torch, args, step, n_marks)
    out = {}
    if args.cold_trace:
        out["cold_ms_per_step"] = round(cold_trace(torch, args, step, args.cold_trace), 4)
        pms, psteps = r.precondition()
        out["preconditioning_ms"] = round(pms, 1)
        out["preconditioning_steps"] = psteps
    elif args.precondition_ms > 0:
        out["cold_ms_per_step"] = round(r.cold(), 4)
        pms, psteps = r.precondition()
        out["preconditioning_ms"] = round(pms, 1)
        out["preconditioning_steps"] = psteps
    else:
        out["cold_ms_per_step"] = None
        out["preconditioning_ms"] = 0.0
        out["preconditioning_steps"] = 0
    wall, spans = r.timed()
    out["wall_ms"] = wall
    out["spans"] = spans
    out["runner"] = r
    return out


def base_line(args, value, wall, config, roofline, prot, spans_summary):
    return {
        "metric": METRIC, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(wall, 4),
        "ms_per_step_median": spans_summary["median_ms"], "ms_per_step_min": spans_summary["min_ms"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": DTYPE, "data": "synthetic",
        "config": config, "roofline": roofline,
        "cold_ms_per_step": prot["cold_ms_per_step"], "preconditioning_ms": prot["preconditioning_ms"],
        "preconditioning_steps": prot["preconditioning_steps"],
        "timing_note": ("ms_per_step = wall clock of the timed steps / steps, after an untimed pre-conditioning phase of the "
                        "same launches; cold_ms_per_step = the same count of warm-up + steps straight after the idle "
                        "period before it; median/min = per-step HIP-event spans of the timed steps"
                        + ("; cache-evicting variant: per-step times from the events only" if args.evict else "")),
    }


# ------------------------------------------------------------------------------------------ c3
def bench_c3(args, lgn, SI, torch, np):
    """Twenty tensors with ResNet-18 activation-gradient shapes, per-tensor parameters: total
    algorithmic bytes / total time."""
    tensors = SI.config_c3()
    rounding = lgn.LGN_ROUND_STOCHASTIC if args.rounding == "stochastic" else lgn.LGN_ROUND_NEAREST_EVEN
    items = []
    for cfg in tensors:
        d = torch.from_numpy(SI.make(cfg)).cuda()
        items.append(dict(cfg=cfg, d=d, out=torch.empty(cfg["n"], dtype=torch.uint8, device="cuda"),
                          st=torch.empty(72, dtype=torch.uint8, device="cuda"),
                          pp=torch.empty(24, dtype=torch.uint8, device="cuda"),
                          fp=torch.empty(32, dtype=torch.uint8, device="cuda")))
    total_n = sum(c["n"] for c in tensors)
    batched = args.c3_mode == "batched"
    merged = args.launches == "merged"
    if batched:
        batch = lgn.make_batch([dict(g=it["d"], out=it["out"], target_sparsity=it["cfg"]["sparsity"],
                                     n_bits=it["cfg"]["n_bits"], seed=it["cfg"]["rng_seed"],
                                     st=it["st"], p=it["pp"], f=it["fp"]) for it in items])
        ws = lgn.workspace(items[0]["d"].device)

        def one_step(marks):
            mark(torch, marks)
            lgn.lgn_batch_stats_solve(batch, ws=ws)
            mark(torch, marks)
            lgn.lgn_batch_prune_quantize_fused(batch, rounding, out_kind=lgn.LGN_OUT_CODE8)
            mark(torch, marks)
        launches, n_marks, how = 2, 3, "one batched statistics+solve launch and one batched fused launch, 1 stream"
    else:
        nstreams = max(1, min(args.streams, 4))
        streams = [torch.cuda.Stream() for _ in range(nstreams)] if nstreams > 1 else [torch.cuda.current_stream()]
        wss = []
        for _ in range(nstreams):   # a workspace per stream: calls that overlap must not share one
            w = torch.empty(lgn.lgn_workspace_bytes(0, lgn.LGN_F32), dtype=torch.uint8, device="cuda")
            lgn.lgn_workspace_init(w)
            wss.append(w)
        torch.cuda.synchronize()

        def one_step(marks):
            mark(torch, marks)
            for i, it in enumerate(items):
                c = it["cfg"]
                with torch.cuda.stream(streams[i % nstreams]):
                    if merged:
                        lgn.lgn_stats_solve(it["d"], c["sparsity"], lgn.LGN_F32, c["n_bits"], st=it["st"],
                                            p=it["pp"], f=it["fp"], ws=wss[i % nstreams])
                    else:
                        lgn.lgn_stats(it["d"], out=it["st"], ws=wss[i % nstreams])
                        lgn.lgn_threshold(it["st"], c["sparsity"], lgn.LGN_F32, out=it["pp"])
                        lgn.lgn_fp_params(it["st"], c["n_bits"], out=it["fp"])
                    lgn.lgn_prune_quantize_fused(it["d"], it["pp"], it["fp"], rounding, c["rng_seed"], 0,
                                                 out=it["out"], out_kind=lgn.LGN_OUT_CODE8)
            if nstreams == 1:
                mark(torch, marks)
            elif marks is not None:
                marks.clear()          # events on one stream say nothing about the others
        launches = (40 if merged else 100)
        n_marks = 2
        how = f"20 whole chains back to back ({'2' if merged else '4'} launches each) on {nstreams} stream(s)"

    prot = protocol(torch, args, one_step, n_marks)
    wall, spans = prot["wall_ms"], prot["spans"]
    alg = total_n * 9
    value = alg / (wall * 1e-3) / 1e9
    summ = summarize(spans) if spans else {"median_ms": None, "min_ms": None, "events_on_steps": 0}
    log(f"[bench] c3: {len(items)} tensors, {total_n} elements, {wall:.4f} ms per step, {value:.0f} GB/s ({how})")
    config = {"workload": "c3: 20 fp32 tensors with ResNet-18 activation-gradient shapes at batch 256, per-tensor mu, "
                          f"sigma and target sparsity; {how}; {args.rounding} rounding, code8 output",
              "elements": total_n, "elements_per_s": round(total_n / (wall * 1e-3)),
              "algorithmic_bytes_per_step": alg, "pct_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2),
              "cache_assisted": "the statistics pass leaves up to 224 MB of what it read last in the 256 MB memory-side "
                                "cache for the fused pass" if not args.evict else "evicted before every step"}
    if batched and spans:
        fused_ms = statistics.fmean(s[1] for s in spans)
        stats_ms = statistics.fmean(s[0] for s in spans)
        roofline = {"bound": "hbm", "kernel": "stream_batch_kernel (fused prune+quantize, all tensors)",
                    "achieved": round(total_n * 5 / (fused_ms * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(total_n * 5 / (fused_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "traffic": None,
                    "algorithmic_bytes": total_n * 5, "avg_launch_ms": round(fused_ms, 4),
                    "other_kernels": {"stats_ms": round(stats_ms, 4),
                                      "stats_GBps": round(total_n * 4 / (stats_ms * 1e-3) / 1e9, 1)}}
    else:
        roofline = {"bound": "hbm", "kernel": "whole chain (%d launches)" % launches, "achieved": round(value, 1),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(value / HBM_PEAK_GBS, 4), "traffic": None}
    line = base_line(args, value, wall, config, roofline, prot, summ)
    line["cpu_baseline"] = None
    return line


# ------------------------------------------------------------------------- one-tensor workloads
def bench_one(args, name, lgn, SI, torch, np):
    cfg = {"c1": SI.config_c1, "c2": SI.config_c2, "c4": SI.config_c4, "c5": SI.config_c5}[name]()
    if args.n:
        cfg["n"] = args.n
    n = cfg["n"]
    prune_only = name == "c2"           # configuration 2: pruning at four sparsities, no quantization
    sparsities = cfg.get("sparsities", (cfg.get("sparsity", 0.85),))
    sparsity = sparsities[-1] if prune_only else cfg.get("sparsity", 0.85)
    n_bits = cfg.get("n_bits", 6)
    rounding = lgn.LGN_ROUND_STOCHASTIC if args.rounding == "stochastic" else lgn.LGN_ROUND_NEAREST_EVEN
    ok_name = args.out_kind or {"c5": "packed", "c2": "value"}.get(name, "code8")
    out_kind = {"code8": lgn.LGN_OUT_CODE8, "packed": lgn.LGN_OUT_PACKED, "value": lgn.LGN_OUT_VALUE}[ok_name]
    seed = cfg["rng_seed"]

    t0 = time.time()
    if cfg["dtype"] == SI.F32:
        d = torch.empty(n, dtype=torch.float32, device="cuda")
        view = d
    else:
        d = torch.empty(n, dtype=torch.bfloat16, device="cuda")
        view = d.view(torch.int16)
    # generate in slices so host memory stays bounded; upload once
    step = 1 << 26
    for s0 in range(0, n, step):
        part = SI.make(cfg, n=min(step, n - s0), start=s0)
        if part.dtype == np.uint16:
            part = part.view(np.int16)
        view[s0:s0 + part.size].copy_(torch.from_numpy(part))
    torch.cuda.synchronize()
    log(f"[bench] {name}: generated {n} {cfg['dtype']} elements in {time.time() - t0:.1f}s")

    in_bytes = 4 if cfg["dtype"] == SI.F32 else 2
    out_bytes_per_elem = {lgn.LGN_OUT_CODE8: 1.0, lgn.LGN_OUT_PACKED: n_bits / 8.0,
                          lgn.LGN_OUT_VALUE: float(in_bytes)}[out_kind]
    if out_kind == lgn.LGN_OUT_VALUE:
        out = torch.empty_like(d)
    elif out_kind == lgn.LGN_OUT_CODE8:
        out = torch.empty(n, dtype=torch.uint8, device="cuda")
    else:
        out = torch.empty(lgn.lgn_packed_bytes(n, n_bits), dtype=torch.uint8, device="cuda")
    st = torch.empty(72, dtype=torch.uint8, device="cuda")
    pp = torch.empty(24, dtype=torch.uint8, device="cuda")
    fp = torch.empty(32, dtype=torch.uint8, device="cuda")
    ws = lgn.workspace(d.device)

    alpha_dt = lgn.LGN_F32 if in_bytes == 4 else lgn.LGN_BF16
    merged = args.launches == "merged"

    if prune_only:
        # one statistics pass, then threshold + pruning pass per sparsity (the statistics do not
        # depend on the target); marks: [start, stats, prune_1, ..., prune_k]
        def one_step(marks):
            mark(torch, marks)
            lgn.lgn_stats_solve(d, sparsities[0], alpha_dt, 0, st=st, p=pp, ws=ws)
            mark(torch, marks)
            for i, s in enumerate(sparsities):
                if i:
                    lgn.lgn_threshold(st, s, alpha_dt, out=pp)
                lgn.lgn_prune(d, pp, seed, 0, out=out)
                mark(torch, marks)
        n_marks = 2 + len(sparsities)
        alg_bytes_step = n * in_bytes * (1 + 2 * len(sparsities))
        fused_bytes = n * in_bytes * 2
        what = (f"one statistics+threshold launch, then threshold + lgn_prune (value output) at sparsities "
                f"{list(sparsities)}: {2 * len(sparsities)} launches")
    else:
        def one_step(marks):
            mark(torch, marks)
            if merged:
                lgn.lgn_stats_solve(d, sparsity, alpha_dt, n_bits, st=st, p=pp, f=fp, ws=ws)
            else:
                lgn.lgn_stats(d, out=st, ws=ws)
                lgn.lgn_threshold(st, sparsity, alpha_dt, out=pp)
                lgn.lgn_fp_params(st, n_bits, out=fp)
            mark(torch, marks)
            lgn.lgn_prune_quantize_fused(d, pp, fp, rounding, seed, 0, out=out, out_kind=out_kind)
            mark(torch, marks)
        n_marks = 3
        alg_bytes_step = n * (2 * in_bytes + out_bytes_per_elem)
        fused_bytes = n * (in_bytes + out_bytes_per_elem)
        what = (f"stats+threshold(S={sparsity})+FP{n_bits} format+fused prune/quantize, {args.rounding} rounding, "
                f"{ok_name} output, " + ("2 launches (stats+solvers merged, fused)" if merged else "4 launches"))

    if args.touch_outputs:
        for buf in (out, st, pp, fp):
            buf.zero_()
        torch.cuda.synchronize()

    if args.copy_probe and cfg["dtype"] == SI.F32:
        probe = torch.empty_like(d)
        torch.mul(d, 1.0, out=probe)  # reads n*4 bytes, writes n*4 bytes
        torch.cuda.synchronize()
        del probe

    prot = protocol(torch, args, one_step, n_marks)
    wall, spans = prot["wall_ms"], prot["spans"]
    summ = summarize(spans)
    t_stats = summ["per_launch_mean_ms"][0]
    t_fused = statistics.fmean(summ["per_launch_mean_ms"][1:])   # c2: mean over the pruning passes
    value = alg_bytes_step / (wall * 1e-3) / 1e9
    stats_bytes = n * in_bytes
    fused_gbs = fused_bytes / (t_fused * 1e-3) / 1e9
    stats_gbs = stats_bytes / (t_stats * 1e-3) / 1e9
    hp, hs = lgn.read_prune_params(pp), lgn.read_stats(st)
    hf = lgn.read_fp_params(fp) if not prune_only else None
    log(f"[bench] {name}: mu={hs.mu:.5f} sigma={hs.sigma:.5f} nnz={hs.nnz} alpha={hp.alpha:.6e}"
        + (f" format=1-{hf.e_bits}-{hf.m_bits} s={hf.scale_exp}" if hf else ""))
    log(f"[bench] {name}: per step {wall:.4f} ms wall (events: median {summ['median_ms']}, min {summ['min_ms']}; cold "
        f"{prot['cold_ms_per_step']}): stats {t_stats:.4f} ms ({stats_gbs:.0f} GB/s), "
        f"{'prune' if prune_only else 'fused'} {t_fused:.4f} ms ({fused_gbs:.0f} GB/s)")

    # dominant kernel = the one that takes longer per launch
    stream_name = "stream_kernel (prune)" if prune_only else "stream_kernel (fused prune+quantize)"
    if t_fused >= t_stats:
        dom = dict(kernel=stream_name, achieved=fused_gbs, bytes=fused_bytes, ms=t_fused,
                   key=f"stream_kernel_fused_{name}_{ok_name}_{args.rounding}")
    else:
        dom = dict(kernel="stats_solve_kernel" if merged or prune_only else "stats_stage1", achieved=stats_gbs,
                   bytes=stats_bytes, ms=t_stats, key=f"stats_solve_kernel_{name}")
    roofline = {"bound": "hbm", "kernel": dom["kernel"], "achieved": round(dom["achieved"], 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(dom["achieved"] / HBM_PEAK_GBS, 4),
                "traffic": measured_traffic(dom["key"]), "algorithmic_bytes": int(dom["bytes"]),
                "avg_launch_ms": round(dom["ms"], 4),
                "other_kernels": {"stats_ms": round(t_stats, 4), "stats_GBps": round(stats_gbs, 1),
                                  "stream_ms": round(t_fused, 4), "stream_GBps": round(fused_gbs, 1),
                                  "per_launch_median_ms": summ["per_launch_median_ms"]}}

    # The statistics pass leaves the tensor's tail in the memory-side cache for the pass after it.
    # One more timed loop with that switched off (all loads streaming) shows what it is worth.
    keep_mb = lgn.lgn_get_tuning(lgn.LGN_TUNE_STATS_KEEP_MB)
    cache = {"keep_mb": keep_mb, "ms_per_step_keep0": None,
             "note": "the statistics pass reads the last keep_mb MB of the tensor with cache-allocating loads, so the "
                     "next pass finds them in the 256 MB memory-side cache; ms_per_step_keep0 = same timed loop with "
                     "every load streaming. Counters in front of that cache (roofline.traffic) cannot see the reuse."
                     + (" Tensors below keep_mb (this one) are kept whole." if n * in_bytes <= keep_mb << 20 else "")}
    if not args.no_keep0 and keep_mb:
        try:
            lgn.lgn_set_tuning(lgn.LGN_TUNE_STATS_KEEP_MB, 0)
            w0, _ = prot["runner"].timed()
            cache["ms_per_step_keep0"] = round(w0, 4)
        finally:
            lgn.lgn_set_tuning(lgn.LGN_TUNE_STATS_KEEP_MB, keep_mb)
        one_step(None)   # leave the state as the timed loop had it
        torch.cuda.synchronize()
        log(f"[bench] {name}: all-streaming statistics pass: {cache['ms_per_step_keep0']} ms per step")

    # Outside the timed region: the rows built beyond the hot path, each timed on the same tensor with
    # HIP events.  Reported beside the headline, never part of `value`.
    def timed(fn, reps=30):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    def measure_beyond():
        nchunks = (n + lgn.LGN_PREFIX_CHUNK - 1) // lgn.LGN_PREFIX_CHUNK
        pbuf, ptab = lgn.lgn_prefix_encode(out, lgn.LGN_OUT_CODE8, pp, fp, width=n_bits)
        enc_ms = timed(lambda: lgn.lgn_prefix_encode(out, lgn.LGN_OUT_CODE8, pp, fp, out=pbuf, table=ptab))
        words = int(ptab[nchunks].item())
        dec = torch.empty(n, dtype=torch.uint8, device="cuda")
        dec_ms = timed(lambda: lgn.lgn_prefix_decode(pbuf, ptab, n, lgn.LGN_OUT_CODE8, pp, fp, out=dec))
        if not torch.equal(dec, out):
            raise RuntimeError("prefix round trip differs")
        del pbuf, ptab, dec
        hist = torch.empty(lgn.LGN_HIST_BINS, dtype=torch.int64, device="cuda")
        hist_ms = timed(lambda: lgn.lgn_log_histogram(d, out=hist))
        bmask = (view != 0).to(torch.uint8)              # a ReLU-style byte mask: the non-zero entries
        masked_ms = timed(lambda: lgn.lgn_stats_masked(d, bmask, out=st, ws=ws))
        del bmask
        fmask = d.clone()                                # a second tensor of the same dtype as the mask
        masked_same_ms = timed(lambda: lgn.lgn_stats_masked(d, fmask, out=st, ws=ws))
        del fmask
        gb = lambda b, ms: round(b / (ms * 1e-3) / 1e9, 1)
        return {
            "prefix_encode": {"ms": round(enc_ms, 4), "bits_per_value": round(words * 32 / n, 3),
                              "GBps": gb(2 * n + words * 4, enc_ms),
                              "what": "lgn_prefix_encode of the step's CODE8 output: reads it twice, writes the stream"},
            "prefix_decode": {"ms": round(dec_ms, 4), "GBps": gb(n + words * 4, dec_ms),
                              "what": "lgn_prefix_decode of that stream back to the codes (checked equal)"},
            "log_histogram": {"ms": round(hist_ms, 4), "GBps": gb(n * in_bytes, hist_ms),
                              "what": "lgn_log_histogram of the tensor (one read)"},
            "stats_masked_u8": {"ms": round(masked_ms, 4), "GBps": gb(n * (in_bytes + 1), masked_ms),
                                "what": "lgn_stats_masked with a byte mask (tensor + 1 B/elem)"},
            "stats_masked_same_dtype": {"ms": round(masked_same_ms, 4), "GBps": gb(2 * n * in_bytes, masked_same_ms),
                                        "what": "lgn_stats_masked with a mask tensor of the same dtype (two reads)"},
            "note": "measured after the timed region; not part of the step"}

    extras = None
    if out_kind == lgn.LGN_OUT_CODE8 and not prune_only and not args.no_beyond:
        # a failure here must not take the headline line with it
        try:
            extras = measure_beyond()
            log(f"[bench] {name}: beyond the hot path: { {k: v['ms'] for k, v in extras.items() if isinstance(v, dict)} } ms")
        except Exception as e:  # noqa: BLE001
            extras = {"error": f"{type(e).__name__}: {e}"}
            log(f"[bench] beyond the hot path failed: {extras['error']}")
        # leave the structs as the timed step wrote them
        one_step(None)
        torch.cuda.synchronize()

    def measure_cpu_baseline():
        """The oracle's whole chain on a bounded sample of the same tensor: all host cores, then one."""
        import oracle as O
        threads = O.max_threads()
        o_round = O.ROUND_STOCHASTIC if rounding == lgn.LGN_ROUND_STOCHASTIC else O.ROUND_NEAREST_EVEN
        o_kind = {lgn.LGN_OUT_CODE8: O.OUT_CODE8, lgn.LGN_OUT_PACKED: O.OUT_PACKED, lgn.LGN_OUT_VALUE: O.OUT_VALUE}[out_kind]
        o_dt = O.F32 if in_bytes == 4 else O.BF16

        def chain(sample):
            ost = O.stats(sample)
            if prune_only:
                for s in sparsities:
                    O.prune(sample, O.threshold(ost, s, o_dt).alpha, seed, 0)
            else:
                op = O.threshold(ost, sparsity, o_dt)
                of = O.fp_params(ost, n_bits)
                O.prune_quantize(sample, op.alpha, of.e_bits, of.m_bits, of.scale_exp, o_round, seed, 0, o_kind)

        def run(m, nthreads, reps):
            O.set_threads(nthreads)
            sample = SI.make(cfg, n=m)
            t1 = time.perf_counter()
            for _ in range(reps):
                chain(sample)
            dt = (time.perf_counter() - t1) / reps
            return m * alg_bytes_step / n / dt / 1e9, dt

        m_all = min(n, 1 << 28)        # the whole tensor for configuration 4: ~0.5 s on 16 cores
        v_all, dt_all = run(m_all, threads, 2)
        m_one = min(n, 1 << 25)        # a sixth of it on one core: a few seconds
        v_one, dt_one = run(m_one, 1, 1)
        O.set_threads(threads)
        return {"value": round(v_all, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
                "sample": f"first {m_all} elements of the same tensor, whole chain, 2 repetitions of {dt_all:.2f} s on "
                          f"{threads} threads; single thread: first {m_one} elements, 1 repetition of {dt_one:.2f} s",
                "single_thread_value": round(v_one, 3)}

    cpu = None
    if not args.no_cpu_baseline:
        try:  # a failure here must not take the headline line with it
            cpu = measure_cpu_baseline()
        except Exception as e:  # noqa: BLE001
            cpu = {"value": None, "unit": "GB/s", "cores": 0, "kind": "oracle", "sample": f"failed: {type(e).__name__}: {e}"}
        log(f"[bench] {name}: cpu oracle: {cpu}")

    config = {"workload": f"{cfg['name']}: {n} {cfg['dtype']} elements, zeros {cfg['zero_frac']}, "
                          f"ln|g|~N({cfg['mu']},{cfg['sigma']}^2); {what}",
              "elements": n, "elements_per_s": round(n / (wall * 1e-3)),
              "algorithmic_bytes_per_step": int(alg_bytes_step),
              "pct_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2)}
    line = base_line(args, value, wall, config, roofline, prot, summ)
    line["cache_assisted"] = cache if not args.evict else {"keep_mb": keep_mb, "note": "evicted before every step"}
    if not prune_only:
        # the paper refreshes the statistics once per epoch: between refreshes a step is the fused pass alone
        line["amortised"] = {"ms_per_step": round(t_fused, 4), "GBps": round(fused_gbs, 1),
                             "pct_hbm_peak": round(100 * fused_gbs / HBM_PEAK_GBS, 2),
                             "note": "fused prune+quantize alone (parameters from an earlier statistics pass): "
                                     "n * (input + output bytes) / its average launch time in the timed steps"}
    line["cpu_baseline"] = cpu
    line["beyond_hot_path"] = extras
    del d, out
    torch.cuda.empty_cache()
    return line


def table_text(lines, args):
    rows = ["workload | ms/step (wall) | median | min | cold | GB/s (algorithmic) | % of 8 TB/s | stats ms | stream ms | keep0 ms",
            "---|---|---|---|---|---|---|---|---|---"]
    for name, l in lines.items():
        ok = l["roofline"].get("other_kernels", {})
        rows.append(" | ".join(str(x) for x in (
            name, l["ms_per_step"], l["ms_per_step_median"], l["ms_per_step_min"], l["cold_ms_per_step"], l["value"],
            l["config"]["pct_hbm_peak"], ok.get("stats_ms"), ok.get("stream_ms", l["roofline"].get("avg_launch_ms")),
            (l.get("cache_assisted") or {}).get("ms_per_step_keep0"))))
    head = (f"python3 bench.py --workload all --steps {args.steps} --warmup {args.warmup}"
            + (" --evict" if args.evict else "") + f" --precondition-ms {args.precondition_ms:g}\n")
    return head + "\n".join(rows) + "\n" + "\n".join(f"{k}: {v['config']['workload']}" for k, v in lines.items()) + "\n"


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures one GPU only (gradients are local to a data-parallel rank, "
                 "so the path needs no communication and every rank would run it on its own tensors). "
                 "Run with --gpus 1.")
    import numpy as np
    import torch

    import paper_2006_08173_amd as lgn
    import synth_inputs as SI

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    lgn.load()

    def run(name):
        if name == "c3":
            return bench_c3(args, lgn, SI, torch, np)
        return bench_one(args, name, lgn, SI, torch, np)

    if args.workload != "all":
        print(json.dumps(run(args.workload)), flush=True)
        return
    args.no_beyond = True
    lines = {}
    for name in ("c1", "c2", "c3", "c4", "c5"):
        lines[name] = run(name)
        torch.cuda.empty_cache()
    text = table_text(lines, args)
    log(text)
    if args.table_out:
        with open(args.table_out, "w") as f:
            f.write(text)
    head = dict(lines["c4"])
    head["workloads"] = {k: {kk: v[kk] for kk in ("value", "ms_per_step", "ms_per_step_median", "ms_per_step_min",
                                                  "cold_ms_per_step", "config", "roofline", "cpu_baseline")}
                         for k, v in lines.items()}
    print(json.dumps(head), flush=True)


if __name__ == "__main__":
    main()
