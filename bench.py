#!/usr/bin/env python3
"""Benchmark of the lognormal gradient-compression hot path on one MI355X.

One step = one pass of the whole path over one gradient tensor already resident in HBM:

    lgn_stats -> lgn_threshold -> lgn_fp_params -> lgn_prune_quantize_fused

By default the first three run as ONE launch (lgn_stats_solve: the last workgroup of the statistics
pass runs both solvers; results identical to the separate calls), so a step is two launches;
--launches separate times the calls one by one.

Workload (default): the ResNet-50-style activation gradient of the benchmark configurations,
256x256x56x56 = 205 520 896 fp32 elements, 40 % exact zeros, ln|g| ~ N(-13, 2^2) (seeded
synthetic data standing in for ImageNet gradients); target sparsity 0.85, FP6 with the
closed-form exponent/mantissa split and quantile scale, stochastic rounding, one byte per code.

Metric: GB/s of ALGORITHMIC bytes = (2 reads of the tensor + 1 write of the codes) / time.
Prints exactly one JSON line on stdout.
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

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth

# HBM traffic of the dominant kernel per launch measured with rocprofv3 --pmc (FETCH_SIZE and
# WRITE_SIZE, scaled by the same counters on a copy kernel of known size); see profiles/.
# None until measured for the workload at hand.
MEASURED_TRAFFIC_BYTES = {
    # profiles/hot_path_c4_hbm_traffic.txt: FETCH_SIZE x 2.000 KiB + WRITE_SIZE x 1.000 KiB per launch
    ("c4", "code8", "stochastic", "stream_kernel (fused prune+quantize)"): int((401498.7 * 2.0 + 200704.0) * 1024),
    ("c4", "code8", "stochastic", "stats_solve_kernel"): int((402623.7 * 2.0 + 96.2) * 1024),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # a step takes a third of a millisecond and the device needs some tens of steps to settle into
    # its steady state (the first ~20 steps after an idle period run 15 % slower), hence the counts
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--n", type=int, default=None, help="override the element count")
    ap.add_argument("--out-kind", default="code8", choices=["code8", "packed", "value"])
    ap.add_argument("--rounding", default="stochastic", choices=["stochastic", "nearest"])
    ap.add_argument("--launches", default="merged", choices=["merged", "separate"],
                    help="merged: lgn_stats_solve + lgn_prune_quantize_fused (two launches per step); "
                         "separate: lgn_stats, lgn_threshold, lgn_fp_params, lgn_prune_quantize_fused")
    ap.add_argument("--event-every", type=int, default=10,
                    help="record the per-kernel HIP events on every N-th timed step (each record "
                         "costs a few microseconds of stream time; 1 = every step)")
    ap.add_argument("--streams", type=int, default=3,
                    help="workload c3 only: tensors are dealt round-robin to this many HIP streams (default "
                         "priority, one workspace each), so one tensor's solver tail overlaps the next "
                         "tensor's streaming kernels")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-beyond", action="store_true", help="skip the timings of the rows beyond the hot path")
    ap.add_argument("--copy-probe", action="store_true",
                    help="run one plain elementwise copy of the tensor before the timed region "
                         "(known traffic, to calibrate rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def bench_c3(args, lgn, SI, torch, np):
    """Twenty tensors with ResNet-18 activation-gradient shapes, twenty whole chains dealt round-robin
    to a few streams (no host synchronisation in between): total algorithmic bytes / total time."""
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
    nstreams = max(1, min(args.streams, 4))
    streams = [torch.cuda.Stream() for _ in range(nstreams)]
    wss = []
    for _ in range(nstreams):   # a workspace per stream: calls that overlap must not share one
        w = torch.empty(lgn.lgn_workspace_bytes(0, lgn.LGN_F32), dtype=torch.uint8, device="cuda")
        lgn.lgn_workspace_init(w)
        wss.append(w)
    torch.cuda.synchronize()

    merged = args.launches == "merged"

    def one_step():
        for i, it in enumerate(items):
            c = it["cfg"]
            ws = wss[i % nstreams]
            with torch.cuda.stream(streams[i % nstreams]):
                if merged:
                    lgn.lgn_stats_solve(it["d"], c["sparsity"], lgn.LGN_F32, c["n_bits"], st=it["st"],
                                        p=it["pp"], f=it["fp"], ws=ws)
                else:
                    lgn.lgn_stats(it["d"], out=it["st"], ws=ws)
                    lgn.lgn_threshold(it["st"], c["sparsity"], lgn.LGN_F32, out=it["pp"])
                    lgn.lgn_fp_params(it["st"], c["n_bits"], out=it["fp"])
                lgn.lgn_prune_quantize_fused(it["d"], it["pp"], it["fp"], rounding, c["rng_seed"], 0,
                                             out=it["out"], out_kind=lgn.LGN_OUT_CODE8)

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    alg = total_n * 9
    value = alg / (ms * 1e-3) / 1e9
    log(f"[bench] c3: {len(items)} tensors, {total_n} elements, {ms:.4f} ms per step, {value:.0f} GB/s")
    print(json.dumps({
        "metric": "GB/s and % HBM peak for fused lognormal-stats+prune+FP-n quantize", "value": round(value, 1),
        "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32 (bit-level prune/quantize) + f64 (statistics, solver)", "data": "synthetic",
        "config": {"workload": "c3: 20 fp32 tensors with ResNet-18 activation-gradient shapes at batch 256, "
                               "per-tensor mu, sigma and target sparsity, 20 whole chains back to back "
                               f"({'2' if merged else '5'} launches each) on {nstreams} streams, "
                               f"{args.rounding} rounding, code8 output",
                   "elements": total_n, "algorithmic_bytes_per_step": alg,
                   "pct_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2)},
        "roofline": {"bound": "hbm", "kernel": "whole chain (%d launches)" % (40 if merged else 100), "achieved": round(value, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(value / HBM_PEAK_GBS, 4), "traffic": None},
        "cpu_baseline": None}), flush=True)


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

    if args.workload == "c3":
        return bench_c3(args, lgn, SI, torch, np)
    cfg = {"c1": SI.config_c1, "c2": SI.config_c2, "c4": SI.config_c4, "c5": SI.config_c5}[args.workload]()
    if args.n:
        cfg["n"] = args.n
    n = cfg["n"]
    sparsity = cfg.get("sparsity", 0.85)
    n_bits = cfg.get("n_bits", 6)
    rounding = lgn.LGN_ROUND_STOCHASTIC if args.rounding == "stochastic" else lgn.LGN_ROUND_NEAREST_EVEN
    out_kind = {"code8": lgn.LGN_OUT_CODE8, "packed": lgn.LGN_OUT_PACKED, "value": lgn.LGN_OUT_VALUE}[args.out_kind]
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
    log(f"[bench] generated {n} {cfg['dtype']} elements in {time.time() - t0:.1f}s")

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

    def one_step(ev=None):
        if ev:
            ev[0].record()
        if merged:
            lgn.lgn_stats_solve(d, sparsity, alpha_dt, n_bits, st=st, p=pp, f=fp, ws=ws)
            if ev:
                ev[1] = ev[2]  # no separate solver launches: one record serves both marks
        else:
            lgn.lgn_stats(d, out=st, ws=ws)
            if ev:
                ev[1].record()
            lgn.lgn_threshold(st, sparsity, alpha_dt, out=pp)
            lgn.lgn_fp_params(st, n_bits, out=fp)
        if ev:
            ev[2].record()
        lgn.lgn_prune_quantize_fused(d, pp, fp, rounding, seed, 0, out=out, out_kind=out_kind)
        if ev:
            ev[3].record()

    if args.copy_probe and cfg["dtype"] == SI.F32:
        probe = torch.empty_like(d)
        torch.mul(d, 1.0, out=probe)  # reads n*4 bytes, writes n*4 bytes
        torch.cuda.synchronize()
        del probe

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()

    every = max(1, args.event_every)
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] if k % every == 0 else None
              for k in range(args.steps)]
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for k in range(args.steps):
        one_step(events[k])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed * 1e3 / args.steps

    events = [e for e in events if e is not None]
    t_stats = sum(e[0].elapsed_time(e[1]) for e in events) / len(events)
    t_solve = sum(e[1].elapsed_time(e[2]) for e in events) / len(events)
    t_fused = sum(e[2].elapsed_time(e[3]) for e in events) / len(events)

    alg_bytes_step = n * (2 * in_bytes + out_bytes_per_elem)
    value = alg_bytes_step / (ms_per_step * 1e-3) / 1e9
    fused_bytes = n * (in_bytes + out_bytes_per_elem)
    stats_bytes = n * in_bytes
    fused_gbs = fused_bytes / (t_fused * 1e-3) / 1e9
    stats_gbs = stats_bytes / (t_stats * 1e-3) / 1e9
    hp, hf, hs = lgn.read_prune_params(pp), lgn.read_fp_params(fp), lgn.read_stats(st)
    log(f"[bench] mu={hs.mu:.5f} sigma={hs.sigma:.5f} nnz={hs.nnz} alpha={hp.alpha:.6e} "
        f"format=1-{hf.e_bits}-{hf.m_bits} s={hf.scale_exp}")
    log(f"[bench] per step {ms_per_step:.4f} ms: stats {t_stats:.4f} ms ({stats_gbs:.0f} GB/s), "
        f"solve {t_solve:.4f} ms, fused {t_fused:.4f} ms ({fused_gbs:.0f} GB/s)")

    # dominant kernel = the one that takes longer
    if t_fused >= t_stats:
        dom = dict(kernel="stream_kernel (fused prune+quantize)", achieved=fused_gbs,
                   bytes=fused_bytes, ms=t_fused)
    else:
        dom = dict(kernel="stats_solve_kernel" if merged else "stats_stage1", achieved=stats_gbs,
                   bytes=stats_bytes, ms=t_stats)
    traffic = MEASURED_TRAFFIC_BYTES.get((args.workload, args.out_kind, args.rounding, dom["kernel"]))
    roofline = {"bound": "hbm", "kernel": dom["kernel"], "achieved": round(dom["achieved"], 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(dom["achieved"] / HBM_PEAK_GBS, 4),
                "traffic": traffic, "algorithmic_bytes": int(dom["bytes"]),
                "avg_launch_ms": round(dom["ms"], 4),
                "other_kernels": {"stats_ms": round(t_stats, 4), "stats_GBps": round(stats_gbs, 1),
                                  "solve_ms": round(t_solve, 4), "fused_ms": round(t_fused, 4),
                                  "fused_GBps": round(fused_gbs, 1)}}

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
    if out_kind == lgn.LGN_OUT_CODE8 and not args.no_beyond:
        # a failure here must not take the headline line with it
        try:
            extras = measure_beyond()
            log(f"[bench] beyond the hot path: { {k: v['ms'] for k, v in extras.items() if isinstance(v, dict)} } ms")
        except Exception as e:  # noqa: BLE001
            extras = {"error": f"{type(e).__name__}: {e}"}
            log(f"[bench] beyond the hot path failed: {extras['error']}")
        # leave the structs as the timed step wrote them
        one_step()
        torch.cuda.synchronize()

    def measure_cpu_baseline():
        import oracle as O
        threads = O.max_threads()
        O.set_threads(threads)
        m = min(n, 1 << 28)  # the whole tensor for configuration 4: ~1 s on 16 cores
        sample = SI.make(cfg, n=m)
        reps = 2  # about 17 core-seconds in all
        t1 = time.perf_counter()
        for _ in range(reps):
            ost = O.stats(sample)
            op = O.threshold(ost, sparsity, O.F32 if in_bytes == 4 else O.BF16)
            of = O.fp_params(ost, n_bits)
            O.prune_quantize(sample, op.alpha, of.e_bits, of.m_bits, of.scale_exp,
                             O.ROUND_STOCHASTIC if rounding == lgn.LGN_ROUND_STOCHASTIC else O.ROUND_NEAREST_EVEN,
                             seed, 0, {lgn.LGN_OUT_CODE8: O.OUT_CODE8, lgn.LGN_OUT_PACKED: O.OUT_PACKED,
                                       lgn.LGN_OUT_VALUE: O.OUT_VALUE}[out_kind])
        dt = (time.perf_counter() - t1) / reps
        return {"value": round(m * (2 * in_bytes + out_bytes_per_elem) / dt / 1e9, 3), "unit": "GB/s",
                "cores": threads, "kind": "oracle",
                "sample": f"first {m} elements of the same tensor, whole chain, {reps} repetitions of {dt:.2f} s"}

    cpu = None
    if not args.no_cpu_baseline:
        try:  # a failure here must not take the headline line with it
            cpu = measure_cpu_baseline()
        except Exception as e:  # noqa: BLE001
            cpu = {"value": None, "unit": "GB/s", "cores": 0, "kind": "oracle", "sample": f"failed: {type(e).__name__}: {e}"}
        log(f"[bench] cpu oracle: {cpu}")

    line = {
        "metric": "GB/s and % HBM peak for fused lognormal-stats+prune+FP-n quantize",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u32 (bit-level prune/quantize) + f64 (statistics, solver)",
        "data": "synthetic",
        "config": {"workload": f"{cfg['name']}: {n} {cfg['dtype']} elements, zeros {cfg['zero_frac']}, "
                               f"ln|g|~N({cfg['mu']},{cfg['sigma']}^2); stats+threshold(S={sparsity})"
                               f"+FP{n_bits} format+fused prune/quantize, {args.rounding} rounding, "
                               f"{args.out_kind} output, "
                               + ("2 launches (stats+solvers merged, fused)" if merged else "5 launches"),
                   "elements": n, "elements_per_s": round(n / (ms_per_step * 1e-3)),
                   "algorithmic_bytes_per_step": int(alg_bytes_step),
                   "pct_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2)},
        "roofline": roofline, "cpu_baseline": cpu, "beyond_hot_path": extras,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
