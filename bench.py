#!/usr/bin/env python3
"""Benchmark of the expanded W4A4 linear layer on one MI355X.

One step = one pass of the whole hot path (zero-pad + Hadamard rotation + per-token int4
quantization + int4 GEMM + dequantising epilogue) over one batch of synthetic activations
that already sit in HBM.  Prints one JSON line.

The headline workload is C5 (4096 tokens, 14336 -> 15360, 4096 outputs: the largest single-GPU
configuration); the same line carries a record per other workload (C2, C3, and the decode shape C4,
whose layer GB/s is the metric's decode half) and the measured ceilings the fractions are also
quoted against.
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

PEAK_INT8_TOPS = 5000.0      # MI355X dense int8 MFMA, published
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E, published


def _event_ms(fn, iters: int, repeats: int = 1) -> float:
    """Milliseconds per call of fn: `iters` back-to-back launches between two HIP events (recorded on the
    stream the library launches on, torch's current stream); the median over `repeats` such runs."""
    import torch
    times = []
    for _ in range(repeats):
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        start.record()
        for _ in range(iters):
            fn()
        stop.record()
        torch.cuda.synchronize()
        times.append(start.elapsed_time(stop) / iters)
    times.sort()
    return times[len(times) // 2]


def _graph_ms(fn, iters: int, repeats: int = 5):
    """Milliseconds per call of fn with the host out of the way: `iters` launches captured into one HIP graph,
    the graph replayed `repeats` times between HIP events, median.  For kernels of a few microseconds the
    Python call itself (about 8 us) is otherwise what gets timed.  None if the capture fails."""
    import torch
    try:
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()                                     # warm the shape on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=side):
            for _ in range(iters):
                fn()
        for _ in range(3):                           # untimed: clocks and caches settle before the timed replays
            g.replay()
        torch.cuda.synchronize()
        times = []
        for _ in range(repeats):
            start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            start.record()
            g.replay()
            stop.record()
            torch.cuda.synchronize()
            times.append(start.elapsed_time(stop) / iters)
        times.sort()
        return times[len(times) // 2]
    except Exception as ex:                          # noqa: BLE001 - report and fall back to the plain loop
        print(f"bench: HIP graph timing unavailable ({ex})", file=sys.stderr)
        return None


def _cpu_baseline(wl, budget_s: float = 20.0):
    """The CPU oracle as it stands, timed on the host cores on a bounded sample of the workload."""
    import numpy as np
    import oracle
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    sp = wl.spec

    def timed(tokens):
        t0 = time.perf_counter()
        oracle.expanded_linear(wl.x[:tokens], sp.d_e, wl.qw, wl.sw)
        return time.perf_counter() - t0

    # grow the token sample until one pass takes a few seconds, capped at the full batch
    tokens = min(sp.T, 128)
    while True:
        dt = timed(tokens)
        if tokens >= sp.T or dt * 4 > budget_s * 0.6:
            break
        tokens = min(sp.T, tokens * 4)
    # a workload the oracle finishes quickly is passed over several times (about 10 s of work in all)
    passes = max(1, min(10, int(budget_s * 0.5 / max(dt, 1e-3))))
    if passes > 1:
        dt = sum(timed(tokens) for _ in range(passes)) / passes
    ops = 2.0 * tokens * sp.d_e * sp.N
    out = {"value": ops / dt / 1e12, "unit": "TOPS", "cores": int(threads), "kind": "oracle",
           "sample": f"{tokens} of {sp.T} tokens of {sp.name}, all {sp.N} outputs, mean of {passes} pass(es) of {dt:.2f} s",
           "host_cpus": len(os.sched_getaffinity(0))}
    # the same oracle held to one thread, on a sample sized from the rate just seen
    try:
        from threadpoolctl import threadpool_limits
        t1 = max(16, min(tokens, int(tokens * (budget_s * 0.3) / max(dt * threads, 1e-3))))
        with threadpool_limits(limits=1):
            dt1 = timed(t1)
        out["single_thread"] = {"value": 2.0 * t1 * sp.d_e * sp.N / dt1 / 1e12, "unit": "TOPS", "cores": 1,
                                "sample": f"{t1} tokens, one pass, {dt1:.2f} s"}
    except ImportError:
        pass
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--replays", type=int, default=5,
                    help="timed replays of the HIP graph of K steps; ms_per_step is the median replay / K")
    ap.add_argument("--workload", default="C5", help="C1..C5 (default C5, the largest single-GPU configuration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the records of the other workloads (profiling runs)")
    ap.add_argument("--stages", action="store_true", help="accepted for compatibility: the per-workload stage records are always printed")
    ap.add_argument("--mxfp4", action="store_true",
                    help="also time the MXFP4 variant of the layer (the paper's second quantization setting)")
    ap.add_argument("--asym", action="store_true",
                    help="also time the layer with per-token asymmetric int4 activations (the paper's W4A4 setting)")
    ap.add_argument("--probe-copy", action="store_true",
                    help="time the library's plain 1 GiB copy kernel with 5 launches instead of 2 (the known-size "
                         "dispatch that calibrates the profiler's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--paper-sizes", action="store_true",
                    help="also time the layer at every expanded size of the paper's Tables 1-2 (down projections of the "
                         "1B- and 8B-shaped models: 8192 -> 8704 .. 12288 with N = 2048, 14336 -> 15360 .. 22016 with "
                         "N = 4096; 2048 tokens, random weights quantized by the library's own weight-side call)")
    ap.add_argument("--no-graph", action="store_true",
                    help="time the plain Python loop of library calls instead of a HIP graph replay of it")
    ap.add_argument("--no-probes", action="store_true",
                    help="skip the measured ceilings (streaming copy and read, back-to-back matrix-core instructions, launch floor)")
    ap.add_argument("--cold", action="store_true",
                    help="also time the layer cycling through distinct operand sets larger than twice the 256 MB "
                         "last-level cache, so that nothing is served from cache")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import torch
    import paper_2503_17513_amd as pme
    from workloads import SPECS, algorithmic_bytes_gemm, algorithmic_bytes_rotate_quant, gemm_ops, make_workload

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    def prepare(name):
        wl = make_workload(name)
        sp = wl.spec
        x = torch.from_numpy(wl.x)
        if sp.in_dtype == "bf16":
            x = x.to(torch.bfloat16)
        x = x.cuda()
        qw = pme.pack_int4(torch.from_numpy(wl.qw))
        sw = torch.from_numpy(wl.sw).cuda()
        y = torch.empty((sp.T, sp.N), dtype=torch.bfloat16, device="cuda")
        ws = torch.empty((max(256, pme.workspace_bytes(sp.T, sp.d, sp.d_e, sp.N)),), dtype=torch.uint8, device="cuda")
        qx = torch.empty((sp.T, sp.d_e // 2), dtype=torch.uint8, device="cuda")
        sx = torch.empty((sp.T,), dtype=torch.float32, device="cuda")
        return wl, dict(x=x, qw=qw, sw=sw, y=y, ws=ws, qx=qx, sx=sx)

    def timed(fn, iters):
        if not args.no_graph:
            t = _graph_ms(fn, iters)
            if t is not None:
                return t
        return _event_ms(fn, iters, 5)

    def stage_times(sp, b, iters):
        pme.hadamard_expand_quant(b["x"], sp.d_e, b["qx"], b["sx"])
        rot = lambda: pme.hadamard_expand_quant(b["x"], sp.d_e, b["qx"], b["sx"])
        gemm = lambda: pme.w4a4_gemm(b["qx"], b["sx"], b["qw"], b["sw"], b["y"])
        return timed(rot, iters), timed(gemm, iters)

    def decode_layer_bytes(sp):
        return sp.N * sp.d_e // 2 + 4 * sp.N + sp.T * sp.d * 2 + 2 * sp.T * sp.N

    traffic_file = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    stored_traffic = {}
    if os.path.exists(traffic_file):
        with open(traffic_file) as f:
            stored_traffic = json.load(f)

    def traffic_of(key, stage, kernel_now):
        """HBM bytes per launch from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE, calibrated by the library's
        1 GiB copy kernel; profiles/expanded_linear_<workload>.md), only if they were taken on the kernel
        configuration that is being timed now: the stored record names the instantiation it belongs to."""
        tr = stored_traffic.get(key, {}).get(stage)
        if not tr:
            return None, None
        stored = tr.get("kernel", "")
        # (the weight-streaming kernels are named without their template arguments by pme_gemm_plan)
        if kernel_now is not None and stored != kernel_now and not stored.startswith(kernel_now + "<"):
            return None, f"stored profile is of {tr.get('kernel')}, this run dispatches {kernel_now}: not used"
        return tr["total_bytes"], tr

    def workload_record(sp, b, t_layer, iters):
        """Per-kernel times and roofline fractions of one workload (published peaks)."""
        t_rot, t_gemm = stage_times(sp, b, iters)
        ops = gemm_ops(sp)
        rot_bytes = algorithmic_bytes_rotate_quant(sp)
        rec = {"T": sp.T, "d": sp.d, "d_e": sp.d_e, "N": sp.N,
               "layer_us": t_layer * 1e3, "layer_tops": ops / (t_layer * 1e-3) / 1e12,
               "rotate_us": t_rot * 1e3, "rotate_gbs": rot_bytes / (t_rot * 1e-3) / 1e9,
               "rotate_frac_hbm": rot_bytes / (t_rot * 1e-3) / 1e9 / PEAK_HBM_GBS,
               "gemm_us": t_gemm * 1e3, "gemm_kernel": pme.gemm_plan(sp.T, sp.d_e, sp.N),
               "gemm_tops": ops / (t_gemm * 1e-3) / 1e12, "gemm_gbs": algorithmic_bytes_gemm(sp) / (t_gemm * 1e-3) / 1e9}
        if sp.T <= 32:
            lb = decode_layer_bytes(sp)
            rec.update({"bound": "hbm", "layer_bytes": lb, "layer_gbs": lb / (t_layer * 1e-3) / 1e9,
                        "layer_frac_hbm": lb / (t_layer * 1e-3) / 1e9 / PEAK_HBM_GBS,
                        "gemm_frac_hbm": lb / (t_gemm * 1e-3) / 1e9 / PEAK_HBM_GBS})
        else:
            rec.update({"bound": "mfma", "gemm_frac_int8_peak": ops / (t_gemm * 1e-3) / 1e12 / PEAK_INT8_TOPS,
                        "layer_frac_int8_peak": ops / (t_layer * 1e-3) / 1e12 / PEAK_INT8_TOPS})
        return rec, t_rot, t_gemm

    def measured_ceilings(fp4: bool, copy_launches: int):
        """The microbenchmarks the roofline fractions are also quoted against."""
        res = {}
        src = torch.empty((1 << 30,), dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        pme.probe_copy(src, dst)
        t_copy = _event_ms(lambda: pme.probe_copy(src, dst), copy_launches)
        res["probe_copy"] = {"bytes_read": 1 << 30, "bytes_written": 1 << 30, "us": t_copy * 1e3,
                             "gbs": 2 * (1 << 30) / (t_copy * 1e-3) / 1e9}
        del dst
        sink = torch.zeros((2048 * 256,), dtype=torch.int32, device="cuda")
        pme.probe_read(src, sink)
        t_read = _event_ms(lambda: pme.probe_read(src, sink), max(2, copy_launches))
        res["probe_read"] = {"bytes_read": 1 << 30, "bytes_written": sink.numel() * 4, "us": t_read * 1e3,
                             "gbs": (1 << 30) / (t_read * 1e-3) / 1e9}
        del src
        torch.cuda.empty_cache()
        # a chain of kernels that do nothing, captured in a graph like the timed steps: microseconds per dependent launch
        t_launch = _graph_ms(pme.probe_launch, 200)
        if t_launch is not None:
            res["probe_launch"] = {"us_per_dependent_launch_in_a_graph": t_launch * 1e3}
        # near-constant operands reach the published peak; pseudo-random codes (the bytes a GEMM really feeds the
        # pipe) run slower, the matrix pipe being power-limited: both ceilings are printed
        kinds = ((0, "probe_mfma_int8"), (2, "probe_mfma_int8_random_codes"))
        if fp4:
            kinds += ((1, "probe_mfma_fp4"), (3, "probe_mfma_fp4_random_codes"))
        for kind, key in kinds:
            iters = 20000
            n_ops = pme.probe_mfma(kind, sink, iters)
            t = _event_ms(lambda: pme.probe_mfma(kind, sink, iters), 3)
            res[key] = {"ops_per_launch": n_ops, "us": t * 1e3, "tops": n_ops / (t * 1e-3) / 1e12}
        return res

    wl, b = prepare(args.workload)
    sp = wl.spec
    step = lambda: pme.expanded_linear(b["x"], sp.d_e, b["qw"], b["sw"], b["y"], b["ws"])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record()
    for _ in range(args.steps):
        step()
    stop.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    plain_ms = start.elapsed_time(stop) / args.steps
    # The same K steps captured once into a HIP graph and replayed: what a serving loop would do, and it
    # takes the host's launch path (a ctypes call and two kernel launches per step) out of the timed region.
    # Three untimed replays, then `replays` timed replays of exactly K steps each; the median replay is reported.
    ms, launch = plain_ms, "plain loop of K library calls"
    if not args.no_graph:
        g_ms = _graph_ms(step, args.steps, max(1, args.replays))
        if g_ms is not None:
            ms, launch = g_ms, f"HIP graph of K library calls, median of {max(1, args.replays)} timed replays"

    ops = gemm_ops(sp)
    iters = 100                                      # launches per graph for the per-kernel times, whatever K is
    rec, t_rot, t_gemm = workload_record(sp, b, ms, iters)
    decode = sp.T <= 32
    kernel_now = rec["gemm_kernel"]
    if decode:
        # memory-bound shape: the GEMM (the dominant kernel) is priced against HBM bandwidth on the layer's bytes
        layer_bytes = decode_layer_bytes(sp)
        ach = layer_bytes / (t_gemm * 1e-3) / 1e9
        roof = {"bound": "hbm", "kernel": kernel_now, "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": ach / PEAK_HBM_GBS, "traffic": None, "avg_launch_us": t_gemm * 1e3, "algorithmic_bytes": layer_bytes}
    else:
        ach = ops / (t_gemm * 1e-3) / 1e12
        roof = {"bound": "mfma", "kernel": kernel_now, "achieved": ach, "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                "frac": ach / PEAK_INT8_TOPS, "traffic": None, "avg_launch_us": t_gemm * 1e3,
                "algorithmic_ops": ops, "algorithmic_bytes": algorithmic_bytes_gemm(sp),
                "note": "int8 MFMA ops (2 per multiply-add) over the expanded d_e; dtype peak: int8 dense 5.0 POP/s"}
    tr_bytes, tr_detail = traffic_of(sp.name, "w4a4_gemm", kernel_now)
    roof["traffic"] = tr_bytes
    if isinstance(tr_detail, dict):
        roof["traffic_detail"] = tr_detail
    elif tr_detail:
        roof["traffic_note"] = tr_detail
    rot_bytes = algorithmic_bytes_rotate_quant(sp)
    rot_gbs = rot_bytes / (t_rot * 1e-3) / 1e9

    probes = None
    if not args.no_probes:
        probes = measured_ceilings(args.mxfp4, 5 if args.probe_copy else 2)
        if decode:
            roof["measured_peak"] = probes["probe_read"]["gbs"]
        else:
            roof["measured_peak"] = probes["probe_mfma_int8"]["tops"]
            roof["measured_peak_random_codes"] = probes["probe_mfma_int8_random_codes"]["tops"]
            roof["frac_of_measured_random_codes"] = roof["achieved"] / roof["measured_peak_random_codes"]
        roof["frac_of_measured"] = roof["achieved"] / roof["measured_peak"]

    out = {
        "metric": "expanded W4A4 linear TOPS (prefill) + rotate/quant HBM GB/s (decode), 1 MI355X",
        "value": ops / (ms * 1e-3) / 1e12,
        "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "plain_loop_ms_per_step": plain_ms, "wall_ms_per_step": wall_ms,
        # the same time priced at the unexpanded layer's 2 T d N operations (what the expansion costs in useful work)
        "effective_tops_unexpanded": 2.0 * sp.T * sp.d * sp.N / (ms * 1e-3) / 1e12,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"{sp.name}: T={sp.T} d={sp.d} d_e={sp.d_e} N={sp.N} in={sp.in_dtype}",
                   "step": "pme_expanded_linear (rotate+quantize, then W4A4 GEMM with bf16 epilogue)",
                   "launch": launch, "replays": max(1, args.replays)},
        "roofline": roof,
        "rotate_quant": {"bound": "hbm", "kernel": "hadamard_expand_quant", "achieved": rot_gbs, "peak": PEAK_HBM_GBS,
                         "unit": "GB/s", "frac": rot_gbs / PEAK_HBM_GBS, "avg_launch_us": t_rot * 1e3,
                         "algorithmic_bytes": rot_bytes},
        "workloads": {sp.name: rec},
    }
    tr_rot, _ = traffic_of(sp.name, "hadamard_expand_quant", None)
    out["rotate_quant"]["traffic"] = tr_rot
    if not args.no_others:
        for name in SPECS:
            if name in (sp.name, "C1"):
                continue
            wl2, b2 = prepare(name)
            s2 = wl2.spec
            layer2 = lambda: pme.expanded_linear(b2["x"], s2.d_e, b2["qw"], b2["sw"], b2["y"], b2["ws"])
            for _ in range(10):
                layer2()
            it = 100
            rec2, _, _ = workload_record(s2, b2, timed(layer2, it), it)
            out["workloads"][name] = rec2
            del wl2, b2
            torch.cuda.empty_cache()
    # the metric's decode half: the memory-bound shape's whole layer against HBM bandwidth
    for name, r in out["workloads"].items():
        if r.get("bound") == "hbm":
            out["decode"] = {"workload": name, "metric": "layer HBM GB/s (weights + activations + outputs once)",
                             "value": r["layer_gbs"], "unit": "GB/s", "frac": r["layer_frac_hbm"], "layer_us": r["layer_us"],
                             "rotate_us": r["rotate_us"], "gemm_us": r["gemm_us"], "algorithmic_bytes": r["layer_bytes"]}
    if args.paper_sizes:
        rows = []
        for d, N, sizes in ((8192, 2048, (8704, 8960, 9728, 10240, 12288)), (14336, 4096, (15360, 18432, 19968, 22016))):
            T = 2048
            xs = (torch.randn((T, d), device="cuda") * (1 + 20 * (torch.rand(d, device="cuda") < 0.01))).to(torch.bfloat16)
            wt = torch.randn((N, d), device="cuda").to(torch.bfloat16)
            for d_e in sizes:
                qw_, sw_ = pme.expand_quantize_weights(wt, d_e)
                y_ = torch.empty((T, N), dtype=torch.bfloat16, device="cuda")
                ws_ = torch.empty((pme.workspace_bytes(T, d, d_e, N),), dtype=torch.uint8, device="cuda")
                qx_ = torch.empty((T, d_e // 2), dtype=torch.uint8, device="cuda")
                sx_ = torch.empty((T,), dtype=torch.float32, device="cuda")
                layer_ = lambda: pme.expanded_linear(xs, d_e, qw_, sw_, y_, ws_)
                rot_ = lambda: pme.hadamard_expand_quant(xs, d_e, qx_, sx_)
                for _ in range(5):
                    layer_()
                rot_()
                tl = _graph_ms(layer_, 30) or _event_ms(layer_, 30, 3)
                tr = _graph_ms(rot_, 30) or _event_ms(rot_, 30, 3)
                b_, k_ = pme.factor_order(d_e)
                rows.append({"T": T, "d": d, "d_e": d_e, "N": N, "ratio": round(d_e / d, 3), "order": f"{b_} x 2^{k_}",
                             "layer_us": tl * 1e3, "rotate_quant_us": tr * 1e3,
                             "layer_tops": 2.0 * T * d_e * N / (tl * 1e-3) / 1e12})
                del qw_, sw_, y_, ws_, qx_, sx_
            del xs, wt
            torch.cuda.empty_cache()
        out["paper_sizes"] = rows
    if args.asym:
        wsum = pme.weight_rowsum(b["qw"])
        zx = torch.empty((sp.T,), dtype=torch.int32, device="cuda")
        layer_a = lambda: pme.expanded_linear_asym(b["x"], sp.d_e, b["qw"], b["sw"], wsum, b["y"], b["ws"])
        rot_a = lambda: pme.hadamard_expand_quant_asym(b["x"], sp.d_e, b["qx"], b["sx"], zx)
        gemm_a = lambda: pme.w4a4_gemm_asym(b["qx"], b["sx"], zx, b["qw"], b["sw"], wsum, b["y"])
        for f in (layer_a, rot_a, gemm_a):
            for _ in range(3):
                f()
        t_l, t_r, t_g = (timed(f, iters) for f in (layer_a, rot_a, gemm_a))
        out["asym"] = {"layer_us": t_l * 1e3, "layer_tops": ops / (t_l * 1e-3) / 1e12, "rotate_quant_us": t_r * 1e3,
                       "gemm_us": t_g * 1e3, "gemm_tops": ops / (t_g * 1e-3) / 1e12,
                       "gemm_kernel": pme.gemm_plan(sp.T, sp.d_e, sp.N, 1)}
    if args.mxfp4:
        wt = torch.randn((sp.N, sp.d), device="cuda").to(torch.bfloat16)     # any weights: timing only
        qw4, ew4 = pme.hadamard_expand_quant_mxfp4(wt, sp.d_e)
        qx4, ex4 = pme.hadamard_expand_quant_mxfp4(b["x"], sp.d_e)
        for _ in range(5):
            pme.expanded_linear_mxfp4(b["x"], sp.d_e, qw4, ew4, b["y"], b["ws"])
        layer_m = lambda: pme.expanded_linear_mxfp4(b["x"], sp.d_e, qw4, ew4, b["y"], b["ws"])
        rot_m = lambda: pme.hadamard_expand_quant_mxfp4(b["x"], sp.d_e, qx4, ex4)
        gemm_m = lambda: pme.mxfp4_gemm(qx4, ex4, qw4, ew4, b["y"])
        t_l, t_r, t_g = (timed(f, iters) for f in (layer_m, rot_m, gemm_m))
        mx_kernel = pme.gemm_plan(sp.T, sp.d_e, sp.N, 2)
        out["mxfp4"] = {"layer_us": t_l * 1e3, "layer_tflops": ops / (t_l * 1e-3) / 1e12, "rotate_quant_us": t_r * 1e3,
                        "gemm_us": t_g * 1e3, "gemm_kernel": mx_kernel, "gemm_tflops": ops / (t_g * 1e-3) / 1e12,
                        "gemm_peak_tflops": 10100.0, "gemm_frac": ops / (t_g * 1e-3) / 1e12 / 10100.0, "gemm_traffic": None}
        out["mxfp4"]["gemm_traffic"], _ = traffic_of(sp.name + "_mxfp4", "w4a4_gemm", mx_kernel)
    if probes:
        # rotate + quantize reads four bytes for each one it writes: the read-only stream is its yardstick
        out["rotate_quant"]["measured_peak"] = probes["probe_read"]["gbs"]
        out["rotate_quant"]["frac_of_measured"] = rot_gbs / probes["probe_read"]["gbs"]
        out["rotate_quant"]["frac_of_measured_copy"] = rot_gbs / probes["probe_copy"]["gbs"]
        out["measured_ceilings"] = probes
        if "decode" in out and "probe_launch" in probes:
            # two dependent launches per layer: what two kernels that do nothing cost in the same kind of graph
            out["decode"]["two_empty_launches_us"] = 2 * probes["probe_launch"]["us_per_dependent_launch_in_a_graph"]
        if args.mxfp4 and "probe_mfma_fp4" in probes:
            out["mxfp4"]["gemm_measured_peak_tflops"] = probes["probe_mfma_fp4"]["tops"]
            out["mxfp4"]["gemm_measured_peak_random_codes_tflops"] = probes["probe_mfma_fp4_random_codes"]["tops"]
    if args.cold:
        per_set = (b["x"].numel() * b["x"].element_size() + b["qw"].numel() + b["y"].numel() * 2 + b["ws"].numel())
        nsets = max(2, -(-(600 << 20) // per_set))
        sets = [b] + [dict(x=b["x"].clone(), qw=b["qw"].clone(), sw=b["sw"], y=torch.empty_like(b["y"]),
                           ws=torch.empty_like(b["ws"])) for _ in range(nsets - 1)]
        state = {"i": 0}

        def cold_step():
            c = sets[state["i"] % nsets]
            state["i"] += 1
            pme.expanded_linear(c["x"], sp.d_e, c["qw"], c["sw"], c["y"], c["ws"])

        for _ in range(nsets):
            cold_step()
        t_cold = _event_ms(cold_step, nsets * max(2, 200 // nsets), 3)
        out["cold"] = {"layer_us": t_cold * 1e3, "layer_tops": ops / (t_cold * 1e-3) / 1e12, "operand_sets": nsets,
                       "bytes_per_set": per_set}
        del sets
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = _cpu_baseline(wl)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
