#!/usr/bin/env python3
"""Benchmark of the expanded W4A4 linear layer on one MI355X.

One step = one pass of the whole hot path (zero-pad + Hadamard rotation + per-token int4
quantization + int4 GEMM + dequantising epilogue) over one batch of synthetic activations
that already sit in HBM.  Prints one JSON line.
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


def _event_ms(fn, iters: int) -> float:
    """Average milliseconds per call of fn over `iters` back-to-back launches (HIP events on the
    stream the library launches on: torch's current stream)."""
    import torch
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for _ in range(iters):
        fn()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / iters


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
    # grow the token sample until one pass takes a few seconds, capped at the full batch
    tokens = min(sp.T, 128)
    while True:
        t0 = time.perf_counter()
        oracle.expanded_linear(wl.x[:tokens], sp.d_e, wl.qw, wl.sw)
        dt = time.perf_counter() - t0
        if tokens >= sp.T or dt * 4 > budget_s:
            break
        tokens = min(sp.T, tokens * 4)
    ops = 2.0 * tokens * sp.d_e * sp.N
    return {"value": ops / dt / 1e12, "unit": "TOPS", "cores": int(threads), "kind": "oracle",
            "sample": f"{tokens} of {sp.T} tokens of {sp.name}, all {sp.N} outputs, one pass, {dt:.2f} s",
            "host_cpus": len(os.sched_getaffinity(0))}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="C2", help="C1..C5 (default C2, the configuration the metric is quoted on)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stages", action="store_true", help="also time each stage and every other workload")
    ap.add_argument("--mxfp4", action="store_true",
                    help="also time the MXFP4 variant of the layer (the paper's second quantization setting)")
    ap.add_argument("--probe-copy", action="store_true",
                    help="also run the library's plain 1 GiB copy kernel (the known-size dispatch that calibrates "
                         "the profiler's FETCH_SIZE / WRITE_SIZE counters)")
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
        qw = pme.pack_int4_codes(torch.from_numpy(wl.qw)).cuda()
        sw = torch.from_numpy(wl.sw).cuda()
        y = torch.empty((sp.T, sp.N), dtype=torch.bfloat16, device="cuda")
        ws = torch.empty((max(256, pme.workspace_bytes(sp.T, sp.d, sp.d_e, sp.N)),), dtype=torch.uint8, device="cuda")
        qx = torch.empty((sp.T, sp.d_e // 2), dtype=torch.uint8, device="cuda")
        sx = torch.empty((sp.T,), dtype=torch.float32, device="cuda")
        return wl, dict(x=x, qw=qw, sw=sw, y=y, ws=ws, qx=qx, sx=sx)

    def stage_times(sp, b, iters):
        pme.hadamard_expand_quant(b["x"], sp.d_e, b["qx"], b["sx"])
        t_rot = _event_ms(lambda: pme.hadamard_expand_quant(b["x"], sp.d_e, b["qx"], b["sx"]), iters)
        t_gemm = _event_ms(lambda: pme.w4a4_gemm(b["qx"], b["sx"], b["qw"], b["sw"], b["y"]), iters)
        return t_rot, t_gemm

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
    ms = start.elapsed_time(stop) / args.steps

    ops = gemm_ops(sp)
    t_rot, t_gemm = stage_times(sp, b, max(20, args.steps))
    decode = sp.T <= 32
    if decode:
        # memory-bound shape: the whole layer is priced against HBM bandwidth
        layer_bytes = sp.N * sp.d_e // 2 + 4 * sp.N + sp.T * sp.d * 2 + 2 * sp.T * sp.N
        ach = layer_bytes / (t_gemm * 1e-3) / 1e9
        roof = {"bound": "hbm", "kernel": "w4a4_gemm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": ach / PEAK_HBM_GBS, "traffic": None, "avg_launch_us": t_gemm * 1e3}
    else:
        ach = ops / (t_gemm * 1e-3) / 1e12
        roof = {"bound": "mfma", "kernel": "w4a4_gemm", "achieved": ach, "peak": PEAK_INT8_TOPS, "unit": "TFLOP/s",
                "frac": ach / PEAK_INT8_TOPS, "traffic": None, "avg_launch_us": t_gemm * 1e3,
                "algorithmic_ops": ops, "algorithmic_bytes": algorithmic_bytes_gemm(sp),
                "note": "int8 MFMA ops (2 per multiply-add) over the expanded d_e"}
    traffic_file = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(traffic_file):
        with open(traffic_file) as f:
            tr = json.load(f).get(sp.name, {}).get("w4a4_gemm")
        if tr:
            # HBM bytes per launch from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE), calibrated by the
            # library's 1 GiB copy kernel; see profiles/expanded_linear_<workload>.md
            roof["traffic"] = tr["total_bytes"]
            roof["traffic_detail"] = tr
    rot_bytes = algorithmic_bytes_rotate_quant(sp)
    rot_gbs = rot_bytes / (t_rot * 1e-3) / 1e9

    out = {
        "metric": "expanded W4A4 linear TOPS (prefill) + rotate/quant HBM GB/s (decode), 1 MI355X",
        "value": ops / (ms * 1e-3) / 1e12,
        "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "wall_ms_per_step": wall_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"{sp.name}: T={sp.T} d={sp.d} d_e={sp.d_e} N={sp.N} in={sp.in_dtype}",
                   "step": "pme_expanded_linear (rotate+quantize, then W4A4 GEMM with bf16 epilogue)"},
        "roofline": roof,
        "rotate_quant": {"bound": "hbm", "kernel": "hadamard_expand_quant", "achieved": rot_gbs, "peak": PEAK_HBM_GBS,
                         "unit": "GB/s", "frac": rot_gbs / PEAK_HBM_GBS, "avg_launch_us": t_rot * 1e3,
                         "algorithmic_bytes": rot_bytes},
    }
    if args.stages:
        others = {}
        for name in SPECS:
            if name == sp.name:
                continue
            wl2, b2 = prepare(name)
            s2 = wl2.spec
            for _ in range(5):
                pme.expanded_linear(b2["x"], s2.d_e, b2["qw"], b2["sw"], b2["y"], b2["ws"])
            it = 50
            t_all = _event_ms(lambda: pme.expanded_linear(b2["x"], s2.d_e, b2["qw"], b2["sw"], b2["y"], b2["ws"]), it)
            tr, tg = stage_times(s2, b2, it)
            others[name] = {"layer_us": t_all * 1e3, "layer_tops": gemm_ops(s2) / (t_all * 1e-3) / 1e12,
                            "rotate_us": tr * 1e3, "rotate_gbs": algorithmic_bytes_rotate_quant(s2) / (tr * 1e-3) / 1e9,
                            "gemm_us": tg * 1e3, "gemm_tops": gemm_ops(s2) / (tg * 1e-3) / 1e12,
                            "gemm_gbs": algorithmic_bytes_gemm(s2) / (tg * 1e-3) / 1e9}
            del wl2, b2
            torch.cuda.empty_cache()
        out["other_workloads"] = others
    if args.mxfp4:
        wt = torch.randn((sp.N, sp.d), device="cuda").to(torch.bfloat16)     # any weights: timing only
        qw4, ew4 = pme.hadamard_expand_quant_mxfp4(wt, sp.d_e)
        qx4, ex4 = pme.hadamard_expand_quant_mxfp4(b["x"], sp.d_e)
        for _ in range(5):
            pme.expanded_linear_mxfp4(b["x"], sp.d_e, qw4, ew4, b["y"], b["ws"])
        it = max(20, args.steps)
        t_l = _event_ms(lambda: pme.expanded_linear_mxfp4(b["x"], sp.d_e, qw4, ew4, b["y"], b["ws"]), it)
        t_r = _event_ms(lambda: pme.hadamard_expand_quant_mxfp4(b["x"], sp.d_e), it)
        t_g = _event_ms(lambda: pme.mxfp4_gemm(qx4, ex4, qw4, ew4, b["y"]), it)
        out["mxfp4"] = {"layer_us": t_l * 1e3, "layer_tflops": ops / (t_l * 1e-3) / 1e12, "rotate_quant_us": t_r * 1e3,
                        "gemm_us": t_g * 1e3, "gemm_tflops": ops / (t_g * 1e-3) / 1e12, "gemm_peak_tflops": 10100.0,
                        "gemm_frac": ops / (t_g * 1e-3) / 1e12 / 10100.0}
    if args.probe_copy:
        src = torch.empty((1 << 30,), dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            pme.probe_copy(src, dst)
        t_copy = _event_ms(lambda: pme.probe_copy(src, dst), 5)
        out["probe_copy"] = {"bytes_read": 1 << 30, "bytes_written": 1 << 30, "us": t_copy * 1e3,
                             "gbs": 2 * (1 << 30) / (t_copy * 1e-3) / 1e9}
        del src, dst
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = _cpu_baseline(wl)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
