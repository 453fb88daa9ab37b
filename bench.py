#!/usr/bin/env python3
"""Benchmark of the TurboQuant hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input that
is already resident in HBM:  tq_quantize_prod over every key  ->
tq_dequantize of every code  ->  tq_score of every query head against the
codes of its KV head (query rotation included).  The default workload is the
KV-cache configuration (8 KV heads x 16384 bf16 keys, d = 128, b = 3 =
2-bit MSE stage + 1-bit QJL, 32 query heads, GQA 4:1).

Prints ONE JSON line.  `value` is vectors quantised per second through the
whole step.  `rooflines` prices every call of the step against the roofline
that bounds it, from its ALGORITHMIC flops or bytes and its HIP-event time on
the launch stream inside the timed region; `roofline` is the entry of the call
that takes the largest share of the step.  A contraction that the library
feeds to the bf16 matrix cores as pieces of its fp32 factors is priced
against the bf16 peak on its algorithmic flops (`frac`); the share of the
peak that the executed piece products reach (`executed_frac`) and the
fp32-equivalent rate are given beside it, and `fp32_mfma_reference` times the
same calls with TQ_FLAG_FP32_MFMA (every contraction on fp32 MFMA).
`d1536` is the same step on the d = 1536 configuration (C4: 10^6 database
vectors, 1000 queries, top-10), a few timed steps after the headline region.
`cpu_baseline` is the CPU oracle on a bounded sample of the headline workload
(a reported baseline, not a target).
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

PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_BF16_MFMA_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0


def build_workload(name: str):
    import numpy as np
    import torch

    import paper_2504_19874_amd as tq
    import workloads as W

    cfg = W.CONFIGS[name]
    prod = cfg.kind == "prod"
    S = W.sketch_matrix(cfg.d, cfg.seed_s) if prod else None
    p = tq.make_params(cfg.d, cfg.bits_mse, W.gaussian_matrix(cfg.d, cfg.seed_pi), S)
    n = cfg.n * cfg.n_groups
    if cfg.in_dtype == "bf16":
        keys = W.kv_keys(cfg.n_groups, cfg.n, cfg.d, cfg.seed_x).reshape(n, cfg.d)
        x = torch.from_numpy(keys.view(np.int16)).view(torch.bfloat16).cuda()
        q = W.gaussian_queries(cfg.nq, cfg.d, cfg.seed_q, unit=False)
        host_x = keys
    else:
        host_x = W.mixture_all(n, cfg.d, cfg.seed_x, cfg.seed_x) if cfg.n > 4096 else W.unit_gaussian_rows(n, cfg.d, cfg.seed_x)
        x = torch.from_numpy(host_x).cuda()
        q = (W.mixture_chunk(0, cfg.nq, cfg.d, cfg.seed_q, W.mixture_centers(cfg.d, cfg.seed_x))
             if cfg.n > 4096 else W.unit_gaussian_rows(cfg.nq, cfg.d, cfg.seed_q))
    bufs = dict(
        x=x, q=torch.from_numpy(q).cuda(),
        idx=torch.zeros((n, max(1, p.idx_words)), dtype=torch.int32, device="cuda"),
        qjl=torch.zeros((n, p.qjl_words), dtype=torch.int32, device="cuda") if prod else None,
        gamma=torch.zeros(n, dtype=torch.float32, device="cuda") if prod else None,
        norm=None if cfg.unit_norm else torch.zeros(n, dtype=torch.float32, device="cuda"),
        xt=torch.zeros((n, cfg.d), dtype=torch.float32, device="cuda"),
        scores=torch.zeros((cfg.nq, cfg.n), dtype=torch.float32, device="cuda") if cfg.topk == 0 else None,
        topk_idx=torch.zeros((cfg.nq, max(1, cfg.topk)), dtype=torch.int32, device="cuda"),
        topk_val=torch.zeros((cfg.nq, max(1, cfg.topk)), dtype=torch.float32, device="cuda"),
    )
    p.reserve(n, cfg.nq, 0).reserve_score(cfg.n_groups, cfg.q_per_group, cfg.n, prod, cfg.topk == 0, cfg.topk)
    return cfg, p, bufs, host_x, q


def make_calls(tq, cfg, p, b):
    prod = cfg.kind == "prod"

    def quantize():
        if prod:
            tq.tq_quantize_prod(p, b["x"], b["idx"], b["qjl"], b["gamma"], b["norm"])
        else:
            tq.tq_quantize_mse(p, b["x"], b["idx"], b["norm"])

    def dequantize():
        tq.tq_dequantize(p, b["idx"], b["qjl"], b["gamma"], b["norm"], b["xt"])

    def score():
        tq.tq_score(p, b["q"], cfg.n_groups, cfg.q_per_group, b["idx"], b["qjl"], b["gamma"], b["norm"],
                    cfg.n, b["scores"], cfg.topk, b["topk_idx"] if cfg.topk else None,
                    b["topk_val"] if cfg.topk else None)

    return [("quantize", quantize), ("dequantize", dequantize), ("score", score)]


def piece_products(cfg, call: str):
    """bf16 piece products the library executes per fp32 contraction of `call`, or 0 when the call runs on the
    fp32 matrix cores.  Mirrors the library's routing (d = 128, one instance): large bf16 batches are quantised
    with x as one piece against three pieces of Pi, and the residual's two pieces against two of S Pi^T (three
    products each); DeQuant takes three products for the centroid part and three for the sign part."""
    n, prod = cfg.n * cfg.n_groups, cfg.kind == "prod"
    if cfg.d != 128:
        # the generic kernel: rotation with three pieces of Pi against the two leading pieces of an fp32 vector
        # (five products; three against the single piece of a bf16 vector), the sketch with two of each (three)
        if call == "quantize":
            rot = 3.0 if cfg.in_dtype == "bf16" else 5.0
            return (rot + 3.0) / 2 if prod else rot
        if call == "dequantize" or cfg.q_per_group > 32 or cfg.d > 512:
            # the many-query scoring kernel (also DeQuant, with the rows of Pi^T as queries): two pieces of a query
            # coordinate against two of a centroid (three products; two for a 1-bit table) or against a sign (two)
            cen = 0 if cfg.bits_mse == 0 else 2 if cfg.bits_mse == 1 else 3
            return (cen + (2 if prod else 0)) / ((1 if cfg.bits_mse else 0) + (1 if prod else 0))
        return 0.0
    if getattr(cfg, "d_hi", 0):
        return 0.0
    if call == "quantize" and cfg.in_dtype == "bf16" and n > 8192:
        return 3.0
    if call == "dequantize" and n > 8192:
        return 3.0  # two pieces of each factor, three products, for the centroid part and for the sign part alike
    return 0.0


def arithmetic(cfg):
    """What each call of this workload multiplies in (every result meets the fp32 tolerances of the parity tests)."""
    if cfg.d == 128:
        q = ("bf16 MFMA on exact pieces: bf16 input x three pieces of Pi (rotation), two pieces of the residual x two "
             "of S Pi^T (signs only); fp32 accumulation and bucket decision") if piece_products(cfg, "quantize") else \
            "fp32 MFMA (rotation and sketch), fp32 bucket decision"
        dq = "bf16 MFMA on two-piece splits of the fp32 factors (error < 3e-5 of a coordinate), fp32 accumulation" \
            if piece_products(cfg, "dequantize") else "fp32 MFMA"
    else:
        q = ("bf16 MFMA on pieces: three (exact) pieces of Pi x the two leading pieces of x (rotation, y to 8e-6 |x|; a bf16 "
             "x is one exact piece), two x two for the sketch (signs only); fp32 accumulation and bucket decision")
        dq = "bf16 MFMA on two-piece splits of the fp32 factors (the scoring kernel with the rows of Pi^T as queries), fp32 accumulation"
    few = cfg.q_per_group <= 32 and cfg.d <= 512
    sc = "int8 MFMA on exact base-128 digits of 2^-19-scaled rotated queries, fp32 combination" if few else \
        "bf16 MFMA on two-piece splits of the rotated queries and centroids (scores within 3e-6 |q| norm), fp32 accumulation"
    return {"quantize": q, "dequantize": dq, "score": sc}


def algorithmic_work(cfg, call: str):
    """(flops, bytes) of one call, counting only what the method needs."""
    n, d, nq = cfg.n * cfg.n_groups, cfg.d, cfg.nq
    prod = cfg.kind == "prod"
    in_b = 2 if cfg.in_dtype == "bf16" else 4
    code_b = cfg.bits_mse * d / 8 + (d / 8 + 4 if prod else 0) + (0 if cfg.unit_norm else 4)
    if call == "quantize":
        return 2.0 * n * d * d * (2 if prod else 1), n * (d * in_b + code_b)
    if call == "dequantize":
        return 2.0 * n * d * d * (2 if prod else 1), n * (code_b + 4 * d)
    pairs = float(cfg.nq) * cfg.n  # every query against the codes of its group
    flops = 2.0 * pairs * d * (2 if prod else 1) + 2.0 * nq * d * d * (2 if prod else 1)
    return flops, n * code_b + 4 * pairs + 4 * nq * d


def measured_traffic(workload: str, kernel: str):
    """HBM bytes per launch of the dominant call, from the rocprofv3 --pmc FETCH_SIZE and
    WRITE_SIZE runs recorded under profiles/ (scaled there by a plain copy of known size);
    None when no measurement has been recorded for this workload and call."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            table = json.load(f)
        return table[workload][kernel]["traffic_bytes"]
    except (OSError, KeyError, ValueError):
        return None


def cpu_baseline(cfg, host_x, q, budget_s=20.0):
    """The oracle, untuned, on a bounded sample of the same workload."""
    import numpy as np
    from oracle import turboquant_oracle as o
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        cores = 1
    prod = cfg.kind == "prod"
    Pi = o.rotation_from_gaussian(__import__("workloads").gaussian_matrix(cfg.d, cfg.seed_pi))
    S = __import__("workloads").sketch_matrix(cfg.d, cfg.seed_s) if prod else None
    c32, t32, _ = o.codebook_fp32(cfg.d, cfg.bits_mse)
    n_total = host_x.shape[0]
    rows = min(n_total, 4096)
    def one_pass(rows):
        xs = host_x[:rows]
        xs = o.bf16_bits_to_f64(xs) if cfg.in_dtype == "bf16" else xs
        qs = q[: max(1, min(cfg.nq, cfg.q_per_group))]
        t0 = time.perf_counter()
        if prod:
            r = o.quant_prod(xs, Pi, S, c32, t32, normalise=not cfg.unit_norm)
            o.pack_planes(r["idx"], cfg.bits_mse), o.pack_signs(r["qjl"])
            xt = o.dequant_prod(r["idx"], r["qjl"], r["gamma"], Pi, S, c32, r["norm"])
        else:
            idx, nu, _ = o.quant_mse(xs, Pi, t32, normalise=not cfg.unit_norm)
            o.pack_planes(idx, cfg.bits_mse)
            xt = o.dequant_mse(idx, Pi, c32, nu)
        o.score(qs, xt)
        return time.perf_counter() - t0, qs.shape[0]

    # grow the sample until a pass takes a fair share of the budget; a workload that is done sooner is repeated
    while True:
        dt, n_q = one_pass(rows)
        if rows >= n_total or dt * 4 > budget_s:
            break
        rows = min(n_total, rows * 4)
    passes, elapsed = 1, dt
    while elapsed + dt < budget_s / 2 and passes < 64:
        elapsed += one_pass(rows)[0]
        passes += 1
    done_rows = rows * passes
    return {"value": done_rows / elapsed, "unit": "vectors/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {rows} of {n_total} vectors, {passes} pass(es): quantize + pack + dequantize + score "
                      f"against {n_q} queries, {elapsed:.2f} s"}


def call_roofline(cfg, name: str, ms: float):
    """Roofline entry of one call from its algorithmic work and its measured time."""
    flops, nbytes = algorithmic_work(cfg, name)
    sec = ms * 1e-3
    pieces = piece_products(cfg, name)
    few_q = name == "score" and not pieces  # few queries per code: integer digits or fp32 lanes, graded against HBM
    peak_tf = PEAK_BF16_MFMA_TFLOPS if pieces else PEAK_FP32_MFMA_TFLOPS
    t_mfma, t_hbm = flops / (peak_tf * 1e12), nbytes / (PEAK_HBM_GBS * 1e9)
    kernel = f"tq_{name}" + ("_prod" if name == "quantize" and cfg.kind == "prod" else "_mse" if name == "quantize" else "")
    if few_q or t_hbm > t_mfma and not pieces:
        r = {"bound": "hbm", "achieved": nbytes / sec / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
             "frac": nbytes / sec / 1e9 / PEAK_HBM_GBS}
    else:
        r = {"bound": "mfma", "achieved": flops / sec / 1e12, "peak": peak_tf, "unit": "TFLOP/s",
             "frac": flops / sec / 1e12 / peak_tf,
             "dtype": "bf16 pieces of fp32 factors, fp32 accumulate" if pieces else "f32"}
        if pieces:
            r["piece_products_per_fp32_product"] = pieces
            r["executed_frac"] = flops * pieces / sec / 1e12 / PEAK_BF16_MFMA_TFLOPS
            r["of_fp32_mfma_peak"] = flops / sec / 1e12 / PEAK_FP32_MFMA_TFLOPS
        r["hbm_frac"] = nbytes / sec / 1e9 / PEAK_HBM_GBS
    r.update({"kernel": kernel, "avg_ms": ms, "algorithmic_flops": flops, "algorithmic_bytes": nbytes,
              "traffic": measured_traffic(cfg.name, kernel)})
    return r


def path_dtype(cfg):
    """The arithmetic type the step computes in, from the library's routing for this workload."""
    parts = []
    for name in ("quantize", "dequantize", "score"):
        pc = piece_products(cfg, name)
        if pc:
            parts.append(f"{name}: bf16 pieces of fp32 factors ({pc:g} products per fp32 product), f32 accumulate")
        elif name == "score" and cfg.q_per_group <= 32 and cfg.d <= 512:
            parts.append("score: i8 digits of a 2^-19 fixed-point query, i32 accumulate")
        else:
            parts.append(f"{name}: f32")
    return "; ".join(parts)


def time_step(calls, steps, warmup):
    """W untimed steps, then exactly `steps` timed ones between device synchronisations.  Per-call times come from
    events on torch's current stream (the stream every launch uses), recorded inside the timed region around the
    calls of every `stride`-th step: an event between two launches keeps the second from being set up behind the
    first (about 4 us each, 15 us on the 60 us step of the d = 128 workloads), so only a sample of the steps
    carries them."""
    import torch
    for _ in range(warmup):
        for _, fn in calls:
            fn()
    torch.cuda.synchronize()
    stride = max(steps // 25, 8 if steps >= 16 else 1)  # at most one step in eight, about 25 in a long run
    sampled = [s for s in range(steps) if s % stride == 0]
    ev = {s: [torch.cuda.Event(enable_timing=True) for _ in range(len(calls) + 1)] for s in sampled}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        if s in ev:
            ev[s][0].record()
            for k, (_, fn) in enumerate(calls):
                fn()
                ev[s][k + 1].record()
        else:
            for _, fn in calls:
                fn()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_call = [sum(ev[s][k].elapsed_time(ev[s][k + 1]) for s in sampled) / len(sampled) for k in range(len(calls))]
    return wall * 1e3 / steps, per_call


def workload_label(cfg):
    return (f"{cfg.name}: TurboQuant_{cfg.kind} b={cfg.bits} d={cfg.d}, {cfg.n_groups}x{cfg.n} {cfg.in_dtype} vectors, "
            f"{cfg.nq} queries ({cfg.q_per_group} per group)" + (f", top-{cfg.topk}" if cfg.topk else ""))


def second_config_record(name: str, steps: int, warmup: int):
    """The same step on another configuration (the d = 1536 half of the metric), timed after the headline region."""
    import torch

    import paper_2504_19874_amd as tq
    cfg, p, bufs, _, _ = build_workload(name)
    calls = make_calls(tq, cfg, p, bufs)
    ms_per_step, per_call = time_step(calls, steps, warmup)
    n = cfg.n * cfg.n_groups
    rec = {"workload": workload_label(cfg), "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
           "vectors_per_s_whole_step": n / (ms_per_step * 1e-3),
           "per_call_ms": {nm: per_call[k] for k, (nm, _) in enumerate(calls)},
           "quantize_vectors_per_s": n / (per_call[0] * 1e-3),
           "scores_per_s": float(cfg.nq) * cfg.n / (per_call[2] * 1e-3),
           "dtype": path_dtype(cfg),
           "rooflines": {nm: call_roofline(cfg, nm, per_call[k]) for k, (nm, _) in enumerate(calls)}}
    del bufs, p, calls
    torch.cuda.empty_cache()
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="C2", choices=["C1", "C2", "C3", "C3b4", "C4", "C5"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-fp32-reference", action="store_true",
                    help="skip the TQ_FLAG_FP32_MFMA leg (profiler runs that should see one kernel per call)")
    ap.add_argument("--no-d1536", action="store_true", help="skip the d = 1536 record (C4)")
    ap.add_argument("--d1536-steps", type=int, default=3)
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2504_19874_amd as tq

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    cfg, p, bufs, host_x, q = build_workload(args.workload)
    calls = make_calls(tq, cfg, p, bufs)
    n = cfg.n * cfg.n_groups

    if args.calibration_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)  # 256 MiB read + 256 MiB written, shows up as one elementwise kernel
        torch.cuda.synchronize()
        del src, dst

    ms_per_step, per_call_ms = time_step(calls, args.steps, args.warmup)
    rooflines = {name: call_roofline(cfg, name, per_call_ms[k]) for k, (name, _) in enumerate(calls)}
    dom_name = max(rooflines, key=lambda k: rooflines[k]["avg_ms"])

    out = {
        "metric": "vectors quantized/s through quantize+dequantize+score (one GPU)",
        "value": n / (ms_per_step * 1e-3),
        "unit": "vectors/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": path_dtype(cfg),
        "data": "synthetic",
        "config": {"workload": workload_label(cfg)},
        "per_call_ms": {name: per_call_ms[k] for k, (name, _) in enumerate(calls)},
        "quantize_vectors_per_s": n / (per_call_ms[0] * 1e-3),
        "scores_per_s": float(cfg.nq) * cfg.n / (per_call_ms[2] * 1e-3),
        "roofline": rooflines[dom_name],
        "rooflines": rooflines,
        # what each call multiplies in; every result meets the fp32 tolerances of the parity tests
        "arithmetic": arithmetic(cfg),
    }
    if not args.no_fp32_reference and any(piece_products(cfg, name) for name, _ in calls):
        # the same calls with every contraction kept on the fp32 matrix instructions (TQ_FLAG_FP32_MFMA in the
        # parameters): the figure the fp32 MFMA peak applies to directly.  Outside the timed region, not part
        # of `value`.
        p.fp32_mfma = True
        try:
            # without a score buffer the fp32 route keeps a score matrix in the workspace
            p.reserve_score(cfg.n_groups, cfg.q_per_group, cfg.n, cfg.kind == "prod", cfg.topk == 0, cfg.topk)
            reps = max(20, args.steps // 4) if n * cfg.d < (1 << 30) else 2
            ref = {}
            for name, fn in calls:
                if not piece_products(cfg, name):
                    continue
                for _ in range(5 if reps > 2 else 1):
                    fn()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(reps):
                    fn()
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / reps
                fl, _ = algorithmic_work(cfg, name)
                ref[name] = {"avg_ms": ms, "achieved": fl / (ms * 1e-3) / 1e12, "unit": "TFLOP/s",
                             "frac_of_fp32_mfma_peak": fl / (ms * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS}
            out["fp32_mfma_reference"] = ref
        finally:
            p.fp32_mfma = False
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, host_x, q)
    if not args.no_d1536 and args.workload != "C4":
        del bufs, calls, host_x
        torch.cuda.empty_cache()
        out["d1536"] = second_config_record("C4", args.d1536_steps, 1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
