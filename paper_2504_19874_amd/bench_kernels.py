"""Per-entry-point timings against the MFMA / HBM rooflines for the five
benchmark configurations.

    python -m paper_2504_19874_amd.bench_kernels --config C2 [--reps 50]

Prints one JSON object per entry point: average milliseconds (HIP events on the
launch stream), algorithmic flops and bytes (nothing the kernels execute beyond
the definition is counted), and what that is of the HBM peak (8 TB/s) or, for a
contraction, of both dense MFMA peaks: fp32 (157.3 TFLOP/s) and bf16 (2.5
PFLOP/s, the type the piece kernels multiply in).
For configurations whose working set fits the 256 MB last-level cache the
inputs are rotated through several buffer sets so HBM-bound figures are not
cache figures ("cold"); `--warm` disables that.  Inputs come from the seeded
generators in workloads/.  Also times a plain device-to-device copy of the
same size as the stage kernels' traffic, as the reference for what a
streaming kernel reaches on this chip.  `--only intake` runs no entry point
but a probe: how long one workgroup per compute unit needs to take in N KB.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TF, PEAK_BF16_TF, PEAK_GBS = 157.3, 2500.0, 8000.0


def timed(fn, reps, warmup=3):
    import torch
    for _ in range(warmup):
        fn(0)
    torch.cuda.synchronize()
    e0 = [torch.cuda.Event(enable_timing=True) for _ in range(reps)]
    e1 = [torch.cuda.Event(enable_timing=True) for _ in range(reps)]
    for r in range(reps):
        e0[r].record()
        fn(r)
        e1[r].record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) for a, b in zip(e0, e1))
    return sum(ts) / len(ts), ts[0], ts[len(ts) // 2]


def report(name, cfg, ms, flops, nbytes, extra=None, bound=None):
    avg, mn, med = ms
    t_mfma, t_hbm = flops / (PEAK_TF * 1e12), nbytes / (PEAK_GBS * 1e9)
    bound = bound or ("mfma" if t_mfma >= t_hbm else "hbm")
    out = {"config": cfg.name, "call": name, "avg_ms": round(avg, 5), "min_ms": round(mn, 5),
           "median_ms": round(med, 5), "flops": flops, "bytes": nbytes, "bound": bound,
           "tflops": round(flops / (avg * 1e-3) / 1e12, 2), "gbs": round(nbytes / (avg * 1e-3) / 1e9, 1)}
    if bound == "mfma":
        out["frac_of_fp32_mfma_peak"] = round(out["tflops"] / PEAK_TF, 4)
        out["frac_of_bf16_mfma_peak"] = round(out["tflops"] / PEAK_BF16_TF, 4)
    else:
        out["frac_of_hbm_peak"] = round(t_hbm / (avg * 1e-3), 4)
    if extra:
        out.update(extra)
    print(json.dumps(out), flush=True)


def intake_probe(torch):
    """`--only intake`: time for one workgroup per compute unit to take in a given number of KB, part of it a
    region all workgroups share (the parameter matrices of the few-query scoring kernel) and part its own (its
    codes), from the probe kernel in libtqprobe.so.  Own regions are rotated through 12 buffers (cold)."""
    import ctypes as C
    lib = C.CDLL(os.path.join(os.path.dirname(os.path.abspath(__file__)), "libtqprobe.so"))
    lib.tq_probe_intake.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p]
    lib.tq_probe_intake.restype = C.c_int
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sets = 12
    shared = torch.empty(128 << 10, dtype=torch.uint8, device="cuda").random_(0, 255)
    own = [torch.empty(cus * (240 << 10), dtype=torch.uint8, device="cuda").random_(0, 255) for _ in range(sets)]
    out = torch.empty(cus * 512, dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    for shared_kb, own_kb in ((0, 8), (0, 56), (0, 112), (0, 176), (0, 240), (64, 0), (128, 0), (32, 112), (64, 112),
                              (128, 112), (64, 56), (128, 56)):
        def run(r):
            rc = lib.tq_probe_intake(shared.data_ptr(), shared_kb, own[r % sets].data_ptr(), own_kb, out.data_ptr(), cus,
                                     stream)
            if rc != 0:
                raise RuntimeError(f"tq_probe_intake({shared_kb}, {own_kb}) returned {rc}")
        avg, mn, med = timed(run, 60)
        kb = shared_kb + own_kb
        print(json.dumps({"probe": "intake", "workgroups": cus, "shared_kb": shared_kb, "own_kb": own_kb,
                          "avg_us": round(avg * 1e3, 2), "min_us": round(mn * 1e3, 2), "median_us": round(med * 1e3, 2),
                          "hbm_gbs": round(cus * own_kb * 1024 / (med * 1e-3) / 1e9, 1),
                          "bytes_per_us_per_cu": round(kb * 1024 / (med * 1e3), 1)}), flush=True)

    # when each wavefront's loads come back (own region of 112 KB per workgroup, 14 loads per thread, cold)
    lib.tq_probe_arrival.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
    lib.tq_probe_arrival.restype = C.c_int
    stamps = torch.zeros(cus * 8 * 16, dtype=torch.int64, device="cuda")
    for r in range(6):
        rc = lib.tq_probe_arrival(own[r % sets].data_ptr(), out.data_ptr(), stamps.data_ptr(), cus, stream)
        if rc != 0:
            raise RuntimeError(f"tq_probe_arrival returned {rc}")
        torch.cuda.synchronize()
    t = stamps.cpu().numpy().reshape(cus * 8, 16)[:, :15].astype("float64")
    t = (t - t[:, 0].min()) * 0.01  # 100 MHz clock -> microseconds after the first wavefront's start
    import numpy as np
    rows = {}
    for k in (0, 1, 2, 4, 7, 10, 12, 14):
        rows[f"after_{k}_loads" if k else "start"] = [round(float(np.percentile(t[:, k], q)), 2) for q in (5, 25, 50, 75, 95)]
    print(json.dumps({"probe": "arrival", "workgroups": cus, "own_kb": 112, "loads_per_thread": 14,
                      "us_percentiles_5_25_50_75_95": rows}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="C2")
    ap.add_argument("--reps", type=int, default=0)
    ap.add_argument("--warm", action="store_true")
    ap.add_argument("--only", default="")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--no-images", action="store_true",
                    help="d = 128: split the matrices in every launch instead of using the images of tq_build_images")
    ap.add_argument("--f32-input", action="store_true",
                    help="hand the vectors of a bf16 configuration to the quantiser as fp32 (same values)")
    ap.add_argument("--value-bits", type=int, default=2, help="attend: bits of the MSE stage of the value codes")
    ap.add_argument("--value-prod", action="store_true", help="attend: value codes from TurboQuant_prod")
    ap.add_argument("--value-split", type=int, default=0, metavar="D_HI",
                    help="attend: value codes in two MSE instances, D_HI outlier channels with one more bit")
    args = ap.parse_args()

    import numpy as np
    import torch

    import paper_2504_19874_amd as tq
    import workloads as W

    if args.calibration_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)  # 256 MiB read + 256 MiB written
        torch.cuda.synchronize()
        del src, dst

    if args.only == "intake":
        intake_probe(torch)
        return

    cfg = W.CONFIGS[args.config]
    prod = cfg.kind == "prod"
    d, n, nq = cfg.d, cfg.n * cfg.n_groups, cfg.nq
    big = n * d * 4 > (1 << 30)
    reps = args.reps or (5 if big else 100)
    if cfg.d_hi:
        # two instances over a channel split: cfg.bits belongs to the d - d_hi ordinary channels
        hi = W.kv_hi_channels(cfg.n_groups, d, cfg.seed_x, cfg.d_hi)
        p = tq.make_mixed_params(d, hi, cfg.bits_mse + 1, cfg.bits_mse, W.gaussian_matrix(cfg.d_hi, cfg.seed_pi),
                                 W.gaussian_matrix(d - cfg.d_hi, cfg.seed_pi + 1),
                                 W.sketch_matrix(cfg.d_hi, cfg.seed_s) if prod else None,
                                 W.sketch_matrix(d - cfg.d_hi, cfg.seed_s + 1) if prod else None)
    else:
        S = W.sketch_matrix(d, cfg.seed_s) if prod else None
        p = tq.make_params(d, cfg.bits_mse, W.gaussian_matrix(d, cfg.seed_pi), S)
    if args.no_images:
        p.drop_images()
    # quantisation scratch, then exactly what this configuration's scoring call takes (no score matrix
    # where the top-k selection runs inside the scoring kernel)
    p.reserve(n, nq, 0).reserve_score(cfg.n_groups, cfg.q_per_group, cfg.n, prod, not cfg.topk, cfg.topk)
    spv = p.scalars_per_vector

    # input sets: rotate through several when the working set would sit in cache
    in_b = 2 if cfg.in_dtype == "bf16" and not args.f32_input else 4
    sets = 1 if (big or args.warm) else max(1, min(12, int(300e6 // max(1, n * d * in_b)) + 1))
    xs = []
    for s in range(sets):
        if cfg.in_dtype == "bf16":
            keys = W.kv_keys(cfg.n_groups, cfg.n, d, cfg.seed_x + 1000 * s).reshape(n, d)
            xs.append(torch.from_numpy(keys.view(np.int16)).view(torch.bfloat16).cuda())
            if args.f32_input:
                xs[-1] = xs[-1].float()
        elif big:
            x = torch.empty((n, d), dtype=torch.float32, device="cuda")
            for start, blk in W.mixture_rows(n, d, cfg.seed_x, cfg.seed_x):
                x[start:start + blk.shape[0]] = torch.from_numpy(blk).cuda()
            xs.append(x)
        else:
            xs.append(torch.from_numpy(W.unit_gaussian_rows(n, d, cfg.seed_x + 1000 * s)).cuda())
    if big:
        q = W.mixture_chunk(0, nq, d, cfg.seed_q, W.mixture_centers(d, cfg.seed_x))
    else:
        q = W.gaussian_queries(nq, d, cfg.seed_q, unit=cfg.unit_norm)
    q = torch.from_numpy(q).cuda()

    def new_codes():
        return dict(idx=torch.zeros((n, max(1, p.idx_words)), dtype=torch.int32, device="cuda"),
                    qjl=torch.zeros((n, p.qjl_words), dtype=torch.int32, device="cuda") if prod else None,
                    gamma=torch.zeros((n, spv), dtype=torch.float32, device="cuda") if prod else None,
                    norm=None if cfg.unit_norm else torch.zeros((n, spv), dtype=torch.float32, device="cuda"))

    codes = [new_codes() for _ in range(sets)]

    def quantize(r):
        c, x = codes[r % sets], xs[r % sets]
        if prod:
            tq.tq_quantize_prod(p, x, c["idx"], c["qjl"], c["gamma"], c["norm"])
        else:
            tq.tq_quantize_mse(p, x, c["idx"], c["norm"])

    code_b = 4 * p.idx_words + (d / 8 + 4 * spv if prod else 0) + (0 if cfg.unit_norm else 4 * spv)
    # algorithmic contraction size per vector: two instances rotate their own channels only
    dd = float(cfg.d_hi ** 2 + (d - cfg.d_hi) ** 2) if cfg.d_hi else float(d * d)
    want = [w for w in args.only.split(",") if w]

    def on(name):
        return not want or name in want

    for s in range(sets):
        quantize(s)
    torch.cuda.synchronize()

    if on("quantize"):
        report("quantize", cfg, timed(quantize, reps), 2.0 * n * dd * (2 if prod else 1), n * (d * in_b + code_b),
               {"vectors_per_s": None, "input_sets": sets})

    if on("dequantize"):
        xt = [torch.empty((n, d), dtype=torch.float32, device="cuda") for _ in range(min(sets, 4) if not big else 1)]

        def dequantize(r):
            c = codes[r % sets]
            tq.tq_dequantize(p, c["idx"], c["qjl"], c["gamma"], c["norm"], xt[r % len(xt)])

        report("dequantize", cfg, timed(dequantize, reps), 2.0 * n * dd * (2 if prod else 1), n * (code_b + 4 * d))
        del xt

    if on("score"):
        sc = None if cfg.topk else [torch.empty((nq, cfg.n), dtype=torch.float32, device="cuda")
                                    for _ in range(min(sets, 8))]
        ti = torch.zeros((nq, max(1, cfg.topk)), dtype=torch.int32, device="cuda")
        tv = torch.zeros((nq, max(1, cfg.topk)), dtype=torch.float32, device="cuda")

        def score(r):
            c = codes[r % sets]
            tq.tq_score(p, q, cfg.n_groups, cfg.q_per_group, c["idx"], c["qjl"], c["gamma"], c["norm"], cfg.n,
                        None if cfg.topk else sc[r % len(sc)], cfg.topk, ti if cfg.topk else None,
                        tv if cfg.topk else None)

        pairs = float(nq) * cfg.n
        out_b = 0 if cfg.topk else 4 * pairs
        report("score" + (f"+top{cfg.topk}" if cfg.topk else ""), cfg, timed(score, reps),
               2.0 * pairs * d * (2 if prod else 1) + 2.0 * nq * dd * (2 if prod else 1),
               n * code_b + out_b + 4 * nq * d, {"scores_per_s": None, "pairs": pairs},
               # a few queries per code run on the int8 cores and read the codes once per four queries
               bound="hbm" if cfg.q_per_group <= 16 and d > 128 else None)

    if on("attend") and not cfg.topk and cfg.q_per_group <= 32 and not big:
        # attention read-out: the key codes above plus a value cache of the same shape
        vprod = args.value_prod
        if args.value_split:
            vhi = W.kv_hi_channels(cfg.n_groups, d, cfg.seed_x + 9, args.value_split)
            pv = tq.make_mixed_params(d, vhi, args.value_bits + 1, args.value_bits,
                                      W.gaussian_matrix(args.value_split, cfg.seed_pi + 7),
                                      W.gaussian_matrix(d - args.value_split, cfg.seed_pi + 8), None, None).reserve(n, nq, 0)
        else:
            pv = tq.make_params(d, args.value_bits, W.gaussian_matrix(d, cfg.seed_pi + 7),
                                W.sketch_matrix(d, cfg.seed_s + 7) if vprod else None).reserve(n, nq, 0)
        vsets = []
        for s in range(sets):
            v = torch.from_numpy(W.unit_gaussian_rows(n, d, cfg.seed_x + 500 + s)).cuda() * 2.0
            vc = dict(idx=torch.zeros((n, max(1, pv.idx_words)), dtype=torch.int32, device="cuda"),
                      qjl=torch.zeros((n, pv.qjl_words), dtype=torch.int32, device="cuda") if vprod else None,
                      gamma=torch.zeros(n, dtype=torch.float32, device="cuda") if vprod else None,
                      norm=torch.zeros((n, pv.scalars_per_vector), dtype=torch.float32, device="cuda"))
            if vprod:
                tq.tq_quantize_prod(pv, v, vc["idx"], vc["qjl"], vc["gamma"], vc["norm"])
            else:
                tq.tq_quantize_mse(pv, v, vc["idx"], vc["norm"])
            vsets.append(vc)
        outs = [torch.empty((nq, d), dtype=torch.float32, device="cuda") for _ in range(min(sets, 8))]
        knorm = [c["norm"] if c["norm"] is not None else torch.ones((n, spv), dtype=torch.float32, device="cuda")
                 for c in codes]

        def attend(r):
            c, vc = codes[r % sets], vsets[r % sets]
            tq.tq_attend(p, pv, q, cfg.n_groups, cfg.q_per_group, (c["idx"], c["qjl"], c["gamma"], knorm[r % sets]),
                         (vc["idx"], vc["qjl"], vc["gamma"], vc["norm"]), cfg.n, 1.0 / d ** 0.5, outs[r % len(outs)])

        pairs = float(nq) * cfg.n
        vcode_b = 4 * pv.idx_words + 4 * pv.scalars_per_vector + (d / 8 + 4 if vprod else 0)
        vname = f"split{args.value_split}:{args.value_bits + 1}+{args.value_bits}" if args.value_split else \
            f"{'prod' if vprod else 'mse'}{args.value_bits}"
        report(f"attend(v{vname})", cfg, timed(attend, reps),
               2.0 * pairs * d * ((2 if prod else 1) + (2 if vprod else 1)), n * (code_b + vcode_b) + 8 * nq * d,
               {"pairs": pairs}, bound="hbm")  # the contractions run on the int8 cores; the codes are read once

        if d == 128 and not cfg.d_hi and p.PiT is not None:
            # one decoding step on a cache laid out [head][capacity = n]: the last slot of every head is
            # rewritten with a new key and a new value, then the queries read the whole cache
            newk = torch.randn((cfg.n_groups, d), dtype=torch.float32, device="cuda")
            newv = torch.randn((cfg.n_groups, d), dtype=torch.float32, device="cuda")

            def decode_step(r):
                c, vc = codes[r % sets], vsets[r % sets]
                kn = knorm[r % sets]
                tq.tq_append(p, newk, c["idx"], c["qjl"], c["gamma"], kn, cfg.n - 1, cfg.n)
                tq.tq_append(pv, newv, vc["idx"], vc["qjl"], vc["gamma"], vc["norm"], cfg.n - 1, cfg.n)
                tq.tq_attend(p, pv, q, cfg.n_groups, cfg.q_per_group, (c["idx"], c["qjl"], c["gamma"], kn),
                             (vc["idx"], vc["qjl"], vc["gamma"], vc["norm"]), cfg.n, 1.0 / d ** 0.5, outs[r % len(outs)],
                             group_stride=cfg.n)

            report(f"decode_step(v{vname})", cfg, timed(decode_step, reps),
                   2.0 * pairs * d * ((2 if prod else 1) + (2 if vprod else 1)), n * (code_b + vcode_b) + 8 * nq * d,
                   {"pairs": pairs}, bound="hbm")

    if on("stage") and cfg.bits_mse > 0 and not cfg.d_hi:
        # codec stages on rotated coordinates of the same shape
        rows = n if not big else min(n, 1 << 20)
        ysets = 1 if big else sets
        ys = [torch.randn((rows, d), dtype=torch.float32, device="cuda") / d ** 0.5 for _ in range(ysets)]
        iw = [torch.zeros((rows, p.idx_words), dtype=torch.int32, device="cuda") for _ in range(ysets)]
        report("stage_pack", cfg, timed(lambda r: tq.tq_stage_pack(p, ys[r % ysets], iw[r % ysets]), reps),
               0.0, rows * (4 * d + cfg.bits_mse * d / 8))
        report("stage_unpack", cfg, timed(lambda r: tq.tq_stage_unpack(p, iw[r % ysets], ys[r % ysets]), reps),
               0.0, rows * (4 * d + cfg.bits_mse * d / 8))
        qw = [torch.zeros((rows, d // 32), dtype=torch.int32, device="cuda") for _ in range(ysets)]
        report("stage_sign_pack", cfg, timed(lambda r: tq.tq_stage_sign_pack(d, ys[r % ysets], qw[r % ysets]), reps),
               0.0, rows * (4 * d + d / 8))
        dst = [torch.empty_like(y) for y in ys]
        report("plain_copy(torch)", cfg, timed(lambda r: dst[r % ysets].copy_(ys[r % ysets]), reps),
               0.0, rows * 8 * d)
        # write-only and read-only streams of the same footprint: what stage_unpack (almost all stores) and
        # stage_pack (almost all loads) can be held against
        report("plain_fill(torch)", cfg, timed(lambda r: dst[r % ysets].fill_(1.0), reps), 0.0, rows * 4 * d)
        report("plain_sum(torch)", cfg, timed(lambda r: ys[r % ysets].sum(), reps), 0.0, rows * 4 * d)


if __name__ == "__main__":
    main()
