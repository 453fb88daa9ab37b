"""Turn rocprofv3 CSV output into the short summaries kept under profiles/.

    python -m paper_2504_19874_amd.profile_summary stats  <dir with *_kernel_stats.csv>
    python -m paper_2504_19874_amd.profile_summary traffic <FETCH_SIZE dir> <WRITE_SIZE dir> \
           --workload C2 [--json profiles/traffic.json]

    python -m paper_2504_19874_amd.profile_summary counters <dir of a --pmc run>

`stats` prints a markdown table of the per-kernel durations (rocprofv3
--kernel-trace --stats --output-format csv).  `counters` prints, per kernel,
the averages of whatever counters the run collected and, when the run has
SQ_VALU_MFMA_BUSY_CYCLES, SQ_ACTIVE_INST_VALU, SQ_WAIT_INST_ANY,
SQ_WAVE_CYCLES and GRBM_GUI_ACTIVE, three shares:
    MFMA busy  = SQ_VALU_MFMA_BUSY_CYCLES / (4 SIMDs x 256 CUs x GRBM_GUI_ACTIVE / 8 XCDs)
    VALU busy  = 4 x SQ_ACTIVE_INST_VALU  / (the same denominator)
    waiting    = SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES   (share of wavefront cycles)
(rocprofv3 sums GRBM_GUI_ACTIVE over the chip's 8 XCDs and the SQ counters over
all SIMDs; SQ_ACTIVE_INST_VALU counts units of 4 cycles).  `traffic` reads the two
--pmc runs (FETCH_SIZE in one, WRITE_SIZE in the other; both made with
bench.py --calibration-copy so that a plain 256 MiB device copy is in the same
trace), derives the scale factor of each counter from that copy, prints the
per-kernel table and, with --json, records bytes per launch for the library's
entry points in the file bench.py reads for `roofline.traffic`.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import re
import os
import sys

COPY_KIB = 256 * 1024  # what bench.py --calibration-copy reads and writes
# kernel name prefix -> entry point whose dominant kernel it is
ENTRY_OF = (("tq::quant128_kernel", "tq_quantize_prod"), ("tq::(anonymous namespace)::quant128_bf3_kernel", "tq_quantize_prod"), ("tq::dequant128_kernel", "tq_dequantize"),
            ("tq::(anonymous namespace)::dequant128_bf3_kernel", "tq_dequantize"),
            ("tq::(anonymous namespace)::score_bf3_kernel", "tq_score"),
            ("tq::score_i8_128_kernel", "tq_score"), ("tq::score_i8_kernel", "tq_score"),
            ("tq::score_small_kernel", "tq_score"), ("tq::gemm_kernel<0, 2", "tq_quantize"),
            ("tq::gemm_kernel<1, 2", "tq_quantize"), ("tq::gemm_kernel<2, 0", "tq_dequantize"),
            ("tq::gemm_kernel<2, 1", "tq_score"), ("tq::stage_pack_kernel", "tq_stage_pack"),
            ("tq::stage_unpack_kernel", "tq_stage_unpack"), ("tq::stage_sign_pack_kernel", "tq_stage_sign_pack"),
            ("tq::(anonymous namespace)::stage_", "tq_stage"))


def find(dirname, suffix):
    hits = sorted(glob.glob(os.path.join(dirname, "**", "*" + suffix), recursive=True))
    if not hits:
        sys.exit(f"no *{suffix} under {dirname}")
    return hits[-1]


def short(name, width=90):
    name = name.replace("void ", "")
    return name if len(name) <= width else name[:width - 3] + "..."


def stats(dirname):
    rows = list(csv.DictReader(open(find(dirname, "kernel_stats.csv"))))
    print("| kernel | calls | avg ns | min ns | max ns | % |")
    print("|---|---|---|---|---|---|")
    for r in rows:
        print(f"| `{short(r['Name'])}` | {r['Calls']} | {float(r['AverageNs']):.0f} | {r['MinNs']} | {r['MaxNs']} | "
              f"{float(r['Percentage']):.2f} |")


def counters(dirname, cus=256, xcds=8):
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(find(dirname, "counter_collection.csv"))):
        name = r["Kernel_Name"].replace("void ", "")
        if name.startswith("tq::"):
            acc[name][r["Counter_Name"]].append(float(r["Counter_Value"]))
    names = sorted({c for v in acc.values() for c in v})
    print("| kernel | launches | " + " | ".join(names) + " | MFMA busy | VALU busy | waiting |")
    print("|---|---|" + "---|" * (len(names) + 3))
    for k in sorted(acc):
        v = {c: sum(x) / len(x) for c, x in acc[k].items()}
        n = max(len(x) for x in acc[k].values())
        den = 4.0 * cus * v["GRBM_GUI_ACTIVE"] / xcds if v.get("GRBM_GUI_ACTIVE") else 0.0
        mfma = f"{100 * v['SQ_VALU_MFMA_BUSY_CYCLES'] / den:.1f} %" if den and "SQ_VALU_MFMA_BUSY_CYCLES" in v else ""
        valu = f"{100 * 4 * v['SQ_ACTIVE_INST_VALU'] / den:.1f} %" if den and "SQ_ACTIVE_INST_VALU" in v else ""
        wait = f"{100 * v['SQ_WAIT_INST_ANY'] / v['SQ_WAVE_CYCLES']:.1f} %" if v.get("SQ_WAVE_CYCLES") and "SQ_WAIT_INST_ANY" in v else ""
        print(f"| `{short(k, 80)}` | {n} | " + " | ".join(f"{v[c]:.4g}" if c in v else "" for c in names) +
              f" | {mfma} | {valu} | {wait} |")


def per_kernel(dirname, counter):
    acc = collections.defaultdict(list)
    for r in csv.DictReader(open(find(dirname, "counter_collection.csv"))):
        if r["Counter_Name"] == counter:
            acc[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return acc


def traffic(fetch_dir, write_dir, workload, json_path):
    fetch, write = per_kernel(fetch_dir, "FETCH_SIZE"), per_kernel(write_dir, "WRITE_SIZE")
    # the calibration copy is the launch of a copy kernel that wrote 256 MiB (WRITE_SIZE counts every byte
    # written, which the copy itself shows); other copies in the trace (inputs being laid out) have other sizes.
    # The two runs execute the same program, so launch i of a kernel is the same launch in both.
    copy, at = None, -1
    for k in write:
        if not ("copyBuffer" in k or "direct_copy" in k or "CUDAFunctor" in k) or k not in fetch:
            continue
        for i, w in enumerate(write[k]):
            if abs(w - COPY_KIB) < 0.05 * COPY_KIB and i < len(fetch[k]):
                copy, at = k, i
    if copy is None:
        sys.exit("no calibration copy in the trace (run bench.py with --calibration-copy)")
    f_copy, w_copy = fetch[copy][at], write[copy][at]
    f_scale = COPY_KIB / f_copy
    w_scale = COPY_KIB / w_copy
    print(f"calibration copy `{short(copy, 60)}`: FETCH_SIZE {f_copy:.1f} KiB -> scale {f_scale:.4f}, "
          f"WRITE_SIZE {w_copy:.1f} KiB -> scale {w_scale:.4f}\n")
    print("| call | kernel | launches | FETCH_SIZE KiB | WRITE_SIZE KiB | HBM bytes (scaled) |")
    print("|---|---|---|---|---|---|")
    table = {}
    for k in sorted(fetch):
        if not k.startswith("void tq::") and not k.startswith("tq::"):
            continue
        name = k.replace("void ", "")
        entry = next((e for p, e in ENTRY_OF if name.startswith(p)), "")
        f, w = sum(fetch[k]) / len(fetch[k]), sum(write[k]) / len(write[k])
        total = (f * f_scale + w * w_scale) * 1024
        print(f"| {entry} | `{short(k, 70)}` | {len(fetch[k])} | {f:.1f} | {w:.1f} | {total / 1e6:.2f} MB |")
        if entry and len(fetch[k]) > 2:
            table[entry] = {"kernel": re.match(r"(.*?kernel(?:<[^>]*>)?)", name).group(1) if "kernel" in name else name.split("(")[0], "fetch_kib_raw": round(f, 1), "write_kib_raw": round(w, 1),
                            "fetch_scale": round(f_scale, 4), "write_scale": round(w_scale, 4),
                            "traffic_bytes": int(total), "launches_averaged": len(fetch[k])}
    if json_path:
        try:
            with open(json_path) as fh:
                doc = json.load(fh)
        except (OSError, ValueError):
            doc = {}
        doc[workload] = table
        with open(json_path, "w") as fh:
            json.dump(doc, fh, indent=1)
            fh.write("\n")


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    s = sub.add_parser("stats")
    s.add_argument("dir")
    c = sub.add_parser("counters")
    c.add_argument("dir")
    t = sub.add_parser("traffic")
    t.add_argument("fetch_dir")
    t.add_argument("write_dir")
    t.add_argument("--workload", required=True)
    t.add_argument("--json", default="")
    args = ap.parse_args()
    if args.cmd == "stats":
        stats(args.dir)
    elif args.cmd == "counters":
        counters(args.dir)
    else:
        traffic(args.fetch_dir, args.write_dir, args.workload, args.json)


if __name__ == "__main__":
    main()
