"""Turns rocprofv3 CSV output of ``bench.py`` runs into the short text summaries kept under
``profiles/`` and into ``profiles/traffic.json``, which ``bench.py`` reads for the
``roofline.traffic`` field.

    python -m paper_2602_00777_amd.profile_summary --workload llama3_8b_32k \\
        --stats out/prof_stats_llama3_8b_32k \\
        --fetch out/prof_fetch_llama3_8b_32k --write out/prof_write_llama3_8b_32k

The three directories come from (run from /tmp with TMPDIR=/tmp, one counter per run):

    rocprofv3 --kernel-trace --stats --output-format csv -d <stats dir> -o stats -- python3 bench.py --workload W
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <fetch dir> -o fetch -- python3 bench.py --workload W --steps 2 --warmup 1 --no-cpu-baseline --no-parity
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <write dir> -o write -- python3 bench.py --workload W --steps 2 --warmup 1 --no-cpu-baseline --no-parity

FETCH_SIZE / WRITE_SIZE (KiB per dispatch) are scaled by what the same counter reads for the
library's plain copy kernel (``hylra_probe_copy`` of 4 GiB, part of every bench run's probes).
Any of the three directories may be left out.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROFILES = os.path.join(ROOT, "profiles")
COPY_KIB = 4 << 20          # the copy probe moves 4 GiB each way

# kernel-name fragments -> the kernel class bench.py reports
CLASSES = (("full_attn", ("full_attn_split_kernel", "full_mfma_kernel", "full_mfma2_kernel")),
           ("full_finalize", ("full_finalize_kernel", "select_", "block_max_kernel", "topk_")),
           ("reuse_attn", ("reuse_attn_split_kernel", "reuse_mfma_kernel", "reuse_mfma2_kernel")))


def kernel_class(name: str):
    for cls, frags in CLASSES:
        if any(f in name for f in frags):
            return cls
    return None


def short(name: str) -> str:
    return name.replace("void ", "").replace("hylra::", "").split("(")[0]


def one_csv(directory: str, pattern: str) -> str:
    hits = glob.glob(os.path.join(directory, "**", pattern), recursive=True)
    if not hits:
        raise FileNotFoundError("no %s under %s" % (pattern, directory))
    return sorted(hits)[0]


def summarise_stats(directory: str, workload: str, command: str) -> str:
    rows = list(csv.DictReader(open(one_csv(directory, "*kernel_stats.csv"))))
    out = ["rocprofv3 --kernel-trace --stats, workload %s, MI355X, one GPU" % workload,
           "command (from /tmp, TMPDIR=/tmp):", "  " + command, "",
           "%-62s %6s %14s %12s %10s %10s" % ("kernel", "calls", "total_ns", "avg_ns", "min_ns", "max_ns")]
    for r in rows:
        if "hylra" in r["Name"]:
            out.append("%-62s %6s %14s %12.0f %10s %10s" % (short(r["Name"])[:62], r["Calls"], r["TotalDurationNs"],
                                                           float(r["AverageNs"]), r["MinNs"], r["MaxNs"]))
    out += ["", "(the remaining rows of the trace are PyTorch kernels that draw the synthetic inputs before the timed region)"]
    return "\n".join(out) + "\n"


def counter_means(directory: str):
    rows = list(csv.DictReader(open(one_csv(directory, "*counter_collection.csv"))))
    agg = collections.defaultdict(list)
    for r in rows:
        if "hylra" in r["Kernel_Name"]:
            agg[short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return rows[0]["Counter_Name"] if rows else "?", agg


def summarise_traffic(fetch_dir: str, write_dir: str, workload: str, algorithmic: dict):
    out = ["rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE (KiB per dispatch), workload %s, MI355X" % workload,
           "commands (from /tmp, TMPDIR=/tmp; one counter per run):",
           "  rocprofv3 --pmc FETCH_SIZE --output-format csv -d %s -o fetch -- python3 bench.py --workload %s --steps 2 --warmup 1 --no-cpu-baseline --no-parity" % (fetch_dir, workload),
           "  rocprofv3 --pmc WRITE_SIZE --output-format csv -d %s -o write -- python3 bench.py --workload %s --steps 2 --warmup 1 --no-cpu-baseline --no-parity" % (write_dir, workload), ""]
    means = {}
    for tag, d in (("fetch", fetch_dir), ("write", write_dir)):
        cname, agg = counter_means(d)
        means[tag] = {k: sum(v) / len(v) for k, v in agg.items()}
        out.append("%s (mean KiB per dispatch):" % cname)
        for k, v in agg.items():
            out.append("   %-48s n=%4d  mean %12.1f KiB  min %12.1f  max %12.1f" % (k[:48], len(v), sum(v) / len(v), min(v), max(v)))
        out.append("")
    copy = [k for k in means["fetch"] if "probe_copy" in k]
    if not copy:
        raise RuntimeError("the copy probe is not in the counter run (bench.py runs it unless --no-probe is given)")
    f_scale = COPY_KIB / means["fetch"][copy[0]]
    w_scale = COPY_KIB / means["write"][copy[0]]
    out += ["calibration: probe_copy_kernel copies 4 GiB (reads %d KiB, writes %d KiB)" % (COPY_KIB, COPY_KIB),
            "   FETCH_SIZE reads %.1f KiB for it -> scale factor %.3f" % (means["fetch"][copy[0]], f_scale),
            "   WRITE_SIZE reads %.1f KiB for it -> scale factor %.3f" % (means["write"][copy[0]], w_scale), "",
            "scaled HBM traffic per launch (bytes) vs algorithmic bytes:"]
    traffic = {}
    for k, fk in means["fetch"].items():
        if "probe" in k:
            continue
        fb, wb = fk * f_scale * 1024, means["write"].get(k, 0.0) * w_scale * 1024
        cls = kernel_class(k)
        alg = algorithmic.get(cls) if cls in ("full_attn", "reuse_attn") else None
        out.append("   %-48s fetch %13.0f + write %11.0f = %13.0f B%s" %
                   (k[:48], fb, wb, fb + wb, "   algorithmic %d B (ratio %.3f)" % (alg, (fb + wb) / alg) if alg else ""))
        if cls in ("full_attn", "reuse_attn"):
            traffic[cls] = int(round(fb + wb))
    return "\n".join(out) + "\n", traffic, {"fetch_scale": round(f_scale, 4), "write_scale": round(w_scale, 4)}


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", required=True)
    ap.add_argument("--stats")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--bench-args", default="", help="extra bench.py arguments of the profiled command, for the record")
    args = ap.parse_args(argv)
    sys.path.insert(0, ROOT)
    from paper_2602_00777_amd import synth

    w = synth.WORKLOADS[args.workload]
    small = w.batch * w.n_q_heads * w.head_dim * 6 + w.batch * w.n_kv_heads * w.top_k * 4
    algorithmic = {"full_attn": 4 * w.batch * w.n_kv_heads * w.ctx_len * w.head_dim + small,
                   "reuse_attn": 4 * w.batch * w.n_kv_heads * w.top_k * w.head_dim + small}
    os.makedirs(PROFILES, exist_ok=True)
    if args.stats:
        cmd = "rocprofv3 --kernel-trace --stats --output-format csv -d %s -o stats -- python3 bench.py --workload %s %s" % (
            args.stats, args.workload, args.bench_args)
        path = os.path.join(PROFILES, "kernel_stats_%s.txt" % args.workload)
        open(path, "w").write(summarise_stats(args.stats, args.workload, cmd.strip()))
        print("wrote", path)
    if args.fetch and args.write:
        text, traffic, calib = summarise_traffic(args.fetch, args.write, args.workload, algorithmic)
        path = os.path.join(PROFILES, "hbm_traffic_%s.txt" % args.workload)
        open(path, "w").write(text)
        print("wrote", path)
        jpath = os.path.join(PROFILES, "traffic.json")
        table = json.load(open(jpath)) if os.path.exists(jpath) else {}
        table[args.workload] = dict(traffic, algorithmic=algorithmic, calibration=calib,
                                    source="profiles/hbm_traffic_%s.txt" % args.workload)
        json.dump(table, open(jpath, "w"), indent=1, sort_keys=True)
        print("wrote", jpath)


if __name__ == "__main__":
    main()
