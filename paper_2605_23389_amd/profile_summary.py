"""Turns the raw rocprofv3 output of three runs of bench.py (kernel trace,
FETCH_SIZE, WRITE_SIZE) into the short summary under profiles/ and into the
HBM-traffic figure bench.py reports as roofline.traffic.

    python -m paper_2605_23389_amd.profile_summary --dir <raw-output-dir> \\
        --kernel attn_kernel --alg-bytes 1969799885 --out profiles/attn_bf16_d128_cfg2_aligned.md \\
        --json-key attn_cfg2_aligned_bytes_per_launch --title "..." --bench-args "" --note "..."

Expects <dir>/trace/t_kernel_stats.csv, <dir>/fetch/f_counter_collection.csv
and <dir>/write/w_counter_collection.csv, each from one run of

    rocprofv3 <--kernel-trace --stats | --pmc FETCH_SIZE | --pmc WRITE_SIZE> --output-format csv \\
        -d <dir>/<trace|fetch|write> -o <t|f|w> -- python3 bench.py --steps S --warmup W \\
        --skip-cpu --skip-extra --copy-calibration --settle-seconds 0 <bench-args>

The counters read KiB per dispatch; they are scaled by what the same counter
reads for the three plain 2 GiB device-to-device copies that
--copy-calibration runs (true traffic: 2 GiB read and 2 GiB written each).
The commit the numbers were taken at is recorded beside them.
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
KNOWN = ("attn_mfma_kernel", "attn_kernel", "combine_kernel", "plan_kernel", "sweep_kernel", "gather_kernel",
         "kv_append_kernel", "copyBuffer", "distribution_elementwise", "FillFunctor")
COPY_KIB = 2 * 1024 * 1024


def short(name: str) -> str:
    for key in KNOWN:
        if key in name:
            return key
    return name[:40]


def counter_by_kernel(path: str, counter: str):
    acc = collections.defaultdict(list)
    with open(path, newline="") as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] == counter:
                acc[short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return acc


def git_head() -> str:
    try:
        r = subprocess.run(["git", "-C", ROOT, "rev-parse", "--short=12", "HEAD"], capture_output=True, text=True)
        return r.stdout.strip() or "unknown"
    except Exception:
        return "unknown"


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--dir", required=True, help="directory holding trace/, fetch/, write/")
    ap.add_argument("--kernel", required=True, help="short kernel name, e.g. attn_kernel")
    ap.add_argument("--alg-bytes", type=int, required=True, help="algorithmic bytes per launch of that kernel")
    ap.add_argument("--out", required=True, help="markdown summary to write (under profiles/)")
    ap.add_argument("--json-key", required=True, help="key in profiles/hbm_traffic.json")
    ap.add_argument("--title", required=True)
    ap.add_argument("--bench-args", default="", help="extra bench.py arguments of the profiled runs")
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--note", default="", help="sentence on what the launches are")
    ap.add_argument("--commit", default="", help="commit the profiled tree was built from (default: HEAD)")
    a = ap.parse_args()

    base = a.dir.rstrip("/")
    rel = os.path.relpath(os.path.abspath(base), ROOT)
    with open(f"{base}/trace/t_kernel_stats.csv", newline="") as f:
        rows = list(csv.DictReader(f))
    commit = a.commit or git_head()
    cmd = (f"python3 $R/bench.py --steps {a.steps} --warmup {a.warmup} --skip-cpu --skip-extra --copy-calibration "
           f"--settle-seconds 0{(' ' + a.bench_args) if a.bench_args else ''}")
    out = [f"# {a.title}\n",
           f"MI355X (gfx950), ROCm 7.2, one GPU, tree at commit {commit}. Each command was run from /tmp with TMPDIR=/tmp, "
           "on a GPU that had been idle for 8 s (a process started right after another one streams a few per cent "
           "slower at first); `$R` is the repository root. Summarised by "
           "`python -m paper_2605_23389_amd.profile_summary`.\n",
           f"## Pass 1: kernel trace\n\n```\nrocprofv3 --kernel-trace --stats --output-format csv -d $R/{rel}/trace -o t -- {cmd}\n```\n",
           "| kernel | calls | total ms | avg us | min us | max us | % |\n|---|---|---|---|---|---|---|"]
    for r in rows:
        out.append(f"| {short(r['Name'])} | {r['Calls']} | {int(r['TotalDurationNs']) / 1e6:.3f} | "
                   f"{float(r['AverageNs']) / 1e3:.2f} | {int(r['MinNs']) / 1e3:.2f} | {int(r['MaxNs']) / 1e3:.2f} | "
                   f"{r['Percentage']} |")
    main_row = [r for r in rows if short(r["Name"]) == a.kernel][0]
    avg_us = float(main_row["AverageNs"]) / 1e3
    gbs = a.alg_bytes / avg_us / 1e3
    out.append(f"\n{a.note} Algorithmic bytes per launch = {a.alg_bytes} B; average `{a.kernel}` duration "
               f"{avg_us:.2f} us => {gbs:.0f} GB/s = {gbs / 80:.1f} % of 8 TB/s.\n")

    fe = counter_by_kernel(f"{base}/fetch/f_counter_collection.csv", "FETCH_SIZE")
    wr = counter_by_kernel(f"{base}/write/w_counter_collection.csv", "WRITE_SIZE")
    big_f = [v for v in fe["copyBuffer"] if v > 1e5]
    big_w = [v for v in wr["copyBuffer"] if v > 1e5]
    if not big_f or not big_w:
        raise SystemExit("no 2 GiB calibration copies in the counter runs: profile with --copy-calibration")
    ff = COPY_KIB / (sum(big_f) / len(big_f))
    wf = COPY_KIB / (sum(big_w) / len(big_w))
    out.append(f"## Pass 2 and 3: HBM traffic counters\n\n```\nrocprofv3 --pmc FETCH_SIZE --output-format csv -d "
               f"$R/{rel}/fetch -o f -- {cmd}\nrocprofv3 --pmc WRITE_SIZE --output-format csv -d $R/{rel}/write -o w "
               f"-- {cmd}\n```\n")
    out.append("Calibration: `--copy-calibration` runs three plain 2 GiB device-to-device copies "
               "(__amd_rocclr_copyBuffer), true traffic 2 GiB read + 2 GiB written each.\n")
    out.append("| counter | copy kernel reading (KiB/dispatch) | true (KiB) | scale factor |\n|---|---|---|---|\n"
               f"| FETCH_SIZE | {sum(big_f) / len(big_f):.1f} | {COPY_KIB} | {ff:.4f} |\n"
               f"| WRITE_SIZE | {sum(big_w) / len(big_w):.1f} | {COPY_KIB} | {wf:.4f} |\n")
    out.append("| kernel | dispatches | FETCH_SIZE avg KiB | scaled read MB | WRITE_SIZE avg KiB | scaled write MB |\n"
               "|---|---|---|---|---|---|")
    res = {}
    for k in (a.kernel, "combine_kernel", "plan_kernel"):
        if k not in fe or k not in wr:
            continue
        f_avg = sum(fe[k]) / len(fe[k])
        w_avg = sum(wr[k]) / len(wr[k])
        res[k] = (f_avg * ff * 1024, w_avg * wf * 1024)
        out.append(f"| {k} | {len(fe[k])} | {f_avg:.1f} | {res[k][0] / 1e6:.2f} | {w_avg:.1f} | {res[k][1] / 1e6:.2f} |")
    tot = sum(res[a.kernel])
    out.append(f"\n`{a.kernel}` HBM traffic per launch = {res[a.kernel][0] / 1e6:.1f} MB read + "
               f"{res[a.kernel][1] / 1e6:.1f} MB written = {tot / 1e6:.1f} MB = {tot / a.alg_bytes:.4f} x the algorithmic "
               f"{a.alg_bytes / 1e6:.1f} MB (whole 16-token blocks are fetched, so the padded rows of each request's last "
               "block are included; writes are the output and the split-KV partials).\n")
    with open(a.out, "w") as f:
        f.write("\n".join(out) + "\n")
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        tj = json.load(open(tpath))
    except Exception:
        tj = {}
    tj[a.json_key] = {"bytes_per_launch": round(tot), "alg_bytes_per_launch": a.alg_bytes,
                      "ratio": round(tot / a.alg_bytes, 4), "avg_kernel_us": round(avg_us, 2),
                      "fetch_scale": round(ff, 4), "write_scale": round(wf, 4), "commit": commit,
                      "summary": os.path.relpath(os.path.abspath(a.out), ROOT)}
    with open(tpath, "w") as f:
        json.dump(tj, f, indent=1)
    print(a.out, f"avg {avg_us:.1f} us, {gbs:.0f} GB/s, traffic ratio {tot / a.alg_bytes:.4f}, commit {commit}")


if __name__ == "__main__":
    main()
