"""Turns the CSV output of four rocprofv3 runs of `bench.py --config NAME` into the text summary kept under
profiles/ and into the table bench.py reads its `roofline.traffic` from (profiles/kernel_traffic.txt).

  python -m paper_2406_17145_amd.profile_summary OUT_DIR NAME [--note TEXT] [--bench-flags "FLAGS"]

OUT_DIR holds, for workload NAME, the output of (run from /tmp with TMPDIR=/tmp; REPO = repository root):

  rocprofv3 --kernel-trace --stats --output-format csv -d OUT_DIR/NAME/stats -o NAME -- python3 REPO/bench.py --config NAME FLAGS --steps 5 --warmup 2
  rocprofv3 --kernel-trace --pmc FETCH_SIZE --output-format csv -d OUT_DIR/NAME/pmc_FETCH_SIZE -o NAME -- python3 REPO/bench.py --config NAME FLAGS --steps 2 --warmup 1
  rocprofv3 --kernel-trace --pmc WRITE_SIZE ...                       -d OUT_DIR/NAME/pmc_WRITE_SIZE   (same command, other counter)
  rocprofv3 --kernel-trace --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_LDS_BANK_CONFLICT SQ_ACTIVE_INST_LDS SQ_WAIT_INST_LDS GRBM_GUI_ACTIVE ...
                                                                       -d OUT_DIR/NAME/pmc_SQ           (same command)

with FLAGS = --no-cpu-baseline --no-kernel-pass --no-step-times --copy-calibration 256 plus a schedule that puts every
launch of the timed configuration on one stream (so that every launch is one row of the kernel trace).  The 256 MiB
elementwise copy of --copy-calibration gives the factor between what FETCH_SIZE / WRITE_SIZE read and bytes moved.

No GPU is needed here: this only reads CSV files.
"""
from __future__ import annotations

import argparse
import collections
import csv
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SQ_COUNTERS = "SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_LDS_BANK_CONFLICT SQ_ACTIVE_INST_LDS SQ_WAIT_INST_LDS GRBM_GUI_ACTIVE"
CAL_MIB = 256

# kernel name (as rocprofv3 prints it, namespace stripped) -> kernel family of bench.py's `kernels` table
FAMILIES = [
    (r"k_gemm_(big|mid)_dw_group|k_gemm_(big|mid)<2", "gemm_big_dw"),
    (r"k_gemm_(big|mid)<0", "gemm_big_fwd"),
    (r"k_gemm_(big|mid)<1", "gemm_big_dx"),
    (r"k_gemm_skinny<0", "gemm_skinny_fwd"),
    (r"k_gemm_skinny<1", "gemm_skinny_dx"),
    (r"k_gemm_bwd_merged", "gemm_bwd_merged_dx_dw"),
    (r"k_gemm_dw_ksplit", "gemm_dw_ksplit"),
    (r"k_emb_fwd", "embedding_fwd"),
    (r"k_sort_|k_emb_bwd_", "embedding_bwd_sort_segsum"),
    (r"k_attn_fwd", "attention_fwd"),
    (r"k_attn_bwd_dq", "attention_bwd_dq"),
    (r"k_attn_bwd_dkv", "attention_bwd_dkv"),
    (r"k_ln_fwd", "layernorm_fwd"),
    (r"k_ln_bwd_vec|k_ln_bwd<", "layernorm_bwd_dx"),
    (r"k_ln_bwd_params", "layernorm_bwd_params"),
    (r"k_interact_fwd", "interact_fwd"),
    (r"k_interact_bwd", "interact_bwd"),
]


def short(name):
    name = name.replace("gpp::", "").replace("void ", "")
    i = name.find("(")
    return (name[:i] if i > 0 else name)[:64]


def family(kernel):
    for pat, fam in FAMILIES:
        if re.search(pat, kernel):
            return fam
    return None


def counters(base, cfg, run):
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    path = os.path.join(base, run, f"{cfg}_counter_collection.csv")
    if not os.path.exists(path):
        return acc
    for r in csv.DictReader(open(path)):
        key = short(r["Kernel_Name"]) + (" grid=%s" % r["Grid_Size"] if "elementwise" in r["Kernel_Name"] else "")
        acc[key][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return acc


def summarise(out_dir, cfg, note, flags):
    base = os.path.join(out_dir, cfg)
    lines = []
    add = lines.append
    add(f"# rocprofv3 summary: one GPP stage, workload {cfg} (bench.py --config {cfg}), MI355X")
    add(f"# commands (from /tmp, TMPDIR=/tmp; <repo> = repository root; {note}):")
    add(f"#   rocprofv3 --kernel-trace --stats --output-format csv -d <out>/{cfg}/stats -o {cfg} -- python3 <repo>/bench.py --config {cfg} {flags} --steps 5 --warmup 2")
    add(f"#   rocprofv3 --kernel-trace --pmc FETCH_SIZE --output-format csv -d <out>/{cfg}/pmc_FETCH_SIZE -o {cfg} -- python3 <repo>/bench.py --config {cfg} {flags} --steps 2 --warmup 1")
    add("#   rocprofv3 --kernel-trace --pmc WRITE_SIZE ...   (same command, other counter)")
    add(f"#   rocprofv3 --kernel-trace --pmc {SQ_COUNTERS} ...   (same command)")
    add(f"#   python -m paper_2406_17145_amd.profile_summary <out> {cfg}      (this file and the {cfg} rows of kernel_traffic.txt)")
    bench_json = os.path.join(base, "stats.json")
    if os.path.exists(bench_json):
        import json
        d = json.loads(open(bench_json).read().strip().splitlines()[-1])
        add(f"# bench line of the stats run (under the profiler): {d['value']:.0f} samples/s, {d['ms_per_step']:.3f} ms/step, {d['config']['workload']}")
    add("# (the at::native / __amd_rocclr rows are the bench's own set-up and the calibration copy, not the stage)")
    add("")
    rows = list(csv.DictReader(open(os.path.join(base, "stats", f"{cfg}_kernel_stats.csv"))))
    add("## kernel durations (rocprofv3 --kernel-trace --stats)")
    add("%-64s %7s %12s %9s %7s" % ("kernel", "calls", "total_us", "avg_us", "share%"))
    for r in rows[:22]:
        add("%-64s %7s %12.1f %9.2f %7.2f" % (short(r["Name"]), r["Calls"], float(r["TotalDurationNs"]) / 1e3,
                                              float(r["AverageNs"]) / 1e3, float(r["Percentage"])))
    f, w = counters(base, cfg, "pmc_FETCH_SIZE"), counters(base, cfg, "pmc_WRITE_SIZE")
    traffic = {}
    if f and w:
        cal = max((k for k in f if "elementwise" in k), key=lambda k: sum(f[k]["FETCH_SIZE"]) / len(f[k]["FETCH_SIZE"]))
        cf = sum(f[cal]["FETCH_SIZE"]) / len(f[cal]["FETCH_SIZE"])
        cw = sum(w[cal]["WRITE_SIZE"]) / len(w[cal]["WRITE_SIZE"])
        kib = CAL_MIB * 1024.0
        sf, sw = kib / cf, kib / cw
        add("")
        add("## HBM traffic per launch (rocprofv3 --pmc FETCH_SIZE / --pmc WRITE_SIZE, KiB per dispatch)")
        add(f"calibration: elementwise copy of {CAL_MIB} MiB ({cal}): FETCH_SIZE reads {cf:.0f} KiB, WRITE_SIZE reads {cw:.0f} KiB for {kib:.0f} KiB each way")
        add(f"scale factors: fetch x{sf:.4f}, write x{sw:.4f}")
        add("%-64s %7s %12s %12s %12s" % ("kernel", "calls", "fetch_MB", "write_MB", "total_MB"))
        fam_bytes, fam_calls = collections.defaultdict(float), collections.defaultdict(int)
        for k in sorted(f, key=lambda k: -sum(f[k]["FETCH_SIZE"])):
            if "elementwise" in k or "rocclr" in k:
                continue
            n = len(f[k]["FETCH_SIZE"])
            fm = sum(f[k]["FETCH_SIZE"]) / n * sf * 1024 / 1e6
            wm = sum(w[k]["WRITE_SIZE"]) / max(1, len(w[k]["WRITE_SIZE"])) * sw * 1024 / 1e6 if k in w else float("nan")
            add("%-64s %7d %12.3f %12.3f %12.3f" % (k, n, fm, wm, fm + wm))
            fam = family(k)
            if fam and wm == wm:
                fam_bytes[fam] += (fm + wm) * 1e6 * n
                fam_calls[fam] += n
        traffic = {fam: fam_bytes[fam] / fam_calls[fam] for fam in fam_bytes}
    s = counters(base, cfg, "pmc_SQ")
    if s:
        add("")
        add(f"## SQ counters per launch (rocprofv3 --pmc {SQ_COUNTERS})")
        add("# mfma_util = SQ_VALU_MFMA_BUSY_CYCLES / (1024 SIMDs x GRBM_GUI_ACTIVE / 8 XCDs): share of SIMD cycles with the matrix pipe busy")
        add("%-64s %7s %10s %12s %12s %12s" % ("kernel", "calls", "gui_cyc/8", "mfma_util", "lds_wait/sq_busy", "bank_confl/lds_active"))
        for k in sorted(s, key=lambda k: -sum(s[k]["GRBM_GUI_ACTIVE"])):
            if "elementwise" in k or "rocclr" in k:
                continue
            c = {n: sum(v) / len(v) for n, v in s[k].items()}
            b = max(c.get("SQ_BUSY_CYCLES", 0), 1)
            add("%-64s %7d %10.0f %12.3f %12.3f %12.3f" % (
                k, len(s[k]["GRBM_GUI_ACTIVE"]), c["GRBM_GUI_ACTIVE"] / 8, c["SQ_VALU_MFMA_BUSY_CYCLES"] / (1024 * c["GRBM_GUI_ACTIVE"] / 8),
                c["SQ_WAIT_INST_LDS"] / b, c["SQ_LDS_BANK_CONFLICT"] / max(c["SQ_ACTIVE_INST_LDS"], 1)))
    return "\n".join(lines) + "\n", traffic


def update_traffic_table(cfg, traffic, path):
    """kernel_traffic.txt: `workload | kernel family | bytes per launch | source`; the rows of `cfg` are replaced."""
    keep = []
    if os.path.exists(path):
        for line in open(path):
            part = [v.strip() for v in line.split("|")]
            if line.startswith("#") or len(part) < 3 or part[0] != cfg:
                keep.append(line.rstrip("\n"))
    if not any(l.startswith("#") for l in keep):
        keep = ["# HBM bytes per launch of a kernel family of a workload, averaged over the family's launches in a step:",
                "# FETCH_SIZE + WRITE_SIZE of two rocprofv3 --pmc runs, scaled by what the same counters read for a 256 MiB copy.",
                "# Written by `python -m paper_2406_17145_amd.profile_summary` from the runs named in the source column; read by bench.py.",
                "# workload | kernel family | bytes per launch | source"] + keep
    for fam in sorted(traffic):
        keep.append(f"{cfg} | {fam} | {traffic[fam]:.0f} | stage_{cfg}_kernels_traffic_counters.txt")
    with open(path, "w") as f:
        f.write("\n".join(keep) + "\n")


def main(argv=None):
    ap = argparse.ArgumentParser(prog="python -m paper_2406_17145_amd.profile_summary")
    ap.add_argument("out_dir")
    ap.add_argument("config")
    ap.add_argument("--note", default="serial schedule, eager launches, so that every launch is one row of the kernel trace")
    ap.add_argument("--bench-flags", default="--no-cpu-baseline --no-kernel-pass --no-step-times --schedule serial --graph off --copy-calibration 256")
    ap.add_argument("--profiles", default=os.path.join(ROOT, "profiles"))
    args = ap.parse_args(argv)
    text, traffic = summarise(args.out_dir, args.config, args.note, args.bench_flags)
    os.makedirs(args.profiles, exist_ok=True)
    out = os.path.join(args.profiles, f"stage_{args.config}_kernels_traffic_counters.txt")
    with open(out, "w") as f:
        f.write(text)
    if traffic:
        update_traffic_table(args.config, traffic, os.path.join(args.profiles, "kernel_traffic.txt"))
    print(f"wrote {out}" + (f" and {len(traffic)} rows of kernel_traffic.txt" if traffic else ""))


if __name__ == "__main__":
    main()
