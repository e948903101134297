"""Summarises two rocprofv3 --pmc runs of bench.py (FETCH_SIZE, then WRITE_SIZE) into the HBM traffic per launch.

    cd /tmp && export TMPDIR=/tmp && cd <repo>
    rocprofv3 --pmc FETCH_SIZE -d gpurun_out/pmc_fetch -o f --output-format csv -- python3 bench.py --steps 1 --warmup 1 --no-cpu-baseline --no-frontier --no-secondary --no-auto-ratio
    rocprofv3 --pmc WRITE_SIZE -d gpurun_out/pmc_write -o w --output-format csv -- python3 bench.py --steps 1 --warmup 1 --no-cpu-baseline --no-frontier --no-secondary --no-auto-ratio
    python3 -m paper_2503_01328_amd.profile_traffic C2 <fetch counter csv> <write counter csv>

Both counters read KiB per dispatch.  They are scaled by what they read for a plain copy kernel of known size in
the same run (po::copy16_kernel copies one [s, h] stage input per launch).  Writes the table to
profiles/hbm_traffic_<workload>.md and the average over all bf16 matrix-core GEMM launches, with the commit the
tree is at, to profiles/gemm_hbm_traffic.txt, which bench.py reads for roofline.traffic.
"""
from __future__ import annotations

import collections
import csv
import os
import subprocess
import sys

from . import inputs as syn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _load(path, counter):
    d = collections.OrderedDict()
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        name = r["Kernel_Name"].split("(")[0].replace("void ", "")
        e = d.setdefault((name, r["Grid_Size"]), [0, 0.0])
        e[0] += 1
        e[1] += float(r["Counter_Value"])
    return d


def main():
    workload, fetch_csv, write_csv = sys.argv[1:4]
    shape = syn.CONFIGS[workload]
    F, W = _load(fetch_csv, "FETCH_SIZE"), _load(write_csv, "WRITE_SIZE")
    ck = [k for k in F if "copy16" in k[0]][0]
    copy_kib = shape.seq * shape.hidden * 2 / 1024.0
    fs, ws = copy_kib / (F[ck][1] / F[ck][0]), copy_kib / (W[ck][1] / W[ck][0])
    rows, gemm_n, gemm_b = [], 0, 0.0
    for k in F:
        if k not in W:
            continue
        n, f, w = F[k][0], F[k][1] / F[k][0], W[k][1] / W[k][0]
        rows.append((k[0], k[1], n, f, w, (f * fs + w * ws) / 1024.0))
        if "gemm_mfma" in k[0]:
            gemm_n += n
            gemm_b += n * (f * fs + w * ws) * 1024.0
    rows.sort(key=lambda r: -r[2] * r[5])
    avg = gemm_b / gemm_n
    commit = subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], capture_output=True,
                            text=True).stdout.strip() or "unknown"
    flags = "--steps 1 --warmup 1 --no-cpu-baseline --no-frontier --no-secondary --no-auto-ratio"
    cfg = "" if workload == "C2" else f" --config {workload}"
    L = [f"# HBM traffic per launch, workload {workload} (rocprofv3 --pmc), tree at {commit}", "",
         "Commands (on the MI355X box, from the repository root; one counter per run):", "",
         f"    rocprofv3 --pmc FETCH_SIZE -d gpurun_out/pmc_fetch -o f --output-format csv -- python3 bench.py{cfg} {flags}",
         f"    rocprofv3 --pmc WRITE_SIZE -d gpurun_out/pmc_write -o w --output-format csv -- python3 bench.py{cfg} {flags}",
         f"    python3 -m paper_2503_01328_amd.profile_traffic {workload} <fetch counter csv> <write counter csv>", "",
         f"Calibration: `po::copy16_kernel` copies exactly {copy_kib:.0f} KiB (one [s, h] bf16 stage input) per launch in "
         f"this workload. FETCH_SIZE reads {F[ck][1] / F[ck][0]:.0f} KiB for it and WRITE_SIZE {W[ck][1] / W[ck][0]:.0f} "
         f"KiB, so readings are scaled by {fs:.3f} (fetch) and {ws:.3f} (write).", "",
         f"All bf16 MFMA GEMM launches of the run ({gemm_n}): scaled traffic {avg / 2 ** 20:.1f} MiB per launch on "
         f"average ({avg:.0f} bytes: the `roofline.traffic` figure of bench.py, read from "
         f"`profiles/gemm_hbm_traffic.txt`). The counters sit at the L2's far side, so what the infinity cache serves "
         f"is counted as traffic too.", "",
         "| kernel | grid (threads) | launches | FETCH_SIZE KiB/launch | WRITE_SIZE KiB/launch | scaled MiB/launch |",
         "|---|---:|---:|---:|---:|---:|"]
    for r in rows[:22]:
        L.append(f"| `{r[0][:80]}` | {r[1]} | {r[2]} | {r[3]:.0f} | {r[4]:.0f} | {r[5]:.1f} |")
    out_md = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload.lower()}.md")
    open(out_md, "w").write("\n".join(L) + "\n")
    table = os.path.join(ROOT, "profiles", "gemm_hbm_traffic.txt")
    lines = []
    if os.path.exists(table):
        lines = [l for l in open(table).read().splitlines() if l and not l.startswith("#") and l.split()[0] != workload]
    head = ["# HBM bytes per bf16 matrix-core GEMM launch (average over all GEMM launches of a bench.py run), from the",
            "# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes summarised in profiles/hbm_traffic_<workload>.md.",
            "# workload bytes_per_launch commit_the_tree_was_at"]
    open(table, "w").write("\n".join(head + lines + [f"{workload} {avg:.0f} {commit}"]) + "\n")
    print(f"{workload}: {avg:.0f} bytes per GEMM launch -> {out_md}, {table}")


if __name__ == "__main__":
    main()
