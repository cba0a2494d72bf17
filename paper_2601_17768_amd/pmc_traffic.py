"""Turns rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of bench.py into the per-launch HBM-side traffic figure
that bench.py reports as roofline.traffic, and records it in profiles/pmc_traffic.txt together with a digest
of the kernel sources it was measured on (bench.py reports the figure only while that digest still matches).

    rocprofv3 --pmc FETCH_SIZE --kernel-include-regex "<kernel regex>|elementwise" -d <fetch dir> -o run \\
        --output-format csv -- python3 bench.py --workload c5 --no-others --layers 2 --steps 1 --warmup 1 \\
        --no-cpu-baseline --no-graph --pmc-calibration
    (the same with WRITE_SIZE into <write dir>)
    python -m paper_2601_17768_amd.pmc_traffic --workload c5 --kernel gate_up --regex "gemm_tiled.*Swiglu" \\
        --fetch <fetch dir> --write <write dir>

The counters come in KiB per dispatch; each is scaled by what the same counter reads for the plain elementwise
kernel that --pmc-calibration adds to the run (256 MiB read, 256 MiB written).
"""
from __future__ import annotations

import argparse
import csv
import glob
import os
import re
import subprocess

from .build import kernel_sources_digest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OUT = os.path.join(ROOT, "profiles", "pmc_traffic.txt")
CAL_BYTES = 256 * 1024 * 1024


def counter_per_launch(directory: str, counter: str, regex: str):
    """(average counter value per launch of the kernels matching regex, the same for the calibration kernel)."""
    rows = []
    for path in glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True):
        rows += list(csv.DictReader(open(path)))
    pick = lambda pat: [float(r["Counter_Value"]) for r in rows
                        if r["Counter_Name"] == counter and re.search(pat, r["Kernel_Name"])]
    # the calibration kernel: bench.py's `torch.add(x, 1.0, out=y)` on 64 Mi floats (torch's fills and copies of the
    # same run are elementwise kernels too, but not this functor)
    kern, cal = pick(regex), pick(r"elementwise.*_add<float>")
    if not kern or not cal:
        raise SystemExit(f"{directory}: no {counter} rows for /{regex}/ ({len(kern)}) or the calibration kernel ({len(cal)})")
    return sum(kern) / len(kern), sum(cal) / len(cal), len(kern)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--kernel", required=True, help="gate_up or attention")
    ap.add_argument("--regex", required=True)
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--out", default=OUT)
    a = ap.parse_args()
    f_k, f_cal, n = counter_per_launch(a.fetch, "FETCH_SIZE", a.regex)
    w_k, w_cal, _ = counter_per_launch(a.write, "WRITE_SIZE", a.regex)
    traffic = f_k * (CAL_BYTES / f_cal) + w_k * (CAL_BYTES / w_cal)
    digest = kernel_sources_digest()
    entries = {}
    if os.path.exists(a.out):
        for line in open(a.out):
            if "=" in line and not line.lstrip().startswith("#"):
                k, v = line.split("=", 1)
                entries[k.strip()] = v.strip()
    if entries.get("kernel_sources_sha256") != digest:
        entries = {}                      # figures measured on other kernels do not carry over
    entries["kernel_sources_sha256"] = digest
    try:
        entries["commit"] = subprocess.check_output(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], text=True).strip()
    except Exception:
        entries.setdefault("commit", "unknown")
    entries[f"{a.workload}.{a.kernel}"] = str(int(round(traffic)))
    entries[f"{a.workload}.{a.kernel}.detail"] = (f"FETCH_SIZE {f_k:.1f} KiB x {CAL_BYTES / f_cal / 1024:.4f} + WRITE_SIZE {w_k:.1f} KiB x "
                                                  f"{CAL_BYTES / w_cal / 1024:.4f}, {n} launches of /{a.regex}/")
    with open(a.out, "w") as f:
        f.write("# HBM-side bytes per launch (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, each scaled by a plain kernel of known\n"
                "# traffic in the same run), written by `python -m paper_2601_17768_amd.pmc_traffic`; read by bench.py, which\n"
                "# reports a figure only while kernel_sources_sha256 matches the sources it runs.\n")
        for k in sorted(entries, key=lambda k: (k not in ("kernel_sources_sha256", "commit"), k)):
            f.write(f"{k} = {entries[k]}\n")
    print(f"{a.workload}.{a.kernel}: {traffic / 1e6:.1f} MB per launch -> {a.out}")


if __name__ == "__main__":
    main()
