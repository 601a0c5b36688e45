"""Turns rocprofv3 CSV output of a bench.py run into the short text summaries kept
under profiles/.

  python -m paper_2505_23219_amd.profile_summary stats   KERNEL_STATS.csv OUT.md --command "..."
  python -m paper_2505_23219_amd.profile_summary traffic FETCH.csv WRITE.csv OUT.md --command "..."
  python -m paper_2505_23219_amd.profile_summary counter COUNTERS.csv NAME OUT.md --command "..."

`stats` lists this library's kernels from a `--kernel-trace --stats` run.  `traffic`
takes the counter_collection CSVs of two `--pmc` runs (FETCH_SIZE, then WRITE_SIZE) of
`bench.py --pmc-calibrate`, scales each counter by what it reads for the calibration
copy kernel of known size, and records the HBM bytes per launch of the linear-layer
kernel together with a digest of the kernel sources the figure belongs to.
"""
from __future__ import annotations

import argparse
import csv
import hashlib
import os
import re
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CALIBRATION_BYTES = 1 << 30          # bench.py --pmc-calibrate copies 1 GiB
LINEAR_KERNEL = re.compile(r"k_linear<4, \d+, \d+>")        # linear-only launches of the M = 64 step
FUSED_KERNEL = re.compile(r"k_qkv_attn<4, \d+, \d+>")      # QKV layer + attention in one launch
COPY_KERNEL = re.compile(r"k_debug_copy")


def source_digest() -> str:
    """sha256 over the kernel sources: a recorded counter figure is only valid for the
    sources it was taken with."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2505_23219_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")):
            with open(os.path.join(d, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()


def _short(name: str) -> str:
    name = name.strip('"')
    return name if len(name) <= 90 else name[:87] + "..."


def stats(path: str, out: str, command: str) -> None:
    rows = [r for r in csv.DictReader(open(path)) if "ghd" in r["Name"]]
    total = sum(int(r["TotalDurationNs"]) for r in rows)
    with open(out, "w") as f:
        f.write("# rocprofv3 kernel statistics: verification step, workload stack7b\n\n")
        f.write("Command (on an MI355X, from the repository root):\n\n    %s\n\n" % command)
        f.write("Kernels of this library only (model set-up and PyTorch fill kernels left out); "
                "the run holds tree steps (M=64: `k_linear<4, R, RB>`, `k_qkv_attn<4, R, 128>`) and 1-token "
                "decode steps (`k_linear<1, R, RB>`, `k_qkv_attn<1, R, 128>`); R = row tiles streamed together, "
                "RB = tiles per row block (4: narrow matrices, split along K).\n\n")
        f.write("| kernel | calls | avg us | min us | max us | total ms | share |\n|---|---|---|---|---|---|---|\n")
        for r in sorted(rows, key=lambda r: -int(r["TotalDurationNs"])):
            f.write("| `%s` | %s | %.2f | %.2f | %.2f | %.3f | %.1f%% |\n" % (
                _short(r["Name"]), r["Calls"], float(r["AverageNs"]) / 1e3, int(r["MinNs"]) / 1e3,
                int(r["MaxNs"]) / 1e3, int(r["TotalDurationNs"]) / 1e6,
                100.0 * int(r["TotalDurationNs"]) / total))


def _counter(path: str, name: str):
    copy, lin, fused = [], [], []
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != name:
            continue
        v = float(r["Counter_Value"])
        if COPY_KERNEL.search(r["Kernel_Name"]):
            copy.append(v)
        elif LINEAR_KERNEL.search(r["Kernel_Name"]):
            lin.append(v)
        elif FUSED_KERNEL.search(r["Kernel_Name"]):
            fused.append(v)
    if not copy or not lin:
        sys.exit("%s: calibration copy or linear-layer dispatches missing" % path)
    avg = lambda v: sum(v) / len(v) if v else 0.0
    return avg(copy), avg(lin), len(lin), avg(fused), len(fused)


def traffic(fetch_csv: str, write_csv: str, out: str, command: str) -> None:
    f_copy, f_lin, n, f_fus, nf = _counter(fetch_csv, "FETCH_SIZE")
    w_copy, w_lin, _, w_fus, _ = _counter(write_csv, "WRITE_SIZE")
    f_scale = CALIBRATION_BYTES / f_copy       # bytes per counter unit
    w_scale = CALIBRATION_BYTES / w_copy
    fetched, written = f_lin * f_scale, w_lin * w_scale
    with open(out, "w") as f:
        f.write("# HBM traffic of the linear-layer kernel `k_linear<4, R, RB>`, workload stack7b\n\n")
        f.write("Commands (on an MI355X, from the repository root; one counter per run):\n\n")
        f.write("    %s\n\n" % command.replace("COUNTER", "FETCH_SIZE"))
        f.write("    %s\n\n" % command.replace("COUNTER", "WRITE_SIZE"))
        f.write("Calibration: the 1 GiB copy kernel of the same run (reads 1 GiB, writes 1 GiB) "
                "reads FETCH_SIZE = %.1f and WRITE_SIZE = %.1f, i.e. %.1f and %.1f bytes per "
                "counter unit.\n\n" % (f_copy, w_copy, f_scale, w_scale))
        f.write("Average over %d dispatches of the linear-only launches (output, gate|up and down "
                "projection of every layer + LM head, M = 64)" % n)
        if nf:
            f.write(" and over %d dispatches of `k_qkv_attn<4, R, 128>` (QKV layer + tree attention)" % nf)
        f.write(":\n\n| kernel | | counter avg | bytes per launch |\n|---|---|---|---|\n")
        f.write("| k_linear | fetched | %.1f | %d |\n| k_linear | written | %.1f | %d |\n" % (f_lin, fetched, w_lin, written))
        if nf:
            f.write("| k_qkv_attn | fetched | %.1f | %d |\n| k_qkv_attn | written | %.1f | %d |\n"
                    % (f_fus, f_fus * f_scale, w_fus, w_fus * w_scale))
        f.write("\ntraffic_bytes_per_launch: %d\n" % int(fetched + written))
        if nf:
            f.write("qkv_attention_traffic_bytes_per_launch: %d\n" % int(f_fus * f_scale + w_fus * w_scale))
        f.write("source_sha256: %s\n" % source_digest())


def counter(path: str, name: str, out: str, command: str) -> None:
    """Average of one (derived) counter per kernel of this library."""
    acc = {}
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != name or "ghd" not in r["Kernel_Name"]:
            continue
        acc.setdefault(_short(r["Kernel_Name"]), []).append(float(r["Counter_Value"]))
    if not acc:
        sys.exit("%s: no %s rows for this library's kernels" % (path, name))
    with open(out, "w") as f:
        f.write("# %s per kernel, workload stack7b\n\n" % name)
        f.write("Command (on an MI355X, from the repository root):\n\n    %s\n\n" % command)
        f.write("| kernel | dispatches | avg %s | min | max |\n|---|---|---|---|---|\n" % name)
        for k, v in sorted(acc.items(), key=lambda kv: -len(kv[1])):
            f.write("| `%s` | %d | %.2f | %.2f | %.2f |\n" % (k, len(v), sum(v) / len(v), min(v), max(v)))


def main() -> None:
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="what", required=True)
    a = sub.add_parser("stats")
    a.add_argument("csv")
    a.add_argument("out")
    a.add_argument("--command", required=True)
    b = sub.add_parser("traffic")
    b.add_argument("fetch_csv")
    b.add_argument("write_csv")
    b.add_argument("out")
    b.add_argument("--command", required=True)
    c = sub.add_parser("counter")
    c.add_argument("csv")
    c.add_argument("name")
    c.add_argument("out")
    c.add_argument("--command", required=True)
    args = ap.parse_args()
    if args.what == "counter":
        counter(args.csv, args.name, args.out, args.command)
    elif args.what == "stats":
        stats(args.csv, args.out, args.command)
    else:
        traffic(args.fetch_csv, args.write_csv, args.out, args.command)


if __name__ == "__main__":
    main()
