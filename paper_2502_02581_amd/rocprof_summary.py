#!/usr/bin/env python3
"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2502_02581_amd.rocprof_summary stats   <kernel_stats.csv> <out.md> --cmd "<command>"
    python -m paper_2502_02581_amd.rocprof_summary traffic <fetch counter csv> <write counter csv> <out.txt>
                                                           --probe-bytes N --cmd "<command>"

`stats` keeps the per-kernel call count and durations of a `--kernel-trace --stats` run.
`traffic` takes two `--pmc` runs of the same command (FETCH_SIZE, then WRITE_SIZE), averages each
counter per dispatch and per kernel, and scales it to bytes with what the same counter reads for
the library's copy_probe_kernel, which moves exactly --probe-bytes bytes each way.
"""
from __future__ import annotations

import argparse
import collections
import csv
import re


def short_name(n: str) -> str:
    n = re.sub(r"void at::native::.*?distribution.*", "at::native::distribution_elementwise (torch.randn: input generation, untimed)", n)
    n = n.replace("void moe::", "moe::")
    return n if len(n) < 220 else n[:217] + "..."


def stats(args):
    rows = list(csv.DictReader(open(args.csv)))
    with open(args.out, "w") as f:
        f.write("# rocprofv3 --kernel-trace --stats summary\n\nCommand (run from the repo root on one MI355X):\n\n")
        f.write(f"    {args.cmd}\n\nCalls include the warm-up steps. Durations in microseconds.\n\n")
        f.write("| kernel | calls | total us | avg us | min us | max us | % |\n|---|---|---|---|---|---|---|\n")
        for r in rows:
            if float(r["Percentage"]) < 0.01:
                continue
            f.write(f"| `{short_name(r['Name'])}` | {r['Calls']} | {int(r['TotalDurationNs']) / 1e3:.1f} | "
                    f"{float(r['AverageNs']) / 1e3:.1f} | {int(r['MinNs']) / 1e3:.1f} | {int(r['MaxNs']) / 1e3:.1f} | "
                    f"{r['Percentage']} |\n")


def per_kernel(path, counter):
    tot, n = collections.defaultdict(float), collections.Counter()
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        tot[r["Kernel_Name"]] += float(r["Counter_Value"])
        n[r["Kernel_Name"]] += 1
    return {k: (tot[k] / n[k], n[k]) for k in tot}


def traffic(args):
    fetch = per_kernel(args.fetch_csv, "FETCH_SIZE")
    write = per_kernel(args.write_csv, "WRITE_SIZE")
    probe = [k for k in fetch if "copy_probe_kernel" in k]
    if not probe or probe[0] not in write:
        raise SystemExit("no copy_probe_kernel dispatch in the counter files: the scale factor cannot be derived")
    f_fac = args.probe_bytes / fetch[probe[0]][0]
    w_fac = args.probe_bytes / write[probe[0]][0]
    with open(args.out, "w") as f:
        f.write("# HBM traffic per launch from rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE\n#\n")
        f.write(f"# Command (run twice, once per counter, from the repo root on one MI355X):\n#     {args.cmd}\n#\n")
        f.write(f"# copy_probe_kernel moves {args.probe_bytes} bytes each way: FETCH_SIZE reads {fetch[probe[0]][0]:.1f}, "
                f"WRITE_SIZE reads {write[probe[0]][0]:.1f}\n")
        f.write(f"# scale: {f_fac:.2f} bytes per FETCH_SIZE unit, {w_fac:.2f} bytes per WRITE_SIZE unit (nominal unit: 1 KiB)\n")
        f.write("# columns: dispatches, fetched bytes per launch, written bytes per launch, their sum, kernel\n")
        for k in sorted(fetch, key=lambda k: -fetch[k][0] * fetch[k][1]):
            if "moe::" not in k:
                continue
            fb = fetch[k][0] * f_fac
            wb = write.get(k, (0.0, 0))[0] * w_fac
            f.write(f"{fetch[k][1]}\t{fb:.0f}\t{wb:.0f}\t{fb + wb:.0f}\t{short_name(k)}\n")


def read_traffic(path):
    """{kernel name: bytes per launch (fetched + written)} from a file written by `traffic`."""
    out = {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        _, _, _, total, name = line.rstrip("\n").split("\t")
        out[name] = float(total)
    return out


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="what", required=True)
    s = sub.add_parser("stats")
    s.add_argument("csv")
    s.add_argument("out")
    s.add_argument("--cmd", required=True)
    s.set_defaults(fn=stats)
    t = sub.add_parser("traffic")
    t.add_argument("fetch_csv")
    t.add_argument("write_csv")
    t.add_argument("out")
    t.add_argument("--probe-bytes", type=int, required=True)
    t.add_argument("--cmd", required=True)
    t.set_defaults(fn=traffic)
    args = ap.parse_args()
    args.fn(args)


if __name__ == "__main__":
    main()
