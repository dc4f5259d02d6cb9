#!/usr/bin/env python3
"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2502_02581_amd.rocprof_summary stats   <kernel_stats.csv> <out.md> --cmd "<command>"
    python -m paper_2502_02581_amd.rocprof_summary traffic <fetch counter csv> <write counter csv> <out.txt>
                                                           --probe-bytes N --cmd "<command>"

    python -m paper_2502_02581_amd.rocprof_summary counters <out.md> <counter csv>... --cmd "<command>" [--cmd ...]

`stats` keeps the per-kernel call count and durations of a `--kernel-trace --stats` run.
`counters` sums every collected counter per kernel and adds MFMA-busy and LDS ratios.
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
    if n.startswith("__amd_rocclr_copyBuffer"):
        n += " (the runtime's staged host<->device copies: inputs up, sampled outputs down; untimed)"
    n = n.replace("void moe::", "moe::")
    return n if len(n) < 220 else n[:217] + "..."


def stats(args):
    rows = list(csv.DictReader(open(args.csv)))
    with open(args.out, "w") as f:
        f.write("# rocprofv3 --kernel-trace --stats summary\n\nCommand (run from the repo root on one MI355X):\n\n")
        f.write(f"    {args.cmd}\n\nKernels of commit {args.commit}.  Calls include the warm-up steps and the profiled pass "
                "(every step runs twice: timed, then with the library's own events). Durations in microseconds.\n\n")
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
        f.write(f"# commit: {args.commit}\n#\n")
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


def counters(args):
    """Per-kernel sums of whatever counters a --pmc run collected, plus the ratios they allow."""
    tot = collections.defaultdict(lambda: collections.defaultdict(float))
    for path in args.csv:
        for r in csv.DictReader(open(path)):
            if "moe::" not in r["Kernel_Name"]:
                continue
            k = short_name(r["Kernel_Name"])
            tot[k][r["Counter_Name"]] += float(r["Counter_Value"])
    with open(args.out, "w") as f:
        f.write("# rocprofv3 --pmc counter sums per kernel (all dispatches of the run)\n\nCommands (from the repo root on one MI355X):\n\n")
        for c in args.cmd:
            f.write(f"    {c}\n")
        f.write(f"\nKernels of commit {args.commit}.\n")
        f.write("\nDerived: MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / (4 SIMDs x SQ_BUSY_CU_CYCLES); executed bf16 MFMA FLOPs = "
                "512 x SQ_INSTS_VALU_MFMA_MOPS_BF16 (padding rows of ragged tiles included); LDS bank conflict share = "
                "SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE; LDS wait share = SQ_WAIT_INST_LDS / SQ_WAVE_CYCLES.\n\n")
        for k in sorted(tot, key=lambda k: -tot[k].get("SQ_BUSY_CU_CYCLES", tot[k].get("SQ_WAVE_CYCLES", 0.0))):
            v = tot[k]
            if not any(c.startswith("SQ_") for c in v):
                continue
            f.write(f"`{k}`\n\n")
            for c in sorted(v):
                f.write(f"    {c:34s} {v[c]:.4g}\n")
            if v.get("SQ_BUSY_CU_CYCLES") and "SQ_VALU_MFMA_BUSY_CYCLES" in v:
                f.write(f"    MFMA busy                          {v['SQ_VALU_MFMA_BUSY_CYCLES'] / (4 * v['SQ_BUSY_CU_CYCLES']):.3f}\n")
            if "SQ_INSTS_VALU_MFMA_MOPS_BF16" in v:
                f.write(f"    executed bf16 MFMA TFLOP           {512 * v['SQ_INSTS_VALU_MFMA_MOPS_BF16'] / 1e12:.3f}\n")
            if v.get("SQ_LDS_IDX_ACTIVE") and "SQ_LDS_BANK_CONFLICT" in v:
                f.write(f"    LDS bank conflict share            {v['SQ_LDS_BANK_CONFLICT'] / v['SQ_LDS_IDX_ACTIVE']:.3f}\n")
            if v.get("SQ_WAVE_CYCLES") and "SQ_WAIT_INST_LDS" in v:
                f.write(f"    LDS wait share                     {v['SQ_WAIT_INST_LDS'] / v['SQ_WAVE_CYCLES']:.3f}\n")
            f.write("\n")


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
    s.add_argument("--commit", default="not recorded")
    s.set_defaults(fn=stats)
    t = sub.add_parser("traffic")
    t.add_argument("fetch_csv")
    t.add_argument("write_csv")
    t.add_argument("out")
    t.add_argument("--probe-bytes", type=int, required=True)
    t.add_argument("--cmd", required=True)
    t.add_argument("--commit", default="not recorded")
    t.set_defaults(fn=traffic)
    c = sub.add_parser("counters")
    c.add_argument("out")
    c.add_argument("csv", nargs="+")
    c.add_argument("--cmd", action="append", required=True)
    c.add_argument("--commit", default="not recorded")
    c.set_defaults(fn=counters)
    args = ap.parse_args()
    args.fn(args)


if __name__ == "__main__":
    main()
