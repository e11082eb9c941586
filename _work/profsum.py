"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

Two uses:
  * `--stats DIR`   : per-kernel duration table from a `--kernel-trace --stats` run;
  * `--fetch DIR --write DIR` : per-kernel HBM traffic from two `--pmc` runs (FETCH_SIZE, then
    WRITE_SIZE) of `bench.py --pmc-mode`.  That mode ends with plain device copies of a known size;
    the counter value of those copies gives the bytes-per-count factor of each counter, which is
    then applied to the library's kernels.

The summary names the command that produced the data (pass it with --command).
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re
import sys

COPY_KERNEL = "__amd_rocclr_copyBuffer"
CALIBRATION_COPIES = 4


def _read_counter(dirname: str, counter: str):
    files = glob.glob(os.path.join(dirname, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit(f"no counter_collection.csv under {dirname}")
    per = collections.defaultdict(list)
    copies = []                      # (dispatch id, value) of the plain device copies
    for f in files:
        for r in csv.DictReader(open(f)):
            if r["Counter_Name"] == counter:
                per[r["Kernel_Name"]].append(float(r["Counter_Value"]))
                if COPY_KERNEL in r["Kernel_Name"]:
                    copies.append((int(r["Dispatch_Id"]), float(r["Counter_Value"])))
    return per, sorted(copies)


def _short(name: str) -> str:
    m = re.search(r"(lc_[a-z_0-9]+)", name)
    return m.group(1) if m else name[:48]


def _label(name: str) -> str:
    """Kernel name with its template arguments, without the parameter list."""
    head = name.split("(")[0]
    if "lc_" not in head:
        return _short(name)
    return _short(head) + (head[head.index("<"):head.rindex(">") + 1] if "<" in head and ">" in head else "")


def traffic(fetch_dir: str, write_dir: str, copy_bytes: int):
    out = {}
    factors = {}
    for counter, d in (("FETCH_SIZE", fetch_dir), ("WRITE_SIZE", write_dir)):
        per, copies = _read_counter(d, counter)
        cal = [v for _, v in copies[-CALIBRATION_COPIES:]]         # bench.py --pmc-mode ends with them
        factor = copy_bytes / (sum(cal) / len(cal))
        factors[counter] = factor
        for k, vs in per.items():
            if "lc_" not in k:
                continue
            e = out.setdefault(_label(k), {})
            e[counter] = (sum(vs) / len(vs), len(vs))
    return out, factors


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--stats")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--copy-bytes", type=int, default=256 << 20)
    ap.add_argument("--command", default="")
    ap.add_argument("--bench-json", default="", help="bench.py output line of the same build, appended verbatim")
    ap.add_argument("--title", default="")
    ap.add_argument("--out", required=True)
    a = ap.parse_args()
    lines = [f"# {a.title or 'rocprofv3 summary'}", ""]
    if a.command:
        lines += ["Command(s), run from the repository root on the MI355X box:", ""]
        lines += [f"    {c.strip()}" for c in a.command.split(";;")] + [""]
    if a.stats:
        files = glob.glob(os.path.join(a.stats, "**", "*kernel_stats.csv"), recursive=True)
        rows = list(csv.DictReader(open(files[0])))
        lines += ["| kernel | calls | avg us | min us | max us | % of GPU time |", "|---|---|---|---|---|---|"]
        for r in rows[:14]:
            lines.append(f"| {_label(r['Name'])} | {r['Calls']} | "
                         f"{float(r['AverageNs']) / 1e3:.2f} | {float(r['MinNs']) / 1e3:.2f} | "
                         f"{float(r['MaxNs']) / 1e3:.2f} | {float(r['Percentage']):.1f} |")
        lines.append("")
    if a.fetch and a.write:
        t, f = traffic(a.fetch, a.write, a.copy_bytes)
        lines += [f"Counter calibration from the plain {a.copy_bytes >> 20} MiB device copy at the end of the run: "
                  f"FETCH_SIZE x {f['FETCH_SIZE']:.1f} bytes per count, WRITE_SIZE x {f['WRITE_SIZE']:.1f} bytes per count.", "",
                  "| kernel | dispatches | FETCH_SIZE avg | WRITE_SIZE avg | HBM read bytes | HBM write bytes | traffic bytes per launch |",
                  "|---|---|---|---|---|---|---|"]
        for k in sorted(t):
            e = t[k]
            if "FETCH_SIZE" not in e or "WRITE_SIZE" not in e:
                continue
            rb = e["FETCH_SIZE"][0] * f["FETCH_SIZE"]
            wb = e["WRITE_SIZE"][0] * f["WRITE_SIZE"]
            lines.append(f"| {k} | {e['FETCH_SIZE'][1]} | {e['FETCH_SIZE'][0]:.1f} | {e['WRITE_SIZE'][0]:.1f} | "
                         f"{rb:.0f} | {wb:.0f} | traffic[{k}] = {rb + wb:.0f} |")
        lines.append("")
    if a.bench_json:
        lines += ["bench.py line of the same build:", "", "    " + open(a.bench_json).read().strip().splitlines()[-1], ""]
    os.makedirs(os.path.dirname(os.path.abspath(a.out)), exist_ok=True)
    open(a.out, "w").write("\n".join(lines))
    print("wrote", a.out)


def read_traffic(path: str, kernel: str):
    """The `traffic[<kernel>] = N` figure of a summary written by this module, or None."""
    try:
        m = re.search(r"traffic\[" + re.escape(kernel) + r"\] = (\d+)", open(path).read())
        return int(m.group(1)) if m else None
    except OSError:
        return None


if __name__ == "__main__":
    main()
