"""Turn the ``*_kernel_stats.csv`` of a ``rocprofv3 --kernel-trace --stats`` run of bench.py into
a short table under ``profiles/``.

    python -m paper_2507_05829_amd.trace_summary STATS.csv --workload NAME \
        --command "<the rocprofv3 command>" [--note "..."] [--out profiles]

Writes ``profiles/kernels_<workload>.md``: calls, total and average duration per kernel, the
figures ``bench.py``'s per-kernel event timings are to be compared with.
"""
from __future__ import annotations

import argparse
import csv
import os

from .pmc_traffic import demangle

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def short(name: str) -> str:
    n = demangle(name).replace("lop::(anonymous namespace)::", "").replace("void ", "")
    return n if len(n) <= 110 else n[:107] + "..."


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("stats_csv")
    ap.add_argument("--workload", required=True)
    ap.add_argument("--command", default="")
    ap.add_argument("--note", default="")
    ap.add_argument("--out", default=os.path.join(ROOT, "profiles"))
    a = ap.parse_args()
    rows = list(csv.DictReader(open(a.stats_csv)))
    lines = [f"# rocprofv3 kernel summary: {a.workload}", "",
             "Command (on the MI355X box, from the repository root, after `cd /tmp && export TMPDIR=/tmp`):",
             "", f"    {a.command}", ""]
    if a.note:
        lines += [a.note, ""]
    lines += ["| kernel | calls | total ms | avg us | min us | max us | % |", "|---|---|---|---|---|---|---|"]
    for r in rows:
        lines.append("| `%s` | %s | %.2f | %.2f | %.2f | %.2f | %.2f |" % (
            short(r["Name"]), r["Calls"], float(r["TotalDurationNs"]) / 1e6,
            float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3,
            float(r["Percentage"])))
    os.makedirs(a.out, exist_ok=True)
    path = os.path.join(a.out, f"kernels_{a.workload}.md")
    with open(path, "w") as fh:
        fh.write("\n".join(lines) + "\n")
    print(path)


if __name__ == "__main__":
    main()
