"""Turn two rocprofv3 counter runs (FETCH_SIZE, then WRITE_SIZE) of bench.py into HBM bytes
per launch for every kernel of the library, scaled by what the same counters read for a
plain device-to-device copy of known size issued by ``bench.py --pmc-calibrate``.

    python -m paper_2507_05829_amd.pmc_traffic FETCH.csv WRITE.csv --workload NAME \
        --command "<the rocprofv3 command>" [--out profiles]

Writes ``profiles/traffic_<workload>.json`` (read by bench.py for ``roofline.traffic``; it
carries a hash of the kernel sources so that stale numbers are dropped) and a short
``profiles/traffic_<workload>.md``.
"""
from __future__ import annotations

import argparse
import collections
import csv
import hashlib
import json
import os
import re

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CALIB_BYTES = 256 << 20          # bench.py --pmc-calibrate copies 64 Mi floats
CALIB_KERNEL = "__amd_rocclr_copyBuffer"


def source_hash() -> str:
    """Hash of the HIP sources: counters taken for other kernels must not be reported."""
    h = hashlib.sha256()
    csrc = os.path.join(HERE, "csrc")
    for f in sorted(os.listdir(csrc)):
        if f.endswith((".hip", ".hpp", ".cpp")):
            h.update(open(os.path.join(csrc, f), "rb").read())
    return h.hexdigest()[:16]


def _per_kernel(path: str, counter: str):
    vals = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == counter:
            vals[r["Kernel_Name"]].append(float(r["Counter_Value"]))     # KiB per dispatch
    return vals


def _factor(vals) -> float:
    """Counter KiB read for the calibration copy divided by the KiB it really moves."""
    cal = [v for k, vs in vals.items() if CALIB_KERNEL in k for v in vs]
    if not cal:
        raise SystemExit("no calibration copy in the counter file: run bench.py --pmc-calibrate")
    return max(cal) / (CALIB_BYTES / 1024.0)


_MANGLED = re.compile(r"^_ZN3lop12_GLOBAL__N_1(\d+)")


def demangle(name: str) -> str:
    """The profiler leaves kernel names with a __bf16 template argument mangled; spell out the
    few forms this library's kernels use (type and integer/bool template arguments)."""
    m = _MANGLED.match(name)
    if not m:
        return name
    start = m.end()
    ident = name[start:start + int(m.group(1))]
    rest = name[start + int(m.group(1)):]
    args = []
    if rest.startswith("I"):
        rest = rest[1:]
        while rest and not rest.startswith("E"):
            if rest.startswith("DF16b"):
                args.append("__bf16"); rest = rest[5:]
            elif rest.startswith("f"):
                args.append("float"); rest = rest[1:]
            elif rest.startswith("Li"):
                end = rest.index("E")
                args.append(rest[2:end]); rest = rest[end + 1:]
            elif rest.startswith("Lb"):
                args.append("true" if rest[2] == "1" else "false"); rest = rest[4:]
            else:
                return name
    return "lop::(anonymous namespace)::" + ident + ("<" + ", ".join(args) + ">" if args else "")


def short(name: str) -> str:
    n = demangle(name).replace("lop::(anonymous namespace)::", "").replace("void ", "")
    return n[:n.index("(")] if "(" in n else n


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("fetch_csv")
    ap.add_argument("write_csv")
    ap.add_argument("--workload", required=True)
    ap.add_argument("--command", default="")
    ap.add_argument("--out", default=os.path.join(ROOT, "profiles"))
    a = ap.parse_args()
    fetch, write = _per_kernel(a.fetch_csv, "FETCH_SIZE"), _per_kernel(a.write_csv, "WRITE_SIZE")
    ff, fw = _factor(fetch), _factor(write)
    kernels = {}
    for name in sorted(set(fetch) | set(write)):
        if "lop::" not in demangle(name):
            continue
        f, w = fetch.get(name, []), write.get(name, [])
        kernels[short(name)] = dict(
            dispatches=len(f),
            fetch_bytes_per_launch=(sum(f) / len(f)) * 1024 / ff if f else None,
            write_bytes_per_launch=(sum(w) / len(w)) * 1024 / fw if w else None)
    doc = dict(workload=a.workload, source_hash=source_hash(), command=a.command,
               calibration=dict(kernel=CALIB_KERNEL, bytes=CALIB_BYTES, fetch_factor=ff,
                                write_factor=fw),
               kernels=kernels)
    os.makedirs(a.out, exist_ok=True)
    with open(os.path.join(a.out, f"traffic_{a.workload}.json"), "w") as fh:
        json.dump(doc, fh, indent=1)
    lines = [f"# HBM traffic per launch from rocprofv3 counters: {a.workload}", "",
             "Two runs of the command below, one with `--pmc FETCH_SIZE`, one with `--pmc WRITE_SIZE`",
             "(KiB per dispatch), averaged over the dispatches of each kernel:", "",
             f"    {a.command}", "",
             f"Scaling: the same counters read for `{CALIB_KERNEL}` copying {CALIB_BYTES >> 20} MiB device to",
             f"device (bench.py --pmc-calibrate) are {ff:.4f} (fetch) and {fw:.4f} (write) of the true size;",
             "the figures below are divided by these factors.", "",
             "| kernel | dispatches | fetch bytes/launch | write bytes/launch |", "|---|---|---|---|"]
    for k, v in kernels.items():
        fb = "-" if v["fetch_bytes_per_launch"] is None else f"{v['fetch_bytes_per_launch']:.0f}"
        wb = "-" if v["write_bytes_per_launch"] is None else f"{v['write_bytes_per_launch']:.0f}"
        lines.append(f"| `{k}` | {v['dispatches']} | {fb} | {wb} |")
    lines += ["", f"Kernel source hash: {doc['source_hash']}"]
    with open(os.path.join(a.out, f"traffic_{a.workload}.md"), "w") as fh:
        fh.write("\n".join(lines) + "\n")
    print(json.dumps(doc["kernels"], indent=1))


if __name__ == "__main__":
    main()
