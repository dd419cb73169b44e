"""Turns rocprofv3 output of bench.py runs into the short summaries kept under profiles/.

  python -m paper_2512_09238_amd.profile_summary traffic FETCH_DIR WRITE_DIR -o profiles/traffic_config3.json
      FETCH_DIR / WRITE_DIR: output folders of two `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE`
      runs of `bench.py --steps 1 --warmup 0 --no-cpu --copy-probe` (one counter per run).  The plain
      1 GiB device copy of --copy-probe, whose traffic is known, gives the factor that turns a
      counter reading into bytes; the file records HBM bytes per launch of every libtca kernel.
  python -m paper_2512_09238_amd.profile_summary stats STATS_CSV
      prints the libtca rows of a `rocprofv3 --kernel-trace --stats` kernel_stats.csv as a table.
  python -m paper_2512_09238_amd.profile_summary counters PMC_DIR
      prints the mean per dispatch of every counter of a `rocprofv3 --pmc ...` run, per libtca kernel.

bench.py reads the traffic file and reports its figures only while `source_sha` still equals the
hash of the kernel sources (source_sha() below): a changed kernel invalidates the measurement.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import hashlib
import json
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
GIB_IN_KIB = float(1 << 20)


def source_sha() -> str:
    """Hash of everything the kernels are built from."""
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(HERE, "csrc", "*")) + glob.glob(os.path.join(ROOT, "include", "*.h")))
    for f in files:
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def short_name(kernel: str) -> str:
    m = re.search(r"tca::(\w+)", kernel)
    return m.group(1) if m else kernel.split("(")[0][:60]


def read_counter(folder: str, counter: str):
    """{kernel name: [values per dispatch]} of one counter from a rocprofv3 --pmc output folder."""
    files = glob.glob(os.path.join(folder, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit(f"no counter_collection.csv under {folder}")
    out = collections.defaultdict(list)
    for f in files:
        for r in csv.DictReader(open(f)):
            if r["Counter_Name"] == counter:
                out[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return out


def copy_factor(values: dict, what: str) -> float:
    """Bytes per counter unit from the 1 GiB copy of --copy-probe: the largest dispatch of the runtime's
    buffer-copy kernel (the other dispatches of that kernel are the small copies of the set-up)."""
    cands = [(max(v), k) for k, v in values.items() if "copyBuffer" in k]
    if not cands or max(cands)[0] <= 0:
        raise SystemExit(f"no buffer-copy kernel found for {what}: was bench.py run with --copy-probe?")
    best = max(cands)
    return GIB_IN_KIB * 1024.0 / best[0], best[1]


def cmd_traffic(args):
    fetch, write = read_counter(args.fetch_dir, "FETCH_SIZE"), read_counter(args.write_dir, "WRITE_SIZE")
    f_fetch, k_fetch = copy_factor(fetch, "FETCH_SIZE")
    f_write, k_write = copy_factor(write, "WRITE_SIZE")
    kernels = {}
    for name in sorted(set(fetch) | set(write)):
        if "tca::" not in name:
            continue
        fv, wv = fetch.get(name, [0.0]), write.get(name, [0.0])
        kernels.setdefault(short_name(name), []).append({
            "kernel": name.split("(")[0], "launches": len(fv),
            "fetch_counter_per_launch": sum(fv) / len(fv), "write_counter_per_launch": sum(wv) / len(wv),
            "read_bytes_per_launch": f_fetch * sum(fv) / len(fv), "written_bytes_per_launch": f_write * sum(wv) / len(wv),
        })
    try:
        head = subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], capture_output=True, text=True).stdout.strip()
    except OSError:
        head = ""
    doc = {
        "what": "HBM traffic per kernel launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (one counter per run) of "
                "`python3 bench.py --steps 1 --warmup 0 --no-cpu --copy-probe`",
        "source_sha": source_sha(), "git_head_at_profiling": head,
        "bytes_per_counter_unit": {"FETCH_SIZE": f_fetch, "WRITE_SIZE": f_write,
                                   "from": "the plain 1 GiB device copy of --copy-probe (reads 1 GiB, writes 1 GiB)",
                                   "copy_kernel": k_fetch.split("(")[0]},
        "kernels": kernels,
    }
    with open(args.output, "w") as f:
        json.dump(doc, f, indent=1)
    print("wrote", args.output)


def load_traffic(path: str):
    """The traffic file if it was measured on the kernels as they are now, else None."""
    if not os.path.exists(path):
        return None
    doc = json.load(open(path))
    return doc if doc.get("source_sha") == source_sha() else None


def kernel_bytes(doc, name: str, pick=max):
    """read + written bytes per launch of kernel `name` (several template instances: the one `pick` chooses)."""
    if doc is None or name not in doc["kernels"]:
        return None
    return pick(e["read_bytes_per_launch"] + e["written_bytes_per_launch"] for e in doc["kernels"][name])


def cmd_stats(args):
    rows = [r for r in csv.DictReader(open(args.stats_csv)) if "tca::" in r["Name"]]
    print("| kernel | calls | avg us | min us | max us | total ms |")
    print("|---|---:|---:|---:|---:|---:|")
    for r in sorted(rows, key=lambda r: -float(r["TotalDurationNs"])):
        name = r["Name"].split("(")[0].replace("void ", "")
        print(f"| `{name}` | {r['Calls']} | {float(r['AverageNs']) / 1e3:.1f} | {float(r['MinNs']) / 1e3:.1f} | "
              f"{float(r['MaxNs']) / 1e3:.1f} | {float(r['TotalDurationNs']) / 1e6:.2f} |")


def cmd_counters(args):
    files = glob.glob(os.path.join(args.pmc_dir, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit(f"no counter_collection.csv under {args.pmc_dir}")
    acc, names = collections.defaultdict(lambda: collections.defaultdict(list)), []
    for f in files:
        for r in csv.DictReader(open(f)):
            if "tca::" not in r["Kernel_Name"]:
                continue
            if r["Counter_Name"] not in names:
                names.append(r["Counter_Name"])
            acc[r["Kernel_Name"].split("(")[0].replace("void ", "")][r["Counter_Name"]].append(float(r["Counter_Value"]))
    print("| kernel | dispatches | " + " | ".join(names) + " |")
    print("|---|---:|" + "---:|" * len(names))
    for k, c in sorted(acc.items(), key=lambda kv: -sum(kv[1].get(names[0], [0.0]))):
        n = max(len(v) for v in c.values())
        print(f"| `{k}` | {n} | " + " | ".join(f"{sum(c[x]) / len(c[x]):.4g}" if c.get(x) else "-" for x in names) + " |")


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    t = sub.add_parser("traffic")
    t.add_argument("fetch_dir")
    t.add_argument("write_dir")
    t.add_argument("-o", "--output", required=True)
    t.set_defaults(fn=cmd_traffic)
    s = sub.add_parser("stats")
    s.add_argument("stats_csv")
    s.set_defaults(fn=cmd_stats)
    c = sub.add_parser("counters")
    c.add_argument("pmc_dir")
    c.set_defaults(fn=cmd_counters)
    args = ap.parse_args()
    args.fn(args)


if __name__ == "__main__":
    main()
