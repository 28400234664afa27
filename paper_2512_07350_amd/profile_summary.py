"""Condense rocprofv3 CSV output of a `bench.py` run into the short tables kept under profiles/.

    python -m paper_2512_07350_amd.profile_summary stats   <dir-or-csv>
    python -m paper_2512_07350_amd.profile_summary traffic <fetch-dir> <write-dir> --workload NAME [--json OUT]
    python -m paper_2512_07350_amd.profile_summary counters <dir> [<dir> ...] [--kernel attention_kernel]

`stats` reads `*_kernel_stats.csv` (from `rocprofv3 --kernel-trace --stats`) and prints one row
per kernel of this library.  `traffic` reads the `*_counter_collection.csv` files of two
`rocprofv3 --pmc` runs (FETCH_SIZE, then WRITE_SIZE; both counters are KiB per dispatch) of
`bench.py --copy-calibration`, scales them by what the same counter reads for the plain device
copy of known size, and prints bytes per launch; with --json it also writes (or replaces) this
workload's record in the file `bench.py` reads for `roofline.traffic`; the record carries the
SHA-256 of the attention source in this tree, so summarise before changing that file.  `counters` prints the mean per dispatch of every
counter found for one kernel in any number of `--pmc` runs.  Host-side text processing only: no GPU, no oracle.
"""
from __future__ import annotations

import argparse
import csv
import glob
import json
import os
import re
import sys

OURS = ("attention_kernel", "combine_kernel", "partition_kernel", "partition_rows_kernel", "reconstruct_kernel", "gemm_kernel",
        "norm_rope_kernel")
COPY_KIB = 256 * 1024          # bench.py --copy-calibration copies 256 MiB


def short(name: str) -> str:
    """`void (anonymous namespace)::attention_kernel<128, 1>(...)` -> `attention_kernel<128,1>`."""
    m = re.search(r"(\w+_kernel)(<[^>]*>)?", name)
    return (m.group(1) + (m.group(2) or "")).replace(" ", "") if m else name[:60]


def find_csv(path: str, suffix: str) -> str:
    if os.path.isfile(path):
        return path
    hits = sorted(glob.glob(os.path.join(path, "**", "*" + suffix), recursive=True))
    if not hits:
        raise SystemExit("no *%s under %s" % (suffix, path))
    return hits[0]


def stats(path: str) -> None:
    rows = list(csv.DictReader(open(find_csv(path, "kernel_stats.csv"))))
    total = sum(float(r["TotalDurationNs"]) for r in rows)
    print("| kernel | calls | total ms | average us | % of GPU time | min us | max us |")
    print("|---|---|---|---|---|---|---|")
    for r in rows:
        if not any(k in r["Name"] for k in OURS):
            continue
        t = float(r["TotalDurationNs"])
        print("| `%s` | %d | %.3f | %.2f | %.2f | %.2f | %.2f |" % (
            short(r["Name"]), int(r["Calls"]), t / 1e6, float(r["AverageNs"]) / 1e3, 100.0 * t / total,
            float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3))


def counter_means(path: str, counter: str):
    """-> {short kernel name: (dispatches, mean KiB)}, plus the copy kernel under 'copy'."""
    acc = {}
    for r in csv.DictReader(open(find_csv(path, "counter_collection.csv"))):
        if r["Counter_Name"] != counter:
            continue
        name = r["Kernel_Name"]
        if any(k in name for k in OURS):
            key = short(name)
        elif "copyBuffer" in name or "copy_buffer" in name.lower():
            key = "copy"
        else:
            continue
        n, s = acc.get(key, (0, 0.0))
        acc[key] = (n + 1, s + float(r["Counter_Value"]))
    return {k: (n, s / n) for k, (n, s) in acc.items()}


def traffic(fetch_dir: str, write_dir: str, workload: str, out_json: str | None, algorithmic: float | None) -> None:
    fetch = counter_means(fetch_dir, "FETCH_SIZE")
    write = counter_means(write_dir, "WRITE_SIZE")
    # Several small copies (host uploads) may share the copy kernel's name; take the maximum reading
    # of a single dispatch instead of the mean for the calibration row.
    def max_copy(path, counter):
        best = 0.0
        for r in csv.DictReader(open(find_csv(path, "counter_collection.csv"))):
            if r["Counter_Name"] == counter and "copyBuffer" in r["Kernel_Name"]:
                best = max(best, float(r["Counter_Value"]))
        if best <= 0:
            raise SystemExit("no copy dispatch found: run bench.py with --copy-calibration")
        return best
    f_scale = COPY_KIB / max_copy(fetch_dir, "FETCH_SIZE")
    w_scale = COPY_KIB / max_copy(write_dir, "WRITE_SIZE")
    print("copy of %d KiB: FETCH_SIZE scale %.4f, WRITE_SIZE scale %.4f" % (COPY_KIB, f_scale, w_scale))
    print("| kernel | dispatches | FETCH_SIZE mean KiB | WRITE_SIZE mean KiB | scaled read MB | scaled write MB |")
    print("|---|---|---|---|---|---|")
    rec = {}
    for key in sorted(set(fetch) | set(write)):
        if key == "copy":
            continue
        n, f = fetch.get(key, (0, 0.0))
        _, wv = write.get(key, (0, 0.0))
        rb, wb = f * 1024 * f_scale, wv * 1024 * w_scale
        rec[key] = dict(launches=n, fetch_bytes=int(rb), write_bytes=int(wb))
        print("| `%s` | %d | %.1f | %.1f | %.2f | %.2f |" % (key, n, f, wv, rb / 1e6, wb / 1e6))
    att = [k for k in rec if k.startswith("attention_kernel")]
    comb = [k for k in rec if k.startswith("combine_kernel")]
    per_call = None
    if att:
        a = rec[att[0]]
        per_call = a["fetch_bytes"] + a["write_bytes"]
        if comb:
            c = rec[comb[0]]
            per_call += (c["fetch_bytes"] + c["write_bytes"]) * c["launches"] / a["launches"]
        print("per lp_attention call (attention kernel + its share of merge kernels): %.1f MB" % (per_call / 1e6))
    if out_json:
        # one record per workload; a record names the attention source it was measured with, so that
        # a reader (bench.py) can tell a stale record from a current one
        rec_doc = {"workload": workload, "attention_source_sha256": source_sha256(),
                   "command": "rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE --kernel-trace -- python3 bench.py --workload <index> --only "
                              "--steps 3 --warmup 1 --no-cpu-baseline --copy-calibration",
                   "fetch_scale": round(f_scale, 4), "write_scale": round(w_scale, 4), "kernels": rec,
                   "attention_bytes_per_launch": int(per_call) if per_call else None,
                   "algorithmic_bytes_per_launch": algorithmic}
        doc = {"records": []}
        if os.path.exists(out_json):
            old = json.load(open(out_json))
            doc["records"] = [r for r in old.get("records", []) if r.get("workload") != workload]
        doc["records"].append(rec_doc)
        with open(out_json, "w") as fh:
            json.dump(doc, fh, indent=1)
            fh.write("\n")


def source_sha256() -> str:
    """SHA-256 of the attention kernel's source file as it is in this tree."""
    import hashlib
    here = os.path.dirname(os.path.abspath(__file__))
    return hashlib.sha256(open(os.path.join(here, "csrc", "lp_attention.hip"), "rb").read()).hexdigest()


def counters(paths, kernel: str) -> None:
    print("| counter | mean per dispatch | dispatches |")
    print("|---|---|---|")
    for path in paths:
        acc = {}
        for r in csv.DictReader(open(find_csv(path, "counter_collection.csv"))):
            if kernel in r["Kernel_Name"]:
                n, t = acc.get(r["Counter_Name"], (0, 0.0))
                acc[r["Counter_Name"]] = (n + 1, t + float(r["Counter_Value"]))
        for name in sorted(acc):
            n, t = acc[name]
            print("| %s | %.6g | %d |" % (name, t / n, n))


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    sub = ap.add_subparsers(dest="cmd", required=True)
    s = sub.add_parser("stats"); s.add_argument("path")
    t = sub.add_parser("traffic")
    t.add_argument("fetch_dir"); t.add_argument("write_dir")
    t.add_argument("--workload", required=True)
    t.add_argument("--json", default=None)
    t.add_argument("--algorithmic-bytes", type=float, default=None)
    c = sub.add_parser("counters")
    c.add_argument("paths", nargs="+"); c.add_argument("--kernel", default="attention_kernel")
    a = ap.parse_args()
    if a.cmd == "stats":
        stats(a.path)
    elif a.cmd == "counters":
        counters(a.paths, a.kernel)
    else:
        traffic(a.fetch_dir, a.write_dir, a.workload, a.json, a.algorithmic_bytes)
    return 0


if __name__ == "__main__":
    sys.exit(main())
