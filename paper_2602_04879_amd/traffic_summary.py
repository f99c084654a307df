"""Turn rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs into HBM bytes per launch.

  python3 -m paper_2602_04879_amd.traffic_summary --workload c3_qwen3_binary_tv --path resident \
      --probe-fetch DIR --probe-write DIR --fetch DIR --write DIR [--out profiles/hbm_traffic.json]

Each DIR is the output directory of one `rocprofv3 --pmc <counter> --output-format csv` run:
the two probe runs of `python3 -m paper_2602_04879_amd.hbm_probe` (a plain copy of known size:
its counter reading per dispatch gives the factor that turns the counter into bytes) and the two
runs of `python3 bench.py`.  The record is stored with a hash of the kernel sources; bench.py
reports it as roofline.traffic only while that hash still matches."""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import hashlib
import json
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def kernel_source_hash(path: str) -> str:
    """Hash of the device code behind one kernel path (its kernel file and the shared device
    helpers): stored HBM-traffic counters hold only for it."""
    h = hashlib.sha256()
    src = os.path.join(ROOT, "paper_2602_04879_amd", "csrc")
    files = ["dppo_common.hpp", f"dppo_{path}.hip"] + (["dppo_resident_parts.hpp"] if path.startswith("resident") else [])
    for fn in files:
        h.update(open(os.path.join(src, fn), "rb").read())
    return h.hexdigest()[:16]


def counter_avg(directory: str, kernel_substr: str, counter: str) -> float:
    vals = []
    for fn in glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True):
        for r in csv.DictReader(open(fn)):
            if kernel_substr in r["Kernel_Name"] and r["Counter_Name"] == counter:
                vals.append(float(r["Counter_Value"]))
    if not vals:
        raise SystemExit(f"no {counter} rows for a kernel matching {kernel_substr!r} under {directory}")
    return sum(vals) / len(vals)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--path", required=True, choices=["resident", "resident_long", "resident_multi", "streaming", "fullvocab", "fullvocab_resident"])
    ap.add_argument("--probe-fetch", required=True)
    ap.add_argument("--probe-write", required=True)
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--probe-bytes", type=int, default=4 << 30, help="bytes the probe copy reads (= writes) per launch")
    ap.add_argument("--out", default=os.path.join(ROOT, "profiles", "hbm_traffic.json"))
    a = ap.parse_args()
    kib = a.probe_bytes / 1024.0
    f_read = kib / counter_avg(a.probe_fetch, "dppo_probe_copy_kernel", "FETCH_SIZE")
    f_write = kib / counter_avg(a.probe_write, "dppo_probe_copy_kernel", "WRITE_SIZE")
    kern = f"dppo_{a.path}_kernel"
    rd = counter_avg(a.fetch, kern, "FETCH_SIZE") * f_read * 1024.0
    wr = counter_avg(a.write, kern, "WRITE_SIZE") * f_write * 1024.0
    rec = {"bytes_per_launch": rd + wr, "read_bytes": rd, "write_bytes": wr, "fetch_size_factor": f_read,
           "write_size_factor": f_write, "kernel": kern, "kernel_source_hash": kernel_source_hash(a.path)}
    allrec = json.load(open(a.out)) if os.path.exists(a.out) else {}
    allrec[f"{a.workload}:{a.path}"] = rec
    json.dump(allrec, open(a.out, "w"), indent=1, sort_keys=True)
    print(json.dumps(rec, indent=1))


if __name__ == "__main__":
    main()
