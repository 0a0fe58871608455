"""HBM traffic per call from rocprofv3 counter files, kept as a small JSON file under profiles/ that bench.py reads.

bench.py cannot read hardware counters itself, so the `traffic` figure of its roofline object comes from separate
`rocprofv3 --pmc` runs of bench.py (FETCH_SIZE in one run, WRITE_SIZE in another; KiB per dispatch), each scaled by what
the same counter reads for a plain copy kernel of known size.  This module turns the counter_collection.csv files of those
runs into one entry of profiles/hbm_traffic.json, stamped with a hash of the kernel sources it was measured on; bench.py
reports the figure only while that hash still matches the sources, so a kernel change cannot leave a stale number behind.

    python -m paper_2605_24058_amd.traffic_profile --call lordba_forward --workload <name> \
        --fetch <call FETCH_SIZE csv> --write <call WRITE_SIZE csv> \
        --copy-fetch <copy FETCH_SIZE csv> --copy-write <copy WRITE_SIZE csv> --copy-kib 16384 \
        --command "<the rocprofv3 command line>" [--out profiles/hbm_traffic.json]
"""
from __future__ import annotations

import argparse
import csv
import hashlib
import json
import os
import subprocess
from collections import OrderedDict

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
DEFAULT_JSON = os.path.join(_ROOT, "profiles", "hbm_traffic.json")

# the sources whose change invalidates a measurement of a call
_FORWARD_SOURCES = ("lordba_fwd_impl.h", "lordba_dev_util.h", "lordba_forward.hip")
SOURCES = {
    "lordba_forward": _FORWARD_SOURCES,
    "lordba_backward": _FORWARD_SOURCES + ("lordba_forward_train.hip", "lordba_forward_multi_train.hip", "lordba_backward.hip"),
}


def source_hash(call: str) -> str:
    h = hashlib.sha256()
    for name in SOURCES[call]:
        with open(os.path.join(_PKG, "csrc", name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read() + b"\0")
    return h.hexdigest()


def per_kernel(csv_path: str, counter: str, match: str) -> "OrderedDict[str, list]":
    """Counter values per dispatch, grouped by kernel name, of the kernels whose name contains `match`."""
    out: "OrderedDict[str, list]" = OrderedDict()
    with open(csv_path, newline="") as f:
        for row in csv.DictReader(f):
            if row["Counter_Name"] != counter:
                continue
            name = row["Kernel_Name"]
            if match not in name:
                continue
            name = name.replace("void ", "").replace("(anonymous namespace)::", "")
            out.setdefault(name, []).append(float(row["Counter_Value"]))
    return out


def kib_per_call(csv_path: str, counter: str, match: str):
    """(KiB per call summed over the call's kernels, {kernel: (dispatches per call, mean KiB per dispatch)}).  Every call
    of the run is the same, so the number of calls is the dispatch count of the kernel that runs once per call."""
    groups = per_kernel(csv_path, counter, match)
    if not groups:
        raise SystemExit("%s: no %s rows for kernels named *%s*" % (csv_path, counter, match))
    calls = min(len(v) for v in groups.values())
    detail = OrderedDict((k, (len(v) / calls, sum(v) / len(v))) for k, v in groups.items())
    return sum(sum(v) for v in groups.values()) / calls, detail


def build_entry(a) -> dict:
    copy_f, _ = kib_per_call(a.copy_fetch, "FETCH_SIZE", "copy_kernel(")
    copy_w, _ = kib_per_call(a.copy_write, "WRITE_SIZE", "copy_kernel(")
    f_scale, w_scale = a.copy_kib / copy_f, a.copy_kib / copy_w
    fetch, f_detail = kib_per_call(a.fetch, "FETCH_SIZE", a.kernel_match)
    write, w_detail = kib_per_call(a.write, "WRITE_SIZE", a.kernel_match)
    try:
        commit = subprocess.run(["git", "-C", _ROOT, "rev-parse", "--short", "HEAD"], capture_output=True, text=True).stdout.strip()
    except OSError:
        commit = ""
    kernels = OrderedDict()
    for k in f_detail:
        kernels[k] = {"dispatches_per_call": f_detail[k][0], "fetch_size_kib": round(f_detail[k][1], 2),
                      "write_size_kib": round(w_detail.get(k, (0, 0.0))[1], 2)}
    return {
        "call": a.call, "workload": a.workload, "variant": a.variant,
        "bytes_per_call": int(round((fetch * f_scale + write * w_scale) * 1024)),
        "fetched_bytes_per_call": int(round(fetch * f_scale * 1024)), "written_bytes_per_call": int(round(write * w_scale * 1024)),
        "fetch_size_scale": round(f_scale, 4), "write_size_scale": round(w_scale, 4),
        "copy_kernel": {"known_kib_each_way": a.copy_kib, "fetch_size_kib": round(copy_f, 2), "write_size_kib": round(copy_w, 2)},
        "kernels": kernels, "source_sha256": source_hash(a.call), "measured_after_commit": commit, "command": a.command,
    }


def lookup(call: str, workload: str, variant: str = "", path: str = DEFAULT_JSON):
    """(bytes per call or None, note) for bench.py: the stored figure if it was measured on the present kernel sources."""
    try:
        with open(path) as f:
            entries = json.load(f)["entries"]
    except (OSError, ValueError, KeyError):
        return None, "no traffic file (%s)" % os.path.relpath(path, _ROOT)
    for e in entries:
        if e["call"] == call and e["workload"] == workload and e.get("variant", "") == variant:
            if e["source_sha256"] != source_hash(call):
                return None, "the kernel sources have changed since %s was measured (after commit %s): measure again" % (
                    os.path.relpath(path, _ROOT), e.get("measured_after_commit", "?"))
            return e["bytes_per_call"], "rocprofv3 FETCH_SIZE + WRITE_SIZE, %s (measured after commit %s, kernel sources unchanged since)" % (
                os.path.relpath(path, _ROOT), e.get("measured_after_commit", "?"))
    return None, "no entry for %s / %s in %s" % (call, workload, os.path.relpath(path, _ROOT))


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--call", required=True, choices=sorted(SOURCES))
    ap.add_argument("--workload", required=True)
    ap.add_argument("--variant", default="", help="e.g. 't kept' for lordba_backward with a kept rank-r intermediate")
    ap.add_argument("--kernel-match", default="lordba_", help="substring of the names of the call's kernels")
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--copy-fetch", required=True)
    ap.add_argument("--copy-write", required=True)
    ap.add_argument("--copy-kib", type=float, required=True, help="KiB the copy kernel reads (and writes) per dispatch")
    ap.add_argument("--command", default="")
    ap.add_argument("--out", default=DEFAULT_JSON)
    a = ap.parse_args()
    entry = build_entry(a)
    try:
        with open(a.out) as f:
            doc = json.load(f)
    except (OSError, ValueError):
        doc = {"what": "HBM bytes per call from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch), each scaled by the "
                       "same counter's reading for a plain copy kernel of known size; written by "
                       "paper_2605_24058_amd/traffic_profile.py, read by bench.py", "entries": []}
    doc["entries"] = [e for e in doc["entries"]
                      if (e["call"], e["workload"], e.get("variant", "")) != (entry["call"], entry["workload"], entry["variant"])]
    doc["entries"].append(entry)
    with open(a.out, "w") as f:
        json.dump(doc, f, indent=1)
        f.write("\n")
    print(json.dumps(entry, indent=1))


if __name__ == "__main__":
    main()
