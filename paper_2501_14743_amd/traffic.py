"""HBM traffic of the pull kernel from two rocprofv3 counter runs.

    python -m paper_2501_14743_amd.traffic <FETCH_SIZE counter_collection.csv> <WRITE_SIZE counter_collection.csv> <workload name>

Both runs must be `bench.py ... --copy-calibration`, which also launches the plain copy kernel on
1 GiB.  FETCH_SIZE / WRITE_SIZE are reported per dispatch in nominal KiB; each is scaled by
(1 GiB in KiB) / (what the same counter reads for the plain 1 GiB copy), so the result does not
depend on the counter's unit.  Adds the workload's record to `hbm_traffic.json` next to this file
(one record per workload); bench.py reports a record's `traffic_bytes_per_launch` only while the
kernel source (comments and white space aside) still has the hash stored with that record.
"""
from __future__ import annotations

import csv
import hashlib
import json
import os
import re
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(PKG, "csrc", "kvd_kernels.h")
RECORD = os.path.join(PKG, "hbm_traffic.json")
COPY_BYTES = 1 << 30


def source_hash() -> str:
    """sha256 of the kernel source (structures and device code) with #include lines, comments and
    white space removed, so that only a change of the kernels' code invalidates a recorded measurement."""
    with open(SOURCE) as f:
        text = f.read()
    text = re.sub(r"^\s*#\s*include[^\n]*$", "", text, flags=re.M)  # host headers come and go
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    text = re.sub(r"//[^\n]*", "", text)
    text = re.sub(r"\s+", "", text)
    return hashlib.sha256(text.encode()).hexdigest()


def load_record(workload: str):
    """The recorded traffic for `workload`, or None if there is none for the current kernel source."""
    rec = _load_all().get(workload)
    if rec is None or rec.get("kernel_source_sha256") != source_hash():
        return None
    return rec


def _load_all() -> dict:
    if not os.path.exists(RECORD):
        return {}
    with open(RECORD) as f:
        return json.load(f).get("records", {})


def _mean_counter(path: str, counter: str, kernel_substr: str) -> tuple[float, int]:
    vals = []
    with open(path) as f:
        for row in csv.DictReader(f):
            if row["Counter_Name"] == counter and kernel_substr in row["Kernel_Name"]:
                vals.append(float(row["Counter_Value"]))
    if not vals:
        raise SystemExit(f"no {counter} rows for a kernel matching {kernel_substr!r} in {path}")
    return sum(vals) / len(vals), len(vals)


def main(argv) -> int:
    if len(argv) != 4:  # two csv files and the workload name
        print(__doc__)
        return 2
    fetch_csv, write_csv, workload = argv[1], argv[2], argv[3]
    pull_f, n1 = _mean_counter(fetch_csv, "FETCH_SIZE", "kvd_pull_kernel")
    copy_f, _ = _mean_counter(fetch_csv, "FETCH_SIZE", "kvd_copy_kernel")
    pull_w, n2 = _mean_counter(write_csv, "WRITE_SIZE", "kvd_pull_kernel")
    copy_w, _ = _mean_counter(write_csv, "WRITE_SIZE", "kvd_copy_kernel")
    kib = COPY_BYTES / 1024
    f_scale, w_scale = kib / copy_f, kib / copy_w
    read_b = pull_f * f_scale * 1024
    write_b = pull_w * w_scale * 1024
    rec = {
        "kernel_source_sha256": source_hash(), "workload": workload,
        "fetch_size_pull": pull_f, "fetch_size_copy_1GiB": copy_f, "fetch_scale": f_scale,
        "write_size_pull": pull_w, "write_size_copy_1GiB": copy_w, "write_scale": w_scale,
        "pull_dispatches_averaged": [n1, n2],
        "read_bytes_per_launch": read_b, "write_bytes_per_launch": write_b,
        "traffic_bytes_per_launch": read_b + write_b,
    }
    records = _load_all()
    records[workload] = rec
    with open(RECORD, "w") as f:
        json.dump({"records": records}, f, indent=1)
    print(json.dumps(rec, indent=1))
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
