"""Turn rocprofv3 counter-collection CSVs into the short summaries kept under
profiles/.

    python -m paper_2605_09402_amd.profile_summary traffic FETCH.csv WRITE.csv OUT.json

reads the per-dispatch FETCH_SIZE and WRITE_SIZE values (KiB) of two
`rocprofv3 --pmc` runs of `bench.py --steps 1 --warmup 0 --traffic-calibration`,
scales each by what the same counter read for the plain 4 GiB device copy in
the same run, and writes the HBM bytes per layer of the library's kernels.
"""
from __future__ import annotations

import csv
import hashlib
import json
import os
import re
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
COPY_BYTES = 4 << 30


def kernel_source_hash() -> str:
    h = hashlib.sha256()
    for name in ("k_aggregate.hip", "k_update.hip"):
        with open(os.path.join(HERE, "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def _per_kernel(path):
    rows = list(csv.DictReader(open(path)))
    copies = [float(r["Counter_Value"]) for r in rows
              if r["Kernel_Name"].startswith("__amd_rocclr_copyBuffer") and float(r["Counter_Value"]) > 1e6]
    if len(copies) < 3:
        raise SystemExit("calibration copies not found in " + path)
    scale = (COPY_BYTES / 1024.0) / (sum(copies[-3:]) / 3.0)
    out = {}
    for r in rows:
        if "atlas" not in r["Kernel_Name"]:
            continue
        name = re.sub(r"[<(].*", "", r["Kernel_Name"].replace("void ", "").replace("atlas::(anonymous namespace)::", ""))
        ent = out.setdefault(name, {"launches": 0, "kib": 0.0})
        ent["launches"] += 1
        ent["kib"] += float(r["Counter_Value"])
    return scale, out


def traffic(fetch_csv: str, write_csv: str, out_json: str) -> None:
    fs, fk = _per_kernel(fetch_csv)
    ws, wk = _per_kernel(write_csv)
    kernels = {}
    for name in fk:
        if name not in wk:
            continue
        rd = fk[name]["kib"] * fs * 1024.0
        wr = wk[name]["kib"] * ws * 1024.0
        kernels[name] = {"launches": fk[name]["launches"], "read_bytes": round(rd), "write_bytes": round(wr),
                         "bytes_per_launch": round((rd + wr) / max(1, fk[name]["launches"]))}
    doc = {"what": "HBM-side bytes (L2 <-> fabric) of one layer of bench.py's workload, from rocprofv3 --pmc "
                   "FETCH_SIZE and WRITE_SIZE, each scaled by the same counter's reading for a plain 4 GiB copy",
           "fetch_scale": round(fs, 4), "write_scale": round(ws, 4), "kernel_source_hash": kernel_source_hash(),
           "kernels": kernels}
    with open(out_json, "w") as f:
        json.dump(doc, f, indent=1)
        f.write("\n")
    print(json.dumps(doc, indent=1))


if __name__ == "__main__":
    if len(sys.argv) == 5 and sys.argv[1] == "traffic":
        traffic(sys.argv[2], sys.argv[3], sys.argv[4])
    else:
        raise SystemExit(__doc__)
