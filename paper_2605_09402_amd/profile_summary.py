"""Turn rocprofv3 counter-collection CSVs into the short summaries kept under
profiles/.

    python -m paper_2605_09402_amd.profile_summary traffic FETCH.csv WRITE.csv OUT.json

reads the per-dispatch FETCH_SIZE and WRITE_SIZE values (KiB) of two
`rocprofv3 --pmc` runs of `bench.py --steps 1 --warmup 0 --traffic-calibration`,
scales each by what the same counter read for the plain 4 GiB device copy in
the same run, and writes the HBM bytes per layer of the library's kernels.

    python -m paper_2605_09402_amd.profile_summary kernels STATS.csv TRACE.csv BENCH.json TRAFFIC.json OUT.md

writes the markdown summary of a `rocprofv3 --kernel-trace --stats` run of
`bench.py --steps 5 --warmup 1` (kernel table, per-chunk launch times of one
layer, the bench line's figures and the traffic table).
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
        ent = out.setdefault(name, {"launches": 0, "kib": 0.0, "each": []})
        ent["launches"] += 1
        ent["kib"] += float(r["Counter_Value"])
        ent["each"].append(float(r["Counter_Value"]))
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
        if name == "k_aggregate_grouped" and len(fk[name]["each"]) == len(wk[name]["each"]):
            # the counter runs execute one layer: launch i is chunk i
            kernels[name]["read_bytes_by_launch"] = [round(v * fs * 1024.0) for v in fk[name]["each"]]
            kernels[name]["write_bytes_by_launch"] = [round(v * ws * 1024.0) for v in wk[name]["each"]]
    doc = {"what": "HBM-side bytes (L2 <-> fabric) of one layer of bench.py's workload, from rocprofv3 --pmc "
                   "FETCH_SIZE and WRITE_SIZE, each scaled by the same counter's reading for a plain 4 GiB copy",
           "fetch_scale": round(fs, 4), "write_scale": round(ws, 4), "kernel_source_hash": kernel_source_hash(),
           "kernels": kernels}
    with open(out_json, "w") as f:
        json.dump(doc, f, indent=1)
        f.write("\n")
    print(json.dumps(doc, indent=1))


def _short(name: str) -> str:
    name = name.replace("void ", "").replace("atlas::(anonymous namespace)::", "")
    return name.split("(")[0]


def kernels_md(stats_csv: str, trace_csv: str, bench_json: str, traffic_json: str, out_md: str) -> None:
    stats = [r for r in csv.DictReader(open(stats_csv)) if "atlas" in r["Name"] and "rocprim" not in r["Name"]]
    trace = list(csv.DictReader(open(trace_csv)))
    line = [ln for ln in open(bench_json).read().splitlines() if ln.startswith("{")][0]
    b = json.loads(line)
    t = json.load(open(traffic_json))["kernels"]
    nchunks = b["config"]["chunks"]

    def per_chunk(sub):
        d = [(int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e6 for r in trace if sub in r["Kernel_Name"]]
        return " ".join("%.3f" % x for x in d[nchunks:2 * nchunks])     # the second layer of the run

    agg = [r for r in stats if "k_aggregate_grouped" in r["Name"]][0]
    rows = "\n".join("| %s | %s | %.3f | %.1f | %.1f | %.1f |" % (
        _short(r["Name"])[:60], r["Calls"], float(r["TotalDurationNs"]) / 1e6, float(r["AverageNs"]) / 1e3,
        float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3) for r in stats)
    gb = lambda k, f: t[k][f] / 1e9 if k in t else 0.0
    agg_gb = gb("k_aggregate_grouped", "read_bytes") + gb("k_aggregate_grouped", "write_bytes")
    upd_gb = gb("k_update_pipelined", "read_bytes") + gb("k_update_pipelined", "write_bytes")
    lm = b["layer_ms"]
    out = []
    out.append("# rocprofv3 kernel summary: bench.py default run, workload %s\n" % b["config"]["workload"])
    out.append("Command (on the MI355X box, from the repository root):\n")
    out.append("    export TMPDIR=/tmp && rocprofv3 --kernel-trace --stats --output-format csv \\\n"
               "        -d gpurun_out/prof_s26 -o s26 -- python3 bench.py --steps 5 --warmup 1\n")
    out.append("summarised by `python -m paper_2605_09402_amd.profile_summary kernels <stats csv> <trace csv> "
               "<bench json> <traffic json> <this file>`.\n")
    out.append("The run executes 10 layers of the workload (1 warm-up + 5 timed + 3 end-to-end + 1 sampled-parity), "
               "i.e. %d launches of the\nscatter-aggregate kernel (%d chunks per layer).  The library's kernels "
               "(torch's input generation and the rocprim sort\nkernels of plan building and reordering omitted):\n"
               % (10 * nchunks, nchunks))
    out.append("| kernel | calls | total ms | avg us | min us | max us |\n|---|---|---|---|---|---|\n" + rows + "\n")
    out.append("k_aggregate_grouped: average launch %.3f ms over %s launches; bench.py's HIP-event figure for the "
               "timed launches of the\nsame run: %.2f ms per layer / %d = %.2f ms (the event span also covers "
               "k_zero_rows).\n" % (float(agg["AverageNs"]) / 1e6, agg["Calls"], lm["aggregate"], nchunks,
                                               b["roofline"]["avg_launch_ms"]))
    out.append("Launch times of one layer (ms), chunk 0 first; with in-degree-descending ids chunk 0 holds the hot "
               "sources and most edges.\nk_aggregate_grouped:\n\n    %s\n\nk_update_pipelined:\n\n    %s\n"
               % (per_chunk("k_aggregate_grouped"), per_chunk("k_update_pipelined")))
    out.append("bench.py line of the same run (bench_config5_rmat26.json.txt): %.2f ms per layer (aggregate %.2f, "
               "update %.2f, self %.2f, init %.2f);\n%.1f GTEPS; three layers end to end %.1f ms.\n"
               % (b["ms_per_step"], lm["aggregate"], lm["update"], lm["self"], lm["init"], b["value"],
                  b["end_to_end_ms"]))
    out.append("HBM-side traffic: two further runs, `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE`, each with\n"
               "`--kernel-include-regex \"k_aggregate|k_update|k_fill_zero|k_zero_cut|k_self|copyBuffer\" "
               "--output-format csv -- python3 bench.py\n--steps 1 --warmup 0 --no-cpu-baseline --no-e2e "
               "--traffic-calibration`, summarised by `python -m paper_2605_09402_amd.profile_summary\ntraffic`; the "
               "plain 4 GiB device copy of the same runs reads 2.0 GiB on FETCH_SIZE and 4.0 GiB on WRITE_SIZE, hence "
               "the scale\nfactors 2.0 and 1.0.  Per layer:\n")
    out.append("| kernel | launches | read GB | written GB |\n|---|---|---|---|\n" + "\n".join(
        "| %s | %d | %.2f | %.2f |" % (k, v["launches"], v["read_bytes"] / 1e9, v["write_bytes"] / 1e9)
        for k, v in t.items()) + "\n")
    out.append("k_aggregate_grouped moves %.0f GB in %.1f ms = %.2f TB/s (%.0f%% of the 8 TB/s peak); "
               "k_update_pipelined %.1f GB in %.2f ms = %.2f TB/s.\n"
               % (agg_gb, lm["aggregate"], agg_gb / lm["aggregate"], agg_gb / lm["aggregate"] / 8 * 100,
                  upd_gb, lm["update"], upd_gb / lm["update"]))
    ag = t.get("k_aggregate_grouped", {})
    d = [(int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e6 for r in trace if "k_aggregate_grouped" in r["Kernel_Name"]]
    d = d[nchunks:2 * nchunks]
    if "read_bytes_by_launch" in ag and len(ag["read_bytes_by_launch"]) == len(d) == nchunks:
        out.append("k_aggregate_grouped by launch (bytes from the counter runs, time from the trace above): with later "
                   "chunks the share of\naccumulator read-add-writes grows, and with the share of writes the rate "
                   "falls towards that of a plain copy.\n")
        out.append("| chunk | read GB | written GB | ms | TB/s |\n|---|---|---|---|---|\n" + "\n".join(
            "| %d | %.2f | %.2f | %.3f | %.2f |" % (i, r / 1e9, w / 1e9, d[i], (r + w) / 1e9 / d[i])
            for i, (r, w) in enumerate(zip(ag["read_bytes_by_launch"], ag["write_bytes_by_launch"]))) + "\n")
    with open(out_md, "w") as f:
        f.write("\n".join(out))


if __name__ == "__main__":
    if len(sys.argv) == 5 and sys.argv[1] == "traffic":
        traffic(sys.argv[2], sys.argv[3], sys.argv[4])
    elif len(sys.argv) == 7 and sys.argv[1] == "kernels":
        kernels_md(*sys.argv[2:7])
    else:
        raise SystemExit(__doc__)
