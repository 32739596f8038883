"""Turns rocprofv3 CSV output (kernel trace and counter collection of profile_driver runs) into the
short text summaries kept under profiles/ and into profiles/traffic.json.

    python -m paper_2511_00603_amd.profile_summary kernels OUT/run_kernel_trace.csv "command" profiles/NAME.txt
    python -m paper_2511_00603_amd.profile_summary traffic OUT/fetch_counter_collection.csv OUT/write_counter_collection.csv WORKLOAD
    python -m paper_2511_00603_amd.profile_summary report OUT WORKLOAD MIX DTYPE      (both, from OUT/{run,fetch,write}_*.csv)

Per-launch figures: the launches of one pass alternate (launch 0, launch 1, ...), so dispatch i of
grouped_kernel belongs to launch i mod L.  HBM traffic of a launch = counter value (KiB) x 1024 x
(known bytes of the copy kernel / what the counter read for it).
"""
import csv
import hashlib
import json
import os
import statistics
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
KERNEL_SOURCE = os.path.join(HERE, "csrc", "epara_kernels.hip")
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "traffic.json")
COPY_BYTES = 1 << 30


def kernel_source_hash():
    return hashlib.sha256(open(KERNEL_SOURCE, "rb").read()).hexdigest()[:16]


def _rows(path):
    return list(csv.DictReader(open(path)))


def kernels(trace_csv, command, out_txt, launches_per_pass):
    rows = _rows(trace_csv)
    by = {}
    for r in rows:
        by.setdefault(r["Kernel_Name"], []).append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    total = sum(sum(v) for v in by.values())
    L = ["rocprofv3 kernel-trace summary (durations in microseconds)", "command: " + command, "",
         "%-78s %6s %12s %10s %7s" % ("kernel", "calls", "total_us", "avg_us", "pct")]
    for name, d in sorted(by.items(), key=lambda kv: -sum(kv[1]))[:8]:
        L.append("%-78s %6d %12.1f %10.2f %7.2f" % (name[:78], len(d), sum(d), sum(d) / len(d), 100 * sum(d) / total))
    g = [(r["Kernel_Name"], (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3, r) for r in rows if "grouped_kernel" in r["Kernel_Name"]]
    g.sort(key=lambda t: int(t[2]["Start_Timestamp"]))
    L += ["", "grouped_kernel per launch of a pass (dispatch i -> launch i mod %d; first pass skipped as warm-up):" % launches_per_pass]
    for l in range(launches_per_pass):
        d = [t[1] for i, t in enumerate(g) if i % launches_per_pass == l and i >= launches_per_pass]
        if d:
            r = g[l][2]
            L.append("  launch %d  n=%3d  avg %9.2f  median %9.2f  min %9.2f  max %9.2f   grid %s x %s threads, scratch %s B/lane"
                     % (l, len(d), sum(d) / len(d), statistics.median(d), min(d), max(d),
                        int(r["Grid_Size_X"]) // int(r["Workgroup_Size_X"]), r["Workgroup_Size_X"], r["Scratch_Size"]))
    open(out_txt, "w").write("\n".join(L) + "\n")
    print("\n".join(L))


def _counter(path, name):
    vals = {}
    for r in _rows(path):
        if r["Counter_Name"] != name:
            continue
        key = (int(r["Dispatch_Id"]), r["Kernel_Name"])
        vals[key] = vals.get(key, 0.0) + float(r["Counter_Value"])
    grouped = [v for (d, k), v in sorted(vals.items()) if "grouped_kernel" in k]
    copy = [v for (d, k), v in sorted(vals.items()) if "copy_kernel" in k]
    return grouped, copy


def traffic(fetch_csv, write_csv, workload, launches_per_pass):
    fg, fc = _counter(fetch_csv, "FETCH_SIZE")
    wg, wc = _counter(write_csv, "WRITE_SIZE")
    f_scale = COPY_BYTES / (fc[-1] * 1024.0)          # the copy kernel reads and writes COPY_BYTES
    w_scale = COPY_BYTES / (wc[-1] * 1024.0)
    out = {"kernel_source_sha256_16": kernel_source_hash(), "fetch_scale": f_scale, "write_scale": w_scale, "launches": []}
    for l in range(launches_per_pass):
        f = [v for i, v in enumerate(fg) if i % launches_per_pass == l and i >= launches_per_pass]
        w = [v for i, v in enumerate(wg) if i % launches_per_pass == l and i >= launches_per_pass]
        out["launches"].append({"launch": l, "fetch_bytes": statistics.median(f) * 1024 * f_scale,
                                "write_bytes": statistics.median(w) * 1024 * w_scale})
    data = json.load(open(TRAFFIC_JSON)) if os.path.exists(TRAFFIC_JSON) else {}
    data[workload] = out
    json.dump(data, open(TRAFFIC_JSON, "w"), indent=1, sort_keys=True)
    print(json.dumps(out, indent=1))


def lookup_traffic(workload, launch):
    """HBM bytes (fetch + write) per launch from the last counter runs, or None if absent / the kernel source changed since."""
    if not os.path.exists(TRAFFIC_JSON):
        return None
    rec = json.load(open(TRAFFIC_JSON)).get(workload)
    if not rec or rec.get("kernel_source_sha256_16") != kernel_source_hash():
        return None
    for l in rec["launches"]:
        if l["launch"] == launch:
            return l["fetch_bytes"] + l["write_bytes"]
    return None


def report(out_dir, workload, mix, dtype, launches_per_pass=2):
    """profiles/grouped_kernel_WORKLOAD.txt and the WORKLOAD entry of profiles/traffic.json from the three
    runs of the profile driver (kernel trace with 8 passes, FETCH_SIZE and WRITE_SIZE with 4 passes each)."""
    drv = "python3 -m paper_2511_00603_amd.profile_driver %s %s" % (mix, dtype)
    txt = os.path.join(ROOT, "profiles", "grouped_kernel_%s.txt" % workload)
    kernels(os.path.join(out_dir, "run_kernel_trace.csv"),
            "rocprofv3 --kernel-trace --stats --output-format csv -d OUT -o run -- %s 8" % drv, txt, launches_per_pass)
    traffic(os.path.join(out_dir, "fetch_counter_collection.csv"), os.path.join(out_dir, "write_counter_collection.csv"),
            workload, launches_per_pass)
    rec = json.load(open(TRAFFIC_JSON))[workload]
    L = ["", "HBM-side traffic per launch (profiles/traffic.json, kernel source %s), from" % rec["kernel_source_sha256_16"],
         "  rocprofv3 --pmc FETCH_SIZE --output-format csv -d OUT -o fetch -- %s 4" % drv,
         "  rocprofv3 --pmc WRITE_SIZE --output-format csv -d OUT -o write -- %s 4" % drv,
         "each scaled by what the same counter reads for the 1 GiB copy kernel of the same run (fetch x %.3f, write x %.3f):"
         % (rec["fetch_scale"], rec["write_scale"])]
    for l in rec["launches"]:
        L.append("  launch %d: fetch %.3f GB, write %.3f GB" % (l["launch"], l["fetch_bytes"] / 1e9, l["write_bytes"] / 1e9))
    open(txt, "a").write("\n".join(L) + "\n")
    print("\n".join(L))


if __name__ == "__main__":
    if sys.argv[1] == "report":
        report(sys.argv[2], sys.argv[3], sys.argv[4], sys.argv[5], int(sys.argv[6]) if len(sys.argv) > 6 else 2)
    elif sys.argv[1] == "kernels":
        kernels(sys.argv[2], sys.argv[3], sys.argv[4], int(sys.argv[5]) if len(sys.argv) > 5 else 2)
    elif sys.argv[1] == "traffic":
        traffic(sys.argv[2], sys.argv[3], sys.argv[4], int(sys.argv[5]) if len(sys.argv) > 5 else 2)
