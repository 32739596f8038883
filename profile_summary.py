"""Turns rocprofv3 CSV output (kernel trace and counter collection of profile_driver runs) into the
short text summaries kept under profiles/ and into profiles/traffic.txt.

    python profile_summary.py kernels OUT/run_kernel_trace.csv "command" profiles/NAME.txt [LAUNCHES [PASSES [FIRST_PASS]]]
    python profile_summary.py traffic OUT/fetch_counter_collection.csv OUT/write_counter_collection.csv WORKLOAD
    python profile_summary.py report OUT WORKLOAD MIX DTYPE      (both, from OUT/{run,fetch,write}_*.csv)
    python profile_summary.py counters OUT WORKLOAD MIX DTYPE    (OUT/{sq,tcc}_counter_collection.csv)
    python profile_summary.py pieces OUT ROWS D                  (OUT/{fetch,write}_counter_collection.csv of `profile_driver.py 3 block N`)

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

ROOT = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(ROOT, "paper_2511_00603_amd", "csrc")
KERNEL_SOURCES = [os.path.join(CSRC, f) for f in ("epara_device.h", "epara_panel.h", "epara_stream.h", "epara_grouped.h")]
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "traffic.txt")
COPY_BYTES = 1 << 30


def kernel_source_hash():
    return hashlib.sha256(b"".join(open(f, "rb").read() for f in KERNEL_SOURCES)).hexdigest()[:16]


def _rows(path):
    return list(csv.DictReader(open(path)))


def kernels(trace_csv, command, out_txt, launches_per_pass, tail_passes=0, first_pass=None):
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
    first, last = launches_per_pass, len(g)
    what = "first pass skipped as warm-up"
    if first_pass is not None:
        first, last = first_pass * launches_per_pass, (first_pass + tail_passes) * launches_per_pass
        what = "passes %d..%d, the ones the benchmark times launch by launch" % (first_pass, first_pass + tail_passes - 1)
    elif tail_passes:
        first = max(launches_per_pass, len(g) - tail_passes * launches_per_pass)
        what = "the last %d passes" % tail_passes
    L += ["", "grouped_kernel per launch of a pass (dispatch i -> launch i mod %d; %s):" % (launches_per_pass, what)]
    for l in range(launches_per_pass):
        d = [t[1] for i, t in enumerate(g) if i % launches_per_pass == l and first <= i < last]
        if d:
            r = g[l][2]
            L.append("  launch %d  n=%3d  avg %9.2f  median %9.2f  min %9.2f  max %9.2f   grid %s x %s threads, scratch %s B/lane"
                     % (l, len(d), sum(d) / len(d), statistics.median(d), min(d), max(d),
                        int(r["Grid_Size_X"]) // int(r["Workgroup_Size_X"]), r["Workgroup_Size_X"], r["Scratch_Size"]))
    # the kernels between the dense layers of a ViT block (bench.py times them after its warm-up dispatches)
    for name in ("attention_kernel", "add_layernorm_kernel"):
        d = [(int(r["Start_Timestamp"]), (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3, r) for r in rows if name in r["Kernel_Name"]]
        d.sort(key=lambda t: t[0])
        if len(d) > 10:
            t = [x[1] for x in d[10:60]]                     # bench.py: 10 warm-up dispatches, 50 timed; the whole-block passes follow
            r = d[10][2]
            L.append("%s, dispatches 10..59 (the ones bench.py times on their own):  n=%3d  avg %9.2f  median %9.2f  min %9.2f  max %9.2f   grid %s x %s threads, LDS %s B, scratch %s B/lane"
                     % (name, len(t), sum(t) / len(t), statistics.median(t), min(t), max(t), int(r["Grid_Size_X"]) // int(r["Workgroup_Size_X"]),
                        r["Workgroup_Size_X"], r["LDS_Block_Size"], r["Scratch_Size"]))
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


def pieces(out_dir, rows, d):
    """profiles/counters_vit_block_pieces.txt: HBM-side bytes per launch of the attention and normalisation kernels."""
    def per_kernel(path, counter):
        vals = {}
        for r in _rows(path):
            if r["Counter_Name"] == counter:
                key = (int(r["Dispatch_Id"]), r["Kernel_Name"])
                vals[key] = vals.get(key, 0.0) + float(r["Counter_Value"])
        pick = lambda name: [v for (i, k), v in sorted(vals.items()) if name in k]
        return pick("attention_kernel"), pick("add_layernorm_kernel"), pick("copy_kernel")
    fa, fn, fc = per_kernel(os.path.join(out_dir, "fetch_counter_collection.csv"), "FETCH_SIZE")
    wa, wn, wc = per_kernel(os.path.join(out_dir, "write_counter_collection.csv"), "WRITE_SIZE")
    f_scale, w_scale = COPY_BYTES / (fc[-1] * 1024.0), COPY_BYTES / (wc[-1] * 1024.0)
    alg = rows * d * 2
    L = ["rocprofv3 counter summary of the kernels between a ViT block's dense layers (medians over the launches, first skipped)",
         "commands: rocprofv3 --pmc FETCH_SIZE --output-format csv -d OUT -o fetch -- python3 profile_driver.py 3 block 6",
         "          rocprofv3 --pmc WRITE_SIZE --output-format csv -d OUT -o write -- python3 profile_driver.py 3 block 6",
         "counter values (KiB per dispatch) scaled by what the same counter reads for a copy kernel of %d bytes: x %.3f (fetch), x %.3f (write)" % (COPY_BYTES, f_scale, w_scale), ""]
    for name, f, w, rd, wr in (("attention_kernel", fa, wa, 3 * alg, alg), ("add_layernorm_kernel", fn, wn, 2 * alg, 2 * alg)):
        fb, wb = statistics.median(f[1:]) * 1024 * f_scale, statistics.median(w[1:]) * 1024 * w_scale
        L.append("%-22s fetched %7.1f MB (algorithmic %6.1f MB)   written %6.1f MB (algorithmic %6.1f MB)   together %.2f x the algorithmic bytes"
                 % (name, fb / 1e6, rd / 1e6, wb / 1e6, wr / 1e6, (fb + wb) / (rd + wr)))
    sq = os.path.join(out_dir, "sq_counter_collection.csv")
    if os.path.exists(sq):
        L += ["", "          rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_WAIT_INST_LDS SQ_WAIT_INST_ANY GRBM_GUI_ACTIVE --output-format csv -d OUT -o sq -- python3 profile_driver.py 3 block 6",
              "(sums over the chip: GRBM_GUI_ACTIVE over 8 dies, SQ_VALU_MFMA_BUSY_CYCLES over 1024 SIMDs)"]
        vals = {}
        for r in _rows(sq):
            name = "attention_kernel" if "attention_kernel" in r["Kernel_Name"] else ("add_layernorm_kernel" if "add_layernorm" in r["Kernel_Name"] else None)
            if name:
                d = vals.setdefault(name, {}).setdefault(int(r["Dispatch_Id"]), {})
                d[r["Counter_Name"]] = d.get(r["Counter_Name"], 0.0) + float(r["Counter_Value"])
        for name, per in vals.items():
            med = lambda c: statistics.median([v[c] for v in list(per.values())[1:]])
            active = med("GRBM_GUI_ACTIVE") / 8
            L.append("%-22s active cycles per die %8.0f   matrix cores busy %5.1f %%   LDS bank conflict cycles %4.1f %% of LDS active   wave cycles waiting on LDS / any %4.1f %% / %4.1f %%"
                     % (name, active, 100 * med("SQ_VALU_MFMA_BUSY_CYCLES") / 1024 / active,
                        100 * med("SQ_LDS_BANK_CONFLICT") / max(med("SQ_LDS_IDX_ACTIVE"), 1.0),
                        100 * med("SQ_WAIT_INST_LDS") / med("SQ_WAVE_CYCLES"), 100 * med("SQ_WAIT_INST_ANY") / med("SQ_WAVE_CYCLES")))
    out = os.path.join(ROOT, "profiles", "counters_vit_block_pieces.txt")
    open(out, "w").write("\n".join(L) + "\n")
    print("\n".join(L))


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
    """profiles/grouped_kernel_WORKLOAD.txt and the WORKLOAD entry of profiles/traffic.txt from the three
    runs of the profile driver (kernel trace with 8 passes, FETCH_SIZE and WRITE_SIZE with 4 passes each)."""
    drv = "python3 profile_driver.py %s %s" % (mix, dtype)
    txt = os.path.join(ROOT, "profiles", "grouped_kernel_%s.txt" % workload)
    kernels(os.path.join(out_dir, "run_kernel_trace.csv"),
            "rocprofv3 --kernel-trace --stats --output-format csv -d OUT -o run -- %s 8" % drv, txt, launches_per_pass)
    traffic(os.path.join(out_dir, "fetch_counter_collection.csv"), os.path.join(out_dir, "write_counter_collection.csv"),
            workload, launches_per_pass)
    rec = json.load(open(TRAFFIC_JSON))[workload]
    L = ["", "HBM-side traffic per launch (profiles/traffic.txt, kernel source %s), from" % rec["kernel_source_sha256_16"],
         "  rocprofv3 --pmc FETCH_SIZE --output-format csv -d OUT -o fetch -- %s 4" % drv,
         "  rocprofv3 --pmc WRITE_SIZE --output-format csv -d OUT -o write -- %s 4" % drv,
         "each scaled by what the same counter reads for the 1 GiB copy kernel of the same run (fetch x %.3f, write x %.3f):"
         % (rec["fetch_scale"], rec["write_scale"])]
    for l in rec["launches"]:
        L.append("  launch %d: fetch %.3f GB, write %.3f GB" % (l["launch"], l["fetch_bytes"] / 1e9, l["write_bytes"] / 1e9))
    open(txt, "a").write("\n".join(L) + "\n")
    print("\n".join(L))


SQ_COUNTERS = "SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_WAIT_INST_LDS SQ_WAIT_INST_ANY GRBM_GUI_ACTIVE"
TCC_COUNTERS = "TCC_HIT_sum TCC_MISS_sum"
N_XCD, N_SIMD = 8, 256 * 4


def _per_launch(path, launches_per_pass):
    """counter name -> list over launches of the median (over passes, first pass skipped) of the per-dispatch sums;
    "_us" -> the same for the dispatch durations."""
    vals, dur = {}, {}
    for r in _rows(path):
        if "grouped_kernel" not in r["Kernel_Name"]:
            continue
        d = int(r["Dispatch_Id"])
        vals.setdefault(r["Counter_Name"], {})
        vals[r["Counter_Name"]][d] = vals[r["Counter_Name"]].get(d, 0.0) + float(r["Counter_Value"])
        dur[d] = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
    order = sorted(dur)
    out = {}
    for name, per in list(vals.items()) + [("_us", dur)]:
        out[name] = [statistics.median([per[d] for i, d in enumerate(order) if i % launches_per_pass == l and i >= launches_per_pass])
                     for l in range(launches_per_pass)]
    return out


def counters(out_dir, workload, mix, dtype, launches_per_pass=2):
    """profiles/counters_WORKLOAD.txt: clocks, matrix-core busy share, LDS bank conflicts and L2 hit rate per launch."""
    drv = "python3 profile_driver.py %s %s 4" % (mix, dtype)
    sq = _per_launch(os.path.join(out_dir, "sq_counter_collection.csv"), launches_per_pass)
    tcc = _per_launch(os.path.join(out_dir, "tcc_counter_collection.csv"), launches_per_pass)
    L = ["rocprofv3 counter summary of grouped_kernel, per launch of a pass (medians over passes, first pass skipped)",
         "commands: rocprofv3 --pmc %s --output-format csv -d OUT -o sq -- %s" % (SQ_COUNTERS, drv),
         "          rocprofv3 --pmc %s --output-format csv -d OUT -o tcc -- %s" % (TCC_COUNTERS, drv),
         "counter values are sums over the chip: GRBM_GUI_ACTIVE over %d dies, SQ_VALU_MFMA_BUSY_CYCLES over %d SIMDs" % (N_XCD, N_SIMD), ""]
    for l in range(launches_per_pass):
        clk = sq["GRBM_GUI_ACTIVE"][l] / N_XCD                       # cycles one die was active
        L += ["launch %d (%.0f us under the counter run)" % (l, sq["_us"][l]),
              "  average clock while active        %.2f GHz   (GRBM_GUI_ACTIVE / %d / duration)" % (clk / sq["_us"][l] / 1e3, N_XCD),
              "  matrix cores busy                 %.1f %%     (SQ_VALU_MFMA_BUSY_CYCLES / %d / active cycles)"
              % (100 * sq["SQ_VALU_MFMA_BUSY_CYCLES"][l] / N_SIMD / clk, N_SIMD),
              "  LDS bank conflict cycles          %.2f %%     of SQ_LDS_IDX_ACTIVE (%.3g of %.3g)"
              % (100 * sq["SQ_LDS_BANK_CONFLICT"][l] / max(sq["SQ_LDS_IDX_ACTIVE"][l], 1), sq["SQ_LDS_BANK_CONFLICT"][l], sq["SQ_LDS_IDX_ACTIVE"][l]),
              "  wave cycles waiting on LDS / any  %.1f %% / %.1f %%   (SQ_WAIT_INST_LDS, SQ_WAIT_INST_ANY over SQ_WAVE_CYCLES)"
              % (100 * sq["SQ_WAIT_INST_LDS"][l] / sq["SQ_WAVE_CYCLES"][l], 100 * sq["SQ_WAIT_INST_ANY"][l] / sq["SQ_WAVE_CYCLES"][l]),
              "  L2 hit rate                       %.1f %%     (TCC_HIT_sum / (TCC_HIT_sum + TCC_MISS_sum), %.3g requests)"
              % (100 * tcc["TCC_HIT_sum"][l] / (tcc["TCC_HIT_sum"][l] + tcc["TCC_MISS_sum"][l]), tcc["TCC_HIT_sum"][l] + tcc["TCC_MISS_sum"][l]), ""]
    txt = os.path.join(ROOT, "profiles", "counters_%s.txt" % workload)
    open(txt, "w").write("\n".join(L))
    print("\n".join(L))


if __name__ == "__main__":
    if sys.argv[1] == "counters":
        counters(sys.argv[2], sys.argv[3], sys.argv[4], sys.argv[5], int(sys.argv[6]) if len(sys.argv) > 6 else 2)
    elif sys.argv[1] == "report":
        report(sys.argv[2], sys.argv[3], sys.argv[4], sys.argv[5], int(sys.argv[6]) if len(sys.argv) > 6 else 2)
    elif sys.argv[1] == "kernels":
        kernels(sys.argv[2], sys.argv[3], sys.argv[4], int(sys.argv[5]) if len(sys.argv) > 5 else 2,
                int(sys.argv[6]) if len(sys.argv) > 6 else 0, int(sys.argv[7]) if len(sys.argv) > 7 else None)
    elif sys.argv[1] == "pieces":
        pieces(sys.argv[2], int(sys.argv[3]), int(sys.argv[4]))
    elif sys.argv[1] == "traffic":
        traffic(sys.argv[2], sys.argv[3], sys.argv[4], int(sys.argv[5]) if len(sys.argv) > 5 else 2)
