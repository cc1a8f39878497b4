"""Turns rocprofv3 CSV output of a bench.py run into the short summaries kept under profiles/.

    python -m paper_1404_5997_amd.prof_summary --workload conv_stack \\
        --trace out/prof_kt/kt_kernel_trace.csv \\
        --fetch out/pmc_fetch/fetch_counter_collection.csv \\
        --write out/pmc_write/write_counter_collection.csv \\
        [--sq out/pmc_sq/sq_counter_collection.csv] --out profiles

Only the dispatches of the last steps of the run are used (the steps after the
library's tuning runs); bench.py --copy-calibration ends with three plain
1 GiB copies, which give the factor between the FETCH_SIZE / WRITE_SIZE
counters and real bytes.  Reads files only; needs no GPU and no torch.
"""
import argparse
import collections
import csv
import json
import os

COPY_BYTES = 1024 * 1024 * 1024


def short(name):
    return name.replace("void owt::", "").replace("owt::", "").split("(")[0]


def family(name):
    n = short(name)
    if n.startswith("dconv_bf16_kernel") or n.startswith("dconv16p_kernel"):
        return "dconv16 " + ("fwd" if "EpiFwd" in n else "bwd_data")
    if n.startswith("dconv_kernel"):
        return "dconv " + ("fwd" if "EpiFwd" in n else "bwd_data")
    if n.startswith("dfilter16_kernel"):
        return "dfilter16 bwd_filter"
    if n.startswith("dfilter_kernel"):
        return "dfilter bwd_filter"
    if n.startswith("sconv16_fwd_kernel"):
        return "sconv16 fwd"
    if n.startswith("sfilter16_kernel"):
        return "sfilter16 bwd_filter"
    if n.startswith("sfilter_kernel"):
        return "sfilter bwd_filter"
    if n.startswith("sconv_fwd_kernel"):
        return "sconv fwd"
    if n.startswith("igemm_kernel"):
        return "igemm " + ("fwd" if "FwdA" in n else ("bwd_data" if "DataA" in n else "bwd_filter"))
    return None


def is_step_start(name):
    n = short(name)
    return n.startswith("sconv_pack_filters_kernel") or n.startswith("sconv16_pack_filters_kernel") or \
        (n.startswith("igemm_kernel") and "FwdA" in n and "1, 1, 1, 1" in n)


def is_copy(name):
    return "elementwise" in name or "copyBuffer" in name or "direct_copy" in name


def steady(rows, name_col, order_col, nsteps):
    rows = sorted(rows, key=lambda r: int(r[order_col]))
    starts = [i for i, r in enumerate(rows) if is_step_start(r[name_col])]
    if len(starts) < nsteps:
        raise SystemExit("fewer than %d steps found" % nsteps)
    body = rows[starts[-nsteps]:]
    copies = [r for r in body if is_copy(r[name_col])]
    return [r for r in body if not is_copy(r[name_col])], copies


def counters(path, nsteps):
    rows = list(csv.DictReader(open(path)))
    disp = collections.OrderedDict()
    for r in rows:
        d = disp.setdefault(int(r["Dispatch_Id"]), {"Kernel_Name": r["Kernel_Name"], "Dispatch_Id": r["Dispatch_Id"],
                                                     "Grid_Size": int(r["Grid_Size"]), "c": {}})
        d["c"][r["Counter_Name"]] = float(r["Counter_Value"])
    return steady(list(disp.values()), "Kernel_Name", "Dispatch_Id", nsteps)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--trace")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--sq")
    ap.add_argument("--steps", type=int, default=3, help="steps at the end of the run to average over")
    ap.add_argument("--command", default="", help="the profiled command line, quoted into the summary")
    ap.add_argument("--out", default="profiles")
    a = ap.parse_args()
    os.makedirs(a.out, exist_ok=True)

    if a.trace:
        rows = list(csv.DictReader(open(a.trace)))
        body, _ = steady(rows, "Kernel_Name", "Start_Timestamp", a.steps)
        per = collections.OrderedDict()
        for r in body:
            key = (short(r["Kernel_Name"]), int(r["Grid_Size_X"]) * int(r.get("Grid_Size_Y", 1) or 1) * int(r.get("Grid_Size_Z", 1) or 1))
            per.setdefault(key, []).append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
        wall = (int(body[-1]["End_Timestamp"]) - int(body[0]["Start_Timestamp"])) / 1e3 / a.steps
        tot = sum(sum(v) for v in per.values()) / a.steps
        with open(os.path.join(a.out, "%s_kernel_trace.md" % a.workload), "w") as f:
            f.write("# rocprofv3 kernel trace: %s\n\n" % a.workload)
            f.write("Command: `%s`\n\n" % a.command)
            f.write("Last %d steps of the run (after the library's tuning runs).  Sum of kernel durations "
                    "%.1f us per step, first-start to last-end %.1f us per step.\n\n" % (a.steps, tot, wall))
            f.write("| kernel | grid threads | launches/step | avg us | us/step |\n|---|---|---|---|---|\n")
            for (n, gsz), v in sorted(per.items(), key=lambda kv: -sum(kv[1])):
                f.write("| `%s` | %d | %.2f | %.1f | %.1f |\n" % (n, gsz, len(v) / a.steps, sum(v) / len(v), sum(v) / a.steps))

    traffic = {}
    scale = {}
    for which, path in (("fetch", a.fetch), ("write", a.write)):
        if not path:
            continue
        cname = "FETCH_SIZE" if which == "fetch" else "WRITE_SIZE"
        body, copies = counters(path, a.steps)
        vals = [c["c"][cname] for c in copies if c["c"].get(cname, 0) > 0]
        # the counter reads KiB; a plain copy of COPY_BYTES should read COPY_BYTES / 1024
        scale[which] = (COPY_BYTES / 1024.0) / (sum(vals) / len(vals)) if vals else 1.0
        agg = collections.OrderedDict()
        names = {}
        seen = {"fwd": 0, "bwd_filter": 0, "bwd_data": 0}
        nlayers = sum(1 for d in body if (family(d["Kernel_Name"]) or "").endswith(" fwd")) // a.steps
        for d in body:
            if is_step_start(d["Kernel_Name"]):
                seen = {"fwd": 0, "bwd_filter": 0, "bwd_data": 0}
            fam = family(d["Kernel_Name"])
            if fam is None:
                continue
            agg.setdefault("%s %d" % (fam, d["Grid_Size"]), []).append(d["c"][cname])
            # the same dispatch under the name of the call it serves: forward runs conv1..convL, backward
            # convL..conv1 (filter gradient, then data gradient), one convolution kernel per call
            ps = fam.split()[1]
            layer = seen[ps] + 1 if ps == "fwd" else nlayers - seen[ps]
            seen[ps] += 1
            ck = "call conv%d %s" % (layer, ps)
            agg.setdefault(ck, []).append(d["c"][cname])
            names[ck] = short(d["Kernel_Name"])
        for k, v in agg.items():
            traffic.setdefault(k, {})["%s_bytes" % which] = round(sum(v) / len(v) * 1024.0 * scale[which])
            if k in names:
                traffic[k]["kernel"] = names[k]
    if traffic:
        tpath = os.path.join(a.out, "hbm_traffic.json")
        allw = json.load(open(tpath)) if os.path.exists(tpath) else {}
        merged = dict(allw.get(a.workload, {}))      # variants seen in earlier profile runs stay listed
        merged.update({k: v for k, v in traffic.items() if "fetch_bytes" in v and "write_bytes" in v})
        allw[a.workload] = merged
        allw.setdefault("_calibration", {})[a.workload] = {
            "copy_bytes": COPY_BYTES, "fetch_scale": round(scale.get("fetch", 1.0), 4),
            "write_scale": round(scale.get("write", 1.0), 4),
            "note": "bytes = counter (KiB per dispatch) * 1024 * scale; scale = what a plain 1 GiB device copy should read / what it read"}
        json.dump(allw, open(tpath, "w"), indent=1, sort_keys=True)

    if a.sq:
        body, _ = counters(a.sq, 1)
        with open(os.path.join(a.out, "%s_counters.md" % a.workload), "w") as f:
            f.write("# rocprofv3 --pmc (SQ counters), last step: %s\n\n" % a.workload)
            f.write("Command: `%s`\n\n" % a.command)
            f.write("MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / 1024 SIMDs / (GRBM_GUI_ACTIVE / 8 XCDs); "
                    "LDS conflict = SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE.\n\n")
            f.write("| kernel | grid threads | kcycles | MFMA busy % | LDS bank conflict % |\n|---|---|---|---|---|\n")
            for d in body:
                c = d["c"]
                cyc = c.get("GRBM_GUI_ACTIVE", 0) / 8.0
                if cyc <= 0:
                    continue
                busy = 100.0 * c.get("SQ_VALU_MFMA_BUSY_CYCLES", 0) / 1024.0 / cyc
                conf = 100.0 * c.get("SQ_LDS_BANK_CONFLICT", 0) / c["SQ_LDS_IDX_ACTIVE"] if c.get("SQ_LDS_IDX_ACTIVE") else 0.0
                f.write("| `%s` | %d | %.0f | %.1f | %.1f |\n" % (short(d["Kernel_Name"]), d["Grid_Size"], cyc / 1e3, busy, conf))


if __name__ == "__main__":
    main()
