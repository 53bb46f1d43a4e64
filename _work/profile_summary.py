"""Turn rocprofv3 output of bench.py runs into the short text summaries kept under profiles/.

usage: python _work/profile_summary.py <dir> <workload>
<dir> holds   kt1/<..>_kernel_stats.csv             (rocprofv3 --kernel-trace --stats, bench.py --streams 1)
              kt3/<..>_kernel_stats.csv             (same, default streams)
              pmc_fetch/<..>_counter_collection.csv (rocprofv3 --pmc FETCH_SIZE, bench.py --calibrate-copy)
              pmc_write/<..>_counter_collection.csv (rocprofv3 --pmc WRITE_SIZE, bench.py --calibrate-copy)
              pmc_sq/<..>_counter_collection.csv    (rocprofv3 --pmc SQ_* utilisation counters)
Writes profiles/<workload>_kernels.md and profiles/<workload>_traffic.json (HBM bytes per launch of
each kernel class, scaled by what the same counter reads for the plain 1 GiB copy)."""
import collections
import csv
import glob
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLASSES = {"gather": ("k_gather_mfma", "k_conv3x3_halo", "k_conv3x3_c8"), "wgrad": ("k_wgrad_mfma", "k_wgrad3x3_halo", "k_wgrad3x3_c8"),
           "direct": ("k_conv_",), "pool": ("k_pool_",), "bn": ("k_bn_",), "eltwise": ("k_grad_copy",)}
COPY_BYTES = float(1 << 30)
SQ = "SQ_BUSY_CU_CYCLES SQ_VALU_MFMA_BUSY_CYCLES SQ_WAVE_CYCLES SQ_WAIT_INST_ANY SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE"


def is_copy(name, value):
    return "elementwise" in name and "FillFunctor" not in name and 0.5 * COPY_BYTES < value < 2.0 * COPY_BYTES


def short(name):
    name = name.replace("bapipe::(anonymous namespace)::", "").replace("bapipe::", "").replace("(anonymous namespace)::", "")
    if name.startswith("void at::"):
        return name
    import re
    m = re.search(r"\bk_\w+(<[^(]*>)?", name)
    return (m.group(0) if m else name.split("(")[0]) or name[:60]


def one(pattern):
    f = glob.glob(pattern)
    return f[0] if f else None


def counter_per_kernel(path, scale=1024.0):
    agg = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        agg[short(r["Kernel_Name"])].append(float(r["Counter_Value"]) * scale)
    return agg


def stats_table(path, cmd, lines, top=16):
    lines += ["command: `%s`" % cmd, "", "| kernel | calls | total ms | avg us | % |", "|---|---|---|---|---|"]
    for r in list(csv.DictReader(open(path)))[:top]:
        lines.append("| `%s` | %s | %.3f | %.1f | %s |" % (short(r["Name"])[:70], r["Calls"],
                     int(r["TotalDurationNs"]) / 1e6, float(r["AverageNs"]) / 1e3, r["Percentage"]))


def main():
    d, workload = sys.argv[1], sys.argv[2]
    extra = " ".join(sys.argv[3:])
    base = "python3 bench.py --workload %s" % workload
    out_md = os.path.join(ROOT, "profiles", "%s_kernels.md" % workload)
    lines = ["# %s: rocprofv3 summaries (MI355X)" % workload, ""]
    s1 = one(os.path.join(d, "kt1", "*_kernel_stats.csv"))
    if s1:
        lines += ["## Kernel times, one stream", "",
                  "Every kernel alone on the chip: these averages are what `bench.py`'s roofline tap measures "
                  "(`roofline.avg_launch_ms` is the work-weighted mean over the launches of one class).", ""]
        stats_table(s1, "rocprofv3 --kernel-trace --stats --output-format csv -- %s --streams 1 --steps 5 --warmup 2 --no-cpu-baseline --no-per-config" % base, lines)
    s3 = one(os.path.join(d, "kt3", "*_kernel_stats.csv"))
    if s3:
        lines += ["", "## Kernel times, default streams", "",
                  "Backward passes and their weight-gradient kernels on streams of their own: kernels share the compute units, "
                  "so a kernel's own duration grows while the step gets shorter (the last steps of this run, under the "
                  "roofline tap, are on one stream again).", ""]
        stats_table(s3, "rocprofv3 --kernel-trace --stats --output-format csv -- %s --steps 5 --warmup 2 --no-cpu-baseline --no-per-config" % base, lines, 10)
    sq = one(os.path.join(d, "pmc_sq", "*_counter_collection.csv"))
    if sq:
        rows = list(csv.DictReader(open(sq)))
        agg = collections.OrderedDict()
        for r in rows:
            k = r["Dispatch_Id"]
            e = agg.setdefault(k, {"name": short(r["Kernel_Name"]), "ns": int(r["End_Timestamp"]) - int(r["Start_Timestamp"])})
            e[r["Counter_Name"]] = float(r["Counter_Value"])
        per = collections.OrderedDict()
        for e in agg.values():
            if e.get("SQ_BUSY_CU_CYCLES", 0) < 1e5 or e["name"].startswith("void at::") or e["name"].startswith("__amd"):
                continue
            per.setdefault(e["name"], []).append(e)
        lines += ["", "## Matrix-core utilisation and LDS conflicts per kernel", "",
                  "command: `rocprofv3 --pmc %s --output-format csv -- %s --streams 1 --steps 1 --warmup 0 --tap-steps 1 --no-cpu-baseline --no-per-config --no-peaks`" % (SQ, base), "",
                  "MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / (4 SIMDs x SQ_BUSY_CU_CYCLES): share of the cycles of the BUSY compute units in "
                  "which a matrix core works.  chip = the same over all 256 units for the kernel's whole duration at the clock the counters "
                  "imply (busy cycles / duration / 256 below 1.9-2.0 GHz means units idle at the tail).  wait = SQ_WAIT_INST_ANY / "
                  "SQ_WAVE_CYCLES; LDS conflict = SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE.", "",
                  "| kernel | launches | avg us | MFMA busy | busy GHz-equiv | wait | LDS conflict |", "|---|---|---|---|---|---|---|"]
        order = sorted(per.items(), key=lambda kv: -sum(e["ns"] for e in kv[1]))[:14]
        for name, es in order:
            busy = sum(e["SQ_BUSY_CU_CYCLES"] for e in es)
            ns = sum(e["ns"] for e in es)
            lines.append("| `%s` | %d | %.1f | %.3f | %.2f | %.3f | %.3f |" % (
                name[:60], len(es), ns / len(es) / 1e3, sum(e["SQ_VALU_MFMA_BUSY_CYCLES"] for e in es) / busy / 4,
                busy / 256.0 / ns, sum(e["SQ_WAIT_INST_ANY"] for e in es) / max(1.0, sum(e["SQ_WAVE_CYCLES"] for e in es)),
                sum(e["SQ_LDS_BANK_CONFLICT"] for e in es) / max(1.0, sum(e["SQ_LDS_IDX_ACTIVE"] for e in es))))
    traffic = {}
    fetch, write = one(os.path.join(d, "pmc_fetch", "*_counter_collection.csv")), one(os.path.join(d, "pmc_write", "*_counter_collection.csv"))
    if fetch and write:
        F, W = counter_per_kernel(fetch), counter_per_kernel(write)
        fcopy = [v for k, vs in F.items() for v in vs if is_copy(k, v)]
        wcopy = [v for k, vs in W.items() for v in vs if is_copy(k, v)]
        ff = (sum(fcopy) / len(fcopy)) / COPY_BYTES if fcopy else 1.0
        wf = (sum(wcopy) / len(wcopy)) / COPY_BYTES if wcopy else 1.0
        lines += ["", "## HBM traffic per launch", "",
                  "commands: `rocprofv3 --pmc FETCH_SIZE ...` and `rocprofv3 --pmc WRITE_SIZE ...`, each with "
                  "`--output-format csv -- %s --streams 1 --steps 1 --warmup 0 --tap-steps 1 --no-cpu-baseline --no-per-config --no-peaks "
                  "--calibrate-copy`." % base,
                  "Calibration: the plain 1 GiB copy reads FETCH_SIZE = %.3f GiB and WRITE_SIZE = %.3f GiB, so "
                  "the counters are divided by %.3f and %.3f." % (ff, wf, ff, wf), "",
                  "| kernel | launches | fetch MB/launch | write MB/launch |", "|---|---|---|---|"]
        tot = 0.0
        keys = sorted(set(F) | set(W), key=lambda k: -(sum(F.get(k, [0])) / ff + sum(W.get(k, [0])) / wf))
        for k in keys:
            if not (k.startswith("void at::") or k.startswith("__amd_rocclr_fill")):
                tot += sum(F.get(k, [0])) / ff + sum(W.get(k, [0])) / wf
        for k in keys[:14]:
            fv, wv = F.get(k, [0.0]), W.get(k, [0.0])
            lines.append("| `%s` | %d | %.1f | %.1f |" % (k[:70], len(fv), sum(fv) / len(fv) / ff / 1e6, sum(wv) / len(wv) / wf / 1e6))
        lines += ["", "All library kernels of this run together (see the command for how many steps it holds): %.2f GB." % (tot / 1e9)]
        for cls, pat in CLASSES.items():
            fv = [v for k, vs in F.items() if any(x in k for x in pat) for v in vs]
            wv = [v for k, vs in W.items() if any(x in k for x in pat) for v in vs]
            if fv or wv:
                n = max(len(fv), len(wv))
                traffic[cls] = (sum(fv) / ff + sum(wv) / wf) / n
        json.dump({"workload": workload, "unit": "HBM bytes per kernel launch (FETCH_SIZE + WRITE_SIZE, calibrated)",
                   "per_class": traffic}, open(os.path.join(ROOT, "profiles", "%s_traffic.json" % workload), "w"), indent=1)
    open(out_md, "w").write("\n".join(lines) + "\n")
    print("wrote", out_md, traffic)


if __name__ == "__main__":
    main()
