"""Turn rocprofv3 output of bench.py runs into the short text summaries kept under profiles/.

usage: python _work/profile_summary.py <dir> <workload>
<dir> holds   kt/<tag>_kernel_stats.csv            (rocprofv3 --kernel-trace --stats)
              pmc_fetch/<tag>_counter_collection.csv (rocprofv3 --pmc FETCH_SIZE, bench.py --calibrate-copy)
              pmc_write/<tag>_counter_collection.csv (rocprofv3 --pmc WRITE_SIZE, bench.py --calibrate-copy)
Writes profiles/<workload>_kernels.md and profiles/<workload>_traffic.json (HBM bytes per launch of
each kernel class, scaled by what the same counter reads for the plain 1 GiB copy)."""
import collections
import csv
import glob
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
# kernel class of the library's timing tap -> kernel name fragments
CLASSES = {"gather": ("k_gather_mfma", "k_conv3x3_halo", "k_conv3x3_c8"), "wgrad": ("k_wgrad_mfma", "k_wgrad3x3_halo", "k_wgrad3x3_c8"),
           "direct": ("k_conv_",), "pool": ("k_pool_",), "bn": ("k_bn_",), "eltwise": ("k_grad_copy",)}
COPY_BYTES = float(1 << 30)


def is_copy(name, value):
    """The calibration pass of bench.py --calibrate-copy: torch.mul(src, 1, out=dst) over 1 GiB."""
    return "elementwise" in name and "FillFunctor" not in name and 0.5 * COPY_BYTES < value < 2.0 * COPY_BYTES


def short(name):
    name = name.replace("bapipe::(anonymous namespace)::", "").replace("bapipe::", "")
    return name if name.startswith("void at::") else name.split("(")[0]


def one(pattern):
    f = glob.glob(pattern)
    return f[0] if f else None


def counter_per_kernel(path):
    agg = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        agg[short(r["Kernel_Name"])].append(float(r["Counter_Value"]) * 1024.0)     # KiB -> bytes
    return agg


def main():
    d, workload = sys.argv[1], sys.argv[2]
    out_md = os.path.join(ROOT, "profiles", "%s_kernels.md" % workload)
    lines = ["# %s: rocprofv3 kernel summary (MI355X)" % workload, ""]
    stats = one(os.path.join(d, "kt", "*_kernel_stats.csv"))
    if stats:
        lines += ["command: `rocprofv3 --kernel-trace --stats --output-format csv -- python3 bench.py "
                  "--workload %s --steps 5 --warmup 2 --no-cpu-baseline`" % workload, "",
                  "| kernel | calls | total ms | avg us | % |", "|---|---|---|---|---|"]
        for r in list(csv.DictReader(open(stats)))[:16]:
            lines.append("| `%s` | %s | %.3f | %.1f | %s |" % (short(r["Name"])[:70], r["Calls"],
                         int(r["TotalDurationNs"]) / 1e6, float(r["AverageNs"]) / 1e3, r["Percentage"]))
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
                  "`-- python3 bench.py --workload %s --steps 1 --warmup 0 --no-cpu-baseline --tap gather "
                  "--calibrate-copy`." % workload,
                  "Calibration: the plain 1 GiB copy reads FETCH_SIZE = %.3f GiB and WRITE_SIZE = %.3f GiB, so "
                  "the counters are divided by %.3f and %.3f." % (ff, wf, ff, wf), "",
                  "| kernel | launches | fetch MB/launch | write MB/launch |", "|---|---|---|---|"]
        for k in sorted(set(F) | set(W), key=lambda k: -(sum(F.get(k, [0])) + sum(W.get(k, [0]))))[:14]:
            fv, wv = F.get(k, [0.0]), W.get(k, [0.0])
            lines.append("| `%s` | %d | %.1f | %.1f |" % (k[:70], len(fv), sum(fv) / len(fv) / ff / 1e6, sum(wv) / len(wv) / wf / 1e6))
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
