"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2601_22137_amd.profile_summary stats  <kernel_stats.csv>
    python -m paper_2601_22137_amd.profile_summary pmc    <counter_collection.csv> [<copy_probe_counter_collection.csv>]

`stats` prints calls / total / average duration per kernel.  `pmc` prints the per-dispatch average of
every collected counter per kernel; when the counter collection of `bench.py --copy-probe` (three
1 GiB device copies) is given, FETCH_SIZE / WRITE_SIZE (KiB) are scaled by what the same counter
read for that copy and reported in bytes per launch.
"""
import collections
import csv
import re
import sys


def short(name):
    name = re.sub(r"\(anonymous namespace\)::", "", name)
    name = re.sub(r"^void ", "", name)
    return re.sub(r"\(.*$", "", name)


def stats(path):
    rows = list(csv.DictReader(open(path)))
    total = sum(float(r["TotalDurationNs"]) for r in rows)
    print("| kernel | calls | total ms | avg us | % |")
    print("|---|---:|---:|---:|---:|")
    for r in rows:
        t = float(r["TotalDurationNs"])
        if t / total < 0.002:
            continue
        print("| %s | %d | %.3f | %.2f | %.1f |" % (short(r["Name"]), int(r["Calls"]), t / 1e6,
                                                  float(r["AverageNs"]) / 1e3, 100.0 * t / total))
    print("\nGPU kernel time in total: %.3f ms" % (total / 1e6))


def per_kernel(path):
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        agg[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return agg


def pmc(path, copy_path=None):
    factors = {}
    if copy_path:
        for kern, ctrs in per_kernel(copy_path).items():
            if "copyBuffer" in kern or "copy" in kern.lower():
                for c, v in ctrs.items():
                    if c in ("FETCH_SIZE", "WRITE_SIZE") and max(v) > 1000:
                        factors[c] = (1 << 20) / (sum(v) / len(v))      # 1 GiB = 2^20 KiB per copy
        for c, f in factors.items():
            print("calibration: %s reads %.4f of the true KiB of a 1 GiB copy -> scale by %.4f" % (c, 1.0 / f, f))
    print("| kernel | counter | dispatches | average | bytes per launch (scaled) |")
    print("|---|---|---:|---:|---:|")
    for kern, ctrs in sorted(per_kernel(path).items()):
        for c, v in sorted(ctrs.items()):
            avg = sum(v) / len(v)
            scaled = "%.4g" % (avg * 1024.0 * factors[c]) if c in factors else ""
            if avg > 0:
                print("| %s | %s | %d | %.6g | %s |" % (kern, c, len(v), avg, scaled))


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "stats":
        stats(sys.argv[2])
    elif len(sys.argv) >= 3 and sys.argv[1] == "pmc":
        pmc(sys.argv[2], sys.argv[3] if len(sys.argv) > 3 else None)
    else:
        sys.exit(__doc__)
