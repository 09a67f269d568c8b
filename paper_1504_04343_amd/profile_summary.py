"""Condenses rocprofv3 CSV output into the short text tables kept under profiles/.

Usage:
  python -m paper_1504_04343_amd.profile_summary stats  <dir>/<prefix>_kernel_stats.csv
  python -m paper_1504_04343_amd.profile_summary pmc    <dir>/<prefix>_counter_collection.csv

`stats` prints calls / average / total per kernel (from --kernel-trace --stats).
`pmc` prints, per kernel name, the per-dispatch average of every collected counter (from --pmc),
plus derived figures when their inputs are present: MFMA utilisation
(SQ_VALU_MFMA_BUSY_CYCLES over GRBM_GUI_ACTIVE x SIMDs, as rocprofv3's MfmaUtil defines it), and
FETCH_SIZE / WRITE_SIZE in MiB (the counters count KiB).
"""
import collections
import csv
import re
import sys

SIMDS = 1024      # MI355X: 256 CUs x 4 SIMDs
XCDS = 8          # GRBM_GUI_ACTIVE is reported summed over the 8 XCDs


def short(name):
    name = name.replace("void ", "").replace("cct::(anonymous namespace)::", "")
    name = re.sub(r"\(.*$", "", name)
    return name[:60]


def stats(path):
    rows = list(csv.DictReader(open(path)))
    print("%-60s %7s %12s %12s %7s" % ("kernel", "calls", "avg_us", "total_ms", "pct"))
    for r in rows:
        print("%-60s %7d %12.1f %12.3f %7.2f" % (short(r["Name"]), int(r["Calls"]),
                                                float(r["AverageNs"]) / 1e3,
                                                float(r["TotalDurationNs"]) / 1e6, float(r["Percentage"])))


def pmc(path):
    rows = list(csv.DictReader(open(path)))
    agg = collections.defaultdict(lambda: collections.defaultdict(float))
    disp = collections.defaultdict(set)
    for r in rows:
        k = short(r["Kernel_Name"])
        agg[k][r["Counter_Name"]] += float(r["Counter_Value"])
        disp[k].add(r["Dispatch_Id"])
    for k in sorted(agg, key=lambda k: -len(disp[k])):
        n = len(disp[k])
        v = agg[k]
        parts = ["%s=%.4g" % (c, v[c] / n) for c in sorted(v)]
        extra = []
        if "SQ_VALU_MFMA_BUSY_CYCLES" in v and v.get("GRBM_GUI_ACTIVE"):
            extra.append("MfmaUtil=%.1f%%" % (100.0 * v["SQ_VALU_MFMA_BUSY_CYCLES"] /
                                             (v["GRBM_GUI_ACTIVE"] / XCDS * SIMDS)))
        if "FETCH_SIZE" in v:
            extra.append("FETCH_MiB/dispatch=%.2f" % (v["FETCH_SIZE"] / n / 1024.0))
        if "WRITE_SIZE" in v:
            extra.append("WRITE_MiB/dispatch=%.2f" % (v["WRITE_SIZE"] / n / 1024.0))
        print("%-60s dispatches=%d  %s  %s" % (k, n, "  ".join(extra), "  ".join(parts)))


if __name__ == "__main__":
    if len(sys.argv) != 3 or sys.argv[1] not in ("stats", "pmc"):
        sys.exit(__doc__)
    (stats if sys.argv[1] == "stats" else pmc)(sys.argv[2])
