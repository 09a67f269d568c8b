"""Condenses rocprofv3 CSV output into the short text tables kept under profiles/.

Usage:
  python -m paper_1504_04343_amd.profile_summary stats  <dir>/<prefix>_kernel_stats.csv
  python -m paper_1504_04343_amd.profile_summary pmc    <dir>/<prefix>_counter_collection.csv
  python -m paper_1504_04343_amd.profile_summary traffic <FETCH_SIZE run>.csv <WRITE_SIZE run>.csv

`stats` prints calls / average / total per kernel (from --kernel-trace --stats).
`traffic` combines a --pmc FETCH_SIZE run and a --pmc WRITE_SIZE run of `bench.py
--copy-calibration`: both counters are scaled by what they read for the 1 GiB
`calibration_copy_kernel` (which moves exactly 1 GiB each way), and one line per kernel gives the
scaled HBM bytes per dispatch (`name<TAB>bytes`), the format bench.py reads back.
`pmc` prints, per kernel name, the per-dispatch average of every collected counter (from --pmc),
plus derived figures when their inputs are present: MFMA utilisation
(SQ_VALU_MFMA_BUSY_CYCLES over GRBM_GUI_ACTIVE x SIMDs, as rocprofv3's MfmaUtil defines it), and
FETCH_SIZE / WRITE_SIZE in MiB (the counters count KiB).
"""
import collections
import csv
import hashlib
import os
import re
import sys

SIMDS = 1024      # MI355X: 256 CUs x 4 SIMDs
XCDS = 8          # GRBM_GUI_ACTIVE is reported summed over the 8 XCDs


def kernel_sources_digest():
    """Short hash of the kernel sources (csrc/*.hip, *.h): a counter profile is only quoted for
    the code it was taken from."""
    h = hashlib.sha256()
    d = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()[:12]


def short(name):
    name = name.replace("void ", "").replace("cct::", "").replace("(anonymous namespace)::", "")
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


def per_dispatch(path, counter):
    tot = collections.defaultdict(float)
    disp = collections.defaultdict(set)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        k = short(r["Kernel_Name"])
        tot[k] += float(r["Counter_Value"])
        disp[k].add(r["Dispatch_Id"])
    return {k: tot[k] / len(disp[k]) for k in tot}, {k: len(disp[k]) for k in tot}


def traffic(fetch_csv, write_csv):
    fetch, nd = per_dispatch(fetch_csv, "FETCH_SIZE")      # KiB per dispatch
    write, _ = per_dispatch(write_csv, "WRITE_SIZE")
    cal = "calibration_copy_kernel"
    if cal not in fetch or cal not in write:
        sys.exit("no %s dispatch in the runs: use bench.py --copy-calibration" % cal)
    gib_kib = float(1 << 20)
    fs, ws = gib_kib / fetch[cal], gib_kib / write[cal]
    print("# kernel sources digest: %s" % kernel_sources_digest())
    print("# HBM traffic per dispatch = FETCH_SIZE*%.4f + WRITE_SIZE*%.4f KiB (scales from the 1 GiB "
          "%s: FETCH_SIZE read %.0f KiB, WRITE_SIZE read %.0f KiB)" % (fs, ws, cal, fetch[cal], write[cal]))
    print("# kernel<TAB>bytes_per_dispatch<TAB>dispatches<TAB>fetch_MiB_scaled<TAB>write_MiB_scaled")
    for k in sorted(fetch, key=lambda k: -(fetch[k] * fs + write.get(k, 0.0) * ws)):
        f, w = fetch[k] * fs, write.get(k, 0.0) * ws
        print("%s\t%d\t%d\t%.1f\t%.1f" % (k, int((f + w) * 1024), nd[k], f / 1024, w / 1024))


if __name__ == "__main__":
    if len(sys.argv) == 4 and sys.argv[1] == "traffic":
        traffic(sys.argv[2], sys.argv[3])
    elif len(sys.argv) == 3 and sys.argv[1] in ("stats", "pmc"):
        (stats if sys.argv[1] == "stats" else pmc)(sys.argv[2])
    else:
        sys.exit(__doc__)
