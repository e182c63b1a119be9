"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

  python -m paper_2605_18739_amd.profsum stats  <dir>/<name>_kernel_stats.csv
  python -m paper_2605_18739_amd.profsum pmc    <dir>/<name>_counter_collection.csv <copy_bytes> [COUNTER=factor ...]

`stats` prints calls / average / min / max per kernel.  `pmc` prints the per-dispatch
average of every collected counter per kernel and, for FETCH_SIZE / WRITE_SIZE (KiB), the
bytes after scaling by what the same counter read for the plain device copy of
<copy_bytes> bytes found in the same run (the copy reads and writes that many bytes).
With <copy_bytes> = 0 the factors are taken from the command line instead (those another
run's calibration copy gave, e.g. FETCH_SIZE=2.0 WRITE_SIZE=1.0).
"""
import collections
import csv
import sys


def stats(path):
    rows = list(csv.DictReader(open(path)))
    print(f"{'kernel':100s} {'calls':>6s} {'avg_us':>10s} {'min_us':>10s} {'max_us':>10s} {'pct':>6s}")
    for r in rows:
        print(f"{r['Name'][:100]:100s} {int(r['Calls']):6d} {float(r['AverageNs']) / 1e3:10.2f} "
              f"{float(r['MinNs']) / 1e3:10.2f} {float(r['MaxNs']) / 1e3:10.2f} {float(r['Percentage']):6.2f}")


def pmc(path, copy_bytes, given=None):
    rows = list(csv.DictReader(open(path)))
    agg = collections.OrderedDict()
    for r in rows:
        d = agg.setdefault(r["Kernel_Name"], collections.OrderedDict())
        d.setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
    copy = None
    for k in agg:
        if "copy" in k.lower() or "elementwise" in k.lower():
            copy = k
    factors = dict(given or {})
    for c, f in factors.items():
        print(f"given: {c} is scaled by {f}")
    if copy and copy_bytes > 0:
        for c, vals in agg[copy].items():
            vals = [v for v in vals if v > 0.5 * max(vals)]         # the 1 GiB copies, not small ones
            if c in ("FETCH_SIZE", "WRITE_SIZE") and vals:
                factors[c] = copy_bytes / (sum(vals) / len(vals) * 1024.0)
                print(f"calibration: {copy[:60]} {c} avg {sum(vals) / len(vals):.1f} KiB for {copy_bytes} B "
                      f"-> factor {factors[c]:.4f}")
    for k, v in agg.items():
        print(k[:110])
        for c, vals in v.items():
            avg = sum(vals) / len(vals)
            line = f"    {c:28s} dispatches={len(vals):4d} avg={avg:.6g}"
            if c in factors:
                line += f"  -> {avg * 1024.0 * factors[c] / 1e6:.2f} MB per dispatch (scaled)"
                big = [x for x in vals if x > 0.5 * max(vals)]   # a kernel name may cover tensors of very different sizes
                if len(big) != len(vals):
                    line += (f"; the {len(big)} largest dispatches: "
                             f"{sum(big) / len(big) * 1024.0 * factors[c] / 1e6:.2f} MB each")
            print(line)


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "stats":
        stats(sys.argv[2])
    elif len(sys.argv) >= 4 and sys.argv[1] == "pmc":
        pmc(sys.argv[2], float(sys.argv[3]), {a.split("=")[0]: float(a.split("=")[1]) for a in sys.argv[4:]})
    else:
        sys.exit(__doc__)
