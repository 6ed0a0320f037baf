"""Condense rocprofv3 CSV output into the short text summaries kept under profiles/.

  python profile_summary.py stats  <kernel_stats.csv>
  python profile_summary.py pmc    <counter_collection.csv> [...]

`stats` prints calls / average / total per kernel.  `pmc` prints, per kernel, the
mean counter value per dispatch, and scales FETCH_SIZE / WRITE_SIZE (KiB) by what
the same counter reads for the library's plain copy kernel of known size
(bamboo::calibration_copy_kernel, launched by `bench.py --calibration-copy`).
"""
import csv
import collections
import sys


def _short(name):
    name = name.replace("void ", "").replace("bamboo::", "")
    if name.startswith("_ZN6bamboo"):
        import re
        m = re.match(r"_ZN6bamboo(\d+)", name)
        n = int(m.group(1))
        name = name[len(m.group(0)):][:n] + "<...>"
    return name[:78]


def stats(path, top=24):
    rows = list(csv.DictReader(open(path)))
    total = sum(float(r["TotalDurationNs"]) for r in rows)
    print("%-78s %7s %10s %10s %6s" % ("kernel", "calls", "avg us", "total ms", "%"))
    for r in rows[:top]:
        print("%-78s %7d %10.2f %10.2f %6.2f" % (_short(r["Name"]), int(r["Calls"]), float(r["AverageNs"]) / 1e3,
                                                float(r["TotalDurationNs"]) / 1e6, 100 * float(r["TotalDurationNs"]) / total))
    print("all kernels: %.2f ms" % (total / 1e6))


def pmc(paths, copy_bytes=256 << 20):
    gemm_bytes, group_bytes = {}, {}
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for path in paths:
        for r in csv.DictReader(open(path)):
            acc[r["Counter_Name"]][_short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    for counter, per_kernel in acc.items():
        cal = [v for k, vals in per_kernel.items() if k.startswith("calibration_copy_kernel") for v in vals]
        factor = None
        if cal and counter in ("FETCH_SIZE", "WRITE_SIZE"):
            factor = (copy_bytes / 1024.0) / (sum(cal) / len(cal))
        print("counter %s%s" % (counter, "" if factor is None else
                                 "   (copy kernel of %d MiB reads %.0f KiB -> scale factor %.4f)"
                                 % (copy_bytes >> 20, sum(cal) / len(cal), factor)))
        print("  %-78s %7s %14s %14s" % ("kernel", "calls", "mean/dispatch", "scaled MiB"))
        if factor is not None:
            g = [(len(v), sum(v)) for k, v in per_kernel.items() if k.startswith("gemm_mfma")]
            if g:
                gemm_bytes[counter] = sum(t for _, t in g) / sum(n for n, _ in g) * factor * 1024.0
            w = [(len(v), sum(v)) for k, v in per_kernel.items() if k.startswith("gemm_mfma_pl_group_kernel")]
            if w:
                group_bytes[counter] = sum(t for _, t in w) / sum(n for n, _ in w) * factor * 1024.0
        items = sorted(per_kernel.items(), key=lambda kv: -sum(kv[1]))
        for k, vals in items[:20]:
            mean = sum(vals) / len(vals)
            print("  %-78s %7d %14.1f %14s" % (k, len(vals), mean,
                                               "" if factor is None else "%.2f" % (mean * factor / 1024.0)))


    if len(gemm_bytes) == 2:
        print("call-weighted mean over the stage GEMM kernels (gemm_mfma*), scaled: fetch %.2f MiB + write %.2f MiB"
              % (gemm_bytes["FETCH_SIZE"] / 2 ** 20, gemm_bytes["WRITE_SIZE"] / 2 ** 20))
        print("stage_gemm_traffic_bytes_per_launch=%d" % round(sum(gemm_bytes.values())))
    if len(group_bytes) == 2:
        print("grouped weight-gradient launch (gemm_mfma_pl_group_kernel), scaled: fetch %.2f MiB + write %.2f MiB"
              % (group_bytes["FETCH_SIZE"] / 2 ** 20, group_bytes["WRITE_SIZE"] / 2 ** 20))
        print("wgrad_group_traffic_bytes_per_launch=%d" % round(sum(group_bytes.values())))


if __name__ == "__main__":
    if len(sys.argv) < 3 or sys.argv[1] not in ("stats", "pmc"):
        sys.exit(__doc__)
    if sys.argv[1] == "stats":
        stats(sys.argv[2])
    else:
        pmc(sys.argv[2:])
