"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

    python3 -m paper_2107_06925_amd.prof_summary stats  <..._kernel_stats.csv>
    python3 -m paper_2107_06925_amd.prof_summary pmc    <..._counter_collection.csv> [name-substring]

`stats`: per kernel calls, total and average duration, share.  `pmc`: per
kernel name (shortened) and counter, the mean counter value per dispatch.
"""
import collections
import csv
import re
import sys


def short(name):
    name = re.sub(r"chimera::\(anonymous namespace\)::", "", name)
    m = re.match(r"_ZN7chimera12_GLOBAL__N_1\d+(\w+?)I(.*?)EEv", name)
    if m:
        args = re.findall(r"L[ib](\d+)E", m.group(2))
        types = "".join("f" if t == "f" else "b" for t in re.findall(r"(?<![A-Za-z])(f|DF16b)(?=[A-Z_]|$)", m.group(2).split("L")[0]))
        return "%s<%s%s>" % (m.group(1), (types + ";") if types else "", ",".join(args))
    return name.replace("bool _Accum", "bf16").split("(")[0][:70]        # some demanglers print __bf16 that way


def stats(path):
    rows = list(csv.DictReader(open(path)))
    total = sum(float(r["TotalDurationNs"]) for r in rows)
    print("%-64s %7s %12s %11s %6s" % ("kernel", "calls", "total_ms", "avg_us", "%"))
    for r in sorted(rows, key=lambda r: -float(r["TotalDurationNs"])):
        t = float(r["TotalDurationNs"])
        if t / total < 0.001:
            continue
        print("%-64s %7d %12.3f %11.2f %6.2f" % (short(r["Name"])[:64], int(r["Calls"]), t / 1e6,
                                                  float(r["AverageNs"]) / 1e3, 100 * t / total))
    print("total kernel time %.3f ms" % (total / 1e6))


def pmc(path, needle=""):
    agg = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if needle in r["Kernel_Name"]:
            agg[(short(r["Kernel_Name"]), r["Counter_Name"])].append(float(r["Counter_Value"]))
    print("%-64s %-14s %8s %14s" % ("kernel", "counter", "launches", "mean/launch"))
    for (k, c), v in sorted(agg.items()):
        print("%-64s %-14s %8d %14.1f" % (k[:64], c, len(v), sum(v) / len(v)))


if __name__ == "__main__":
    if len(sys.argv) < 3 or sys.argv[1] not in ("stats", "pmc"):
        sys.exit(__doc__)
    if sys.argv[1] == "stats":
        stats(sys.argv[2])
    else:
        pmc(sys.argv[2], sys.argv[3] if len(sys.argv) > 3 else "")
