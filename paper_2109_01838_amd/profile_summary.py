"""Condense rocprofv3 CSV output into the short text tables kept under profiles/.

  python -m paper_2109_01838_amd.profile_summary stats  <..._kernel_stats.csv> [n_solves]
  python -m paper_2109_01838_amd.profile_summary pmc    <..._counter_collection.csv> <COUNTER> [kernel substrings..]
"""
import csv
import sys
from collections import defaultdict


def short(name):
    for junk in ("rama::", "(anonymous namespace)::", "void "):
        name = name.replace(junk, "")
    return name.split("(")[0]


def stats(path, n_solves=1):
    rows = list(csv.DictReader(open(path)))
    tot = sum(int(r["TotalDurationNs"]) for r in rows)
    print(f"total kernel time {tot / 1e6:.2f} ms over {n_solves} solve(s) = {tot / 1e6 / n_solves:.2f} ms per solve")
    print(f"{'kernel':<70} {'calls':>7} {'total_ms':>10} {'avg_us':>10} {'max_us':>10} {'share':>7}")
    for r in rows[:40]:
        print(f"{short(r['Name'])[:70]:<70} {int(r['Calls']):>7} {int(r['TotalDurationNs']) / 1e6:>10.3f} "
              f"{float(r['AverageNs']) / 1e3:>10.1f} {int(r['MaxNs']) / 1e3:>10.1f} {float(r['Percentage']):>6.2f}%")


def pmc(path, counter, subs):
    acc = defaultdict(lambda: [0, 0.0])
    for r in csv.DictReader(open(path)):
        if r.get("Counter_Name") != counter:
            continue
        name = short(r["Kernel_Name"])
        if subs and not any(s in name for s in subs):
            continue
        a = acc[name]
        a[0] += 1
        a[1] += float(r["Counter_Value"])
    print(f"{'kernel':<70} {'dispatches':>10} {counter + ' sum':>18} {'per dispatch':>16}")
    for name, (n, v) in sorted(acc.items(), key=lambda kv: -kv[1][1])[:40]:
        print(f"{name[:70]:<70} {n:>10} {v:>18.1f} {v / n:>16.1f}")


if __name__ == "__main__":
    if sys.argv[1] == "stats":
        stats(sys.argv[2], int(sys.argv[3]) if len(sys.argv) > 3 else 1)
    else:
        pmc(sys.argv[2], sys.argv[3], sys.argv[4:])
