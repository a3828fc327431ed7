"""Condense rocprofv3 CSV output into the short text tables kept under profiles/.

  python -m paper_2109_01838_amd.profile_summary stats  <..._kernel_stats.csv> [n_solves]
  python -m paper_2109_01838_amd.profile_summary pmc    <..._counter_collection.csv> <COUNTER> [kernel substrings..]
  python -m paper_2109_01838_amd.profile_summary traffic <fetch.csv> <write.csv> <fetch_scale> <write_scale> <out.json>
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


def event_name(rocprof_name):
    """Kernel name as the library's own timers spell it (bench.py's `kernels` table)."""
    n = short(rocprof_name)
    n = n.replace("unsigned long", "u64").replace("unsigned int", "u32").replace(", ", ",")
    if n.startswith("k_rs_scatter<"):
        # <key, value, has values, offsets by local scan>: the timers name key and value types only
        args = n[len("k_rs_scatter<"):].rstrip(">").split(",")
        return f"k_rs_scatter<{args[0]},{args[1]}>" if args[2] == "true" else f"k_rs_scatter<{args[0]}>"
    if n.startswith(("k_scan_", "k_sum_partial")) and "<" in n:
        head, args = n.split("<", 1)
        functor = args.rstrip(">").split(",")[-1].split("<")[0].strip()
        return f"{head}<{functor}>"
    if "<" in n and not n.startswith("k_rs_hist<"):
        return n.split("<", 1)[0]     # plain template arguments (lengths, flags) are not part of the timers' names
    return n


def traffic_json(fetch_csv, write_csv, fetch_scale, write_scale, out_path):
    """Per kernel: average HBM bytes per launch = scale*FETCH_SIZE + scale*WRITE_SIZE (KiB -> bytes)."""
    import json
    acc = defaultdict(lambda: [0, 0.0, 0, 0.0])
    for path, counter, slot in ((fetch_csv, "FETCH_SIZE", 0), (write_csv, "WRITE_SIZE", 2)):
        for r in csv.DictReader(open(path)):
            if r.get("Counter_Name") != counter:
                continue
            a = acc[event_name(r["Kernel_Name"])]
            a[slot] += 1
            a[slot + 1] += float(r["Counter_Value"])
    out = {}
    for name, (nf, f, nw, w) in acc.items():
        if nf and nw and (name.startswith("k_") or name.startswith("__amd")):
            out[name] = {"launches": nf, "read_bytes_per_launch": 1024.0 * fetch_scale * f / nf,
                         "written_bytes_per_launch": 1024.0 * write_scale * w / nw}
    json.dump({"fetch_scale": fetch_scale, "write_scale": write_scale, "kernels": out}, open(out_path, "w"), indent=1,
              sort_keys=True)


if __name__ == "__main__":
    if sys.argv[1] == "traffic":
        traffic_json(sys.argv[2], sys.argv[3], float(sys.argv[4]), float(sys.argv[5]), sys.argv[6])
    elif sys.argv[1] == "stats":
        stats(sys.argv[2], int(sys.argv[3]) if len(sys.argv) > 3 else 1)
    else:
        pmc(sys.argv[2], sys.argv[3], sys.argv[4:])
