"""Condense rocprofv3 CSV output into the short text tables kept under profiles/.

  python -m paper_2109_01838_amd.profile_summary stats  <..._kernel_stats.csv> [n_solves]
  python -m paper_2109_01838_amd.profile_summary pmc    <..._counter_collection.csv> <COUNTER> [kernel substrings..]
  python -m paper_2109_01838_amd.profile_summary traffic <fetch.csv> <write.csv> <fetch_scale> <write_scale> <out.json>
  python -m paper_2109_01838_amd.profile_summary report-workload <raw output dir> <profiles dir> <cfg2|cfg3|..>
  python -m paper_2109_01838_amd.profile_summary report  <raw output dir> <profiles dir>
      (all of the above for bench.py's default workload: expects prof_bench/, pmc_fetch/, pmc_write/ and
       bench_rocprof.log as the commands in the written files' headers leave them)
"""
import csv
import sys
from collections import defaultdict


def short(name):
    for junk in ("rama::", "(anonymous namespace)::", "void "):
        name = name.replace(junk, "")
    return name.split("(")[0]


def stats(path, n_solves=1, top=40):
    rows = list(csv.DictReader(open(path)))
    tot = sum(int(r["TotalDurationNs"]) for r in rows)
    print(f"total kernel time {tot / 1e6:.2f} ms over {n_solves} solve(s) = {tot / 1e6 / n_solves:.2f} ms per solve")
    print(f"{'kernel':<70} {'calls':>7} {'total_ms':>10} {'avg_us':>10} {'max_us':>10} {'share':>7}")
    for r in rows[:top]:
        print(f"{short(r['Name'])[:70]:<70} {int(r['Calls']):>7} {int(r['TotalDurationNs']) / 1e6:>10.3f} "
              f"{float(r['AverageNs']) / 1e3:>10.1f} {int(r['MaxNs']) / 1e3:>10.1f} {float(r['Percentage']):>6.2f}%")
    # instantiations that the library's own timers count as one kernel, taken together
    merged = defaultdict(lambda: [0, 0, 0])
    for r in rows:
        a = merged[event_name(r["Name"])]
        a[0] += 1
        a[1] += int(r["Calls"])
        a[2] += int(r["TotalDurationNs"])
    for name, (k, calls, ns) in sorted(merged.items(), key=lambda kv: -kv[1][2])[:12]:
        if k > 1:
            print(f"{name + ' (its ' + str(k) + ' instantiations together)':<70} {calls:>7} {ns / 1e6:>10.3f} {ns / 1e3 / calls:>10.1f}")


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
    if n.startswith("k_rs_local<"):
        # <key, value, has values, key type inside LDS>
        args = n[len("k_rs_local<"):].rstrip(">").split(",")
        wide = ",wide" if args[3] == "u64" else ""
        return f"k_rs_local<{args[0]},{args[1]}{wide}>" if args[2] == "true" else f"k_rs_local<{args[0]}{wide}>"
    if n.startswith(("k_scan_", "k_sum_partial")) and "<" in n:
        # the timers name the last functor by its tag: the class name without "Emit"; functors templated on a
        # key type or a length append it where the library does (HeadFlagT<u64> -> HeadFlag64)
        head, args = n.split("<", 1)
        last = args.strip().rstrip(">").strip().split(",")[-1].strip()
        functor, _, targ = last.partition("<")
        targ = targ.strip().rstrip(">").strip()
        if functor.endswith("Emit"):
            functor = functor[:-4]
        if functor == "HeadFlagT":
            functor = "HeadFlag64" if targ == "u64" else "HeadFlag32"
        elif functor == "Triangles" and targ == "u64":
            functor = "Triangles64"
        elif functor == "HasCycles" and targ == "7":
            functor = "HasCycles7"
        return f"{head}<{functor}>"
    if n.startswith(("k_count_cycles<", "k_fill_cycles<")):
        # <longest walk, last level closes from the far endpoint>: the timers name the walk length only
        return n.split(",")[0].rstrip(">") + ">"
    if "<" in n and not n.startswith(("k_rs_hist<", "k_edge_update<")):
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
    json.dump({"fetch_scale": fetch_scale, "write_scale": write_scale, "solves": 1, "kernels": out}, open(out_path, "w"),
              indent=1, sort_keys=True)


def capture(fn, *args):
    import contextlib
    import io
    buf = io.StringIO()
    with contextlib.redirect_stdout(buf):
        fn(*args)
    return buf.getvalue()


def copy_calibration(path, counter):
    """The runtime's own device-to-device copies of 1 GiB (bench.py --copy-calibration issues three)."""
    vals = [float(r["Counter_Value"]) for r in csv.DictReader(open(path))
            if r.get("Counter_Name") == counter and "copyBuffer" in r["Kernel_Name"]]
    return [v for v in vals if v > 400000.0][:3]     # the 1 GiB copies, not the small read-backs


def report(raw, out):
    import json
    import os
    n_solves = 5      # bench.py default: 1 warm-up + 1 all-kernel-timed + 3 timed solves
    d = json.loads([l for l in open(os.path.join(raw, "bench_rocprof.log")) if l.startswith("{")][-1])
    r = d["roofline"]
    stats_txt = capture(stats, os.path.join(raw, "prof_bench", "bench_kernel_stats.csv"), n_solves, 26)
    with open(os.path.join(out, "cfg5_solve_kernel_trace.txt"), "w") as f:
        f.write(f"""# rocprofv3 kernel-trace summary: bench.py default run ({d['config']['workload']}, {d['config']['n_edges']} edges; 1 warm-up + 1 all-kernel-timed + 3 timed solves = {n_solves} solves)
# command (on the GPU box; $REPO = repository root, $OUT = any scratch directory):
#   cd /tmp && export TMPDIR=/tmp && rocprofv3 --kernel-trace --stats -d $OUT/prof_bench -o bench --output-format csv -- python3 $REPO/bench.py --other-workloads '' --cpu-config none > $OUT/bench_rocprof.log
# condensed with: python -m paper_2109_01838_amd.profile_summary report $OUT profiles
# bench.py's own HIP-event figures for the dominant kernel in the same run:
#   {r['kernel']} avg_launch_ms {r['avg_launch_ms']:.5f} launches_per_step {r['launches_per_step']} achieved GB/s {r['achieved']:.1f} frac {r['frac']:.4f}
#   ms_per_step {d['ms_per_step']:.2f} edges/s {d['value']:.0f} (under the profiler, whose interception lengthens what the
#   events see: the run without it measures the trace's average, see the merged row at the end of the table)

""")
        f.write(stats_txt)
    fetch = os.path.join(raw, "pmc_fetch", "fetch_counter_collection.csv")
    write = os.path.join(raw, "pmc_write", "write_counter_collection.csv")
    cf, cw = copy_calibration(fetch, "FETCH_SIZE"), copy_calibration(write, "WRITE_SIZE")
    kib = 1048576.0
    fs, ws = round(kib / (sum(cf) / len(cf)), 2), round(kib / (sum(cw) / len(cw)), 2)
    traffic_json(fetch, write, fs, ws, os.path.join(out, "cfg5_solve_hbm_traffic.json"))
    with open(os.path.join(out, "cfg5_solve_hbm_traffic.txt"), "w") as f:
        f.write(f"""# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch), two separate runs, {d['config']['workload']}, one solve each
# commands (on the GPU box; $REPO = repository root, $OUT = any scratch directory):
#   rocprofv3 --pmc FETCH_SIZE -d $OUT/pmc_fetch -o fetch --output-format csv -- python3 $REPO/bench.py --steps 1 --warmup 0 --no-profile --other-workloads '' --cpu-config none --copy-calibration
#   rocprofv3 --pmc WRITE_SIZE -d $OUT/pmc_write -o write --output-format csv -- python3 $REPO/bench.py --steps 1 --warmup 0 --no-profile --other-workloads '' --cpu-config none --copy-calibration
# condensed with: python -m paper_2109_01838_amd.profile_summary report $OUT profiles
# calibration: a plain 1 GiB -> 1 GiB device copy (1048576 KiB read, 1048576 KiB written) reads
#   FETCH_SIZE {', '.join(f'{v:.1f}' for v in cf)}
#   WRITE_SIZE {', '.join(f'{v:.1f}' for v in cw)}
# => actual KiB read = {fs} x FETCH_SIZE, actual KiB written = {ws} x WRITE_SIZE
# per-kernel bytes per launch (scaled) are in cfg5_solve_hbm_traffic.json

""")
        f.write("\n".join(capture(pmc, fetch, "FETCH_SIZE", ["k_"]).splitlines()[:25]) + "\n\n")
        f.write("\n".join(capture(pmc, write, "WRITE_SIZE", ["k_"]).splitlines()[:25]) + "\n")


def report_workload(raw, out, workload):
    """Kernel-trace summary of a bench.py run on another named configuration (expects prof_<workload>/ and
    bench_<workload>_rocprof.log in `raw`, as the command in the written file's header leaves them)."""
    import json
    import os
    n_solves = 5
    d = json.loads([l for l in open(os.path.join(raw, f"bench_{workload}_rocprof.log")) if l.startswith("{")][-1])
    stats_txt = capture(stats, os.path.join(raw, f"prof_{workload}", f"{workload}_kernel_stats.csv"), n_solves, 32)
    with open(os.path.join(out, f"{workload}_solve_kernel_trace.txt"), "w") as f:
        f.write(f"""# rocprofv3 kernel-trace summary: bench.py on {d['config']['workload']} ({d['config']['n_edges']} edges; 1 warm-up + 1 all-kernel-timed + 3 timed solves = {n_solves} solves)
# command (on the GPU box; $REPO = repository root, $OUT = any scratch directory):
#   cd /tmp && export TMPDIR=/tmp && rocprofv3 --kernel-trace --stats -d $OUT/prof_{workload} -o {workload} --output-format csv -- python3 $REPO/bench.py --workload {workload} --other-workloads '' --cpu-config none > $OUT/bench_{workload}_rocprof.log
# condensed with: python -m paper_2109_01838_amd.profile_summary report-workload $OUT profiles {workload}
# bench.py in the same run: ms_per_step {d['ms_per_step']:.2f} (under the profiler), rounds {d['rounds']}, cycles found in round 1 {d['n_cycles_first'][:3]}

""")
        f.write(stats_txt)


if __name__ == "__main__":
    if sys.argv[1] == "report":
        report(sys.argv[2], sys.argv[3])
    elif sys.argv[1] == "report-workload":
        report_workload(sys.argv[2], sys.argv[3], sys.argv[4])
    elif sys.argv[1] == "traffic":
        traffic_json(sys.argv[2], sys.argv[3], float(sys.argv[4]), float(sys.argv[5]), sys.argv[6])
    elif sys.argv[1] == "stats":
        stats(sys.argv[2], int(sys.argv[3]) if len(sys.argv) > 3 else 1)
    else:
        pmc(sys.argv[2], sys.argv[3], sys.argv[4:])
