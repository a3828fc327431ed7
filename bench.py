#!/usr/bin/env python3
"""Benchmark of the primal-dual multicut solver on one MI355X.

A "step" is one full rama_solve (canonicalise -> rounds of {cycle separation, message passing,
contraction} -> labels, primal cost, lower bound) on a synthetic instance that is already in
device memory when the timed region starts.  Default workload: cfg5, the 320^3 6-connected
grid with ~9.8e7 edges (see paper_2109_01838_amd/inputs.py).

Prints ONE JSON line: edges/s and solve time, the roofline record of the dominant kernel
(measured with HIP events by the library's built-in per-kernel timers over the timed steps),
and the CPU oracle timed on a bounded sample of the same recipe.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published


def make_workload(name):
    from paper_2109_01838_amd import inputs
    if name == "cfg5":
        return inputs.cfg5()
    if name.startswith("cfg5crop"):
        return inputs.cfg5_crop(int(name[len("cfg5crop"):]))
    return inputs.make(name)


def solver_kwargs(args):
    return dict(max_cycle_len_first=args.cycle_len[0], max_cycle_len_later=args.cycle_len[1],
                shortest_only=args.shortest_only, dual_rounds=args.dual_rounds)


def cpu_baseline(name, args, gpu_result, g):
    """The CPU oracle, as it stands, timed on a named configuration small enough for ~10-30 s of CPU work
    (default cfg3: 1e6 nodes, ~3.5e6 edges), and compared with the GPU solve of the same instance."""
    import numpy as np
    import oracle
    o = oracle.Oracle("f32")
    t0 = time.perf_counter()
    r = o.solve(g["n_nodes"], g["i"], g["j"], g["c"], **solver_kwargs(args))
    dt = time.perf_counter() - t0
    labels = gpu_result["labels"].cpu().numpy()
    return {"value": g["i"].size / dt, "unit": "edges/s", "cores": 1, "kind": "oracle",
            "sample": f"{name} ({g['name']}: {g['n_nodes']} nodes, {g['i'].size} edges), full solve, {dt:.1f} s, "
                      f"single-threaded C oracle, host has {os.cpu_count()} cores",
            "seconds": dt, "rounds": r["rounds"], "primal": r["primal"], "lower_bound": r["lower_bound"],
            "parity": {"labels_identical": bool(np.array_equal(labels, r["labels"])),
                       "primal_rel": abs(gpu_result["primal"] - r["primal"]) / abs(r["primal"]) if r["primal"] else 0.0,
                       "lb_rel": abs(gpu_result["lower_bound"] - r["lower_bound"]) / abs(r["lower_bound"]) if r["lower_bound"] else 0.0,
                       "rounds_equal": gpu_result["rounds"] == r["rounds"]}}


def stored_oracle(name, gpu_result):
    """What the oracle's stored full-size result (tests/golden/<cfg>_oracle.json, written by the oracle alone) says
    about this GPU solve: its seconds, and whether labels / costs agree."""
    import hashlib
    import numpy as np
    path = os.path.join(ROOT, "tests", "golden", f"{name}_oracle.json")
    if not os.path.exists(path):
        return None
    want = json.load(open(path))
    labels = np.ascontiguousarray(gpu_result["labels"].cpu().numpy().astype("<i4"))
    return {"oracle_seconds_stored": want["oracle_seconds"], "oracle_edges_per_s_stored": want["n_edges"] / want["oracle_seconds"],
            "labels_identical": hashlib.sha256(labels.tobytes()).hexdigest() == want["labels_sha256"],
            "primal_rel": abs(gpu_result["primal"] - want["primal"]) / abs(want["primal"]),
            "lb_rel": abs(gpu_result["lower_bound"] - want["lower_bound"]) / abs(want["lower_bound"]),
            "rounds_equal": gpu_result["rounds"] == want["rounds"]}


def time_solves(rama, n, i, j, c, params, steps, warmup):
    import torch
    res = None
    for _ in range(warmup):
        res = rama.solve(n, i, j, c, params)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        res = rama.solve(n, i, j, c, params)
    torch.cuda.synchronize()
    return 1e3 * (time.perf_counter() - t0) / steps, res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg5")
    ap.add_argument("--cpu-config", default="cfg3",
                    help="named configuration the CPU oracle is timed on and compared with the GPU solve ('none' = skip)")
    ap.add_argument("--cpu-side", type=int, default=None, help="0 = skip the oracle (same as --cpu-config none)")
    ap.add_argument("--other-workloads", default="cfg1,cfg2,cfg3,cfg4",
                    help="named configurations solved besides the timed workload and listed under `workloads` ('' = none)")
    ap.add_argument("--no-profile", action="store_true", help="skip the per-kernel event timers")
    ap.add_argument("--max-rounds", type=int, default=0, help="stop the solver after this many rounds (0 = run to the end)")
    ap.add_argument("--cycle-len", type=int, nargs=2, default=[5, 3], metavar=("FIRST", "LATER"),
                    help="longest conflicted cycle separated in the first / later rounds (default: solver PD, 5 3)")
    ap.add_argument("--shortest-only", action="store_true",
                    help="per repulsive edge separate only its shortest conflicted cycles")
    ap.add_argument("--dual-rounds", type=int, default=1,
                    help="separation + message-passing blocks per round on the same graph (default 1: the paper's loop)")
    ap.add_argument("--cycle-search", type=int, default=0, choices=[0, 1, 2, 3],
                    help="cycles of length 4-5: 0 = default choice, 1 = plain per-thread walk, 2 = cooperative search, 3 = walk whose last level closes from the far endpoint")
    ap.add_argument("--kernels", type=int, default=16, help="how many kernels the per-kernel table lists")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run a plain 1 GiB device copy three times (reference reading for rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2109_01838_amd import Rama, default_params

    g = make_workload(args.workload)
    n, m = g["n_nodes"], int(g["i"].size)
    dev = torch.device("cuda:0")
    i, j, c = (torch.as_tensor(g[k]).to(dev) for k in ("i", "j", "c"))
    rama = Rama("cuda:0")
    rama.set_cycle_search(args.cycle_search)
    plain = args.cycle_len == [5, 3] and not args.shortest_only and args.dual_rounds == 1
    solver_name = ("PD" if plain else "PD variant") + \
        f" (cycles<={args.cycle_len[0]} then <={args.cycle_len[1]}" + (", shortest only" if args.shortest_only else "") + \
        (f", {args.dual_rounds} dual rounds per round" if args.dual_rounds != 1 else "") + ", k=10 then 5)"
    params = default_params(max_rounds=args.max_rounds, max_cycle_len_first=args.cycle_len[0],
                            max_cycle_len_later=args.cycle_len[1], shortest_cycles_only=int(args.shortest_only), dual_rounds=args.dual_rounds)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # Warm-up.  One extra untimed step runs with every kernel timed: it yields the per-kernel table
    # and names the dominant kernel.  During the timed steps only that kernel carries event timers
    # (two events per launch of one kernel: ~1 % overhead instead of ~15 % for all kernels); the records
    # of the next four kernels come from the all-kernel-timed step.
    res = None
    for _ in range(args.warmup):
        res = rama.solve(n, i, j, c, params)
    kernels, dominant = None, None
    if not args.no_profile:
        rama.profile_enable(True)
        rama.solve(n, i, j, c, params)
        kernels = sorted(rama.profile_get(), key=lambda k: -k["ms"])
        rama.profile_enable(False)
        tot = sum(k["ms"] for k in kernels)
        for k in kernels:
            k["GBps"] = (k["bytes"] / 1e9) / (k["ms"] / 1e3) if k["ms"] > 0 else 0.0
            k["share"] = k["ms"] / tot if tot > 0 else 0.0
        dominant = kernels[0]["name"]
        rama.profile_enable(True, only=dominant)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        res = rama.solve(n, i, j, c, params)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = 1e3 * dt / args.steps
    round_records = rama.round_stats()      # of the last timed solve (later solves on this ctx overwrite them)

    roofline, roofline_top, solve_traffic = None, None, None
    if dominant is not None:
        timed = {k["name"]: k for k in rama.profile_get()}
        rama.profile_enable(False)
        # measured HBM bytes per launch from the committed rocprofv3 --pmc summary (FETCH_SIZE / WRITE_SIZE
        # runs of this same workload, scaled by the copy-kernel calibration)
        tkern = {}
        tpath = os.path.join(ROOT, "profiles", "cfg5_solve_hbm_traffic.json")
        if args.workload == "cfg5" and os.path.exists(tpath):
            tkern = json.load(open(tpath))["kernels"]
            total = sum(t["launches"] * (t["read_bytes_per_launch"] + t["written_bytes_per_launch"]) for t in tkern.values())
            n_solves = json.load(open(tpath)).get("solves", 1)
            solve_traffic = {"bytes_per_solve": total / n_solves, "GBps_over_the_solve": total / n_solves / 1e9 / (ms / 1e3),
                             "input_bytes": 12 * m, "note": "all kernels, measured by rocprofv3 --pmc (profiles/), over this run's time per solve"}

        def record(d, steps, share):
            gbps = (d["bytes"] / 1e9) / (d["ms"] / 1e3) if d["ms"] > 0 else 0.0
            t = tkern.get(d["name"])
            return {"bound": "hbm", "kernel": d["name"], "achieved": gbps, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": gbps / HBM_PEAK_GBS,
                    "traffic": (t["read_bytes_per_launch"] + t["written_bytes_per_launch"]) if t else None,
                    "launches_per_step": d["launches"] / steps, "avg_launch_ms": d["ms"] / max(d["launches"], 1),
                    "algorithmic_bytes_per_launch": d["bytes"] / max(d["launches"], 1),
                    "share_of_kernel_time": share}

        roofline = record(timed[dominant], args.steps, kernels[0]["share"])
        roofline["note"] = ("achieved = summed algorithmic bytes / summed HIP-event time of all launches of this "
                            "kernel inside the timed steps")
        roofline_top = [roofline] + [dict(record(k, 1, k["share"]), note="from the one step with every kernel timed")
                                     for k in kernels[1:5]]

    # the other named configurations: a few untimed-by-the-headline solves each (they take < 1 s of GPU time together)
    workloads = []
    others = [w for w in args.other_workloads.split(",") if w and w != args.workload]
    cpu_name = None if (args.cpu_config == "none" or args.cpu_side == 0) else args.cpu_config
    cpu = None
    for w in others + ([cpu_name] if cpu_name and cpu_name not in others and cpu_name != args.workload else []):
        gw = make_workload(w)
        iw, jw, cw = (torch.as_tensor(gw[k]).to(dev) for k in ("i", "j", "c"))
        msw, rw = time_solves(rama, gw["n_nodes"], iw, jw, cw, params, 5, 2)
        entry = {"workload": gw["name"], "config": w, "n_nodes": gw["n_nodes"], "n_edges": int(gw["i"].size),
                 "ms_per_solve": msw, "edges_per_s": gw["i"].size / (msw / 1e3), "primal": rw["primal"],
                 "lower_bound": rw["lower_bound"], "rounds": rw["rounds"], "n_clusters": rw["n_clusters"],
                 "gap": (rw["primal"] - rw["lower_bound"]) / abs(rw["lower_bound"]) if rw["lower_bound"] else 0.0}
        if plain:
            st = stored_oracle(w, rw)
            if st:
                entry["oracle_stored"] = st
        if w == cpu_name:
            cpu = cpu_baseline(w, args, rw, gw)
            entry["oracle"] = {k: cpu[k] for k in ("seconds", "value", "parity")}
        workloads.append(entry)
        del iw, jw, cw, rw
    if cpu_name == args.workload:
        cpu = cpu_baseline(cpu_name, args, res, g)

    labels = res["labels"]
    gap = (res["primal"] - res["lower_bound"]) / abs(res["lower_bound"]) if res["lower_bound"] else 0.0
    out = {
        "metric": "edges_per_second_full_solve", "value": m / (ms / 1e3), "unit": "edges/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": g["name"], "n_nodes": n, "n_edges": m, "solver": solver_name},
        "solve_seconds": ms / 1e3, "primal": res["primal"], "lower_bound": res["lower_bound"], "gap": gap,
        "rounds": res["rounds"], "n_clusters": res["n_clusters"], "n_cycles_first": res["n_cycles_first"],
        "n_triangles_first": res["n_triangles_first"], "stage_ms_last_step": res["ms"],
        "workspace_GiB": rama.workspace_bytes() / 2**30,
        "rounds_detail": [{"nodes": r["n_nodes"], "edges": r["n_edges"], "repulsive": r["n_repulsive"],
                           "cycles": r["n_cycles"][:3], "triangles": r["n_triangles"], "contracted": r["n_contracted"],
                           "forest": r["used_forest"], "workspace_peak_MiB": round(r["workspace_peak"] / 2**20, 1),
                           "ms": [round(r["ms"][k], 3) for k in ("cycles", "dual", "contract")]}
                          for r in round_records],
        "roofline": roofline,
        "roofline_top5": roofline_top,
        "solve_traffic": solve_traffic,
    }
    if kernels:
        out["kernels"] = [{"name": k["name"], "launches": k["launches"], "ms_per_step": k["ms"],
                           "GBps": round(k["GBps"], 1), "frac_hbm": round(k["GBps"] / HBM_PEAK_GBS, 4),
                           "share": round(k["share"], 4)} for k in kernels[:args.kernels]]
    del labels
    if plain:
        st = stored_oracle(args.workload, res)
        if st:
            out["parity_vs_stored_oracle"] = st
    out["workloads"] = workloads
    out["cpu_baseline"] = cpu
    print(json.dumps(out))


if __name__ == "__main__":
    main()
