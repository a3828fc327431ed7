"""Host-side logic that needs no GPU: the seeded input generators, the mapping between rocprofv3's
kernel names and the library's timer names, bench.py's refusal of more than one GPU."""
import os
import subprocess
import sys

import numpy as np

from paper_2109_01838_amd import inputs, profile_summary

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def canonical(g):
    """i<j, in range, no edge twice (the order is the generator's own; the library sorts)."""
    i, j = g["i"], g["j"]
    key = i.astype(np.int64) * g["n_nodes"] + j
    return bool(np.all(i < j) and np.unique(key).size == key.size and i.min() >= 0 and j.max() < g["n_nodes"])


def test_generators_are_seeded_and_well_formed():
    for make in (inputs.cfg1, lambda: inputs.cfg2(h=24, w=20, n_seeds=5), lambda: inputs.cfg3(n_points=3000, n_seeds=20),
                 lambda: inputs.cfg5_crop(9), inputs.hub_graph):
        a, b = make(), make()
        assert canonical(a) and a["c"].dtype == np.float32 and np.all(np.isfinite(a["c"]))
        assert np.array_equal(a["i"], b["i"]) and np.array_equal(a["j"], b["j"]) and np.array_equal(a["c"], b["c"])
        assert (a["c"] > 0).any() and (a["c"] < 0).any()


def test_grid_recipes_have_the_stated_shape():
    g = inputs.cfg5_crop(7)
    assert g["n_nodes"] == 343 and g["i"].size == 3 * 7 * 7 * 6          # 6-connected: 3 directions x 7*7*6 edges
    d = g["j"] - g["i"]
    assert sorted(np.unique(d).tolist()) == [1, 7, 49]
    g = inputs.cfg2(h=30, w=30, n_seeds=4)
    assert sorted(np.unique(g["j"] - g["i"]).tolist()) == [1, 3, 9, 30, 90, 270]   # offsets 1, 3, 9 in x and y
    g = inputs.cfg1()
    assert g["n_nodes"] == 1024 and g["i"].size == 2 * 32 * 31
    # attractive inside a planted cluster, repulsive across, up to the stated noise
    same = g["truth"][g["i"]] == g["truth"][g["j"]]
    assert (g["c"][same] > 0).mean() > 0.8 and (g["c"][~same] < 0).mean() > 0.8


def test_hub_graph_is_skewed():
    g = inputs.hub_graph()
    deg = np.bincount(np.concatenate([g["i"], g["j"]]), minlength=g["n_nodes"])
    assert deg.max() > 600 and np.median(deg) < 10 and (deg > 128).sum() == 4


def test_profiler_names_map_onto_timer_names():
    f = profile_summary.event_name
    assert f("void rama::k_rs_scatter<unsigned long, unsigned int, true, false>(unsigned long const*, int)") == "k_rs_scatter<u64,u32>"
    assert f("void rama::k_rs_scatter<unsigned long, unsigned int, true, true>(unsigned long const*)") == "k_rs_scatter<u64,u32>"
    assert f("void rama::k_rs_scatter<unsigned int, unsigned int, false, false>(unsigned int const*)") == "k_rs_scatter<u32>"
    assert f("void rama::k_rs_hist<unsigned long>(unsigned long const*, unsigned int*)") == "k_rs_hist<u64>"
    assert f("void rama::k_scan_apply<unsigned int, rama::(anonymous namespace)::HeadFlag>(x)") == "k_scan_apply<HeadFlag>"
    assert f("void rama::k_scan_reduce<unsigned long, rama::PtrInput<unsigned int> >(x)") == "k_scan_reduce<PtrInput>"
    assert f("void rama::(anonymous namespace)::k_count_cycles<5>(unsigned long, int const*)") == "k_count_cycles<5>"
    assert f("void rama::(anonymous namespace)::k_count_cycles<5, true>(unsigned long, int const*)") == "k_count_cycles<5>"
    assert f("void rama::(anonymous namespace)::k_fill_cycles<7, false>(unsigned long)") == "k_fill_cycles<7>"
    assert f("void rama::(anonymous namespace)::k_count_cycles_listed<5, true>(unsigned int const*)") == "k_count_cycles_listed"
    assert f("void rama::(anonymous namespace)::k_count_cycles_coop(unsigned long)") == "k_count_cycles_coop"
    assert f("void rama::(anonymous namespace)::k_edge_update<false>(unsigned long)") == "k_edge_update<false>"
    assert f("void rama::(anonymous namespace)::k_triangle_update<true>(unsigned long)") == "k_triangle_update"
    assert f("void rama::k_row_bounds_fill<int, int>(int const*, unsigned long, long, int*)") == "k_row_bounds_fill"
    assert (f("void rama::k_scan_emit<unsigned int, rama::(anonymous namespace)::ChordIsNew, rama::(anonymous namespace)::ChordKeysEmit>(x)")
            == "k_scan_emit<ChordKeys>")
    assert f("void rama::k_rs_local<unsigned long, unsigned int, true, unsigned int>(unsigned long const*)") == "k_rs_local<u64,u32>"
    assert f("void rama::k_rs_local<unsigned int, unsigned int, false, unsigned int>(unsigned int const*)") == "k_rs_local<u32>"
    assert f("void rama::k_rs_local<unsigned long, unsigned int, true, unsigned long>(unsigned long const*)") == "k_rs_local<u64,u32,wide>"
    assert f("rama::(anonymous namespace)::k_triangle_update(unsigned long, int const*)") == "k_triangle_update"
    A = "rama::(anonymous namespace)::"
    assert f(f"void rama::k_scan_emit<unsigned long, {A}SignFlags, {A}SplitSignEmit>(x)") == "k_scan_emit<SplitSign>"
    assert f(f"void rama::k_scan_emit<unsigned int, {A}HeadFlagT<unsigned int>, {A}TrianglesEmit<unsigned int> >(x)") == "k_scan_emit<Triangles>"
    assert f(f"void rama::k_scan_emit<unsigned int, {A}HeadFlagT<unsigned long>, {A}TrianglesEmit<unsigned long> >(x)") == "k_scan_emit<Triangles64>"
    assert f(f"void rama::k_scan_reduce<unsigned int, {A}HeadFlagT<unsigned long> >(x)") == "k_scan_reduce<HeadFlag64>"
    assert f(f"void rama::k_scan_reduce<unsigned int, {A}HasCycles<5> >(x)") == "k_scan_reduce<HasCycles>"
    assert f(f"void rama::k_scan_reduce<unsigned int, {A}HasCycles<7> >(x)") == "k_scan_reduce<HasCycles7>"
    assert f("rama::k_reduce_runs(unsigned long, unsigned long const*)") == "k_reduce_runs"


def test_traffic_summary_scales_and_averages(tmp_path):
    import json
    head = '"Kernel_Name","Counter_Name","Counter_Value"\n'
    (tmp_path / "f.csv").write_text(head + '"void rama::k_x(int)","FETCH_SIZE",100\n"void rama::k_x(int)","FETCH_SIZE",300\n')
    (tmp_path / "w.csv").write_text(head + '"void rama::k_x(int)","WRITE_SIZE",50\n"void rama::k_x(int)","WRITE_SIZE",150\n')
    out = tmp_path / "t.json"
    profile_summary.traffic_json(str(tmp_path / "f.csv"), str(tmp_path / "w.csv"), 2.0, 1.0, str(out))
    k = json.load(open(out))["kernels"]["k_x"]
    assert k == {"launches": 2, "read_bytes_per_launch": 1024.0 * 2.0 * 200, "written_bytes_per_launch": 1024.0 * 100}


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stdout + r.stderr)


def test_committed_traffic_summary_names_the_dominant_kernel():
    import json
    t = json.load(open(os.path.join(ROOT, "profiles", "cfg5_solve_hbm_traffic.json")))
    k = t["kernels"]["k_rs_scatter<u64,u32>"]
    assert k["launches"] > 0 and k["read_bytes_per_launch"] > 0 and k["written_bytes_per_launch"] > 0
    assert t["fetch_scale"] > 0 and t["write_scale"] > 0
