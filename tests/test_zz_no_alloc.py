"""rama_solve_static -- the entry point for callers that cannot allocate device memory -- against
rama_solve through the C ABI: identical labels, primal cost, lower bound and counts, on two calls in a
row (the second on a smaller input, so whatever the first call left in the shared static array is
stale data the second must not see), plus the size limits and a ctx that never ran anything else."""
import ctypes as C

import numpy as np
import pytest

from paper_2109_01838_amd import inputs

pytestmark = pytest.mark.gpu


def np_(t):
    return t.detach().cpu().numpy()


def same_result(a, b):
    assert np.array_equal(np_(a["labels"]), np_(b["labels"]))
    assert a["primal"] == b["primal"] and a["lower_bound"] == b["lower_bound"]
    for k in ("rounds", "n_clusters", "n_cycles_first", "n_triangles_first", "n_edges_aug_first", "n_edges_final"):
        assert a[k] == b[k], k


def test_static_solve_matches_rama_solve_on_two_calls_in_a_row():
    import torch
    from paper_2109_01838_amd import Rama, RamaError, binding
    big = inputs.cfg2(h=128, w=128, n_seeds=30)          # 16,384 nodes, ~9.6e4 edges: several tiles, 4-cycles, chords
    small = inputs.cfg3(n_points=6000, n_seeds=40)       # irregular, 3-, 4- and 5-cycles
    assert big["i"].size <= binding.STATIC_MAX_EDGES and small["i"].size < big["i"].size
    fresh = Rama("cuda:0")                               # a ctx whose first call ever is the static one
    dev = {}
    for name, g in (("big", big), ("small", small)):
        dev[name] = tuple(torch.as_tensor(g[k]).cuda() for k in ("i", "j", "c"))
    out = {name: torch.empty(g["n_nodes"], dtype=torch.int32, device="cuda:0") for name, g in (("big", big), ("small", small))}
    torch.cuda.synchronize()
    before = fresh.workspace_bytes()
    got_big = fresh.solve(big["n_nodes"], *dev["big"], static=True, labels=out["big"])
    got_small = fresh.solve(small["n_nodes"], *dev["small"], static=True, labels=out["small"])
    assert fresh.workspace_bytes() == before             # the ctx's own cache was never touched
    ref = Rama("cuda:0")
    same_result(got_big, ref.solve(big["n_nodes"], *dev["big"]))
    same_result(got_small, ref.solve(small["n_nodes"], *dev["small"]))
    # and once more the other way round, on the ctx that has used its ordinary workspace in between
    same_result(ref.solve(small["n_nodes"], *dev["small"], static=True), got_small)
    same_result(ref.solve(big["n_nodes"], *dev["big"], static=True), got_big)
    # sizes beyond the stated maximum are refused before anything runs
    n_big = binding.STATIC_MAX_NODES + 1
    z = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    with pytest.raises(RamaError) as ei:
        fresh.solve(n_big, z, z, torch.ones(1, device="cuda:0"), static=True)
    assert ei.value.status == binding.RAMA_ERR_CAPACITY
    m_big = binding.STATIC_MAX_EDGES + 1
    zi = torch.zeros(m_big, dtype=torch.int32, device="cuda:0")
    with pytest.raises(RamaError) as ei:
        fresh.solve(4, zi, zi, torch.ones(m_big, device="cuda:0"), static=True)
    assert ei.value.status == binding.RAMA_ERR_CAPACITY and "at most" in str(ei.value)
    same_result(fresh.solve(small["n_nodes"], *dev["small"], static=True), got_small)
    fresh.close()
    ref.close()
