"""End-to-end parity on the named configurations (cfg2: 512x512 grid
with long-range edges, 1.56e6 edges; cfg3: 1e6-point 6-NN graph, ~3.5e6 edges) at their full
sizes, and on a 110^3 cube of cfg5's recipe (3.96e6 edges), the smallest of these on which the
long sorts of both key widths take the split path (top-bit passes + in-LDS sort) by themselves: primal within 0.5 %, lower bound within 1e-4 relative, and -- because both sides order
their arithmetic identically -- in practice identical labels.  cfg4 (256x256x128 grid, 2.5e7 edges)
takes the oracle minutes, so its result is stored (tests/golden/cfg4_oracle.json, written by the oracle
alone) and compared here; cfg5 is compared the same way in test_gpu_fullsize.py."""
import numpy as np
import pytest

import golden_check
from paper_2109_01838_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rama():
    from paper_2109_01838_amd import Rama
    r = Rama("cuda:0")
    yield r
    r.close()


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", ["cfg2", "cfg3", "cfg5crop110"])
def test_named_config_end_to_end(rama, oracle32, name):
    g = inputs.cfg5_crop(110, seed=5) if name == "cfg5crop110" else inputs.make(name)
    n = g["n_nodes"]
    rama.profile_enable(True)
    got = rama.solve(n, g["i"], g["j"], g["c"])
    kernels = {k["name"] for k in rama.profile_get()}
    rama.profile_enable(False)
    if name == "cfg5crop110":
        assert {"k_rs_local<u64,u32>", "k_rs_local<u32>", "k_seg_bounds"} <= kernels
    print(name, "gpu:", {k: v for k, v in got.items() if k not in ("labels",)}, flush=True)
    want = oracle32.solve(n, g["i"], g["j"], g["c"])
    labels = got["labels"].cpu().numpy()
    assert abs(got["lower_bound"] - want["lower_bound"]) <= 1e-4 * abs(want["lower_bound"])
    assert abs(got["primal"] - want["primal"]) <= 5e-3 * abs(want["primal"])
    assert got["n_cycles_first"] == want["n_cycles_first"]
    assert got["n_edges_aug_first"] == want["n_edges_aug_first"]
    assert abs(oracle32.multicut_cost(g["i"], g["j"], g["c"], labels) - got["primal"]) <= 1e-6 * abs(got["primal"])
    assert got["lower_bound"] <= got["primal"]
    print(name, "labels identical:", bool(np.array_equal(labels, want["labels"])), "rounds", got["rounds"], want["rounds"],
          "primal", got["primal"], want["primal"])


@pytest.mark.timeout(900)
def test_cfg4_end_to_end_against_stored_oracle_result(rama, oracle32):
    g = inputs.cfg4()
    got = rama.solve(g["n_nodes"], g["i"], g["j"], g["c"])
    golden_check.check_against_golden("cfg4", g, got)
    labels = got["labels"].cpu().numpy()
    assert abs(oracle32.multicut_cost(g["i"], g["j"], g["c"], labels) - got["primal"]) <= 1e-6 * abs(got["primal"])
