"""GPU parity: every stage of the HIP library against the CPU oracle on the same seeded inputs,
called through the C ABI (paper_2109_01838_amd.binding -> librama_hip.so).

Stage-wise tests hand each GPU stage the oracle's input for that stage.  Integer results
(cycle lists, edge lists, contraction mappings, labels) must match bit-exactly; fp32 reduced
costs and lower bounds within 1e-4 relative; end to end the primal cost within 0.5 % and the
lower bound within 1e-4 relative.
"""
import numpy as np
import pytest

from paper_2109_01838_amd import inputs

pytestmark = pytest.mark.gpu

REL = 1e-4


@pytest.fixture(scope="module")
def rama():
    from paper_2109_01838_amd import Rama
    r = Rama("cuda:0")
    yield r
    r.close()


def np_(t):
    return t.detach().cpu().numpy()


def signed(g, seed, pos=0.7):
    rng = np.random.default_rng(seed)
    c = np.where(rng.random(g["c"].size) < pos, np.abs(g["c"]), -np.abs(g["c"])).astype(np.float32)
    return dict(g, c=c)


def cases():
    """name -> instance; sizes span several sort tiles (5120 or 6144 keys), on both sides of the 32-tile switch between the two offset schemes, and several 2048-item scan tiles, with ragged tails."""
    out = {}
    out["cfg1"] = inputs.cfg1()
    out["grid2d_longrange_96"] = inputs.cfg2(h=96, w=96, n_seeds=20)
    out["knn_20000"] = inputs.cfg3(n_points=20000, n_seeds=100)
    out["grid3d_24"] = inputs.cfg5_crop(24)
    out["random_dense"] = signed(inputs.random_graph(300, 6000, 11), 11, 0.6)
    out["random_sparse"] = signed(inputs.random_graph(5000, 14000, 12), 12, 0.8)
    out["messy"] = inputs.random_graph(200, 3000, 13, allow_messy=True)
    return out


CASES = cases()


def rel_close(a, b, rel=REL):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    scale = max(1.0, float(np.abs(b).max()) if b.size else 1.0)
    return np.all(np.abs(a - b) <= rel * scale)


# --------------------------------------------------------------------------------------------
# a1 cycles
# --------------------------------------------------------------------------------------------
@pytest.fixture
def search_mode(rama, request):
    """The ways of finding the cycles of length 4 and more: 1 = the per-thread walk that fetches a row per path
    at its last level, 3 = the walk whose last level closes from the far endpoint's side, 2 = the cooperative
    search for lengths 4 and 5 (rows beyond its staged sizes fall back to walk 3 edge by edge)."""
    rama.set_cycle_search(request.param)
    yield request.param
    rama.set_cycle_search(0)


BOTH_SEARCHES = pytest.mark.parametrize("search_mode", [1, 2, 3], indirect=True, ids=["walk", "cooperative", "walk-meet"])


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("lmax", [3, 4, 5])
@BOTH_SEARCHES
def test_cycles_bit_exact(rama, oracle32, name, lmax, search_mode):
    g = CASES[name]
    if name == "random_dense" and lmax == 5:
        g = dict(g, i=g["i"][:2500], j=g["j"][:2500], c=g["c"][:2500])
    want = oracle32.find_conflicted_cycles(g["n_nodes"], g["i"], g["j"], g["c"], lmax)
    got = rama.find_conflicted_cycles(g["n_nodes"], g["i"], g["j"], g["c"], lmax)
    assert len(got) == len(want) == lmax - 2
    for L in range(lmax - 2):
        assert np.array_equal(np_(got[L]), want[L]), (name, lmax, L + 3, got[L].shape, want[L].shape)


# cycles of length 6 and 7 (named as future work in Sec. 5) and the shortest-only separation; the
# cases are the ones whose plain enumeration the oracle finishes in seconds
LONG_CASES = [("cfg1", 7), ("grid3d_24", 7), ("random_sparse", 7), ("knn_20000", 7), ("knn_20000", 6),
              ("grid2d_longrange_96", 6), ("messy", 6)]


@pytest.mark.parametrize("name,lmax", LONG_CASES)
@BOTH_SEARCHES
def test_longer_cycles_bit_exact(rama, oracle32, name, lmax, search_mode):
    g = CASES[name]
    want = oracle32.find_conflicted_cycles(g["n_nodes"], g["i"], g["j"], g["c"], lmax)
    got = rama.find_conflicted_cycles(g["n_nodes"], g["i"], g["j"], g["c"], lmax)
    assert len(got) == lmax - 2
    for L in range(lmax - 2):
        assert np.array_equal(np_(got[L]), want[L]), (name, lmax, L + 3, got[L].shape, want[L].shape)
    print(name, lmax, [x.shape[0] for x in want])


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("lmax", [3, 4, 5, 7])
@BOTH_SEARCHES
def test_shortest_only_cycles_bit_exact(rama, oracle32, name, lmax, search_mode):
    g = CASES[name]
    if name in ("random_dense", "messy") and lmax == 7:
        g = dict(g, i=g["i"][:1500], j=g["j"][:1500], c=g["c"][:1500])
    want = oracle32.find_conflicted_cycles(g["n_nodes"], g["i"], g["j"], g["c"], lmax, shortest_only=True)
    got = rama.find_conflicted_cycles(g["n_nodes"], g["i"], g["j"], g["c"], lmax, shortest_only=True)
    for L in range(lmax - 2):
        assert np.array_equal(np_(got[L]), want[L]), (name, lmax, L + 3, got[L].shape, want[L].shape)
    # every repulsive edge appears with one length only
    seen = {}
    for L, x in enumerate(np_(q) for q in got):
        for a, b in set(zip(x[:, 0].tolist(), x[:, -1].tolist())):
            assert seen.setdefault((a, b), L) == L


# skewed degrees: repulsive edges at hubs (attractive rows of ~600 entries) take the wave-per-edge path
@pytest.fixture(scope="module")
def hubs():
    return inputs.hub_graph()


@pytest.mark.parametrize("lmax,shortest", [(3, False), (4, False), (5, False), (4, True), (5, True), (7, True)])
@BOTH_SEARCHES
def test_heavy_rows_cycles_bit_exact(rama, oracle32, hubs, lmax, shortest, search_mode):
    g = hubs
    deg = np.bincount(np.concatenate([g["i"][g["c"] > 0], g["j"][g["c"] > 0]]), minlength=g["n_nodes"])
    assert deg.max() > 500 and np.median(deg) < 10
    want = oracle32.find_conflicted_cycles(g["n_nodes"], g["i"], g["j"], g["c"], lmax, shortest_only=shortest)
    got = rama.find_conflicted_cycles(g["n_nodes"], g["i"], g["j"], g["c"], lmax, shortest_only=shortest)
    for L in range(lmax - 2):
        assert np.array_equal(np_(got[L]), want[L]), (lmax, shortest, L + 3, got[L].shape, want[L].shape)
    # the hubs' own repulsive edges are among the results
    heavy = set(np.where(deg > 128)[0].tolist())
    assert any(int(v) in heavy for L in range(lmax - 2) for v in np.unique(want[L][:, 0]))
    print(lmax, shortest, [x.shape[0] for x in want])


def test_heavy_rows_solve(rama, oracle32, hubs):
    g = hubs
    n = g["n_nodes"]
    want = oracle32.solve(n, g["i"], g["j"], g["c"])
    got = rama.solve(n, g["i"], g["j"], g["c"])
    assert got["n_cycles_first"] == want["n_cycles_first"]
    assert abs(got["lower_bound"] - want["lower_bound"]) <= REL * max(1.0, abs(want["lower_bound"]))
    assert abs(got["primal"] - want["primal"]) <= 5e-3 * max(1.0, abs(want["primal"]))
    print("hubs: labels identical:", bool(np.array_equal(np_(got["labels"]), want["labels"])), got["primal"], want["primal"])


def test_cycles_capacity_protocol(rama):
    import ctypes as C
    import torch
    from paper_2109_01838_amd import binding
    g = CASES["cfg1"]
    i, j, c = (torch.as_tensor(g[k], device="cuda") for k in ("i", "j", "c"))
    cnt = (C.c_int64 * 5)()
    args = (rama.ctx, g["n_nodes"], i.numel(), i.data_ptr(), j.data_ptr(), c.data_ptr())
    st = rama.lib.rama_find_conflicted_cycles(*args, 5, 0, None, None, cnt)
    assert st == binding.RAMA_ERR_CAPACITY and cnt[1] > 0 and cnt[0] == 0 and cnt[2] == 0
    buf = torch.full((4 * (cnt[1] - 1) + 1,), -7, dtype=torch.int32, device="cuda")
    cap = (C.c_int64 * 3)(0, cnt[1] - 1, 0)
    ptrs = (C.c_void_p * 3)(None, buf.data_ptr(), None)
    st = rama.lib.rama_find_conflicted_cycles(*args, 5, 0, cap, ptrs, cnt)
    assert st == binding.RAMA_ERR_CAPACITY
    assert bool((buf == -7).all())          # nothing written on capacity failure
    cap[1] = cnt[1]
    buf = torch.full((4 * cnt[1] + 1,), -7, dtype=torch.int32, device="cuda")
    ptrs[1] = buf.data_ptr()
    st = rama.lib.rama_find_conflicted_cycles(*args, 5, 0, cap, ptrs, cnt)
    assert st == binding.RAMA_OK and int(buf[-1]) == -7 and bool((buf[:-1] >= 0).all())
    for bad_len in (2, binding.MAX_CYCLE_LEN + 1):
        st = rama.lib.rama_find_conflicted_cycles(*args, bad_len, 0, None, None, cnt)
        assert st == binding.RAMA_ERR_INVALID_ARG
    cap[1] = -1
    assert rama.lib.rama_find_conflicted_cycles(*args, 5, 0, cap, ptrs, cnt) == binding.RAMA_ERR_INVALID_ARG
    cap[1] = 5
    ptrs[1] = None
    assert rama.lib.rama_find_conflicted_cycles(*args, 5, 0, cap, ptrs, cnt) == binding.RAMA_ERR_INVALID_ARG


# --------------------------------------------------------------------------------------------
# a2 + a3 message passing
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("k", [0, 1, 10])
def test_message_passing_parity(rama, oracle32, name, k):
    g = CASES[name]
    n = g["n_nodes"]
    lmax = 4 if name == "random_dense" else 5
    cyc = oracle32.find_conflicted_cycles(n, g["i"], g["j"], g["c"], lmax)
    want = oracle32.message_passing(n, g["i"], g["j"], g["c"], cyc, k, trace=True)
    got = rama.message_passing(n, g["i"], g["j"], g["c"], cyc, k, trace=True)
    assert np.array_equal(np_(got["i"]), want["i"]) and np.array_equal(np_(got["j"]), want["j"])
    assert rel_close(np_(got["c"]), want["c"])
    assert abs(got["lower_bound"] - want["lower_bound"]) <= REL * max(1.0, abs(want["lower_bound"]))
    assert rel_close(got["lb_trace"], want["lb_trace"])
    tr = np.asarray(got["lb_trace"])
    assert np.all(np.diff(tr) >= -1e-5 * (1.0 + np.abs(tr[:-1])))       # monotone (Appendix, LB lemma)
    # the arithmetic is ordered identically on both sides, so in practice the match is exact
    print(name, k, "max |dc| =", float(np.abs(np_(got["c"]) - want["c"]).max()) if want["c"].size else 0.0,
          "bit-exact:", bool(np.array_equal(np_(got["c"]), want["c"])))


@pytest.mark.parametrize("name,lmax", LONG_CASES)
@pytest.mark.parametrize("shortest", [False, True])
def test_message_passing_parity_longer_cycles(rama, oracle32, name, lmax, shortest):
    g = CASES[name]
    n = g["n_nodes"]
    cyc = oracle32.find_conflicted_cycles(n, g["i"], g["j"], g["c"], lmax, shortest_only=shortest)
    want = oracle32.message_passing(n, g["i"], g["j"], g["c"], cyc, 5, trace=True)
    got = rama.message_passing(n, g["i"], g["j"], g["c"], cyc, 5, trace=True)
    assert np.array_equal(np_(got["i"]), want["i"]) and np.array_equal(np_(got["j"]), want["j"])
    assert rel_close(np_(got["c"]), want["c"])
    assert rel_close(got["lb_trace"], want["lb_trace"])
    print(name, lmax, shortest, "edges", want["i"].size, "bit-exact:", bool(np.array_equal(np_(got["c"]), want["c"])))


# dual rounds on one graph: the triangle set and its costs persist from round to round
DUAL_CASES = [(name, L, R) for name in CASES for (L, R) in ((3, 3), (4, 2), (5, 2))
              if not (name in ("random_dense", "messy") and L > 3) and not (name == "grid2d_longrange_96" and L == 5)]


@pytest.mark.parametrize("name,lmax,rounds", DUAL_CASES)
def test_dual_rounds_parity(rama, oracle32, name, lmax, rounds):
    from paper_2109_01838_amd import default_params
    g = CASES[name]
    n = g["n_nodes"]
    want = oracle32.dual_rounds(n, g["i"], g["j"], g["c"], lmax, 5, rounds)
    got = rama.dual_rounds(n, g["i"], g["j"], g["c"],
                           default_params(max_cycle_len_first=lmax, mp_iters_first=5, dual_rounds=rounds))
    assert np.array_equal(np_(got["i"]), want["i"]) and np.array_equal(np_(got["j"]), want["j"])
    assert rel_close(np_(got["c"]), want["c"])
    assert rel_close(got["lb_trace"], want["lb_trace"])
    assert abs(got["lower_bound"] - want["lower_bound"]) <= REL * max(1.0, abs(want["lower_bound"]))
    assert got["n_triangles"] == want["n_triangles"]
    tr = np.asarray(got["lb_trace"])
    assert np.all(np.diff(tr) >= -1e-5 * (1.0 + np.abs(tr[:-1])))
    print(name, lmax, rounds, "LB", list(tr), "triangles", got["n_triangles"], "bit-exact:",
          bool(np.array_equal(np_(got["c"]), want["c"])))


def test_dual_rounds_one_round_is_separation_plus_message_passing(rama):
    from paper_2109_01838_amd import default_params
    g = CASES["knn_20000"]
    n = g["n_nodes"]
    cyc = rama.find_conflicted_cycles(n, g["i"], g["j"], g["c"], 5)
    mp = rama.message_passing(n, g["i"], g["j"], g["c"], cyc, 10)
    one = rama.dual_rounds(n, g["i"], g["j"], g["c"], default_params(dual_rounds=1))
    assert np.array_equal(np_(one["c"]), np_(mp["c"])) and one["lower_bound"] == mp["lower_bound"]
    zero = rama.dual_rounds(n, g["i"], g["j"], g["c"], default_params(dual_rounds=0))
    assert zero["lb_trace"] == [zero["lower_bound"]] and zero["n_triangles"] == 0
    assert abs(zero["lower_bound"] - float(np.minimum(g["c"], 0).astype(np.float64).sum())) <= 1e-9 * abs(zero["lower_bound"])


def test_message_passing_cycle_order_is_irrelevant(rama, oracle32):
    g = CASES["knn_20000"]
    n = g["n_nodes"]
    cyc = oracle32.find_conflicted_cycles(n, g["i"], g["j"], g["c"], 5)
    rng = np.random.default_rng(0)
    shuffled = [x[rng.permutation(x.shape[0])] for x in cyc]
    a = rama.message_passing(n, g["i"], g["j"], g["c"], cyc, 3)
    b = rama.message_passing(n, g["i"], g["j"], g["c"], shuffled, 3)
    assert np.array_equal(np_(a["c"]), np_(b["c"])) and a["lower_bound"] == b["lower_bound"]


def test_message_passing_rejects_foreign_cycles(rama):
    from paper_2109_01838_amd import RamaError, binding
    g = CASES["cfg1"]
    bad = [np.array([[0, 1, 40]], np.int32), np.zeros((0, 4), np.int32), np.zeros((0, 5), np.int32)]
    with pytest.raises(RamaError) as ei:
        rama.message_passing(g["n_nodes"], g["i"], g["j"], g["c"], bad, 1)
    assert ei.value.status == binding.RAMA_ERR_BAD_GRAPH
    bad[0] = np.array([[0, 1, 5000]], np.int32)
    with pytest.raises(RamaError):
        rama.message_passing(g["n_nodes"], g["i"], g["j"], g["c"], bad, 1)


# --------------------------------------------------------------------------------------------
# a4-a6 contraction
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("repeat", [1, 0])
def test_contract_parity(rama, oracle32, name, repeat):
    g = CASES[name]
    n = g["n_nodes"]
    # the stage input is what the oracle's dual step hands over: reduced costs incl. chords
    cyc = oracle32.find_conflicted_cycles(n, g["i"], g["j"], g["c"], 4)
    mp = oracle32.message_passing(n, g["i"], g["j"], g["c"], cyc, 5)
    want = oracle32.contract(n, mp["i"], mp["j"], mp["c"], repeat=repeat)
    got = rama.contract(n, mp["i"], mp["j"], mp["c"], repeat=repeat)
    assert got["n_nodes"] == want["n_nodes"]
    assert np.array_equal(np_(got["mapping"]), want["mapping"])
    assert np.array_equal(np_(got["i"]), want["i"]) and np.array_equal(np_(got["j"]), want["j"])
    assert rel_close(np_(got["c"]), want["c"])
    assert rel_close(np_(got["diag"]), want["diag"])
    print(name, repeat, "costs bit-exact:", bool(np.array_equal(np_(got["c"]), want["c"])),
          "diag bit-exact:", bool(np.array_equal(np_(got["diag"]), want["diag"])))


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("repeat", [1, 0])
def test_contract_forest_parity(rama, oracle32, name, repeat):
    """forest_ratio=1 forces the spanning forest without conflicts in every primal update."""
    from paper_2109_01838_amd import default_params
    g = CASES[name]
    n = g["n_nodes"]
    cyc = oracle32.find_conflicted_cycles(n, g["i"], g["j"], g["c"], 4)
    mp = oracle32.message_passing(n, g["i"], g["j"], g["c"], cyc, 5)
    want = oracle32.contract(n, mp["i"], mp["j"], mp["c"], repeat=repeat, forest_ratio=1.0)
    got = rama.contract(n, mp["i"], mp["j"], mp["c"], params=default_params(forest_ratio=1.0), repeat=repeat)
    assert got["n_nodes"] == want["n_nodes"]
    assert np.array_equal(np_(got["mapping"]), want["mapping"])
    assert np.array_equal(np_(got["i"]), want["i"]) and np.array_equal(np_(got["j"]), want["j"])
    assert rel_close(np_(got["c"]), want["c"])
    assert rel_close(np_(got["diag"]), want["diag"])
    # no repulsive input edge ends up inside a cluster after ONE forest update
    if repeat == 1:
        mp_ = want["mapping"]
        assert not np.any((mp["c"] < 0) & (mp_[mp["i"]] == mp_[mp["j"]]))


@pytest.mark.parametrize("n", [9, 26, 30, 31, 32, 33, 41, 6000])
def test_forest_deep_tree(rama, oracle32, n):
    # a long attractive path with a few repulsive chords: one tree as deep as the graph has nodes (the
    # small sizes put the deepest level on either side of the rooting loop's check interval)
    i = np.arange(n - 1, dtype=np.int32)
    j = i + 1
    rng = np.random.default_rng(3)
    c = rng.uniform(0.5, 1.5, n - 1).astype(np.float32)
    k = max(1, min(40, n // 8))
    span = max(3, min(200, n // 2))
    ci = rng.integers(0, n - span, k).astype(np.int32)
    cj = (ci + rng.integers(2, span, k)).astype(np.int32)
    ii, jj = np.concatenate([i, ci]), np.concatenate([j, cj])
    cc = np.concatenate([c, -np.ones(k, np.float32)])
    from paper_2109_01838_amd import default_params
    want = oracle32.contract(n, ii, jj, cc, repeat=1, forest_ratio=1.0)
    got = rama.contract(n, ii, jj, cc, params=default_params(forest_ratio=1.0), repeat=1)
    assert np.array_equal(np_(got["mapping"]), want["mapping"]) and got["n_nodes"] == want["n_nodes"]
    assert np.array_equal(np_(got["c"]), want["c"])


def test_contract_fig2_graph(rama, oracle32):
    # the graph of the paper's Fig. 2; with the matching rule S={st} (cost 4 is the best edge at s and t;
    # rs=3 loses at s), so only the mechanics are compared with the oracle here
    i = np.array([0, 0, 1, 1, 2, 3, 2], np.int32)
    j = np.array([1, 2, 3, 4, 3, 4, 4], np.int32)
    c = np.array([1, -2, -3, 1, 3, 4, 1], np.float32)
    want = oracle32.contract(5, i, j, c, repeat=1)
    got = rama.contract(5, i, j, c, repeat=1)
    assert np.array_equal(np_(got["mapping"]), want["mapping"])
    assert np.array_equal(np_(got["c"]), want["c"]) and np.array_equal(np_(got["diag"]), want["diag"])


def test_canonicalisation_of_large_shuffled_input(rama, oracle32):
    # no attractive edge -> rama_contract returns the canonical form of its input: this drives the
    # 64-bit radix sort, the run reduction and the scans over many tiles with a ragged tail
    g = inputs.random_graph(3000, 100003, 21, allow_messy=True)
    c = -np.abs(g["c"]) - 0.01
    wi, wj, wc = oracle32.canonicalise(3000, g["i"], g["j"], c)
    got = rama.contract(3000, g["i"], g["j"], c, repeat=1)
    assert got["n_nodes"] == 3000 and np.array_equal(np_(got["mapping"]), np.arange(3000))
    assert np.array_equal(np_(got["i"]), wi) and np.array_equal(np_(got["j"]), wj)
    assert np.array_equal(np_(got["c"]), wc)       # duplicates are added in input order on both sides


@pytest.mark.parametrize("n,m", [(3, 20001), (2, 2049), (5, 4096), (40, 70000)])
def test_canonicalisation_sums_long_runs_in_input_order(rama, oracle32, n, m):
    # few nodes, many parallel edges: every run of equal pairs is thousands of entries long and crosses
    # the 2048-entry tiles of the run reduction, some exactly at a tile's end; costs of mixed magnitude
    # make the float sum depend on the order of the adds
    rng = np.random.default_rng(n * 1000 + m)
    i = rng.integers(0, n, m).astype(np.int32)
    j = ((i + 1 + rng.integers(0, max(n - 1, 1), m)) % n).astype(np.int32)
    c = (-np.abs(rng.normal(size=m)) * 10.0 ** rng.integers(-3, 4, m) - 1e-3).astype(np.float32)
    wi, wj, wc = oracle32.canonicalise(n, i, j, c)
    got = rama.contract(n, i, j, c, repeat=1)
    assert np.array_equal(np_(got["i"]), wi) and np.array_equal(np_(got["j"]), wj)
    assert np.array_equal(np_(got["c"]), wc)


@pytest.mark.parametrize("runs", [2, 3, 5, 8, 9])
def test_canonicalisation_of_a_few_sorted_runs(rama, oracle32, runs):
    # an edge list made of `runs` sorted pieces (as a grid written direction by direction): up to eight pieces are
    # merged instead of sorted; pairs that occur in several pieces, flipped pairs and self-loops included
    rng = np.random.default_rng(100 + runs)
    n, m = 40000, 120000
    a = rng.integers(0, n, m); b = rng.integers(0, n, m)
    loops = rng.random(m) < 0.01
    b = np.where(loops, a, b)
    lo, hi = np.minimum(a, b), np.maximum(a, b)
    piece = rng.integers(0, runs, m)
    dup = rng.random(m) < 0.1                                    # a tenth of the pairs also goes into another piece
    lo = np.concatenate([lo, lo[dup]]); hi = np.concatenate([hi, hi[dup]])
    piece = np.concatenate([piece, (piece[dup] + 1) % runs])
    order = np.lexsort((hi, lo, piece))                          # piece by piece, each sorted by (lo, hi)
    lo, hi = lo[order], hi[order]
    flip = rng.random(lo.size) < 0.3
    i = np.where(flip, hi, lo).astype(np.int32); j = np.where(flip, lo, hi).astype(np.int32)
    c = (-np.abs(rng.normal(size=i.size)) * 10.0 ** rng.integers(-2, 3, i.size) - 1e-3).astype(np.float32)
    wi, wj, wc = oracle32.canonicalise(n, i, j, c)
    got = rama.contract(n, i, j, c, repeat=1)                    # no attractive edge: the canonical form comes back
    assert np.array_equal(np_(got["i"]), wi) and np.array_equal(np_(got["j"]), wj)
    assert np.array_equal(np_(got["c"]), wc)


# --------------------------------------------------------------------------------------------
# end to end
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name", list(CASES))
def test_solve_end_to_end(rama, oracle32, name):
    g = CASES[name]
    n = g["n_nodes"]
    want = oracle32.solve(n, g["i"], g["j"], g["c"])
    got = rama.solve(n, g["i"], g["j"], g["c"])
    labels = np_(got["labels"])
    assert abs(got["lower_bound"] - want["lower_bound"]) <= REL * max(1.0, abs(want["lower_bound"]))
    assert abs(got["primal"] - want["primal"]) <= 5e-3 * max(1.0, abs(want["primal"]))
    # the reported primal is the cost of the returned labels, and labels are canonical
    assert abs(oracle32.multicut_cost(g["i"], g["j"], g["c"], labels) - got["primal"]) <= 1e-6 * max(1.0, abs(got["primal"]))
    assert np.all(labels[labels] == labels) and np.all(labels <= np.arange(n))
    assert got["lower_bound"] <= got["primal"] + 1e-6 * max(1.0, abs(got["primal"]))
    assert got["n_cycles_first"] == want["n_cycles_first"]
    assert got["n_edges_aug_first"] == want["n_edges_aug_first"]
    print(name, "labels identical:", bool(np.array_equal(labels, want["labels"])), "rounds", got["rounds"],
          want["rounds"], "primal", got["primal"], want["primal"], "LB", got["lower_bound"], want["lower_bound"])


@pytest.mark.parametrize("variant", ["P", "PD+", "D", "PD-matching-only", "PD-forest-always", "PD-shortest",
                                     "PD-7-then-4", "PD-7-shortest", "PD-2-dual-rounds", "D-3-dual-rounds"])
def test_solver_variants(rama, oracle32, variant):
    from paper_2109_01838_amd import default_params
    g = CASES["knn_20000"]
    n = g["n_nodes"]
    kw = {"P": dict(max_cycle_len_first=0, max_cycle_len_later=0),
          "PD+": dict(max_cycle_len_later=5),
          "D": dict(max_rounds=1),
          "PD-matching-only": dict(forest_ratio=0.0),
          "PD-forest-always": dict(forest_ratio=1.0),
          "PD-shortest": dict(shortest_only=True),
          "PD-7-then-4": dict(max_cycle_len_first=7, max_cycle_len_later=4),
          "PD-7-shortest": dict(max_cycle_len_first=7, max_cycle_len_later=7, shortest_only=True),
          "PD-2-dual-rounds": dict(dual_rounds=2),
          "D-3-dual-rounds": dict(max_rounds=1, dual_rounds=3, max_cycle_len_first=4)}[variant]
    want = oracle32.solve(n, g["i"], g["j"], g["c"], **kw)
    kw = {("shortest_cycles_only" if key == "shortest_only" else key): int(v) if key == "shortest_only" else v
          for key, v in kw.items()}
    got = rama.solve(n, g["i"], g["j"], g["c"], default_params(**kw))
    assert got["n_cycles_first"] == want["n_cycles_first"]
    print(variant, "cycles", got["n_cycles_first"], "labels identical:", bool(np.array_equal(np_(got["labels"]), want["labels"])),
          "primal", got["primal"], want["primal"], "LB", got["lower_bound"], want["lower_bound"])
    assert abs(got["lower_bound"] - want["lower_bound"]) <= REL * max(1.0, abs(want["lower_bound"]))
    assert abs(got["primal"] - want["primal"]) <= 5e-3 * max(1.0, abs(want["primal"]))


def test_determinism(rama):
    g = CASES["knn_20000"]
    n = g["n_nodes"]
    a = rama.solve(n, g["i"], g["j"], g["c"])
    b = rama.solve(n, g["i"], g["j"], g["c"])
    assert np.array_equal(np_(a["labels"]), np_(b["labels"]))
    assert a["primal"] == b["primal"] and a["lower_bound"] == b["lower_bound"]
    c1 = rama.find_conflicted_cycles(n, g["i"], g["j"], g["c"], 5)
    m1 = rama.message_passing(n, g["i"], g["j"], g["c"], c1, 4)
    m2 = rama.message_passing(n, g["i"], g["j"], g["c"], c1, 4)
    assert np.array_equal(np_(m1["c"]), np_(m2["c"])) and m1["lower_bound"] == m2["lower_bound"]


def test_degenerate_inputs(rama):
    from paper_2109_01838_amd import RamaError, binding
    e32, ef = np.zeros(0, np.int32), np.zeros(0, np.float32)
    r = rama.solve(4, e32, e32, ef)
    assert np_(r["labels"]).tolist() == [0, 1, 2, 3] and r["primal"] == 0.0 and r["lower_bound"] == 0.0
    i, j = np.array([0, 1], np.int32), np.array([1, 2], np.int32)
    r = rama.solve(3, i, j, np.array([-1.0, -2.0], np.float32))
    assert np_(r["labels"]).tolist() == [0, 1, 2] and r["primal"] == -3.0 and r["lower_bound"] == -3.0
    r = rama.solve(3, i, j, np.array([1.0, 2.0], np.float32))
    assert np_(r["labels"]).tolist() == [0, 0, 0] and r["primal"] == 0.0
    # no nodes at all
    r = rama.solve(0, e32, e32, ef)
    assert r["labels"].numel() == 0 and r["primal"] == 0.0 and r["n_clusters"] == 0
    r = rama.contract(0, e32, e32, ef)
    assert r["n_nodes"] == 0 and r["i"].numel() == 0
    # only self-loops
    r = rama.solve(2, np.array([0, 1], np.int32), np.array([0, 1], np.int32), np.array([1.0, -1.0], np.float32))
    assert np_(r["labels"]).tolist() == [0, 1]
    cyc = rama.find_conflicted_cycles(3, i, j, np.array([1.0, 2.0], np.float32), 5)
    assert [x.shape[0] for x in cyc] == [0, 0, 0]
    with pytest.raises(RamaError) as ei:
        rama.solve(3, i, np.array([1, 3], np.int32), np.array([1.0, 1.0], np.float32))
    assert ei.value.status == binding.RAMA_ERR_BAD_GRAPH
    with pytest.raises(RamaError) as ei:
        rama.solve(3, i, j, np.array([1.0, np.inf], np.float32))
    assert ei.value.status == binding.RAMA_ERR_BAD_GRAPH
    # the context stays usable after an error
    r = rama.solve(3, i, j, np.array([1.0, 2.0], np.float32))
    assert np_(r["labels"]).tolist() == [0, 0, 0]


def test_profile_hooks_and_workspace(rama):
    g = CASES["grid3d_24"]
    rama.profile_enable(True)
    rama.solve(g["n_nodes"], g["i"], g["j"], g["c"])
    prof = rama.profile_get()
    rama.profile_enable(False)
    names = {k["name"] for k in prof}
    assert {"k_triangle_update", "k_edge_update<false>", "k_edge_update<true>", "k_count_cycles<5>", "k_count_cycles<3>", "k_scan_emit<PackCands>", "k_reduce_runs"} <= names
    assert any(n.startswith("k_rs_scatter<") for n in names) and any(n.startswith("k_scan_apply<") for n in names)
    for k in prof:
        assert k["launches"] > 0 and k["ms"] >= 0.0 and k["bytes"] >= 0.0
    # a name filter restricts the timers
    rama.profile_enable(True, only="k_rs_scatter")
    rama.solve(g["n_nodes"], g["i"], g["j"], g["c"])
    only = rama.profile_get()
    rama.profile_enable(False)
    assert only and all(k["name"].startswith("k_rs_scatter") for k in only)
    assert rama.workspace_bytes() > 0


def test_random_sweep_of_small_instances_and_parameters(rama, oracle32):
    """Seeded sweep: small random / grid instances with random solver parameters (cycle lengths,
    iteration counts, forest switch, round limit, dual rounds, shortest-only) and a random choice of the
    cycle search (0..3) and of the entry point (rama_solve / rama_solve_static).  Labels, cycle counts,
    rounds and bounds must agree with the oracle on every one.  (Such a sweep found a rooting loop
    that gave up one check too early on trees about as deep as the graph has nodes.)"""
    from paper_2109_01838_amd import default_params
    rng = np.random.default_rng(7)
    mode_rng = np.random.default_rng(8)   # a stream of its own: the instances stay the ones of earlier versions of this test
    bad = []
    for it in range(160):
        kind = int(rng.integers(0, 4))
        seed = int(rng.integers(0, 1 << 30))
        if kind == 0:
            g = inputs.random_graph(int(rng.integers(2, 60)), int(rng.integers(1, 400)), seed, allow_messy=bool(rng.integers(0, 2)))
        elif kind == 1:
            n = int(rng.integers(50, 2000))
            g = inputs.random_graph(n, int(n * rng.uniform(1.0, 3.0)), seed)
            g = signed(g, seed, float(rng.uniform(0.5, 0.95)))
        elif kind == 2:
            g = inputs.cfg5_crop(int(rng.integers(3, 12)), seed=seed % 1000)
        else:
            g = inputs.cfg2(seed=seed % 1000, h=int(rng.integers(10, 30)), w=int(rng.integers(10, 30)), n_seeds=int(rng.integers(2, 12)))
        n = g["n_nodes"]
        shortest = bool(rng.integers(0, 2))
        kw = dict(max_cycle_len_first=int(rng.choice([0, 3, 4, 5, 6])), max_cycle_len_later=int(rng.choice([0, 3, 4])),
                  mp_iters_first=int(rng.integers(0, 8)), mp_iters_later=int(rng.integers(0, 5)),
                  forest_ratio=float(rng.choice([0.0, 0.1, 0.5, 1.0])), max_rounds=int(rng.choice([0, 0, 0, 1, 2, 3])),
                  dual_rounds=int(rng.choice([1, 1, 2, 3])))
        if kw["dual_rounds"] > 1 or (kind == 3 and not shortest):   # keeps the oracle's enumeration in seconds
            kw["max_cycle_len_first"] = min(kw["max_cycle_len_first"], 4 if kw["dual_rounds"] > 1 else 5)
            kw["max_cycle_len_later"] = min(kw["max_cycle_len_later"], 3)
        want = oracle32.solve(n, g["i"], g["j"], g["c"], shortest_only=shortest, **kw)
        rama.set_cycle_search(int(mode_rng.integers(0, 4)))
        got = rama.solve(n, g["i"], g["j"], g["c"], default_params(shortest_cycles_only=int(shortest), **kw),
                         static=bool(mode_rng.integers(0, 3) == 0))
        rama.set_cycle_search(0)
        ok = (np.array_equal(np_(got["labels"]), want["labels"]) and got["n_cycles_first"] == want["n_cycles_first"]
              and got["rounds"] == want["rounds"]
              and abs(got["lower_bound"] - want["lower_bound"]) <= REL * max(1.0, abs(want["lower_bound"]))
              and abs(got["primal"] - want["primal"]) <= 5e-3 * max(1.0, abs(want["primal"])))
        if not ok:
            bad.append((it, kind, seed, n, kw, shortest))
    assert not bad, bad


# --------------------------------------------------------------------------------------------
# the split sort (top-bit passes + one in-LDS sort) is the same stable sort as passes over all bits
# --------------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def rama_split():
    from paper_2109_01838_amd import Rama
    r = Rama("cuda:0")
    r.set_sort_split(0, 0)          # every sort of two or more elements takes the split path
    yield r
    r.close()


def star_graph(n_leaves, seed):
    """Node 0 joined to every other node, plus a sparse ring: all edges of the hub share their
    first endpoint, so the hub's segment exceeds what a workgroup can sort in LDS."""
    rng = np.random.default_rng(seed)
    leaves = np.arange(1, n_leaves + 1, dtype=np.int32)
    i = np.concatenate([np.zeros(n_leaves, np.int32), leaves[:-1]])
    j = np.concatenate([leaves, leaves[1:]])
    mag = np.abs(rng.normal(0.0, 1.0, i.size)).astype(np.float32) + 0.05
    c = np.where(rng.random(i.size) < 0.7, mag, -mag).astype(np.float32)
    perm = rng.permutation(i.size)
    return dict(name=f"star_{n_leaves}", n_nodes=n_leaves + 1, i=i[perm], j=j[perm], c=c[perm])


def gappy_graph(n, kind, seed):
    """Graphs whose node rows have long empty stretches.  'clusters': dense little cliques-with-noise far apart
    in the node numbering (many edges, gaps of thousands of rows between them); 'sparse': a few triangles
    scattered over many nodes (far fewer edges than rows); 'tail': all edges among the last few nodes."""
    rng = np.random.default_rng(seed)
    ii, jj = [], []
    if kind == "clusters":
        for base in range(0, n - 64, max(64, n // 40)):
            nodes = base + np.arange(48)
            a = rng.choice(nodes, 400); b = rng.choice(nodes, 400)
            ii.append(a); jj.append(b)
    elif kind == "sparse":
        for base in rng.choice(n - 3, 60, replace=False):
            ii.append(np.array([base, base + 1, base])); jj.append(np.array([base + 1, base + 2, base + 2]))
    else:
        nodes = n - 40 + np.arange(40)
        ii.append(rng.choice(nodes, 500)); jj.append(rng.choice(nodes, 500))
    i = np.concatenate(ii).astype(np.int32); j = np.concatenate(jj).astype(np.int32)
    keep = i != j
    i, j = i[keep], j[keep]
    mag = np.abs(rng.normal(0.0, 1.0, i.size)).astype(np.float32) + 0.05
    c = np.where(rng.random(i.size) < 0.65, mag, -mag).astype(np.float32)
    return dict(n_nodes=n, i=i, j=j, c=c)


@pytest.mark.parametrize("kind", ["clusters", "sparse", "tail"])
@pytest.mark.parametrize("n", [5000, 60000, 300000])
def test_rows_with_long_empty_stretches(rama, oracle32, kind, n):
    """Row pointers over node sets that are mostly empty: long gaps are filled by whole workgroups, sparse key
    sets are searched per row; cycles, message passing and the whole solve must not notice."""
    g = gappy_graph(n, kind, 11)
    want = oracle32.find_conflicted_cycles(n, g["i"], g["j"], g["c"], 5)
    got = rama.find_conflicted_cycles(n, g["i"], g["j"], g["c"], 5)
    for a, b in zip(got, want):
        assert np.array_equal(np_(a), b)
    wmp = oracle32.message_passing(n, g["i"], g["j"], g["c"], want, 3)
    mp = rama.message_passing(n, g["i"], g["j"], g["c"], want, 3)
    assert np.array_equal(np_(mp["i"]), wmp["i"]) and np.array_equal(np_(mp["j"]), wmp["j"])
    assert rel_close(np_(mp["c"]), wmp["c"])
    ws = oracle32.solve(n, g["i"], g["j"], g["c"])
    gs = rama.solve(n, g["i"], g["j"], g["c"])
    assert gs["n_cycles_first"] == ws["n_cycles_first"] and gs["rounds"] == ws["rounds"]
    assert np.array_equal(np_(gs["labels"]), ws["labels"])
    assert abs(gs["lower_bound"] - ws["lower_bound"]) <= REL * max(1.0, abs(ws["lower_bound"]))
    print(kind, n, [x.shape[0] for x in want], gs["rounds"])


@pytest.mark.parametrize("name", list(CASES))
def test_split_sort_stagewise(rama_split, oracle32, name):
    from paper_2109_01838_amd import default_params
    g = CASES[name]
    n = g["n_nodes"]
    lmax = 4 if name == "random_dense" else 5
    cyc = oracle32.find_conflicted_cycles(n, g["i"], g["j"], g["c"], lmax)
    got = rama_split.find_conflicted_cycles(n, g["i"], g["j"], g["c"], lmax)
    for a, b in zip(got, cyc):
        assert np.array_equal(np_(a), b)
    want = oracle32.message_passing(n, g["i"], g["j"], g["c"], cyc, 3)
    mp = rama_split.message_passing(n, g["i"], g["j"], g["c"], cyc, 3)
    assert np.array_equal(np_(mp["i"]), want["i"]) and np.array_equal(np_(mp["j"]), want["j"])
    assert rel_close(np_(mp["c"]), want["c"])
    for forest_ratio in (0.1, 1.0):
        w = oracle32.contract(n, want["i"], want["j"], want["c"], forest_ratio=forest_ratio)
        con = rama_split.contract(n, want["i"], want["j"], want["c"], params=default_params(forest_ratio=forest_ratio))
        assert np.array_equal(np_(con["mapping"]), w["mapping"])
        assert np.array_equal(np_(con["i"]), w["i"]) and np.array_equal(np_(con["j"]), w["j"])
        assert rel_close(np_(con["c"]), w["c"])


@pytest.mark.parametrize("name", list(CASES) + ["hubs", "star_9", "star_40000"])
def test_split_sort_solve(rama, rama_split, oracle32, name):
    """Same labels, bounds and counts from both sort paths (bit for bit: both are the same stable
    sort), and both agree with the oracle.  star_40000 holds a segment no workgroup can take, which
    sends the split path back to passes over all bits after its top-bit passes."""
    g = CASES[name] if name in CASES else (inputs.hub_graph() if name == "hubs" else star_graph(int(name[5:]), 3))
    n = g["n_nodes"]
    a = rama.solve(n, g["i"], g["j"], g["c"])
    b = rama_split.solve(n, g["i"], g["j"], g["c"])
    want = oracle32.solve(n, g["i"], g["j"], g["c"])
    assert np.array_equal(np_(a["labels"]), np_(b["labels"]))
    assert a["primal"] == b["primal"] and a["lower_bound"] == b["lower_bound"]
    assert a["n_cycles_first"] == b["n_cycles_first"] == want["n_cycles_first"]
    assert a["rounds"] == b["rounds"]
    assert np.array_equal(np_(b["labels"]), want["labels"])
    assert abs(b["lower_bound"] - want["lower_bound"]) <= REL * max(1.0, abs(want["lower_bound"]))


def test_split_sort_takes_its_kernels(rama_split):
    g = CASES["knn_20000"]
    rama_split.profile_enable(True)
    rama_split.solve(g["n_nodes"], g["i"], g["j"], g["c"])
    names = {k["name"] for k in rama_split.profile_get()}
    rama_split.profile_enable(False)
    assert "k_seg_bounds" in names and "k_rs_local<u64,u32>" in names and "k_rs_local<u32,u32>" in names


def test_split_sort_with_wide_local_keys(rama_split, oracle32):
    """Few edges over many nodes: one pass over the top bits leaves more than 26 low bits, which do
    not fit the 32-bit keys of the in-LDS sort, so its 64-bit variant runs."""
    from paper_2109_01838_amd import default_params
    g = signed(inputs.random_graph(200000, 400000, 21), 21, 0.75)
    perm = np.random.default_rng(5).permutation(g["i"].size)     # unsorted input: canonicalising it sorts (key, cost) pairs
    g = dict(g, i=g["i"][perm], j=g["j"][perm], c=g["c"][perm])
    n = g["n_nodes"]
    rama_split.profile_enable(True)
    got = rama_split.solve(n, g["i"], g["j"], g["c"])
    names = {k["name"] for k in rama_split.profile_get()}
    rama_split.profile_enable(False)
    assert {"k_rs_local<u64,u32,wide>", "k_rs_local<u64,wide>"} <= names
    want = oracle32.solve(n, g["i"], g["j"], g["c"])
    assert np.array_equal(np_(got["labels"]), want["labels"])
    assert got["n_cycles_first"] == want["n_cycles_first"] and got["rounds"] == want["rounds"]
    assert abs(got["lower_bound"] - want["lower_bound"]) <= REL * max(1.0, abs(want["lower_bound"]))
    for forest_ratio in (0.1, 1.0):
        w = oracle32.contract(n, g["i"], g["j"], g["c"], forest_ratio=forest_ratio)
        con = rama_split.contract(n, g["i"], g["j"], g["c"], params=default_params(forest_ratio=forest_ratio))
        assert np.array_equal(np_(con["mapping"]), w["mapping"])
        assert np.array_equal(np_(con["i"]), w["i"]) and np.array_equal(np_(con["j"]), w["j"])
        assert rel_close(np_(con["c"]), w["c"])


def test_context_on_a_side_stream_and_two_contexts(rama):
    """A context bound to a non-default stream (default priority) gives the same result as the
    default-stream context, also when the two are used in turn."""
    import torch
    from paper_2109_01838_amd import Rama
    g = CASES["grid3d_24"]
    n = g["n_nodes"]
    base = rama.solve(n, g["i"], g["j"], g["c"])
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        other = Rama("cuda:0")
        assert other.stream.cuda_stream == side.cuda_stream and other.stream.cuda_stream != rama.stream.cuda_stream
        a = other.solve(n, g["i"], g["j"], g["c"])
        cyc = other.find_conflicted_cycles(n, g["i"], g["j"], g["c"], 5)
    side.synchronize()
    b = rama.solve(n, g["i"], g["j"], g["c"])
    with torch.cuda.stream(side):
        a2 = other.solve(n, g["i"], g["j"], g["c"])
    side.synchronize()
    for r in (a, b, a2):
        assert np.array_equal(np_(r["labels"]), np_(base["labels"])) and r["primal"] == base["primal"]
        assert r["lower_bound"] == base["lower_bound"]
    want = rama.find_conflicted_cycles(n, g["i"], g["j"], g["c"], 5)
    assert all(np.array_equal(np_(x), np_(y)) for x, y in zip(cyc, want))
    other.close()


# --------------------------------------------------------------------------------------------
# workspace allocator callbacks and per-round records
# --------------------------------------------------------------------------------------------
def test_allocator_callbacks_and_injected_out_of_memory(rama):
    """The workspace comes from the caller's allocator; an allocator that runs dry at its n-th call makes the
    call in progress end with RAMA_ERR_OOM, everything taken so far goes back, and the ctx stays usable."""
    import torch
    from paper_2109_01838_amd import Rama, RamaError, binding
    g = CASES["grid3d_24"]
    n = g["n_nodes"]
    base = rama.solve(n, g["i"], g["j"], g["c"])
    live, calls, fail_from = {}, [0], [None]

    def alloc(nbytes):
        calls[0] += 1
        if fail_from[0] is not None and calls[0] >= fail_from[0]:
            return None
        p = torch.cuda.caching_allocator_alloc(int(nbytes), 0)
        live[p] = nbytes
        return p

    def free(ptr):
        assert ptr in live
        del live[ptr]
        torch.cuda.caching_allocator_delete(ptr)

    r = Rama("cuda:0", allocator=(alloc, free))
    at_create = calls[0]                             # the ctx's own few words
    a = r.solve(n, g["i"], g["j"], g["c"])
    assert np.array_equal(np_(a["labels"]), np_(base["labels"])) and a["primal"] == base["primal"]
    total_calls = calls[0] - at_create               # allocator calls of one solve on a fresh ctx
    assert total_calls > 5 and len(live) > 0 and sum(live.values()) == r.workspace_bytes()
    r.close()
    assert not live                                  # every block went back through the callback
    for k in (1, 3, total_calls // 2, total_calls):
        r = Rama("cuda:0", allocator=(alloc, free))
        calls[0], fail_from[0] = 0, k
        with pytest.raises(RamaError) as ei:
            r.solve(n, g["i"], g["j"], g["c"])
        assert ei.value.status == binding.RAMA_ERR_OOM, ei.value
        assert sum(live.values()) == r.workspace_bytes()   # what was in use at the failure is cached, nothing is lost
        fail_from[0] = None
        b = r.solve(n, g["i"], g["j"], g["c"])       # same ctx, allocator working again
        assert np.array_equal(np_(b["labels"]), np_(base["labels"])) and b["lower_bound"] == base["lower_bound"]
        r.close()
        assert not live
    # the library's own hipMalloc path still exists
    r = Rama("cuda:0", allocator="hip")
    c = r.solve(n, g["i"], g["j"], g["c"])
    assert np.array_equal(np_(c["labels"]), np_(base["labels"]))
    r.close()


def test_round_records(rama, oracle32):
    g = CASES["knn_20000"]
    n = g["n_nodes"]
    got = rama.solve(n, g["i"], g["j"], g["c"])
    rounds = rama.round_stats()
    assert len(rounds) == got["rounds"] >= 2
    ic, jc, cc = oracle32.canonicalise(n, g["i"], g["j"], g["c"])
    first = rounds[0]
    assert first["n_nodes"] == n and first["n_edges"] == ic.size
    assert first["n_attractive"] == int((cc > 0).sum()) and first["n_repulsive"] == int((cc < 0).sum())
    assert first["n_cycles"] == got["n_cycles_first"] and first["n_triangles"] == got["n_triangles_first"]
    assert first["n_edges_aug"] == got["n_edges_aug_first"]
    want = oracle32.find_conflicted_cycles(n, g["i"], g["j"], g["c"], 5)
    assert first["n_cycles"][:3] == [w.shape[0] for w in want]
    for a, b in zip(rounds, rounds[1:]):
        assert b["n_nodes"] < a["n_nodes"]
        assert a["n_contracted"] > 0 and b["n_edges"] <= a["n_edges_aug"]
        if not a["used_forest"]:
            assert b["n_nodes"] == a["n_nodes"] - a["n_contracted"]     # a matching joins pairs
    assert rounds[-1]["n_contracted"] == 0
    assert all(r["workspace_peak"] > 0 for r in rounds)
    assert all(r["ms"]["cycles"] >= 0 and r["ms"]["dual"] >= 0 and r["ms"]["contract"] > 0 for r in rounds)
    s = got["ms"]
    assert abs(sum(r["ms"]["contract"] for r in rounds) - s["contract"]) < 1e-6 and s["total"] > s["contract"]
