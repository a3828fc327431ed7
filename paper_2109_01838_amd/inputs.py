"""Seeded synthetic multicut instances (graph + fp32 edge costs).

This module only *draws inputs*: node grids / point clouds, planted clusters and
random edge costs.  It contains none of the solver's arithmetic and is the one
piece of code that both the CPU oracle's tests and the HIP path's tests/bench
use, so that the two never have to reproduce each other's random numbers.

Every instance is a dict with
  n_nodes : int
  i, j    : int32[E]  edge endpoints (i < j, row-major linear node ids, fixed order)
  c       : float32[E] edge costs, positive = attractive (paper Sec. 3, eq. 2)
  truth   : int32[n_nodes] planted cluster id (informational only)
  name    : str

The five named configurations stand in for the paper's data sets (Sec. 4,
"Datasets"), which are not redistributed with this repository:
  cfg1  2D 4-connected grid 32x32, 16 planted 8x8 blocks            (parity, seconds on a CPU)
  cfg2  2D grid 512x512 + long-range offsets 3 and 9 (Cityscapes-shaped)
  cfg3  1M random points, symmetric 6-NN graph (Connectomics-SP-shaped, irregular)
  cfg4  3D 6-connected grid 256x256x128 (Connectomics-Raw-shaped)
  cfg5  3D 6-connected grid 320^3, ~9.8e7 edges (headline size)
All sizes can be scaled down with the keyword arguments for quick tests.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "grid_edges", "voronoi_truth", "gaussian_costs", "block_truth_2d",
    "cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "make", "random_graph",
]


def grid_edges(shape, offsets):
    """Edges of a regular grid: for every offset vector `d` connect x -> x+d when in range.

    Node id = row-major linear index.  Edges are emitted offset by offset, each
    block in ascending source-node order; always i < j (every offset must be
    lexicographically positive).
    """
    shape = tuple(int(s) for s in shape)
    n = int(np.prod(shape))
    ids = np.arange(n, dtype=np.int32).reshape(shape)
    ii, jj = [], []
    for d in offsets:
        d = tuple(int(x) for x in d)
        assert len(d) == len(shape)
        src = tuple(slice(max(0, -dk), s - max(0, dk)) for dk, s in zip(d, shape))
        dst = tuple(slice(max(0, dk), s - max(0, -dk)) for dk, s in zip(d, shape))
        a = ids[src].ravel()
        b = ids[dst].ravel()
        assert a.size == 0 or np.all(a < b)
        ii.append(a)
        jj.append(b)
    return n, np.concatenate(ii).astype(np.int32), np.concatenate(jj).astype(np.int32)


def block_truth_2d(h, w, bh, bw):
    y, x = np.mgrid[0:h, 0:w]
    return ((y // bh) * ((w + bw - 1) // bw) + (x // bw)).astype(np.int32).ravel()


def voronoi_truth(points, n_seeds, rng, box):
    """Planted clusters: every point is labelled by its nearest of `n_seeds` uniform seeds."""
    from scipy.spatial import cKDTree

    box = np.asarray(box, dtype=np.float64)
    seeds = rng.random((int(n_seeds), box.size)) * box
    tree = cKDTree(seeds)
    out = np.empty(points.shape[0], dtype=np.int32)
    step = 1 << 22
    for s in range(0, points.shape[0], step):
        _, idx = tree.query(points[s:s + step], k=1, workers=-1)
        out[s:s + step] = idx.astype(np.int32)
    return out


def _grid_points(shape):
    n = int(np.prod(shape))
    coords = np.empty((n, len(shape)), dtype=np.float32)
    idx = np.arange(n, dtype=np.int64)
    for k in range(len(shape) - 1, -1, -1):
        coords[:, k] = (idx % shape[k]).astype(np.float32) + 0.5
        idx //= shape[k]
    return coords


def gaussian_costs(i, j, truth, rng, mu_in, sd_in, mu_out, sd_out, flip=0.0):
    """fp32 costs: N(mu_in, sd_in) inside a planted cluster, N(mu_out, sd_out) across;
    then an i.i.d. Bernoulli(flip) subset gets its sign flipped."""
    same = truth[i] == truth[j]
    z = rng.standard_normal(i.size, dtype=np.float32)
    c = np.where(same, np.float32(mu_in) + np.float32(sd_in) * z,
                 np.float32(mu_out) + np.float32(sd_out) * z).astype(np.float32)
    if flip > 0.0:
        f = rng.random(i.size, dtype=np.float32) < np.float32(flip)
        c = np.where(f, -c, c).astype(np.float32)
    return c


def cfg1(seed=0, h=32, w=32, block=8):
    rng = np.random.default_rng(seed)
    n, i, j = grid_edges((h, w), [(0, 1), (1, 0)])
    truth = block_truth_2d(h, w, block, block)
    c = gaussian_costs(i, j, truth, rng, 1.0, 0.5, -1.0, 0.5)
    return dict(name=f"cfg1_grid2d_{h}x{w}", n_nodes=n, i=i, j=j, c=c, truth=truth)


def cfg2(seed=0, h=512, w=512, n_seeds=500):
    rng = np.random.default_rng(seed)
    offs = [(0, 1), (1, 0), (0, 3), (3, 0), (0, 9), (9, 0)]
    n, i, j = grid_edges((h, w), offs)
    truth = voronoi_truth(_grid_points((h, w)), n_seeds, rng, (h, w))
    c = gaussian_costs(i, j, truth, rng, 0.8, 0.6, -0.8, 0.6, flip=0.05)
    return dict(name=f"cfg2_grid2d_longrange_{h}x{w}", n_nodes=n, i=i, j=j, c=c, truth=truth)


def cfg3(seed=0, n_points=1_000_000, k=6, n_seeds=5000):
    from scipy.spatial import cKDTree

    rng = np.random.default_rng(seed)
    pts = rng.random((int(n_points), 2))
    tree = cKDTree(pts)
    _, nb = tree.query(pts, k=k + 1, workers=-1)
    a = np.repeat(np.arange(n_points, dtype=np.int64), k)
    b = nb[:, 1:].reshape(-1).astype(np.int64)
    lo, hi = np.minimum(a, b), np.maximum(a, b)
    keep = lo != hi
    key = np.unique(lo[keep] * np.int64(n_points) + hi[keep])
    i = (key // n_points).astype(np.int32)
    j = (key % n_points).astype(np.int32)
    truth = voronoi_truth(pts, n_seeds, rng, (1.0, 1.0))
    same = truth[i] == truth[j]
    p = np.where(same, rng.beta(5.0, 2.0, i.size), rng.beta(2.0, 5.0, i.size))
    p = np.clip(p, 1e-6, 1.0 - 1e-6)
    c = np.log(p / (1.0 - p)).astype(np.float32)
    return dict(name=f"cfg3_knn{k}_{n_points}", n_nodes=int(n_points), i=i, j=j, c=c, truth=truth)


def _grid3d(seed, shape, n_seeds, mu, sd, flip, tag):
    rng = np.random.default_rng(seed)
    n, i, j = grid_edges(shape, [(0, 0, 1), (0, 1, 0), (1, 0, 0)])
    truth = voronoi_truth(_grid_points(shape), n_seeds, rng, shape)
    c = gaussian_costs(i, j, truth, rng, mu, sd, -mu, sd, flip=flip)
    return dict(name=f"{tag}_grid3d_{shape[0]}x{shape[1]}x{shape[2]}", n_nodes=n, i=i, j=j, c=c,
                truth=truth)


def cfg4(seed=0, shape=(128, 256, 256), n_seeds=20000):
    return _grid3d(seed, shape, n_seeds, 1.0, 0.7, 0.03, "cfg4")


def cfg5(seed=0, shape=(320, 320, 320), n_seeds=100000):
    return _grid3d(seed, shape, n_seeds, 0.7, 0.7, 0.05, "cfg5")


def cfg5_crop(side, seed=0):
    """A cube of side `side` drawn with cfg5's recipe and seed density (seeds scale with volume)."""
    n_seeds = max(2, int(round(100000 * (side / 320.0) ** 3)))
    return _grid3d(seed, (side, side, side), n_seeds, 0.7, 0.7, 0.05, f"cfg5crop{side}")


def make(name, **kw):
    return {"cfg1": cfg1, "cfg2": cfg2, "cfg3": cfg3, "cfg4": cfg4, "cfg5": cfg5}[name](**kw)


def hub_graph(n_nodes=4000, hubs=(0, 1, 2000, 3999), hub_degree=700, n_background=9000, seed=0, p_attractive=0.85):
    """Skewed degrees: a sparse random background plus a few hubs joined to hub_degree random nodes each
    (and to each other); N(0,1) magnitudes, attractive with probability p_attractive."""
    rng = np.random.default_rng(seed)
    a = rng.integers(0, n_nodes, n_background)
    b = rng.integers(0, n_nodes, n_background)
    for h in hubs:
        others = rng.choice(n_nodes, hub_degree, replace=False)
        a = np.concatenate([a, np.full(hub_degree, h)])
        b = np.concatenate([b, others])
    hh = np.array([(x, y) for x in hubs for y in hubs if x < y])
    a, b = np.concatenate([a, hh[:, 0]]), np.concatenate([b, hh[:, 1]])
    lo, hi = np.minimum(a, b), np.maximum(a, b)
    key = np.unique(lo[lo != hi].astype(np.int64) * n_nodes + hi[lo != hi])
    i, j = (key // n_nodes).astype(np.int32), (key % n_nodes).astype(np.int32)
    mag = np.abs(rng.normal(0.0, 1.0, i.size)) + 0.05
    c = np.where(rng.random(i.size) < p_attractive, mag, -mag).astype(np.float32)
    return dict(name=f"hubs_{n_nodes}", n_nodes=int(n_nodes), i=i, j=j, c=c)


def random_graph(n_nodes, n_edges, seed, scale=1.0, allow_messy=False):
    """Small random graph with N(0, scale) costs.  With allow_messy the edge list also
    contains self-loops, antiparallel duplicates and exact-zero costs (boundary hygiene tests)."""
    rng = np.random.default_rng(seed)
    if allow_messy:
        i = rng.integers(0, n_nodes, n_edges).astype(np.int32)
        j = rng.integers(0, n_nodes, n_edges).astype(np.int32)
        c = (scale * rng.standard_normal(n_edges)).astype(np.float32)
        c[rng.random(n_edges) < 0.05] = 0.0
        return dict(name="random_messy", n_nodes=int(n_nodes), i=i, j=j, c=c,
                    truth=np.zeros(n_nodes, np.int32))
    all_pairs = n_nodes * (n_nodes - 1) // 2
    n_edges = min(int(n_edges), all_pairs)
    if all_pairs <= 4_000_000:
        iu, ju = np.triu_indices(n_nodes, 1)
        sel = np.sort(rng.choice(all_pairs, n_edges, replace=False))
        i, j = iu[sel].astype(np.int32), ju[sel].astype(np.int32)
    else:
        a = rng.integers(0, n_nodes, 2 * n_edges)
        b = rng.integers(0, n_nodes, 2 * n_edges)
        lo, hi = np.minimum(a, b), np.maximum(a, b)
        key = np.unique(lo[lo != hi] * np.int64(n_nodes) + hi[lo != hi])
        key = np.sort(rng.permutation(key)[:n_edges])
        i, j = (key // n_nodes).astype(np.int32), (key % n_nodes).astype(np.int32)
    c = (scale * rng.standard_normal(i.size)).astype(np.float32)
    return dict(name="random", n_nodes=int(n_nodes), i=i, j=j, c=c,
                truth=np.zeros(n_nodes, np.int32))
