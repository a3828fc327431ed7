"""Brute-force references used to pin the oracle.  Pure Python / numpy, written from the
definitions only (set partitions, simple cycles, the five triangle labelings); nothing here
calls into oracle/ or the HIP library."""
import itertools

import numpy as np


def set_partitions(n):
    """All partitions of {0..n-1} as label vectors in restricted-growth form."""
    def rec(prefix, mx):
        if len(prefix) == n:
            yield tuple(prefix)
            return
        for v in range(mx + 2):
            prefix.append(v)
            yield from rec(prefix, max(mx, v))
            prefix.pop()
    if n == 0:
        yield ()
        return
    yield from rec([0], 0)


def multicut_cost(i, j, c, labels):
    labels = np.asarray(labels)
    cut = labels[np.asarray(i)] != labels[np.asarray(j)]
    return float(np.sum(np.asarray(c, dtype=np.float64)[cut]))


def optimal_multicut(n, i, j, c):
    """min over all partitions of the cut cost (eq. 2 of the paper)."""
    best, arg = None, None
    i, j = np.asarray(i), np.asarray(j)
    c = np.asarray(c, dtype=np.float64)
    for lab in set_partitions(n):
        lab = np.asarray(lab)
        v = float(c[lab[i] != lab[j]].sum())
        if best is None or v < best:
            best, arg = v, lab
    return best, arg


def conflicted_cycles(n, i, j, c, max_len):
    """All simple cycles of length 3..max_len with exactly one negative edge and all other
    edges positive, found by trying every ordered vertex tuple.  Returned per length as a set
    of tuples (v0,..,v_{L-1}) with (v0,v_{L-1}) the negative edge and v0<v_{L-1}."""
    cost = {}
    for a, b, w in zip(i, j, c):
        a, b = int(a), int(b)
        if a == b:
            continue
        key = (min(a, b), max(a, b))
        cost[key] = cost.get(key, 0.0) + float(w)
    def w(a, b):
        return cost.get((min(a, b), max(a, b)))
    out = {L: set() for L in range(3, max(max_len, 5) + 1)}
    for L in range(3, max_len + 1):
        for tup in itertools.permutations(range(n), L):
            if tup[0] >= tup[-1]:
                continue
            wl = w(tup[0], tup[-1])
            if wl is None or not wl < 0:
                continue
            ok = True
            for q in range(L - 1):
                wq = w(tup[q], tup[q + 1])
                if wq is None or not wq > 0:
                    ok = False
                    break
            if ok:
                out[L].add(tup)
    return out


M_T = [(0, 0, 0), (1, 1, 0), (1, 0, 1), (0, 1, 1), (1, 1, 1)]


def tri_min_marginal(ct, s):
    ct = np.asarray(ct, dtype=np.float64)
    v1 = min(float(np.dot(ct, y)) for y in M_T if y[s] == 1)
    v0 = min(float(np.dot(ct, y)) for y in M_T if y[s] == 0)
    return v1 - v0


def tri_lb(ct):
    ct = np.asarray(ct, dtype=np.float64)
    return min(float(np.dot(ct, y)) for y in M_T)


def forest_path(n, forest_edges, a, b):
    """Edges (as indices into forest_edges) on the unique a-b path of a forest, or None."""
    adj = {v: [] for v in range(n)}
    for k, (u, v) in enumerate(forest_edges):
        adj[u].append((v, k))
        adj[v].append((u, k))
    stack, seen = [(a, [])], {a}
    while stack:
        v, path = stack.pop()
        if v == b:
            return path
        for w, k in adj[v]:
            if w not in seen:
                seen.add(w)
                stack.append((w, path + [k]))
    return None


def hop_distance(n, i, j, c, src, dst):
    """Hop distance src -> dst using attractive edges only (scipy's breadth-first search); inf if none."""
    import scipy.sparse as sp
    from scipy.sparse.csgraph import shortest_path
    cost = {}
    for a, b, w in zip(i, j, c):
        a, b = int(a), int(b)
        if a != b:
            key = (min(a, b), max(a, b))
            cost[key] = cost.get(key, 0.0) + float(w)
    pos = [k for k, w in cost.items() if w > 0]
    A = sp.coo_matrix((np.ones(len(pos)), ([k[0] for k in pos], [k[1] for k in pos])), shape=(n, n)).tocsr()
    return float(shortest_path(A, directed=False, unweighted=True, indices=[src])[0, dst])
