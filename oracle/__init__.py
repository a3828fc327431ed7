"""ctypes view of the CPU oracle (oracle/rama_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product package never imports this module and
this module never imports the product's HIP binding.

Two builds of the same source exist: real=float (decisions taken in the GPU
path's precision; this is the parity twin) and real=double (used to size the
floating-point tolerances).  With RAMA_ORACLE_SANITIZE=1 in the environment both
are built with AddressSanitizer + UndefinedBehaviorSanitizer into libraries of
their own (the process must then have been started with libasan preloaded, see
tests/test_oracle_sanitized.py).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rama_oracle.c")
SANITIZE = os.environ.get("RAMA_ORACLE_SANITIZE", "0") == "1"
_SUFFIX = "_san" if SANITIZE else ""
_LIBS = {"f32": os.path.join(_HERE, f"librama_oracle_f32{_SUFFIX}.so"),
         "f64": os.path.join(_HERE, f"librama_oracle_f64{_SUFFIX}.so")}
_CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-std=c11", "-shared", "-fPIC", "-Wall", "-Wextra"]
if SANITIZE:   # same arithmetic flags; every finding aborts the process
    _CFLAGS = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"] + _CFLAGS[1:]

OK, ERR_ARG, ERR_GRAPH, ERR_CAP, ERR_OOM = 0, -1, -2, -3, -4
MAX_CYCLE_LEN = 7   # longest cycle the C source separates


def build(force=True):
    """Compile both precisions of the oracle with gcc."""
    for tag, path in _LIBS.items():
        if not force and os.path.exists(path) and os.path.getmtime(path) >= os.path.getmtime(_SRC):
            continue
        real = "float" if tag == "f32" else "double"
        cmd = ["gcc", *_CFLAGS, f"-DORACLE_REAL={real}", "-o", path, _SRC, "-lm"]
        subprocess.run(cmd, check=True)


_p32 = np.ctypeslib.ndpointer(np.int32, flags="C_CONTIGUOUS")
_pf = np.ctypeslib.ndpointer(np.float32, flags="C_CONTIGUOUS")


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class OracleError(RuntimeError):
    def __init__(self, status, where):
        super().__init__(f"oracle {where} failed with status {status}")
        self.status = status


class Oracle:
    """One precision of the oracle."""

    def __init__(self, precision="f32"):
        path = _LIBS[precision]
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_SRC):
            build(force=False)
        self.lib = C.CDLL(path)
        self.precision = precision
        L = self.lib
        L.rama_oracle_min_marginal.restype = C.c_double
        L.rama_oracle_triangle_lb.restype = C.c_double
        L.rama_oracle_lower_bound.restype = C.c_double
        L.rama_oracle_multicut_cost.restype = C.c_double
        L.rama_oracle_matching.restype = C.c_int64
        assert L.rama_oracle_real_bytes() == (4 if precision == "f32" else 8)

    # -- a0 -----------------------------------------------------------------------------------
    def canonicalise(self, n, i, j, c):
        i, j, c = _i32(i), _i32(j), _f32(c)
        m = i.size
        io, jo, co = np.empty(m, np.int32), np.empty(m, np.int32), np.empty(m, np.float32)
        mo = C.c_int64(0)
        st = self.lib.rama_oracle_canonicalise(C.c_int32(n), C.c_int64(m), _ptr(i), _ptr(j), _ptr(c),
                                               _ptr(io), _ptr(jo), _ptr(co), C.byref(mo))
        if st != OK:
            raise OracleError(st, "canonicalise")
        k = mo.value
        return io[:k].copy(), jo[:k].copy(), co[:k].copy()

    # -- a1 -----------------------------------------------------------------------------------
    @staticmethod
    def _lists(cycles):
        """list of [n_L, L] arrays, L = 3.. -> (max_cycle_len, arrays, pointer array, count array)"""
        arrs = [_i32(x).reshape(-1, k + 3) for k, x in enumerate(cycles)]
        while len(arrs) < 1:
            arrs.append(np.empty((0, 3), np.int32))
        ptrs = (C.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])
        cnts = (C.c_int64 * len(arrs))(*[a.shape[0] for a in arrs])
        return len(arrs) + 2, arrs, ptrs, cnts

    def find_conflicted_cycles(self, n, i, j, c, max_cycle_len=5, shortest_only=False):
        """Returns max_cycle_len-2 arrays: entry L-3 is [n_L, L], the conflicted L-cycles."""
        i, j, c = _i32(i), _i32(j), _f32(c)
        nl = max_cycle_len - 2
        cnt = (C.c_int64 * max(nl, 1))()
        st = self.lib.rama_oracle_find_conflicted_cycles(
            C.c_int32(n), C.c_int64(i.size), _ptr(i), _ptr(j), _ptr(c), C.c_int32(max_cycle_len),
            C.c_int32(int(shortest_only)), None, None, cnt)
        if st not in (OK, ERR_CAP):
            raise OracleError(st, "find_conflicted_cycles(count)")
        outs = [np.empty((cnt[k], k + 3), np.int32) for k in range(nl)]
        ptrs = (C.c_void_p * nl)(*[o.ctypes.data for o in outs])
        cap = (C.c_int64 * nl)(*[cnt[k] for k in range(nl)])
        st = self.lib.rama_oracle_find_conflicted_cycles(
            C.c_int32(n), C.c_int64(i.size), _ptr(i), _ptr(j), _ptr(c), C.c_int32(max_cycle_len),
            C.c_int32(int(shortest_only)), cap, ptrs, cnt)
        if st != OK:
            raise OracleError(st, "find_conflicted_cycles")
        return outs

    # -- a2 -----------------------------------------------------------------------------------
    def triangulate(self, n, i, j, c, cycles):
        """Input must be canonical.  Returns (ia, ja, ca, tri_nodes[T,3], tri_edge[T,3])."""
        i, j, c = _i32(i), _i32(j), _f32(c)
        lmax, arrs, ptrs, cnts = self._lists(cycles)
        room = i.size + sum(k * a.shape[0] for k, a in enumerate(arrs))
        tmax = sum((k + 1) * a.shape[0] for k, a in enumerate(arrs))
        ia, ja, ca = np.empty(room, np.int32), np.empty(room, np.int32), np.empty(room, np.float32)
        tn, te = np.empty((tmax, 3), np.int32), np.empty((tmax, 3), np.int32)
        ma, nt = C.c_int64(0), C.c_int64(0)
        st = self.lib.rama_oracle_triangulate(
            C.c_int32(n), C.c_int64(i.size), _ptr(i), _ptr(j), _ptr(c), C.c_int32(lmax), ptrs, cnts,
            _ptr(ia), _ptr(ja), _ptr(ca), C.byref(ma), _ptr(tn), _ptr(te), C.byref(nt))
        if st != OK:
            raise OracleError(st, "triangulate")
        return (ia[:ma.value].copy(), ja[:ma.value].copy(), ca[:ma.value].copy(),
                tn[:nt.value].copy(), te[:nt.value].copy())

    # -- a3 -----------------------------------------------------------------------------------
    def min_marginal(self, ct, slot):
        ct = _f32(ct)
        return self.lib.rama_oracle_min_marginal(_ptr(ct), C.c_int32(slot))

    def triangle_lb(self, ct):
        ct = _f32(ct)
        return self.lib.rama_oracle_triangle_lb(_ptr(ct))

    def mp_half_step(self, ce, tri_edge, ct, which):
        """which=0: edges->triangles, 1: triangles->edges.  Returns new (ce, ct)."""
        ce, ct, te = _f32(ce).copy(), _f32(ct).copy().reshape(-1), _i32(tri_edge).reshape(-1)
        st = self.lib.rama_oracle_mp_half_step(C.c_int64(ce.size), _ptr(ce), C.c_int64(te.size // 3),
                                               _ptr(te), _ptr(ct), C.c_int32(which))
        if st != OK:
            raise OracleError(st, "mp_half_step")
        return ce, ct.reshape(-1, 3)

    def lower_bound(self, ce, ct):
        ce, ct = _f32(ce), _f32(ct).reshape(-1)
        return self.lib.rama_oracle_lower_bound(C.c_int64(ce.size), _ptr(ce), C.c_int64(ct.size // 3), _ptr(ct))

    def message_passing(self, n, i, j, c, cycles, k_iters, trace=False):
        i, j, c = _i32(i), _i32(j), _f32(c)
        lmax, arrs, ptrs, cnts = self._lists(cycles)
        room = i.size + sum(k * a.shape[0] for k, a in enumerate(arrs))
        io, jo, co = np.empty(room, np.int32), np.empty(room, np.int32), np.empty(room, np.float32)
        mo, lb = C.c_int64(0), C.c_double(0.0)
        tr = np.zeros(k_iters + 1, np.float64) if trace else None
        st = self.lib.rama_oracle_message_passing(
            C.c_int32(n), C.c_int64(i.size), _ptr(i), _ptr(j), _ptr(c), C.c_int32(lmax), ptrs, cnts,
            C.c_int32(k_iters), C.c_int64(room), _ptr(io), _ptr(jo), _ptr(co), C.byref(mo), C.byref(lb), _ptr(tr))
        if st != OK:
            raise OracleError(st, "message_passing")
        k = mo.value
        return dict(i=io[:k].copy(), j=jo[:k].copy(), c=co[:k].copy(), lower_bound=lb.value, lb_trace=tr)

    def dual_rounds(self, n, i, j, c, max_cycle_len=5, k_iters=10, dual_rounds=1, shortest_only=False,
                    want_triangles=False):
        """Separation + k message-passing iterations, repeated dual_rounds times on the same graph."""
        i, j, c = _i32(i), _i32(j), _f32(c)
        lb = C.c_double(0.0)
        tr = np.zeros(dual_rounds + 1, np.float64)
        room = max(i.size, 1)
        tcap = 0
        while True:     # the sizes are only known afterwards: grow and repeat on a capacity miss
            io, jo, co = np.empty(room, np.int32), np.empty(room, np.int32), np.empty(room, np.float32)
            tn, ct = np.empty((max(tcap, 1), 3), np.int32), np.empty((max(tcap, 1), 3), np.float32)
            mo, nt = C.c_int64(0), C.c_int64(0)
            st = self.lib.rama_oracle_dual_rounds(
                C.c_int32(n), C.c_int64(i.size), _ptr(i), _ptr(j), _ptr(c), C.c_int32(max_cycle_len),
                C.c_int32(int(shortest_only)), C.c_int32(k_iters), C.c_int32(dual_rounds), C.c_int64(room),
                _ptr(io), _ptr(jo), _ptr(co), C.byref(mo), C.byref(lb), _ptr(tr),
                C.c_int64(tcap), _ptr(tn), _ptr(ct), C.byref(nt))
            if st == ERR_CAP or (st == OK and want_triangles and nt.value > tcap):
                room, tcap = max(room, mo.value), nt.value if want_triangles else 0
                continue
            if st != OK:
                raise OracleError(st, "dual_rounds")
            break
        k = mo.value
        out = dict(i=io[:k].copy(), j=jo[:k].copy(), c=co[:k].copy(), lower_bound=lb.value, lb_trace=tr,
                   n_triangles=nt.value)
        if want_triangles:
            out["tri_nodes"], out["ct"] = tn[:nt.value].copy(), ct[:nt.value].copy()
        return out

    # -- a4 / a5 / a6 -------------------------------------------------------------------------
    def matching(self, n, i, j, c, tau=0.0, rounds_cap=32):
        """Input must be canonical.  Returns mate[n]."""
        i, j, c = _i32(i), _i32(j), _f32(c)
        mate = np.empty(n, np.int32)
        r = self.lib.rama_oracle_matching(C.c_int32(n), C.c_int64(i.size), _ptr(i), _ptr(j), _ptr(c),
                                          C.c_float(tau), C.c_int32(rounds_cap), _ptr(mate))
        if r < 0:
            raise OracleError(r, "matching")
        return mate

    def forest_set(self, n, i, j, c, tau=0.0):
        """Input must be canonical.  Returns (in_forest[m], removed[m], S as (si, sj))."""
        i, j, c = _i32(i), _i32(j), _f32(c)
        inf, rem = np.zeros(max(i.size, 1), np.uint8), np.zeros(max(i.size, 1), np.uint8)
        si, sj = np.empty(n + 1, np.int32), np.empty(n + 1, np.int32)
        self.lib.rama_oracle_forest_set.restype = C.c_int64
        ns = self.lib.rama_oracle_forest_set(C.c_int32(n), C.c_int64(i.size), _ptr(i), _ptr(j), _ptr(c), C.c_float(tau),
                                             _ptr(inf), _ptr(rem), _ptr(si), _ptr(sj))
        if ns < 0:
            raise OracleError(ns, "forest_set")
        return inf[:i.size].astype(bool), rem[:i.size].astype(bool), si[:ns].copy(), sj[:ns].copy()

    def components(self, n, si, sj):
        si, sj = _i32(si), _i32(sj)
        rep, fmap = np.empty(n, np.int32), np.empty(n, np.int32)
        nn = C.c_int32(0)
        st = self.lib.rama_oracle_components(C.c_int32(n), C.c_int64(si.size), _ptr(si), _ptr(sj),
                                             _ptr(rep), _ptr(fmap), C.byref(nn))
        if st != OK:
            raise OracleError(st, "components")
        return rep, fmap, nn.value

    def contract_with_mapping(self, n, i, j, c, fmap, n_new):
        i, j, c, fmap = _i32(i), _i32(j), _f32(c), _i32(fmap)
        m = i.size
        io, jo, co = np.empty(m, np.int32), np.empty(m, np.int32), np.empty(m, np.float32)
        diag = np.empty(n_new, np.float32)
        mo = C.c_int64(0)
        st = self.lib.rama_oracle_contract_with_mapping(
            C.c_int32(n), C.c_int64(m), _ptr(i), _ptr(j), _ptr(c), _ptr(fmap), C.c_int32(n_new),
            _ptr(io), _ptr(jo), _ptr(co), C.byref(mo), _ptr(diag))
        if st != OK:
            raise OracleError(st, "contract_with_mapping")
        k = mo.value
        return io[:k].copy(), jo[:k].copy(), co[:k].copy(), diag

    def contract(self, n, i, j, c, tau=0.0, rounds_cap=32, repeat=1, forest_ratio=0.1):
        i, j, c = _i32(i), _i32(j), _f32(c)
        m = max(i.size, 1)
        mapping = np.empty(n, np.int32)
        io, jo, co = np.empty(m, np.int32), np.empty(m, np.int32), np.empty(m, np.float32)
        diag = np.zeros(max(n, 1), np.float32)
        nn, mo = C.c_int32(0), C.c_int64(0)
        st = self.lib.rama_oracle_contract(
            C.c_int32(n), C.c_int64(i.size), _ptr(i), _ptr(j), _ptr(c), C.c_float(tau), C.c_int32(rounds_cap),
            C.c_float(forest_ratio), C.c_int32(repeat), _ptr(mapping), _ptr(io), _ptr(jo), _ptr(co), _ptr(diag), C.byref(nn), C.byref(mo))
        if st != OK:
            raise OracleError(st, "contract")
        k = mo.value
        return dict(mapping=mapping, i=io[:k].copy(), j=jo[:k].copy(), c=co[:k].copy(),
                    diag=diag[:nn.value].copy(), n_nodes=nn.value)

    # -- objective + driver -------------------------------------------------------------------
    def multicut_cost(self, i, j, c, labels):
        i, j, c, labels = _i32(i), _i32(j), _f32(c), _i32(labels)
        return self.lib.rama_oracle_multicut_cost(C.c_int64(i.size), _ptr(i), _ptr(j), _ptr(c), _ptr(labels))

    def solve(self, n, i, j, c, max_cycle_len_first=5, max_cycle_len_later=3, mp_iters_first=10,
              mp_iters_later=5, matching_rounds_cap=32, tau=0.0, max_rounds=0, forest_ratio=0.1,
              shortest_only=False, dual_rounds=1):
        i, j, c = _i32(i), _i32(j), _f32(c)
        labels = np.empty(n, np.int32)
        primal, lb = C.c_double(0.0), C.c_double(0.0)
        stats = (C.c_int64 * 16)()
        st = self.lib.rama_oracle_solve(
            C.c_int32(n), C.c_int64(i.size), _ptr(i), _ptr(j), _ptr(c),
            C.c_int32(max_cycle_len_first), C.c_int32(max_cycle_len_later), C.c_int32(int(shortest_only)),
            C.c_int32(dual_rounds), C.c_int32(mp_iters_first), C.c_int32(mp_iters_later),
            C.c_int32(matching_rounds_cap), C.c_float(tau), C.c_float(forest_ratio), C.c_int32(max_rounds),
            _ptr(labels), C.byref(primal), C.byref(lb), stats)
        if st != OK:
            raise OracleError(st, "solve")
        return dict(labels=labels, primal=primal.value, lower_bound=lb.value, rounds=int(stats[0]),
                    n_clusters=int(stats[1]), n_cycles_first=[int(stats[5 + q]) for q in range(MAX_CYCLE_LEN - 2)],
                    n_edges_aug_first=int(stats[3]), n_edges_final=int(stats[4]))
