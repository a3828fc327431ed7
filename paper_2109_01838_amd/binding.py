"""Thin ctypes binding of librama_hip.so (include/rama.h).  Argument marshalling only: torch
supplies device memory (inputs, outputs and -- through the allocator callbacks of rama_create --
the library's workspace, which so lives in torch's caching allocator) and the stream; every step
of the method runs inside the library.

There is no CPU fallback: if the library is missing or no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "librama_hip.so")

RAMA_OK, RAMA_ERR_INVALID_ARG, RAMA_ERR_BAD_GRAPH, RAMA_ERR_CAPACITY, RAMA_ERR_OOM, RAMA_ERR_HIP = 0, -1, -2, -3, -4, -5

EXPORTS = [
    "rama_create", "rama_destroy", "rama_last_error", "rama_params_default", "rama_workspace_bytes",
    "rama_round_count", "rama_round_get",
    "rama_profile_enable", "rama_profile_count", "rama_profile_get", "rama_set_sort_split", "rama_set_cycle_search",
    "rama_find_conflicted_cycles", "rama_message_passing", "rama_dual_rounds", "rama_contract", "rama_solve",
    "rama_solve_static",
]
STATIC_MAX_NODES, STATIC_MAX_EDGES = 1 << 17, 1 << 18   # RAMA_STATIC_MAX_* of include/rama.h


MAX_CYCLE_LEN = 7   # RAMA_MAX_CYCLE_LEN of include/rama.h


class RamaParams(C.Structure):
    _fields_ = [
        ("max_cycle_len_first", C.c_int32), ("max_cycle_len_later", C.c_int32),
        ("mp_iters_first", C.c_int32), ("mp_iters_later", C.c_int32),
        ("matching_rounds_cap", C.c_int32), ("contract_threshold", C.c_float),
        ("forest_ratio", C.c_float), ("max_rounds", C.c_int32), ("shortest_cycles_only", C.c_int32),
        ("dual_rounds", C.c_int32),
    ]


class RamaStats(C.Structure):
    _fields_ = [
        ("rounds", C.c_int32), ("n_clusters", C.c_int32), ("n_cycles_first", C.c_int64 * (MAX_CYCLE_LEN - 2)),
        ("n_triangles_first", C.c_int64), ("n_edges_aug_first", C.c_int64), ("n_edges_final", C.c_int64),
        ("ms_total", C.c_double), ("ms_cycles", C.c_double), ("ms_dual", C.c_double),
        ("ms_contract", C.c_double), ("ms_other", C.c_double),
    ]


class RamaRoundStats(C.Structure):
    _fields_ = [
        ("n_nodes", C.c_int32), ("used_forest", C.c_int32), ("n_edges", C.c_int64),
        ("n_attractive", C.c_int64), ("n_repulsive", C.c_int64), ("n_cycles", C.c_int64 * (MAX_CYCLE_LEN - 2)),
        ("n_triangles", C.c_int64), ("n_edges_aug", C.c_int64), ("n_contracted", C.c_int64),
        ("workspace_peak", C.c_int64),
        ("ms_cycles", C.c_double), ("ms_dual", C.c_double), ("ms_contract", C.c_double),
    ]


ALLOC_FN = C.CFUNCTYPE(C.c_void_p, C.c_void_p, C.c_size_t)
FREE_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p)


class RamaAlloc(C.Structure):
    _fields_ = [("alloc", ALLOC_FN), ("free", FREE_FN), ("user", C.c_void_p)]


class RamaError(RuntimeError):
    def __init__(self, status, where, msg):
        super().__init__(f"{where} failed with status {status}: {msg}")
        self.status = status


_lib = None


def load_library():
    """Load librama_hip.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    # torch ships its own HIP runtime (same soname as ROCm's).  Import torch first so that the
    # library binds to that one runtime; loaded the other way round the process ends up with two
    # runtimes and torch's streams and pointers mean nothing to the library.
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2109_01838_amd.build` "
                           "(or __graft_entry__.build()); there is no CPU fallback")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.rama_create.argtypes = [C.POINTER(vp), vp, C.POINTER(RamaAlloc)]
    lib.rama_round_count.argtypes = [vp]
    lib.rama_round_count.restype = i32
    lib.rama_round_get.argtypes = [vp, i32, C.POINTER(RamaRoundStats)]
    lib.rama_destroy.argtypes = [vp]
    lib.rama_last_error.argtypes = [vp]
    lib.rama_last_error.restype = C.c_char_p
    lib.rama_params_default.argtypes = [C.POINTER(RamaParams)]
    lib.rama_params_default.restype = None
    lib.rama_workspace_bytes.argtypes = [vp]
    lib.rama_workspace_bytes.restype = i64
    lib.rama_find_conflicted_cycles.argtypes = [vp, i32, i64, vp, vp, vp, i32, i32, C.POINTER(i64), C.POINTER(vp),
                                                C.POINTER(i64)]
    lib.rama_message_passing.argtypes = [vp, i32, i64, vp, vp, vp, i32, C.POINTER(vp), C.POINTER(i64), i32, i64,
                                         vp, vp, vp, C.POINTER(i64), C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.rama_dual_rounds.argtypes = [vp, i32, i64, vp, vp, vp, C.POINTER(RamaParams), i64, vp, vp, vp, C.POINTER(i64),
                                     C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(i64)]
    lib.rama_contract.argtypes = [vp, i32, i64, vp, vp, vp, C.POINTER(RamaParams), i32, vp, vp, vp, vp, vp,
                                  C.POINTER(i32), C.POINTER(i64)]
    lib.rama_solve.argtypes = [vp, i32, i64, vp, vp, vp, C.POINTER(RamaParams), vp, C.POINTER(C.c_double),
                               C.POINTER(C.c_double), C.POINTER(RamaStats)]
    lib.rama_solve_static.argtypes = lib.rama_solve.argtypes
    lib.rama_profile_enable.argtypes = [vp, i32, C.c_char_p]
    lib.rama_set_sort_split.argtypes = [vp, i64, i32]
    lib.rama_set_cycle_search.argtypes = [vp, i32]
    lib.rama_profile_count.argtypes = [vp]
    lib.rama_profile_count.restype = i32
    lib.rama_profile_get.argtypes = [vp, i32, C.POINTER(C.c_char_p), C.POINTER(i64), C.POINTER(C.c_double),
                                     C.POINTER(C.c_double)]
    for name in EXPORTS:
        if name not in ("rama_last_error", "rama_params_default", "rama_workspace_bytes", "rama_profile_count",
                        "rama_round_count"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def default_params(**overrides):
    p = RamaParams()
    load_library().rama_params_default(C.byref(p))
    for k, v in overrides.items():
        if not hasattr(p, k):
            raise TypeError(f"unknown parameter {k}")
        setattr(p, k, v)
    return p


def _dev(t, dtype, torch):
    if t.device.type != "cuda":
        raise ValueError("device tensors required")
    if t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"expected contiguous {dtype} tensor, got {t.dtype}")
    return t


class Rama:
    """One library context bound to the current torch device and stream.

    allocator: "torch" (default) -- the library's workspace comes from torch's caching allocator;
               "hip"             -- the library calls hipMalloc / hipFree itself;
               (alloc, free)     -- two callables, alloc(nbytes) -> device address (int) or None, free(address)
    """

    def __init__(self, device="cuda:0", allocator="torch"):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the HIP path cannot run and there is no CPU fallback")
        self.torch = torch
        self.lib = load_library()
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.stream = torch.cuda.current_stream(self.device)
        self.ctx = C.c_void_p()
        self._alloc = None
        if allocator == "torch":
            dev_index, stream = self.device.index or 0, self.stream

            def t_alloc(nbytes):
                return torch.cuda.caching_allocator_alloc(int(nbytes), dev_index, stream)

            allocator = (t_alloc, torch.cuda.caching_allocator_delete)
        if allocator != "hip":
            py_alloc, py_free = allocator

            def c_alloc(_user, nbytes):     # no exception may cross the C boundary: failure is a null pointer
                try:
                    return py_alloc(nbytes) or None
                except Exception:
                    return None

            def c_free(_user, ptr):
                try:
                    py_free(ptr)
                except Exception:
                    pass

            # the callback objects must live as long as the ctx
            self._alloc = RamaAlloc(ALLOC_FN(c_alloc), FREE_FN(c_free), None)
        st = self.lib.rama_create(C.byref(self.ctx), C.c_void_p(self.stream.cuda_stream),
                                  C.byref(self._alloc) if self._alloc is not None else None)
        if st != RAMA_OK:
            raise RamaError(st, "rama_create", "")

    def close(self):
        if self.ctx:
            self.lib.rama_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- helpers ------------------------------------------------------------------------------
    def _check(self, st, where):
        if st != RAMA_OK:
            raise RamaError(st, where, self.lib.rama_last_error(self.ctx).decode())

    def _graph(self, i, j, c):
        t = self.torch
        i = _dev(t.as_tensor(i, device=self.device), t.int32, t)
        j = _dev(t.as_tensor(j, device=self.device), t.int32, t)
        c = _dev(t.as_tensor(c, device=self.device), t.float32, t)
        if not (i.numel() == j.numel() == c.numel()):
            raise ValueError("i, j, c must have equal length")
        return i, j, c

    def _empty(self, n, dtype):
        return self.torch.empty(max(int(n), 1), dtype=dtype, device=self.device)

    def workspace_bytes(self):
        return int(self.lib.rama_workspace_bytes(self.ctx))

    def round_stats(self):
        """Per-round record of the last solve: sizes, cycles per length, triangles, |S|, stage ms."""
        out = []
        for k in range(self.lib.rama_round_count(self.ctx)):
            r = RamaRoundStats()
            self._check(self.lib.rama_round_get(self.ctx, k, C.byref(r)), "rama_round_get")
            out.append(dict(n_nodes=r.n_nodes, n_edges=r.n_edges, n_attractive=r.n_attractive, n_repulsive=r.n_repulsive,
                            n_cycles=list(r.n_cycles), n_triangles=r.n_triangles, n_edges_aug=r.n_edges_aug,
                            n_contracted=r.n_contracted, used_forest=bool(r.used_forest),
                            workspace_peak=r.workspace_peak,
                            ms=dict(cycles=r.ms_cycles, dual=r.ms_dual, contract=r.ms_contract)))
        return out

    def profile_enable(self, on=True, only=None):
        self._check(self.lib.rama_profile_enable(self.ctx, 1 if on else 0, only.encode() if only else None),
                    "rama_profile_enable")

    def set_sort_split(self, n_min, min_passes_replaced=2):
        """Arrays of at least n_min elements take the split sort (top-bit passes + one in-LDS sort)
        when that replaces at least min_passes_replaced radix passes."""
        self._check(self.lib.rama_set_sort_split(self.ctx, int(n_min), int(min_passes_replaced)), "rama_set_sort_split")

    def set_cycle_search(self, mode):
        """0: cooperative search for cycles of length 4-5 on graphs with short rows (default), 1: always the
        per-thread walk, 2: always cooperative.  The lists are the same either way."""
        self._check(self.lib.rama_set_cycle_search(self.ctx, int(mode)), "rama_set_cycle_search")

    def profile_get(self):
        """Per-kernel totals since profiling was enabled: name, launches, ms, algorithmic bytes."""
        self.torch.cuda.synchronize()
        out = []
        for k in range(self.lib.rama_profile_count(self.ctx)):
            name, n, ms, by = C.c_char_p(), C.c_int64(0), C.c_double(0.0), C.c_double(0.0)
            self._check(self.lib.rama_profile_get(self.ctx, k, C.byref(name), C.byref(n), C.byref(ms), C.byref(by)),
                        "rama_profile_get")
            out.append(dict(name=name.value.decode(), launches=n.value, ms=ms.value, bytes=by.value))
        return out

    # -- entry points ---------------------------------------------------------------------------
    def find_conflicted_cycles(self, n_nodes, i, j, c, max_cycle_len=5, shortest_only=False):
        """max_cycle_len-2 device tensors; entry L-3 is [n_L, L], the conflicted L-cycles."""
        t = self.torch
        i, j, c = self._graph(i, j, c)
        nl = max_cycle_len - 2
        if nl < 1 or max_cycle_len > MAX_CYCLE_LEN:
            raise ValueError("max_cycle_len out of range")
        cnt = (C.c_int64 * nl)()
        st = self.lib.rama_find_conflicted_cycles(self.ctx, n_nodes, i.numel(), i.data_ptr(), j.data_ptr(),
                                                  c.data_ptr(), max_cycle_len, int(shortest_only), None, None, cnt)
        if st not in (RAMA_OK, RAMA_ERR_CAPACITY):
            self._check(st, "rama_find_conflicted_cycles")
        want = [cnt[k] for k in range(nl)]
        outs = [self._empty(want[k] * (k + 3), t.int32) for k in range(nl)]
        cap = (C.c_int64 * nl)(*want)
        ptrs = (C.c_void_p * nl)(*[o.data_ptr() for o in outs])
        st = self.lib.rama_find_conflicted_cycles(self.ctx, n_nodes, i.numel(), i.data_ptr(), j.data_ptr(),
                                                  c.data_ptr(), max_cycle_len, int(shortest_only), cap, ptrs, cnt)
        self._check(st, "rama_find_conflicted_cycles")
        return [outs[k][: want[k] * (k + 3)].view(-1, k + 3) for k in range(nl)]

    def message_passing(self, n_nodes, i, j, c, cycles, k_iters, trace=False):
        """cycles: list whose entry q holds the (q+3)-cycles, as returned by find_conflicted_cycles."""
        t = self.torch
        i, j, c = self._graph(i, j, c)
        cyc = [_dev(t.as_tensor(x, device=self.device).reshape(-1), t.int32, t) for x in cycles]
        nl = len(cyc)
        ncyc = [cyc[q].numel() // (q + 3) for q in range(nl)]
        cap = i.numel() + sum(q * ncyc[q] for q in range(nl))
        io, jo, co = self._empty(cap, t.int32), self._empty(cap, t.int32), self._empty(cap, t.float32)
        mo, lb = C.c_int64(0), C.c_double(0.0)
        tr = (C.c_double * (k_iters + 1))() if trace else None
        ptrs = (C.c_void_p * max(nl, 1))(*[x.data_ptr() for x in cyc])
        cnts = (C.c_int64 * max(nl, 1))(*ncyc)
        st = self.lib.rama_message_passing(self.ctx, n_nodes, i.numel(), i.data_ptr(), j.data_ptr(), c.data_ptr(),
                                           nl + 2, ptrs, cnts, k_iters, cap, io.data_ptr(), jo.data_ptr(),
                                           co.data_ptr(), C.byref(mo), C.byref(lb), tr)
        self._check(st, "rama_message_passing")
        k = mo.value
        return dict(i=io[:k], j=jo[:k], c=co[:k], lower_bound=lb.value,
                    lb_trace=None if tr is None else list(tr))

    def dual_rounds(self, n_nodes, i, j, c, params=None):
        """Separation + message passing, params.dual_rounds times on the same graph (cycle length
        params.max_cycle_len_first, params.mp_iters_first iterations per round)."""
        t = self.torch
        i, j, c = self._graph(i, j, c)
        params = params or default_params()
        mo, nt, lb = C.c_int64(0), C.c_int64(0), C.c_double(0.0)
        tr = (C.c_double * (params.dual_rounds + 1))()
        cap = i.numel()
        while True:     # the number of chords is only known afterwards: grow and repeat on a capacity miss
            io, jo, co = self._empty(cap, t.int32), self._empty(cap, t.int32), self._empty(cap, t.float32)
            st = self.lib.rama_dual_rounds(self.ctx, n_nodes, i.numel(), i.data_ptr(), j.data_ptr(), c.data_ptr(),
                                           C.byref(params), cap, io.data_ptr(), jo.data_ptr(), co.data_ptr(),
                                           C.byref(mo), C.byref(lb), tr, C.byref(nt))
            if st == RAMA_ERR_CAPACITY and mo.value > cap:
                cap = mo.value
                continue
            self._check(st, "rama_dual_rounds")
            break
        k = mo.value
        return dict(i=io[:k], j=jo[:k], c=co[:k], lower_bound=lb.value, lb_trace=list(tr), n_triangles=nt.value)

    def contract(self, n_nodes, i, j, c, params=None, repeat=1, want_diag=True):
        t = self.torch
        i, j, c = self._graph(i, j, c)
        params = params or default_params()
        m = i.numel()
        mapping = self._empty(n_nodes, t.int32)
        io, jo, co = self._empty(m, t.int32), self._empty(m, t.int32), self._empty(m, t.float32)
        diag = self._empty(n_nodes, t.float32) if want_diag else None
        nn, mo = C.c_int32(0), C.c_int64(0)
        st = self.lib.rama_contract(self.ctx, n_nodes, m, i.data_ptr(), j.data_ptr(), c.data_ptr(), C.byref(params),
                                    repeat, mapping.data_ptr(), io.data_ptr(), jo.data_ptr(), co.data_ptr(),
                                    diag.data_ptr() if want_diag else None, C.byref(nn), C.byref(mo))
        self._check(st, "rama_contract")
        k = mo.value
        return dict(mapping=mapping[:n_nodes], i=io[:k], j=jo[:k], c=co[:k],
                    diag=diag[: nn.value] if want_diag else None, n_nodes=nn.value)

    def solve(self, n_nodes, i, j, c, params=None, static=False, labels=None):
        """static=True: rama_solve_static (workspace from the library's static device array, no allocation
        inside the call; the caller may hand in the labels tensor so that this wrapper allocates nothing either)."""
        t = self.torch
        i, j, c = self._graph(i, j, c)
        params = params or default_params()
        if labels is None:
            labels = self._empty(n_nodes, t.int32)
        primal, lb = C.c_double(0.0), C.c_double(0.0)
        stats = RamaStats()
        fn, name = (self.lib.rama_solve_static, "rama_solve_static") if static else (self.lib.rama_solve, "rama_solve")
        st = fn(self.ctx, n_nodes, i.numel(), i.data_ptr(), j.data_ptr(), c.data_ptr(),
                C.byref(params), labels.data_ptr(), C.byref(primal), C.byref(lb), C.byref(stats))
        self._check(st, name)
        return dict(labels=labels[:n_nodes], primal=primal.value, lower_bound=lb.value,
                    rounds=stats.rounds, n_clusters=stats.n_clusters,
                    n_cycles_first=list(stats.n_cycles_first), n_triangles_first=stats.n_triangles_first,
                    n_edges_aug_first=stats.n_edges_aug_first, n_edges_final=stats.n_edges_final,
                    ms=dict(total=stats.ms_total, cycles=stats.ms_cycles, dual=stats.ms_dual,
                            contract=stats.ms_contract, other=stats.ms_other))
