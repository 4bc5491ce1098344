"""ctypes access to the CPU oracle (oracle/dagsched_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
CPU-baseline leg.  The product package never imports this module.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading
from typing import Optional, Tuple

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "dagsched_oracle.c")
_LIB = os.path.join(_DIR, "libdagsched_oracle.so")

OK, EINVAL, ECYCLE, EOVERFLOW, ENOMEM = 0, -1, -2, -3, -4
FLAG_CYCLIC, FLAG_BAD_PLACEMENT, FLAG_BAD_RANK, FLAG_OVER_MEMORY, FLAG_NO_CHANNEL = 1, 2, 4, 16, 32
NO_CHANNEL = -1      # off-diagonal comm entry of a machine pair without a channel (eq. (10))
CAND_MAJOR, CAND_MINOR = 0, 1

_lib = None


def build() -> str:
    """gcc -> oracle/libdagsched_oracle.so (always recompiles)."""
    tmp = _LIB + ".tmp"
    proc = subprocess.run(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra", _SRC, "-o", tmp],
                          stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("oracle build failed:\n" + proc.stdout)
    os.replace(tmp, _LIB)
    build_coarsen()
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
            build()
        lib = ctypes.CDLL(_LIB)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        lib.dagsched_oracle_check_problem.restype = ctypes.c_int
        lib.dagsched_oracle_check_problem.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp]
        lib.dagsched_oracle_evaluate_mem.restype = ctypes.c_int
        lib.dagsched_oracle_evaluate_mem.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, i32, i64, vp, vp,
                                                     i64, i64, vp, vp, vp, vp]
        lib.dagsched_oracle_schedule_mem.restype = ctypes.c_int
        lib.dagsched_oracle_schedule_mem.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.dagsched_oracle_evaluate_contended.restype = ctypes.c_int
        lib.dagsched_oracle_evaluate_contended.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, i32, i64, vp, vp, vp,
                                                           i64, i64, vp, vp, vp, vp, vp, vp, vp]
        _lib = lib
    return _lib


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


def _ptr(a):
    return a.ctypes.data if a.size else None


class Problem:
    """The candidate-independent part: DAG CSR, durations, comm matrix, memory deltas, and optionally the
    static memory W_i of every operation (eq. (16)) and the memory limit of every machine."""

    def __init__(self, n_devices, row_ptr, col_idx, dur, comm, mem_delta, weight=None, mem_limit=None):
        self.P = int(n_devices)
        self.row_ptr = _c(row_ptr, np.int32)
        self.col_idx = _c(col_idx, np.int32)
        self.dur = _c(dur, np.int32)
        self.comm = _c(comm, np.int32).reshape(-1)
        self.mem_delta = _c(mem_delta, np.int64)
        self.N = len(self.row_ptr) - 1
        self.E = len(self.col_idx)
        self.weight = None if weight is None else _c(weight, np.int64)
        self.mem_limit = None if mem_limit is None else _c(mem_limit, np.int64)
        assert self.weight is None or self.weight.shape == (self.N,)
        assert self.mem_limit is None or self.mem_limit.shape == (self.P,)

    @classmethod
    def of(cls, w) -> "Problem":
        return cls(w.n_devices, w.row_ptr, w.col_idx, w.dur, w.comm, w.mem_delta,
                   getattr(w, "weight", None), getattr(w, "mem_limit", None))

    def _mem(self):
        return (None if self.weight is None else _ptr(self.weight),
                None if self.mem_limit is None else _ptr(self.mem_limit))

    def _head(self):
        return (self.N, self.E, self.P, _ptr(self.row_ptr), _ptr(self.col_idx), _ptr(self.dur),
                _ptr(self.comm), _ptr(self.mem_delta))

    def check(self) -> int:
        return _load().dagsched_oracle_check_problem(*self._head())

    def evaluate(self, placement, rank, layout: int = CAND_MAJOR, threads: int = 1
                 ) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
        """-> (makespan int32 [C], bubble int64 [C], peak_mem int64 [C,P] or [P,C], flags int32 [C]).

        ``threads`` > 1 only fans contiguous candidate chunks out over Python threads (the C call
        releases the GIL); every chunk runs the same serial routine.
        """
        placement = _c(placement, np.int32)
        rank = _c(rank, np.int32)
        if layout == CAND_MAJOR:
            C = placement.shape[0]
            assert placement.shape == (C, self.N) and rank.shape == (C, self.N)
            peak = np.empty((C, self.P), dtype=np.int64)
        else:
            C = placement.shape[1]
            assert placement.shape == (self.N, C) and rank.shape == (self.N, C)
            peak = np.empty((self.P, C), dtype=np.int64)
        makespan = np.empty(C, dtype=np.int32)
        bubble = np.empty(C, dtype=np.int64)
        flags = np.empty(C, dtype=np.int32)
        lib = _load()
        rcs = []

        def run(first, count):
            rcs.append(lib.dagsched_oracle_evaluate_mem(*self._head(), *self._mem(), layout, C, _ptr(placement),
                                                        _ptr(rank), first, count, _ptr(makespan), _ptr(bubble),
                                                        _ptr(peak), _ptr(flags)))

        threads = max(1, min(int(threads), C if C else 1))
        if threads == 1:
            run(0, C)
        else:
            bounds = np.linspace(0, C, threads + 1).astype(np.int64)
            ts = [threading.Thread(target=run, args=(int(bounds[i]), int(bounds[i + 1] - bounds[i])))
                  for i in range(threads)]
            for t in ts:
                t.start()
            for t in ts:
                t.join()
        for rc in rcs:
            if rc != OK:
                raise OracleError(rc)
        return makespan, bubble, peak, flags

    def evaluate_contended(self, placement, rank, edge_rank, layout: int = CAND_MAJOR, threads: int = 1):
        """With channel contention (eqs. (11)-(15)): edge_rank [C, E] (or [E, C]) is the rank of every edge's transfer
        on its channel.  -> (makespan, bubble, peak_mem, flags) as evaluate."""
        placement, rank, edge_rank = _c(placement, np.int32), _c(rank, np.int32), _c(edge_rank, np.int32)
        if layout == CAND_MAJOR:
            C = placement.shape[0]
            assert placement.shape == (C, self.N) and rank.shape == (C, self.N) and edge_rank.shape == (C, self.E)
            peak = np.empty((C, self.P), dtype=np.int64)
        else:
            C = placement.shape[1]
            assert placement.shape == (self.N, C) and rank.shape == (self.N, C) and edge_rank.shape == (self.E, C)
            peak = np.empty((self.P, C), dtype=np.int64)
        makespan, bubble, flags = np.empty(C, np.int32), np.empty(C, np.int64), np.empty(C, np.int32)
        lib = _load()
        rcs = []

        def run(first, count):
            rcs.append(lib.dagsched_oracle_evaluate_contended(
                *self._head(), *self._mem(), layout, C, _ptr(placement), _ptr(rank), _ptr(edge_rank), first, count,
                _ptr(makespan), _ptr(bubble), _ptr(peak), _ptr(flags), None, None, None))

        threads = max(1, min(int(threads), C if C else 1))
        bounds = np.linspace(0, C, threads + 1).astype(np.int64)
        ts = [threading.Thread(target=run, args=(int(bounds[i]), int(bounds[i + 1] - bounds[i]))) for i in range(threads)]
        for t in ts:
            t.start()
        for t in ts:
            t.join()
        for rc in rcs:
            if rc != OK:
                raise OracleError(rc)
        return makespan, bubble, peak, flags

    def schedule_contended(self, placement, rank, edge_rank):
        """One candidate with channel contention -> (flag, makespan, start [N], end [N], transfer_end [E]; -1 for
        edges inside a machine); the arrays are valid when the flag is 0 or OVER_MEMORY."""
        placement, rank = _c(placement, np.int32).reshape(1, -1), _c(rank, np.int32).reshape(1, -1)
        edge_rank = _c(edge_rank, np.int32).reshape(1, -1)
        assert placement.shape == (1, self.N) and rank.shape == (1, self.N) and edge_rank.shape == (1, self.E)
        z, b, f = np.empty(1, np.int32), np.empty(1, np.int64), np.empty(1, np.int32)
        peak = np.empty((1, self.P), np.int64)
        start, end, t_end = np.zeros(self.N, np.int64), np.zeros(self.N, np.int64), np.zeros(max(self.E, 1), np.int64)
        rc = _load().dagsched_oracle_evaluate_contended(
            *self._head(), *self._mem(), CAND_MAJOR, 1, _ptr(placement), _ptr(rank), _ptr(edge_rank), 0, 1,
            _ptr(z), _ptr(b), _ptr(peak), _ptr(f), _ptr(start), _ptr(end), _ptr(t_end))
        if rc != OK:
            raise OracleError(rc)
        return int(f[0]), int(z[0]), start, end, t_end[:self.E]

    def schedule(self, placement, rank):
        """One candidate -> (flag, start, end, m_minus, m_plus); arrays valid when flag == 0."""
        placement = _c(placement, np.int32).reshape(-1)
        rank = _c(rank, np.int32).reshape(-1)
        assert placement.shape == (self.N,) and rank.shape == (self.N,)
        out = [np.zeros(self.N, dtype=np.int64) for _ in range(4)]
        rc = _load().dagsched_oracle_schedule_mem(*self._head(), self._mem()[0], _ptr(placement), _ptr(rank),
                                                  *[_ptr(o) for o in out])
        if rc < 0:
            raise OracleError(rc)
        return (rc, *out)


class OracleError(RuntimeError):
    def __init__(self, code: int):
        super().__init__("oracle returned %d" % code)
        self.code = code


def evaluate_workload(w, layout: int = CAND_MAJOR, threads: int = 1):
    """Convenience: evaluate every candidate of a workload object (candidate-major arrays)."""
    prob = Problem.of(w)
    if layout == CAND_MAJOR:
        return prob.evaluate(w.placement, w.rank, layout, threads)
    return prob.evaluate(np.ascontiguousarray(w.placement.T), np.ascontiguousarray(w.rank.T), layout, threads)


# --------------------------------------------------------------------------- graph coarsening (Sec. IV, Alg. 1)

_CO_SRC = os.path.join(_DIR, "coarsen_oracle.c")
_CO_LIB = os.path.join(_DIR, "libcoarsen_oracle.so")
_co_lib = None


def build_coarsen() -> str:
    """gcc -> oracle/libcoarsen_oracle.so (always recompiles)."""
    tmp = _CO_LIB + ".tmp"
    proc = subprocess.run(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra", _CO_SRC, "-o", tmp],
                          stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("coarsening oracle build failed:\n" + proc.stdout)
    os.replace(tmp, _CO_LIB)
    return _CO_LIB


NO_MERGES = -1       # a threshold that no pair passes (sums are never negative)
NO_LIMIT = 2 ** 62


def coarsen(row_ptr, col_idx, dur, mem_delta, mem_req=None, target=1, edge_dur_max=NO_LIMIT, edge_mem_max=NO_LIMIT,
            nonedge_dur_max=NO_LIMIT, nonedge_mem_max=NO_LIMIT):
    """Alg. 1 -> dict(n_coarse, node_map [N], row_ptr, col_idx, dur, mem_delta, mem_req, merges_edge, merges_nonedge)."""
    global _co_lib
    if _co_lib is None:
        if not os.path.exists(_CO_LIB) or os.path.getmtime(_CO_LIB) < os.path.getmtime(_CO_SRC):
            build_coarsen()
        _co_lib = ctypes.CDLL(_CO_LIB)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        _co_lib.coarsen_oracle.restype = ctypes.c_int
        _co_lib.coarsen_oracle.argtypes = [i32, i32, vp, vp, vp, vp, vp, i32, i64, i64, i64, i64] + [vp] * 9
    rp, ci = _c(row_ptr, np.int32), _c(col_idx, np.int32)
    n, e = len(rp) - 1, len(ci)
    d, m = _c(dur, np.int64), _c(mem_delta, np.int64)
    r = None if mem_req is None else _c(mem_req, np.int64)
    assert d.shape == (n,) and m.shape == (n,) and (r is None or r.shape == (n,))
    n_coarse, me, mn = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    node_map = np.empty(n, np.int32)
    c_rp, c_ci = np.empty(n + 1, np.int32), np.empty(max(e, 1), np.int32)
    c_d, c_m, c_r = np.empty(n, np.int64), np.empty(n, np.int64), np.empty(n, np.int64)
    rc = _co_lib.coarsen_oracle(n, e, _ptr(rp), _ptr(ci), _ptr(d), _ptr(m), None if r is None else _ptr(r), int(target),
                                int(edge_dur_max), int(edge_mem_max), int(nonedge_dur_max), int(nonedge_mem_max),
                                ctypes.addressof(n_coarse), _ptr(node_map), _ptr(c_rp), _ptr(c_ci), _ptr(c_d), _ptr(c_m),
                                _ptr(c_r), ctypes.addressof(me), ctypes.addressof(mn))
    if rc != OK:
        raise OracleError(rc)
    k = n_coarse.value
    return dict(n_coarse=k, node_map=node_map, row_ptr=c_rp[:k + 1].copy(), col_idx=c_ci[:c_rp[k]].copy(),
                dur=c_d[:k].copy(), mem_delta=c_m[:k].copy(), mem_req=c_r[:k].copy(),
                merges_edge=me.value, merges_nonedge=mn.value)
