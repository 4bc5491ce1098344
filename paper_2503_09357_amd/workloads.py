"""Seeded synthetic workloads: operator DAGs plus batches of candidate schedules.

This module only *draws inputs*.  It contains none of the evaluator's arithmetic (no
start/end times, makespans, bubbles or memory levels), so the CPU oracle and the HIP path can
both consume its arrays without sharing any of the method's code.

Vocabulary (Sec. III, notation table): the operator DAG G_m(I, B) is given as a successor CSR
(``row_ptr``, ``col_idx``); ``dur`` is D^o_i; ``comm[a, b]`` is the communication duration
D^c on the channel from machine a to machine b (machine-dimension form, footnote of Sec. III);
``mem_delta`` is A_i; a *candidate* fixes the allocation x (``placement[c, i]``, eq. (6)) and
the per-machine total orders y/u (``rank[c, i]`` = position of i on its machine, eqs. (7)-(8)).

The five named configurations stand in for the paper's pipeline (DualPipe experiments,
Sec. V-A) and random-graph (Sec. V-B) workloads, which are not published as data.
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import _build

MASTER_SEED = 20250309

_gen_lib = None


def _gen():
    global _gen_lib
    if _gen_lib is None:
        lib = ctypes.CDLL(_build.ensure_workload_gen())
        fn = lib.dagsched_workload_list_schedules
        fn.restype = ctypes.c_int
        fn.argtypes = [ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                       ctypes.c_int64, ctypes.c_int64, ctypes.c_uint64,
                       ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                       ctypes.c_void_p, ctypes.c_void_p]
        _gen_lib = lib
    return _gen_lib


@dataclass
class Workload:
    name: str
    n_devices: int
    row_ptr: np.ndarray      # int32 [N+1]
    col_idx: np.ndarray      # int32 [E]
    dur: np.ndarray          # int32 [N]
    comm: np.ndarray         # int32 [P, P]
    mem_delta: np.ndarray    # int64 [N]
    placement: np.ndarray    # int32 [C, N]
    rank: np.ndarray         # int32 [C, N]
    meta: Dict = field(default_factory=dict)
    weight: Optional[np.ndarray] = None      # int64 [N] static memory per operation, or None
    mem_limit: Optional[np.ndarray] = None   # int64 [P] memory limit per machine, or None

    @property
    def n_nodes(self) -> int:
        return int(self.dur.shape[0])

    @property
    def n_edges(self) -> int:
        return int(self.col_idx.shape[0])

    @property
    def n_cand(self) -> int:
        return int(self.placement.shape[0])


# ----------------------------------------------------------------------------- helpers

def csr_from_edges(n_nodes: int, src: Sequence[int], dst: Sequence[int]) -> Tuple[np.ndarray, np.ndarray]:
    """Successor CSR of the edge list (u -> v); edges keep their relative order per source."""
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    order = np.argsort(src, kind="stable")
    counts = np.bincount(src, minlength=n_nodes)
    row_ptr = np.zeros(n_nodes + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum(counts)
    return row_ptr, dst[order].astype(np.int32)


def edges_from_csr(row_ptr: np.ndarray, col_idx: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    n = len(row_ptr) - 1
    src = np.repeat(np.arange(n, dtype=np.int32), np.diff(row_ptr))
    return src, np.asarray(col_idx, dtype=np.int32)


def ranks_from_orders(n_nodes: int, orders: Sequence[Sequence[int]]) -> Tuple[np.ndarray, np.ndarray]:
    """Per-machine operation lists -> (placement[N], rank[N])."""
    placement = np.full(n_nodes, -1, dtype=np.int32)
    rank = np.full(n_nodes, -1, dtype=np.int32)
    for j, lst in enumerate(orders):
        for r, v in enumerate(lst):
            placement[v] = j
            rank[v] = r
    if (placement < 0).any():
        raise ValueError("orders do not cover every node")
    return placement, rank


def list_schedules(row_ptr: np.ndarray, col_idx: np.ndarray, n_devices: int, n_cand: int, seed: int,
                   fixed_placement: Optional[np.ndarray] = None, group: Optional[np.ndarray] = None,
                   first_cand: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Randomized list scheduling (uniform pick among ready operations), one stream per candidate.

    ``fixed_placement`` [N] pins every candidate to one placement; otherwise each candidate draws
    a machine uniformly for every value of ``group`` (operations of a group share their machine).
    """
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    n = len(row_ptr) - 1
    placement = np.empty((n_cand, n), dtype=np.int32)
    rank = np.empty((n_cand, n), dtype=np.int32)
    fp = gp = None
    n_groups = 0
    if fixed_placement is not None:
        fp = np.ascontiguousarray(fixed_placement, dtype=np.int32)
        assert fp.shape == (n,) and fp.min() >= 0 and fp.max() < n_devices
    else:
        gp = np.ascontiguousarray(np.arange(n) if group is None else group, dtype=np.int32)
        assert gp.shape == (n,) and gp.min() >= 0
        n_groups = int(gp.max()) + 1
    rc = _gen().dagsched_workload_list_schedules(
        n, row_ptr.ctypes.data, col_idx.ctypes.data if len(col_idx) else None, n_devices,
        first_cand, n_cand, seed & 0xFFFFFFFFFFFFFFFF,
        fp.ctypes.data if fp is not None else None, gp.ctypes.data if gp is not None else None, n_groups,
        placement.ctypes.data, rank.ctypes.data)
    if rc != 0:
        raise RuntimeError("candidate generator failed (cyclic DAG or bad arguments)")
    return placement, rank


# ----------------------------------------------------------------------------- pipeline DAGs

def pipeline_nodes(p: int, m: int, kinds: str) -> Dict[Tuple[str, int, int], int]:
    """Node ids in traced-program order: micro-batch major; inside a micro-batch the forward
    ops stage 0..p-1, then for stage p-1..0 the remaining kinds (B, then W if present)."""
    ids: Dict[Tuple[str, int, int], int] = {}
    nxt = 0
    back = [k for k in kinds if k != "F"]
    for k in range(m):
        for s in range(p):
            ids[("F", s, k)] = nxt
            nxt += 1
        for s in range(p - 1, -1, -1):
            for kind in back:
                ids[(kind, s, k)] = nxt
                nxt += 1
    return ids


def pipeline_dag(p: int, m: int, split_w: bool) -> Tuple[Dict, np.ndarray, np.ndarray]:
    """F/B (and W when ``split_w``) pipeline DAG over p stages and m micro-batches.

    Edges: F(s,k)->F(s+1,k); B(s+1,k)->B(s,k); F(s,k)->B(s,k); with W also B(s,k)->W(s,k).
    """
    kinds = "FBW" if split_w else "FB"
    ids = pipeline_nodes(p, m, kinds)
    src: List[int] = []
    dst: List[int] = []
    for k in range(m):
        for s in range(p):
            if s + 1 < p:
                src.append(ids[("F", s, k)]); dst.append(ids[("F", s + 1, k)])
                src.append(ids[("B", s + 1, k)]); dst.append(ids[("B", s, k)])
            src.append(ids[("F", s, k)]); dst.append(ids[("B", s, k)])
            if split_w:
                src.append(ids[("B", s, k)]); dst.append(ids[("W", s, k)])
    return ids, np.asarray(src), np.asarray(dst)


def order_1f1b(ids: Dict, p: int, m: int) -> List[List[int]]:
    """Canonical one-forward-one-backward order: stage s runs min(p-1-s, m) warm-up forwards,
    then alternates forward/backward, then drains the remaining backwards."""
    orders = []
    for s in range(p):
        w = min(p - 1 - s, m)
        lst = [ids[("F", s, k)] for k in range(w)]
        for i in range(m - w):
            lst.append(ids[("F", s, w + i)])
            lst.append(ids[("B", s, i)])
        lst += [ids[("B", s, k)] for k in range(m - w, m)]
        orders.append(lst)
    return orders


def order_gpipe(ids: Dict, p: int, m: int) -> List[List[int]]:
    """All forwards in micro-batch order, then all backwards in micro-batch order."""
    return [[ids[("F", s, k)] for k in range(m)] + [ids[("B", s, k)] for k in range(m)] for s in range(p)]


def uniform_pipeline(p: int, m: int, t_f: int, t_b: int, lam: int, schedule: str = "1f1b") -> Workload:
    """One-candidate uniform pipeline used by the closed-form checks (stage s on machine s)."""
    ids, src, dst = pipeline_dag(p, m, split_w=False)
    n = 2 * p * m
    row_ptr, col_idx = csr_from_edges(n, src, dst)
    dur = np.zeros(n, dtype=np.int32)
    mem = np.zeros(n, dtype=np.int64)
    for (kind, s, k), v in ids.items():
        dur[v] = t_f if kind == "F" else t_b
        mem[v] = 1 if kind == "F" else -1
    comm = np.full((p, p), lam, dtype=np.int32)
    np.fill_diagonal(comm, 0)
    orders = order_1f1b(ids, p, m) if schedule == "1f1b" else order_gpipe(ids, p, m)
    pl, rk = ranks_from_orders(n, orders)
    return Workload("uniform-%s p=%d m=%d" % (schedule, p, m), p, row_ptr, col_idx, dur, comm, mem,
                    pl[None, :].copy(), rk[None, :].copy(), {"ids": ids, "p": p, "m": m})


# ----------------------------------------------------------------------------- the five configurations

def _cfg1(n_cand: int, seed: int) -> Workload:
    p, m = 4, 8
    rng = np.random.Generator(np.random.PCG64(seed))
    ids, src, dst = pipeline_dag(p, m, split_w=False)
    n = 2 * p * m
    row_ptr, col_idx = csr_from_edges(n, src, dst)
    dur = np.zeros(n, dtype=np.int32)
    mem = np.zeros(n, dtype=np.int64)
    fixed = np.zeros(n, dtype=np.int32)
    for (kind, s, k), v in ids.items():
        fixed[v] = s
        if kind == "F":
            dur[v] = 2 + rng.integers(0, 3)
            mem[v] = 1
        else:
            dur[v] = 4 + rng.integers(0, 5)
            mem[v] = -1
    comm = np.ones((p, p), dtype=np.int32)
    np.fill_diagonal(comm, 0)
    pl, rk = list_schedules(row_ptr, col_idx, p, n_cand, seed, fixed_placement=fixed)
    # candidate 0: the canonical 1F1B order, as an anchor
    pl0, rk0 = ranks_from_orders(n, order_1f1b(ids, p, m))
    pl[0], rk[0] = pl0, rk0
    return Workload("cfg1 1F1B pipeline p=4 m=8", p, row_ptr, col_idx, dur, comm, mem, pl, rk,
                    {"ids": ids, "p": p, "m": m})


def _cfg2(n_cand: int, seed: int) -> Workload:
    p, m = 8, 32
    rng = np.random.Generator(np.random.PCG64(seed))
    ids, src, dst = pipeline_dag(p, m, split_w=True)
    n = 3 * p * m
    row_ptr, col_idx = csr_from_edges(n, src, dst)
    dur = np.zeros(n, dtype=np.int32)
    mem = np.zeros(n, dtype=np.int64)
    fixed = np.zeros(n, dtype=np.int32)
    for (kind, s, k), v in ids.items():
        fixed[v] = s
        if kind == "W":
            dur[v] = rng.integers(2, 5)
            mem[v] = -1
        else:
            dur[v] = rng.integers(3, 7)
            mem[v] = 2 if kind == "F" else -1
    comm = np.zeros((p, p), dtype=np.int32)
    for a in range(p):
        for b in range(a + 1, p):
            comm[a, b] = comm[b, a] = rng.integers(1, 4)
    pl, rk = list_schedules(row_ptr, col_idx, p, n_cand, seed, fixed_placement=fixed)
    # ~1% of the candidates are made cyclic on purpose: swapping the ranks of F(s,k) and
    # B(s,k) (same machine) makes the chain run B before F while the DAG says F -> B.
    cyc = np.nonzero(rng.random(n_cand) < 0.01)[0]
    ss = rng.integers(0, p, size=len(cyc))
    kk = rng.integers(0, m, size=len(cyc))
    for c, s, k in zip(cyc, ss, kk):
        f, b = ids[("F", int(s), int(k))], ids[("B", int(s), int(k))]
        rk[c, f], rk[c, b] = rk[c, b], rk[c, f]
    return Workload("cfg2 zero-bubble-style pipeline p=8 m=32", p, row_ptr, col_idx, dur, comm, mem, pl, rk,
                    {"ids": ids, "p": p, "m": m, "cyclic": cyc})


def _cfg3(n_cand: int, seed: int) -> Workload:
    p, m = 16, 64
    rng = np.random.Generator(np.random.PCG64(seed))
    per_mb = 6 * p
    n = per_mb * m

    def nid(kind: str, s: int, k: int) -> int:
        if kind == "F":
            off = 2 * s
        elif kind == "CF":
            off = 2 * s + 1
        else:
            off = 2 * p + 4 * (p - 1 - s) + {"B": 0, "CB": 1, "W": 2, "CW": 3}[kind]
        return k * per_mb + off

    src: List[int] = []
    dst: List[int] = []
    fixed = np.zeros(n, dtype=np.int32)
    mem = np.zeros(n, dtype=np.int64)
    for k in range(m):
        for s in range(p):
            dev = s if k < m // 2 else p - 1 - s
            for kind in ("F", "CF", "B", "CB", "W", "CW"):
                fixed[nid(kind, s, k)] = dev
            a = int(rng.integers(1, 4))
            mem[nid("F", s, k)] = a
            mem[nid("W", s, k)] = -a
            src += [nid("F", s, k), nid("F", s, k), nid("B", s, k), nid("B", s, k), nid("W", s, k)]
            dst += [nid("CF", s, k), nid("B", s, k), nid("CB", s, k), nid("W", s, k), nid("CW", s, k)]
            if s + 1 < p:
                src += [nid("CF", s, k), nid("CB", s + 1, k)]
                dst += [nid("F", s + 1, k), nid("B", s, k)]
    row_ptr, col_idx = csr_from_edges(n, src, dst)
    dur = rng.integers(2, 9, size=n).astype(np.int32)
    comm = rng.integers(1, 5, size=(p, p)).astype(np.int32)
    np.fill_diagonal(comm, 0)
    pl, rk = list_schedules(row_ptr, col_idx, p, n_cand, seed, fixed_placement=fixed)
    return Workload("cfg3 bidirectional pipeline P=16 m=64", p, row_ptr, col_idx, dur, comm, mem, pl, rk,
                    {"p": p, "m": m})


def _cfg4(n_cand: int, seed: int) -> Workload:
    layers, mbs, roles, p = 61, 8, 12, 32      # roles: A, G, D, X0..X7, M
    A, G, D, X0, M = 0, 1, 2, 3, 11
    rng = np.random.Generator(np.random.PCG64(seed))
    per_dir = layers * roles
    per_mb = 2 * per_dir
    n = per_mb * mbs

    def fwd(l: int, r: int, k: int) -> int:
        return k * per_mb + l * roles + r

    def bwd(l: int, r: int, k: int) -> int:      # traced backward order: last layer first, roles reversed
        return k * per_mb + per_dir + (layers - 1 - l) * roles + (roles - 1 - r)

    fe: List[Tuple[Tuple[int, int], Tuple[int, int]]] = []   # forward edges on (layer, role)
    for l in range(layers):
        fe.append(((l, A), (l, G)))
        fe.append(((l, G), (l, D)))
        for e in range(8):
            fe.append(((l, D), (l, X0 + e)))
            fe.append(((l, X0 + e), (l, M)))
        fe.append(((l, A), (l, M)))
        if l + 1 < layers:
            fe.append(((l, M), (l + 1, A)))
    src: List[int] = []
    dst: List[int] = []
    for k in range(mbs):
        for (a, b) in fe:
            src.append(fwd(a[0], a[1], k)); dst.append(fwd(b[0], b[1], k))
            src.append(bwd(b[0], b[1], k)); dst.append(bwd(a[0], a[1], k))     # mirror image
        for l in range(layers):
            for r in range(roles):
                src.append(fwd(l, r, k)); dst.append(bwd(l, r, k))             # saved activation
    row_ptr, col_idx = csr_from_edges(n, src, dst)
    # one duration per operator and direction, shared by the micro-batches
    d_op = np.maximum(1, np.rint(np.exp(1.5 + 0.5 * rng.standard_normal((2, layers, roles))))).astype(np.int32)
    dur = np.zeros(n, dtype=np.int32)
    mem = np.zeros(n, dtype=np.int64)
    group = np.zeros(n, dtype=np.int32)
    for k in range(mbs):
        for l in range(layers):
            for r in range(roles):
                f, b = fwd(l, r, k), bwd(l, r, k)
                dur[f], dur[b] = d_op[0, l, r], d_op[1, l, r]
                mem[f], mem[b] = 1, -1
                group[f] = group[b] = l * roles + r
    comm = np.full((p, p), 4, dtype=np.int32)
    for a in range(p):
        for b in range(p):
            if a // 8 == b // 8:
                comm[a, b] = 1
    np.fill_diagonal(comm, 0)
    pl, rk = list_schedules(row_ptr, col_idx, p, n_cand, seed, group=group)
    return Workload("cfg4 MoE operator DAG 61 layers x 8 micro-batches, P=32", p, row_ptr, col_idx, dur, comm, mem,
                    pl, rk, {"layers": layers, "mbs": mbs})


def _cfg5(n_cand: int, seed: int) -> Workload:
    levels, width, p, merge = 400, 125, 64, 150
    rng = np.random.Generator(np.random.PCG64(seed))
    n = levels * width
    split = 62                                  # branch 0: columns 0..61, branch 1: 62..124 (levels < merge)
    src: List[int] = []
    dst: List[int] = []
    for l in range(1, levels):
        for i in range(width):
            v = l * width + i
            fan = int(rng.integers(1, 5))
            # before the merge a node only sees its own encoder branch; from the merge on, every column
            if l < merge:
                lo, hi = (0, split) if i < split else (split, width)
            else:
                lo, hi = 0, width
            chosen: List[int] = []
            tries = 0
            while len(chosen) < fan and tries < 64:
                tries += 1
                # first predecessor from the level just above (pins the level), the rest from l-1..l-3
                p_level = l - 1 if not chosen else l - 1 - int(rng.integers(0, min(3, l)))
                u = p_level * width + int(rng.integers(lo, hi))
                if u not in chosen:                      # duplicates are re-drawn
                    chosen.append(u)
            for u in chosen:
                src.append(u); dst.append(v)
    row_ptr, col_idx = csr_from_edges(n, src, dst)
    dur = np.maximum(1, np.rint(np.exp(2.0 + 0.7 * rng.standard_normal(n)))).astype(np.int32)
    comm = rng.integers(1, 9, size=(p, p)).astype(np.int32)
    np.fill_diagonal(comm, 0)
    mem = rng.integers(-4, 5, size=n).astype(np.int64)
    pl, rk = list_schedules(row_ptr, col_idx, p, n_cand, seed, group=None)
    return Workload("cfg5 multi-modal layered DAG 50k nodes, P=64", p, row_ptr, col_idx, dur, comm, mem, pl, rk,
                    {"levels": levels, "width": width})


_CONFIGS = {1: (_cfg1, 1024), 2: (_cfg2, 65536), 3: (_cfg3, 16384), 4: (_cfg4, 4096), 5: (_cfg5, 1024)}


def config_sizes(cfg: int) -> int:
    """Full candidate count of configuration ``cfg`` (1-based)."""
    return _CONFIGS[cfg][1]


def gen_config(cfg: int, n_cand: Optional[int] = None, seed: Optional[int] = None) -> Workload:
    """Configuration ``cfg`` in 1..5; ``n_cand`` below the full count gives a prefix-consistent
    subset for the list-scheduled candidates (each candidate has its own random stream)."""
    fn, full = _CONFIGS[cfg]
    return fn(full if n_cand is None else int(n_cand), MASTER_SEED + cfg if seed is None else int(seed))


# ----------------------------------------------------------------------------- small random instances (tests)

def random_dag(rng: np.random.Generator, n: int, max_fanin: int = 3, window: Optional[int] = None,
               dup_prob: float = 0.0) -> Tuple[np.ndarray, np.ndarray]:
    """Random DAG on nodes 0..n-1 under a random relabelling; optional duplicate edges."""
    perm = rng.permutation(n)
    src: List[int] = []
    dst: List[int] = []
    for v in range(1, n):
        fan = int(rng.integers(0, max_fanin + 1))
        lo = 0 if window is None else max(0, v - window)
        for _ in range(fan):
            u = int(rng.integers(lo, v))
            src.append(int(perm[u])); dst.append(int(perm[v]))
            if dup_prob and rng.random() < dup_prob:
                src.append(int(perm[u])); dst.append(int(perm[v]))
    return csr_from_edges(n, src, dst)


def fcfs_edge_ranks(row_ptr: np.ndarray, col_idx: np.ndarray, n_devices: int, placement: np.ndarray,
                    rank: np.ndarray) -> np.ndarray:
    """Channel orders for the evaluation with contention: [C, E] int32, for every candidate and every DAG edge (in
    successor-CSR order) the rank of the edge's transfer among the transfers of its channel (the ordered pair of its
    ends' machines), first come first served: by the producer's rank on its machine, then by edge index.  The
    producers of one channel share a machine, so this order never contradicts the candidate's own orders.  Edges
    inside a machine, and edges of candidates with a placement out of range, get 0."""
    n = len(row_ptr) - 1
    e = len(col_idx)
    src = np.repeat(np.arange(n, dtype=np.int64), np.diff(row_ptr))
    dst = np.asarray(col_idx, dtype=np.int64)
    out = np.zeros((placement.shape[0], e), dtype=np.int32)
    edge_no = np.arange(e, dtype=np.int64)
    for c in range(placement.shape[0]):
        a, b = placement[c, src].astype(np.int64), placement[c, dst].astype(np.int64)
        if e == 0 or a.min() < 0 or a.max() >= n_devices or b.min() < 0 or b.max() >= n_devices:
            continue
        cross = np.nonzero(a != b)[0]
        if len(cross) == 0:
            continue
        ch = a[cross] * n_devices + b[cross]
        order = np.lexsort((edge_no[cross], rank[c, src[cross]], ch))
        ch_sorted = ch[order]
        first = np.r_[0, np.nonzero(np.diff(ch_sorted))[0] + 1]
        start_of = np.repeat(first, np.diff(np.r_[first, len(order)]))
        out[c, cross[order]] = (np.arange(len(order)) - start_of).astype(np.int32)
    return out


def random_dag_bounded_degree(rng: np.random.Generator, n: int, max_degree: int = 3, window: int = 12
                              ) -> Tuple[np.ndarray, np.ndarray]:
    """Random DAG whose in- and out-degrees are at most max_degree (the shape of the random computational graph of
    Sec. V-B: 200 operations, maximum in- and out-degree 3), under a random relabelling.  Operation v draws up to
    max_degree distinct predecessors among the `window` operations before it that still have an output to give."""
    perm = rng.permutation(n)
    out_left = np.full(n, max_degree, dtype=np.int64)
    src: List[int] = []
    dst: List[int] = []
    for v in range(1, n):
        pool = [u for u in range(max(0, v - window), v) if out_left[u] > 0]
        fan = min(len(pool), int(rng.integers(1, max_degree + 1)))
        for u in rng.choice(pool, size=fan, replace=False) if fan else []:
            src.append(int(perm[int(u)])); dst.append(int(perm[v]))
            out_left[int(u)] -= 1
    return csr_from_edges(n, src, dst)


def random_instance(rng: np.random.Generator, n: int, p: int, n_cand: int, max_fanin: int = 3,
                    max_dur: int = 9, max_comm: int = 5, frac_arbitrary: float = 0.3,
                    frac_bad: float = 0.1, dup_prob: float = 0.05, zero_dur: bool = True) -> Workload:
    """Small random instance mixing list-scheduled (acyclic) candidates, arbitrary per-machine
    permutations (mostly cyclic) and malformed candidates (placement out of range, duplicate
    ranks, rank gaps, negative ranks)."""
    row_ptr, col_idx = random_dag(rng, n, max_fanin, dup_prob=dup_prob)
    dur = rng.integers(0 if zero_dur else 1, max_dur + 1, size=n).astype(np.int32)
    comm = rng.integers(0, max_comm + 1, size=(p, p)).astype(np.int32)
    mem = rng.integers(-6, 7, size=n).astype(np.int64)
    seed = int(rng.integers(0, 2 ** 62))
    pl, rk = list_schedules(row_ptr, col_idx, p, n_cand, seed, group=None)
    kind = np.zeros(n_cand, dtype=np.int32)
    for c in range(n_cand):
        r = rng.random()
        if r < frac_arbitrary:
            kind[c] = 1
            for j in range(p):
                idx = np.nonzero(pl[c] == j)[0]
                rk[c, idx] = rng.permutation(len(idx))
        elif r < frac_arbitrary + frac_bad:
            kind[c] = 2
            v = int(rng.integers(0, n))
            how = int(rng.integers(0, 6))
            if how == 0:
                pl[c, v] = -1 - int(rng.integers(0, 3))
            elif how == 1:
                pl[c, v] = p + int(rng.integers(0, 3))
            elif how == 2:
                rk[c, v] = -1 - int(rng.integers(0, 3))
            elif how == 3:
                rk[c, v] = rk[c, v] + 1 + int(rng.integers(0, n))         # gap or duplicate
            elif how == 4:
                w = int(rng.integers(0, n))
                rk[c, v] = rk[c, w]                                       # duplicate when same machine
            else:
                pl[c, v] = int(rng.integers(0, p))                        # moved without re-ranking
    return Workload("random n=%d p=%d" % (n, p), p, row_ptr, col_idx, dur, comm, mem, pl, rk, {"kind": kind})
